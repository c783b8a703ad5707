// bf16 matrix-core building blocks shared by the forward and backward kernels (gfx950).
//
// One instruction is used throughout: v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] B[16x32].
// Operand layout per lane (lane = 32*hh + ic):
//   A: row ic of A, eight consecutive k starting at 8*hh          (8 bf16 = 16 bytes)
//   B: column ic of B, the same eight k
//   D: column ic of D, rows 8*(r/4) + 4*hh + (r%4) for register r = 0..15
// Since A and B index k the same way, any fixed permutation of k applied to both operands
// leaves the product unchanged.  That is used to feed a D-layout tile straight back in as an
// operand: registers 8c..8c+7 of a D tile are, for this lane, the eight "rows"
// 16c + {0,1,2,3, 8,9,10,11} + 4*hh, so the other operand is stored in LDS with its
// contraction index permuted to match ("slot order", see slot_pos below).
#pragma once
#include "tvm_common.h"

namespace tvm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row (M index) held in register r of a D tile by a lane of half hh.
__device__ __forceinline__ int drow(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

// Position, within a transposed LDS row, of contraction index x (0 <= x < multiple of 16):
// x = 16c + 8g + 4h + t  ->  16c + 8h + 4g + t.  Runs of four consecutive x stay contiguous, and
// the eight values a lane of half h needs for 16-chunk c are the 16 bytes at 16c + 8h.
__device__ __forceinline__ int slot_pos(int x) {
  return (x & ~15) | ((x & 4) << 1) | ((x & 8) >> 1) | (x & 3);
}

// Copies rows [r0, r0+ROWS) of a [N,D] bf16 matrix (row pitch sn) into dst[ROWS][PITCH], columns
// [0,DK), zero-filling rows >= N and columns >= D.  D must be a multiple of 8.
template <int ROWS, int DK, int PITCH, int NT>
__device__ __forceinline__ void load_rows(bf16* dst, const bf16* __restrict__ src, long long sn, int r0, int N, int D,
                                          int tid) {
  constexpr int CH = DK / 8;
  for (int idx = tid; idx < ROWS * CH; idx += NT) {
    const int r = idx / CH, c = idx - r * CH;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r0 + r < N && c * 8 < D) val = *reinterpret_cast<const uint4*>(src + (long long)(r0 + r) * sn + c * 8);
    *reinterpret_cast<uint4*>(dst + r * PITCH + c * 8) = val;
  }
}

// Same source rows, stored transposed and in slot order: dst[d][slot_pos(r)] for d in [0,DV).
// Each thread takes four consecutive rows times eight columns and writes eight 8-byte runs.
template <int ROWS, int DV, int PITCH, int NT>
__device__ __forceinline__ void load_transposed(bf16* dst, const bf16* __restrict__ src, long long sn, int r0, int N,
                                                int D, int tid) {
  constexpr int OCT = DV / 8;
  for (int idx = tid; idx < (ROWS / 4) * OCT; idx += NT) {
    const int qd = idx / OCT, oc = idx - qd * OCT;
    uint32_t w[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int row = r0 + 4 * qd + t;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (row < N && oc * 8 < D) val = *reinterpret_cast<const uint4*>(src + (long long)row * sn + oc * 8);
      w[t][0] = val.x;
      w[t][1] = val.y;
      w[t][2] = val.z;
      w[t][3] = val.w;
    }
    const int pos = slot_pos(4 * qd);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int wi = e >> 1;
      uint2 out;
      if (e & 1) {
        out.x = (w[0][wi] >> 16) | (w[1][wi] & 0xffff0000u);
        out.y = (w[2][wi] >> 16) | (w[3][wi] & 0xffff0000u);
      } else {
        out.x = (w[0][wi] & 0xffffu) | (w[1][wi] << 16);
        out.y = (w[2][wi] & 0xffffu) | (w[3][wi] << 16);
      }
      *reinterpret_cast<uint2*>(dst + (oc * 8 + e) * PITCH + pos) = out;
    }
  }
}

__device__ __forceinline__ bf16x8 lds_frag(const bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }

// Eight bf16 from global memory (16-byte aligned) or zeros.
__device__ __forceinline__ bf16x8 gld_frag(const bf16* p, bool ok) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (ok) v = *reinterpret_cast<const uint4*>(p);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32); }

}  // namespace tvm
