// RMSNorm with a learnable gain as QK-norm (Terminal Velocity Matching, Sec. "Semi-Lipschitz control";
// definition and Jacobian in App. "Lipschitzness of RMSNorm"), with its JVP tangent and its backward, for
// the rows of q and of k in one launch.  Per row x in R^d, with r = 1 / sqrt(mean(x^2) + eps) and
// m = mean(x tx):
//     y  = g o x r                          ty = g o (tx r - x r^3 m)
// Backward of <gy, y> + <gty, ty>, with u = g o gy, w = g o gty, A = <u, x>, Bw = <w, x>, C = <w, tx>:
//     gtx = r w - (r^3 Bw / d) x
//     gx  = r u - r^3 m w - (r^3 Bw / d) tx + x (3 r^5 m Bw - r^3 (A + C)) / d
//     gg  = sum over rows of  gy o x r + gty o (tx r - x r^3 m)
// Memory-bound: every tensor is read once and written once, 16 bytes per lane, 16 lanes to a row (their
// sums meet by lane exchange), float32 arithmetic whatever the storage type.  The gain gradient is summed
// without atomics: each thread keeps the column sums of the rows it worked on, a workgroup adds its 16 row
// slots in LDS and writes one partial row, and a second small kernel adds the partial rows in order, so
// the result does not depend on timing.
#include "tvm_common.h"

#ifndef QKNORM_NT
#define QKNORM_NT 1
#endif

namespace tvm {
namespace {

constexpr int kNT = 256;
constexpr int kLpr = 16;  // lanes per row

template <typename T>
struct alignas(16) Chunk {  // 16 bytes of T, 16-byte aligned: one load or store instruction
  static constexpr int VEC = 16 / sizeof(T);
  T v[VEC];
};

// Elements [c0, c0 + VEC) of the row at p as float32, zero beyond D.  Whole chunks are one 16-byte load
// (rows start on 16-byte boundaries); a chunk that crosses D is read element by element.  FULL: D is a
// multiple of VEC, every chunk is whole or empty, and the load is unconditional (an empty chunk reads the
// row's first one and discards it), so that the loads of a row are all in flight before the first is used.
template <typename T, bool FULL>
__device__ __forceinline__ void load_chunk(float (&out)[Chunk<T>::VEC], const T* p, int c0, int D) {
  constexpr int VEC = Chunk<T>::VEC;
  if (FULL) {
    const bool live = c0 < D;
#if QKNORM_NT  // the rows are touched once: non-temporal (backward 96 -> 91 us at C4, forward unchanged)
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    uint4 raw = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + (live ? c0 : 0))));
#else
    uint4 raw = *reinterpret_cast<const uint4*>(p + (live ? c0 : 0));  // one 16-byte load
#endif
    raw.x = live ? raw.x : 0u;
    raw.y = live ? raw.y : 0u;
    raw.z = live ? raw.z : 0u;
    raw.w = live ? raw.w : 0u;
    const Chunk<T> c = __builtin_bit_cast(Chunk<T>, raw);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = (float)c.v[e];
  } else if (c0 + VEC <= D) {
    const Chunk<T> c = *reinterpret_cast<const Chunk<T>*>(p + c0);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = (float)c.v[e];
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = c0 + e < D ? (float)p[c0 + e] : 0.f;
  }
}
template <typename T, bool FULL>
__device__ __forceinline__ void store_chunk(T* p, int c0, int D, const float (&in)[Chunk<T>::VEC]) {
  constexpr int VEC = Chunk<T>::VEC;
  if (FULL || c0 + VEC <= D) {  // (callers skip chunks that start at or beyond D)
    Chunk<T> c;
#pragma unroll
    for (int e = 0; e < VEC; ++e) c.v[e] = (T)in[e];  // round to nearest even
    *reinterpret_cast<uint4*>(p + c0) = __builtin_bit_cast(uint4, c);  // one 16-byte store
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (c0 + e < D) p[c0 + e] = (T)in[e];
  }
}
// Sum over the 16 lanes of a row (lanes 16k .. 16k+15 of the wave), the same bits in all of them: a butterfly
// of four data-parallel-primitive moves (neighbour, pair, mirrored half, mirrored row; after the first two a
// quad holds one value, so the mirrors pair whole quads and halves), no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row_sum(float x) {
  x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);  // row_half_mirror
  x += dpp_move<0x140>(x);  // row_mirror
  return x;
}

struct RowIter {  // the rows of one side that this thread's row slot works on
  long long row, end, step;
};
__device__ __forceinline__ long long row_offset(const NormArgs& a, const NormSide& s, long long row) {
  const unsigned r = (unsigned)row;  // fewer than 2^31 rows per side: 32-bit divisions
  const unsigned bh = r / (unsigned)s.n, i = r - bh * (unsigned)s.n;
  const unsigned b = bh / (unsigned)a.H, h = bh - b * (unsigned)a.H;
  return (long long)b * s.sb + (long long)h * s.sh + (long long)i * s.sn;
}

// MAXC: chunks per lane (16 lanes x MAXC x VEC >= D).
template <typename T, int MAXC, bool FULL>
__global__ __launch_bounds__(kNT) void qknorm_fwd_kernel(NormArgs a) {
  constexpr int VEC = Chunk<T>::VEC;
  const int sd = (int)blockIdx.x >= a.side[0].nwg ? 1 : 0;
  const NormSide s = sd ? a.side[1] : a.side[0];  // (a select per field: the arguments stay in scalar registers)
  const int wg = blockIdx.x - (sd ? a.side[0].nwg : 0);
  const int lr = threadIdx.x & (kLpr - 1), slot = threadIdx.x / kLpr;
  const long long R = (long long)a.B * a.H * s.n;
  const float invd = 1.0f / (float)a.D;
  float g[MAXC][VEC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const int col = (lr + kLpr * c) * VEC + e;
      g[c][e] = col < a.D ? s.g[col] : 0.f;
    }
  for (long long row = (long long)wg * kNormRowsPerWg + slot; row < R; row += (long long)s.nwg * kNormRowsPerWg) {
    const long long off = row_offset(a, s, row);
    const T* xp = static_cast<const T*>(s.x) + off;
    const T* tp = static_cast<const T*>(s.tx) + off;
    float x[MAXC][VEC], t[MAXC][VEC];
    float sxx = 0.f, sxt = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int c0 = (lr + kLpr * c) * VEC;
      load_chunk<T, FULL>(x[c], xp, c0, a.D);
      load_chunk<T, FULL>(t[c], tp, c0, a.D);
    }
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        sxx = fmaf(x[c][e], x[c][e], sxx);
        sxt = fmaf(x[c][e], t[c][e], sxt);
      }
    sxx = row_sum(sxx);
    sxt = row_sum(sxt);
    const float r = 1.0f / sqrtf(sxx * invd + a.eps);
    const float r3m = r * r * r * (sxt * invd);
    T* yp = static_cast<T*>(s.y) + off;
    T* typ = static_cast<T*>(s.ty) + off;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int c0 = (lr + kLpr * c) * VEC;
      if (c0 >= a.D) continue;
      float y[VEC], ty[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        y[e] = g[c][e] * (x[c][e] * r);
        ty[e] = g[c][e] * (t[c][e] * r - x[c][e] * r3m);
      }
      store_chunk<T, FULL>(yp, c0, a.D, y);
      store_chunk<T, FULL>(typ, c0, a.D, ty);
    }
  }
}

template <typename T, int MAXC, bool FULL>
__global__ __launch_bounds__(kNT) void qknorm_bwd_kernel(NormArgs a) {
  constexpr int VEC = Chunk<T>::VEC;
  __shared__ float red[kNT / kLpr][kLpr * MAXC * VEC];  // one row of column sums per row slot
  const int sd = (int)blockIdx.x >= a.side[0].nwg ? 1 : 0;
  const NormSide s = sd ? a.side[1] : a.side[0];  // (a select per field: the arguments stay in scalar registers)
  const int wg = blockIdx.x - (sd ? a.side[0].nwg : 0);
  const int lr = threadIdx.x & (kLpr - 1), slot = threadIdx.x / kLpr;
  const long long R = (long long)a.B * a.H * s.n;
  const float invd = 1.0f / (float)a.D;
  float g[MAXC][VEC], acc[MAXC][VEC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const int col = (lr + kLpr * c) * VEC + e;
      g[c][e] = col < a.D ? s.g[col] : 0.f;
      acc[c][e] = 0.f;
    }
  for (long long row = (long long)wg * kNormRowsPerWg + slot; row < R; row += (long long)s.nwg * kNormRowsPerWg) {
    const long long off = row_offset(a, s, row);
    const T* xp = static_cast<const T*>(s.x) + off;
    const T* tp = static_cast<const T*>(s.tx) + off;
    const T* gyp = static_cast<const T*>(s.gy) + off;
    const T* gtp = static_cast<const T*>(s.gty) + off;
    float x[MAXC][VEC], t[MAXC][VEC], gy[MAXC][VEC], gt[MAXC][VEC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int c0 = (lr + kLpr * c) * VEC;
      load_chunk<T, FULL>(x[c], xp, c0, a.D);
      load_chunk<T, FULL>(t[c], tp, c0, a.D);
      load_chunk<T, FULL>(gy[c], gyp, c0, a.D);
      load_chunk<T, FULL>(gt[c], gtp, c0, a.D);
    }
    float sxx = 0.f, sxt = 0.f, sA = 0.f, sB = 0.f, sC = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = g[c][e] * gy[c][e], w = g[c][e] * gt[c][e];
        sxx = fmaf(x[c][e], x[c][e], sxx);
        sxt = fmaf(x[c][e], t[c][e], sxt);
        sA = fmaf(u, x[c][e], sA);
        sB = fmaf(w, x[c][e], sB);
        sC = fmaf(w, t[c][e], sC);
      }
    sxx = row_sum(sxx);
    sxt = row_sum(sxt);
    sA = row_sum(sA);
    sB = row_sum(sB);
    sC = row_sum(sC);
    const float r = 1.0f / sqrtf(sxx * invd + a.eps);
    const float r3 = r * r * r, m = sxt * invd;
    const float r3m = r3 * m;
    const float kB = r3 * sB * invd;                                      // r^3 Bw / d
    const float kx = (3.0f * r3 * r * r * m * sB - r3 * (sA + sC)) * invd;  // coefficient of x in gx
    T* gxp = static_cast<T*>(s.y) + off;
    T* gtxp = static_cast<T*>(s.ty) + off;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int c0 = (lr + kLpr * c) * VEC;
      if (c0 >= a.D) continue;
      float gx[VEC], gtx[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = g[c][e] * gy[c][e], w = g[c][e] * gt[c][e];
        gtx[e] = r * w - kB * x[c][e];
        gx[e] = r * u - r3m * w - kB * t[c][e] + kx * x[c][e];
        acc[c][e] += gy[c][e] * (x[c][e] * r) + gt[c][e] * (t[c][e] * r - x[c][e] * r3m);
      }
      store_chunk<T, FULL>(gxp, c0, a.D, gx);
      store_chunk<T, FULL>(gtxp, c0, a.D, gtx);
    }
  }
  // column sums of this workgroup: the 16 row slots added in order
#pragma unroll
  for (int c = 0; c < MAXC; ++c)
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[slot][(lr + kLpr * c) * VEC + e] = acc[c][e];
  __syncthreads();
  for (int col = threadIdx.x; col < a.D; col += kNT) {
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < kNT / kLpr; ++k) sum += red[k][col];
    s.part[(long long)wg * a.D + col] = sum;
  }
}

// gg[col] = sum over the partial rows, in a fixed order: a workgroup takes 64 columns of one side, its 16 row
// slices each add every 16th partial row (eight loads in flight at a time), and the slices are added in order.
constexpr int kRedCols = 64, kRedSlices = 16;
__global__ __launch_bounds__(kRedCols * kRedSlices) void qknorm_gain_grad_kernel(NormArgs a) {
  __shared__ float red[kRedSlices][kRedCols];
  const NormSide s = blockIdx.x ? a.side[1] : a.side[0];
  const int lc = threadIdx.x % kRedCols, sl = threadIdx.x / kRedCols;
  const int col = blockIdx.y * kRedCols + lc;
  float sum = 0.f;
  if (col < a.D) {
    int w = sl;
    for (; w + 7 * kRedSlices < s.nwg; w += 8 * kRedSlices) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = s.part[(long long)(w + u * kRedSlices) * a.D + col];
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += v[u];
    }
    for (; w < s.nwg; w += kRedSlices) sum += s.part[(long long)w * a.D + col];
  }
  red[sl][lc] = sum;
  __syncthreads();
  if (sl == 0 && col < a.D) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < kRedSlices; ++k) t += red[k][lc];
    s.gg[col] = t;
  }
}

// The same for D a multiple of 4 (16-byte aligned partial rows): a thread takes one 16-byte chunk of columns and one
// slice of the rows, as many slices as 1024 threads give (56 at D = 72: 18 rows each of 1024, all loads of a slice in
// flight within two or three round trips instead of eight); the slices meet in LDS and are added in order.
constexpr int kRed4NT = 1024;
__global__ __launch_bounds__(kRed4NT) void qknorm_gain_grad4_kernel(NormArgs a) {
  __shared__ float red[kRed4NT * 4];  // [slices][D], slices * D <= 4096
  const NormSide s = blockIdx.x ? a.side[1] : a.side[0];
  const int nch = a.D >> 2, slices = kRed4NT / nch;
  const int ch = threadIdx.x % nch, sl = threadIdx.x / nch;
  if (sl < slices) {
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4* p = reinterpret_cast<const float4*>(s.part) + ch;
    int w = sl;
    for (; w + 7 * slices < s.nwg; w += 8 * slices) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(long long)(w + u * slices) * nch];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        sum.x += v[u].x;
        sum.y += v[u].y;
        sum.z += v[u].z;
        sum.w += v[u].w;
      }
    }
    for (; w < s.nwg; w += slices) {
      const float4 v = p[(long long)w * nch];
      sum.x += v.x;
      sum.y += v.y;
      sum.z += v.z;
      sum.w += v.w;
    }
    *reinterpret_cast<float4*>(red + sl * a.D + 4 * ch) = sum;
  }
  __syncthreads();
  if ((int)threadIdx.x < a.D) {
    float t = 0.f;
    for (int k = 0; k < slices; ++k) t += red[k * a.D + threadIdx.x];
    s.gg[threadIdx.x] = t;
  }
}

}  // namespace

// Kernel choice: chunks per lane from D, and whether D is a whole number of 16-byte chunks.
#define TVM_NORM_LAUNCH(KERNEL, T, MAXC)                                                         \
  do {                                                                                           \
    if (a.D % Chunk<T>::VEC == 0) hipLaunchKernelGGL((KERNEL<T, MAXC, true>), grid, block, 0, st, a); \
    else hipLaunchKernelGGL((KERNEL<T, MAXC, false>), grid, block, 0, st, a);                   \
  } while (0)
#define TVM_NORM_BY_TYPE(KERNEL)                                   \
  do {                                                             \
    if (dtype == 1) {                                              \
      if (a.D <= 128) TVM_NORM_LAUNCH(KERNEL, bf16, 1);            \
      else TVM_NORM_LAUNCH(KERNEL, bf16, 2);                       \
    } else {                                                       \
      if (a.D <= 64) TVM_NORM_LAUNCH(KERNEL, float, 1);            \
      else if (a.D <= 128) TVM_NORM_LAUNCH(KERNEL, float, 2);      \
      else TVM_NORM_LAUNCH(KERNEL, float, 4);                      \
    }                                                              \
  } while (0)

hipError_t launch_qknorm_fwd(const NormArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.side[0].nwg + a.side[1].nwg), block(kNT);
  TVM_NORM_BY_TYPE(qknorm_fwd_kernel);
  return hipGetLastError();
}

namespace {
void launch_gain_grad(const NormArgs& a, hipStream_t st) {
  if (a.D % 4 == 0 && a.D <= 1024)  // (the norm kernels take D <= 256)
    hipLaunchKernelGGL(qknorm_gain_grad4_kernel, dim3(2), dim3(kRed4NT), 0, st, a);
  else
    hipLaunchKernelGGL(qknorm_gain_grad_kernel, dim3(2, (a.D + kRedCols - 1) / kRedCols), dim3(kRedCols * kRedSlices), 0,
                       st, a);
}
}  // namespace

hipError_t launch_qknorm_bwd(const NormArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.side[0].nwg + a.side[1].nwg), block(kNT);
  TVM_NORM_BY_TYPE(qknorm_bwd_kernel);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  launch_gain_grad(a, st);
  return hipGetLastError();
}


// The same ordered sum for partial rows that other kernels wrote (the attention backward kernels with the
// QK-norm's backward in their epilogues: one row per workgroup).
hipError_t launch_gain_grad_sum(const float* part_q, int rows_q, float* gg_q, const float* part_k, int rows_k, float* gg_k,
                                int D, hipStream_t st) {
  NormArgs a{};
  a.D = D;
  a.side[0].part = const_cast<float*>(part_q);
  a.side[0].nwg = rows_q;
  a.side[0].gg = gg_q;
  a.side[1].part = const_cast<float*>(part_k);
  a.side[1].nwg = rows_k;
  a.side[1].gg = gg_k;
  launch_gain_grad(a, st);
  return hipGetLastError();
}

}  // namespace tvm
