// Linear layers of the block on the bf16 matrix cores (gfx950): a token's features and their tangent through
// y = W x + b, ty = W tx (the weights carry no tangent: the network's JVP runs along its inputs), and the backward
// gx = W^T gy, gtx = W^T gty, gW = sum over tokens (gy x^T + gty tx^T), gb = sum over tokens gy.
//
// One kernel serves the three products.  It computes  OUT[i][j] = sum_c P[i][c] Q[j][c]  with either operand stored
// with its contraction index along the rows of a row-major matrix ("row" access: [i][c]) or along the columns'
// direction, i.e. as [c][i] ("transposed" access):
//     forward   OUT = y  [token][f]:  P = x  [token][k] row,         Q = W [f][k] row          (c = k)
//     grad x    OUT = gx [token][k]:  P = gy [token][f] row,         Q = W [f][k] transposed   (c = f)
//     grad W    OUT = gW [f][k]:      P = gy [token][f] transposed,  Q = x [token][k] transposed (c = token)
// The forward and grad x run once over the stacked rows [x; tx] (two row sets, one launch); grad W contracts over
// both sets.  Everything is computed transposed, D = Q-fragment x P-fragment, so that a lane owns one output ROW
// (32 per 32x32 block) and 16 of its columns: results leave through LDS as whole rows (store_tile_coalesced).
//
// Workgroup: four waves as 2 x 2, each with 2 x 4 blocks of 32 x 32 (128 accumulator registers): a 128 x 256 output
// tile, contraction in steps of 32 through two LDS stages filled by asynchronous global->LDS loads (mfma_tiles.h:
// the same swizzled row-major tiles as the attention kernels; "row" fragments are 16-byte reads, "transposed"
// ones the transposing LDS read, here with the contraction index in natural order so that both kinds pair up).
// Per contraction step of 16 a wave reads 2 + 4 fragments for 8 products.  Two workgroups share a CU.
//
// grad W contracts over all tokens of both sets (32K rows at DiT-XL/2 512 px) for few output tiles, so the token
// range is split over several workgroups per tile; each leaves a float32 partial tile in the workspace and a second
// small kernel adds them in a fixed order (no atomics) and rounds once.  gb is a column sum of gy, done the same way.
#include <type_traits>

#include "mfma_tiles.h"

namespace tvm {
namespace {

constexpr int kNW = 4, kNT = 256;
constexpr int kWI = 2, kWJ = 4;              // 32 x 32 blocks per wave along i (lane dimension) and j
constexpr int kTI = 2 * kWI * 32;            // output rows per workgroup (128)
constexpr int kTJ = 2 * kWJ * 32;            // output columns per workgroup (256)
constexpr int kBK = 32;                      // contraction per LDS tile

// Transposed fragment with the contraction index in natural order: lane (ic, hh) gets, of column 32*db + ic of the
// tile, rows 16*cc + 8*hh + 0..7 (the first transposing read takes rows 8hh..8hh+3, the second 8hh+4..8hh+7;
// four consecutive rows share one swizzle term, as in Tile::taddr).
template <class T>
struct TrNat {
  int lo, hi;
  __device__ __forceinline__ static TrNat make(int ic, int hh) {
    const int i = ic & 15, bq = ic >> 4;
    const int y = 2 * bq + ((i & 3) >> 1);
    const int r0 = 8 * hh + (i >> 2), r1 = r0 + 4;
    const int sub = (i & 1) * 8;
    return TrNat{(r0 * T::PCH + (y ^ ((r0 >> 2) & 3))) * 16 + sub, (r1 * T::PCH + (y ^ ((r1 >> 2) & 3))) * 16 + sub};
  }
  __device__ __forceinline__ bf16x8 frag(const char* p, int cc, int db) const {
    typedef bf16x4 __attribute__((address_space(3))) * lp;
    const int imm = cc * 16 * T::PCH * 16 + db * 64;
    const bf16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(p + lo + imm));
    const bf16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(p + hi + imm));
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};

struct GemmArgs {
  const bf16* P[2];   // two row sets (forward, grad x) or two contraction sets (grad W)
  const bf16* Q[2];
  long long ldP, ldQ; // row pitch in elements of the matrices as stored
  int I, J, C;        // output rows, output columns, contraction length per set
  int csets;          // contraction sets (1, or 2 for grad W)
  bf16* out[2];       // one per row set (forward, grad x); row pitch ldo
  long long ldo;
  const bf16* bias;   // added to out[0] only (the tangent has no bias), may be null
  float* part;        // grad W: float32 partial tiles [splits][I][J]
  int splits;
};

template <bool PTR, bool QTR, bool PARTIAL>
__global__ __launch_bounds__(kNT, 2) void gemm_kernel(GemmArgs g) {
  // tiles: "row" access [rows of the operand][kBK], "transposed" access [kBK][columns of the stored matrix]
  using TP = typename std::conditional<PTR, Tile<kBK, kTI / 8, kNW>, Tile<kTI, kBK / 8, kNW>>::type;
  using TQ = typename std::conditional<QTR, Tile<kBK, kTJ / 8, kNW>, Tile<kTJ, kBK / 8, kNW>>::type;
  constexpr int BUF = TP::BYTES + TQ::BYTES;
  constexpr int STAGE_BYTES = 2 * BUF;
  constexpr int OUT_REGION = 32 * (64 * kWJ + 16);  // per wave, for store_tile_coalesced
  constexpr int LDS_BYTES = STAGE_BYTES > kNW * OUT_REGION ? STAGE_BYTES : kNW * OUT_REGION;
  __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave & 1, wj = wave >> 1;
  const int nI = (g.I + kTI - 1) / kTI, nJ = (g.J + kTJ - 1) / kTJ;
  int wg = blockIdx.x;
  const int jt = wg % nJ;
  wg /= nJ;
  const int it = wg % nI;
  const int zz = wg / nI;  // row set (forward, grad x) or split (grad W)
  const int i0 = it * kTI, j0 = jt * kTJ;
  const int nct = (g.C + kBK - 1) / kBK;  // contraction tiles per set
  const int ntot = g.csets * nct;
  const int t_begin = PARTIAL ? (int)((long long)zz * ntot / g.splits) : 0;
  const int t_end = PARTIAL ? (int)((long long)(zz + 1) * ntot / g.splits) : ntot;
  const int pset = PARTIAL ? 0 : zz;

  const unsigned lds0 = lds_addr_of(lds);
  // per-lane byte offsets of this wave's loads within a tile, worked out once
  typename TP::Offs op_full, op_last;
  typename TQ::Offs oq_full, oq_last;
  {
    const unsigned pitchP = (unsigned)(g.ldP * 2), pitchQ = (unsigned)(g.ldQ * 2);
    const int clast = g.C - (nct - 1) * kBK;  // contraction entries in a set's last tile
    if (PTR) {
      const typename TP::Lane l = TP::lane_setup(min(g.I - i0, kTI), wave, lane);  // columns of the stored matrix = output rows
      op_full = TP::offsets(l, pitchP, kBK);
      op_last = TP::offsets(l, pitchP, clast);
    } else {
      const typename TP::Lane l = TP::lane_setup(kBK, wave, lane);
      op_full = op_last = TP::offsets(l, pitchP, g.I - i0);
    }
    if (QTR) {
      const typename TQ::Lane l = TQ::lane_setup(min(g.J - j0, kTJ), wave, lane);
      oq_full = TQ::offsets(l, pitchQ, kBK);
      oq_last = TQ::offsets(l, pitchQ, clast);
    } else {
      const typename TQ::Lane l = TQ::lane_setup(kBK, wave, lane);
      oq_full = oq_last = TQ::offsets(l, pitchQ, g.J - j0);
    }
  }
  auto issue = [&](int t, unsigned buf) {
    const int set = t / nct, ct = t - set * nct;
    const long long c0 = (long long)ct * kBK;
    const bool last = ct == nct - 1;
    const bf16* pb = g.P[PARTIAL ? set : pset] + (PTR ? c0 * g.ldP + i0 : (long long)i0 * g.ldP + c0);
    const bf16* qb = g.Q[PARTIAL ? set : 0] + (QTR ? c0 * g.ldQ + j0 : (long long)j0 * g.ldQ + c0);
#pragma unroll
    for (int x = 0; x < TP::IPW; ++x) TP::issue_at(last ? op_last.o[x] : op_full.o[x], x, pb, buf, wave);
#pragma unroll
    for (int x = 0; x < TQ::IPW; ++x) TQ::issue_at(last ? oq_last.o[x] : oq_full.o[x], x, qb, buf + TP::BYTES, wave);
  };
  const typename TP::RAddr rp = TP::raddr(ic, hh);
  const typename TQ::RAddr rq = TQ::raddr(ic, hh);
  const TrNat<TP> tp = TrNat<TP>::make(ic, hh);
  const TrNat<TQ> tq = TrNat<TQ>::make(ic, hh);

  f32x16 acc[kWI][kWJ];
#pragma unroll
  for (int a = 0; a < kWI; ++a)
#pragma unroll
    for (int b = 0; b < kWJ; ++b) acc[a][b] = zero16();

  if (t_begin < t_end) issue(t_begin, lds0);
  dma_wait();
  __syncthreads();
  for (int t = t_begin, n = 0; t < t_end; ++t, ++n) {
    const char* sp = lds + (n & 1) * BUF;
    const char* sq = sp + TP::BYTES;
    if (t + 1 < t_end) issue(t + 1, lds0 + ((n + 1) & 1) * BUF);  // uniform: lands during this tile
    // a ragged last contraction tile (transposed access only: a row set's token count is arbitrary): entries beyond
    // the set's end were fetched as copies of its last row; the P fragment gets zeros there
    const int ct = t % nct;
    const int cvalid = (PTR && ct == nct - 1) ? g.C - ct * kBK : kBK;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 pf[kWI], qf[kWJ];
#pragma unroll
      for (int a = 0; a < kWI; ++a) {
        pf[a] = PTR ? tp.frag(sp, kk, wi * kWI + a) : TP::frag_row(sp, rp, wi * kWI + a, kk);
        if (PTR && cvalid < kBK) {
          uint4 v = __builtin_bit_cast(uint4, pf[a]);
          const int k0 = kk * 16 + hh * 8;  // contraction index of the fragment's first element
          v.x = k0 + 0 < cvalid ? (k0 + 1 < cvalid ? v.x : v.x & 0xFFFFu) : 0u;
          v.y = k0 + 2 < cvalid ? (k0 + 3 < cvalid ? v.y : v.y & 0xFFFFu) : 0u;
          v.z = k0 + 4 < cvalid ? (k0 + 5 < cvalid ? v.z : v.z & 0xFFFFu) : 0u;
          v.w = k0 + 6 < cvalid ? (k0 + 7 < cvalid ? v.w : v.w & 0xFFFFu) : 0u;
          pf[a] = __builtin_bit_cast(bf16x8, v);
        }
      }
#pragma unroll
      for (int b = 0; b < kWJ; ++b) qf[b] = QTR ? tq.frag(sq, kk, wj * kWJ + b) : TQ::frag_row(sq, rq, wj * kWJ + b, kk);
#pragma unroll
      for (int a = 0; a < kWI; ++a)
#pragma unroll
        for (int b = 0; b < kWJ; ++b) acc[a][b] = mfma(qf[b], pf[a], acc[a][b]);
    }
    dma_wait();
    __syncthreads();  // the next tile has landed; everyone is done with this one
  }

  const int jw = j0 + wj * (kWJ * 32);  // first output column of this wave
  if (PARTIAL) {
    // float32 partial tile: lane = output row, four consecutive columns per register group
    float* dst = g.part + (long long)zz * g.I * g.J;
#pragma unroll
    for (int a = 0; a < kWI; ++a) {
      const int i = i0 + (wi * kWI + a) * 32 + ic;
      if (i >= g.I) continue;
#pragma unroll
      for (int b = 0; b < kWJ; ++b)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int j = jw + b * 32 + 8 * q4 + 4 * hh;
          if (j < g.J) {  // (J is a multiple of 8: four columns are in range together)
            typedef __attribute__((ext_vector_type(4))) float f32x4;
            const f32x4 v = {acc[a][b][4 * q4], acc[a][b][4 * q4 + 1], acc[a][b][4 * q4 + 2], acc[a][b][4 * q4 + 3]};
            *reinterpret_cast<f32x4*>(dst + (long long)i * g.J + j) = v;
          }
        }
    }
  } else {
    if (g.bias != nullptr && pset == 0) {
#pragma unroll
      for (int b = 0; b < kWJ; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jw + b * 32 + drow(r, hh);
          const float bv = j < g.J ? (float)g.bias[j] : 0.f;
#pragma unroll
          for (int a = 0; a < kWI; ++a) acc[a][b][r] += bv;
        }
    }
    // the loop ended with a barrier and no tile load is in flight: each wave stages its rows through a region of its own
    const unsigned lw = lds0 + (unsigned)wave * OUT_REGION;
    if (jw < g.J) {
#pragma unroll
      for (int a = 0; a < kWI; ++a) {
        const int row0 = i0 + (wi * kWI + a) * 32;
        store_tile_coalesced<kWJ>(lw, g.out[pset] + jw, g.ldo, row0, g.I, g.J - jw, acc[a], 1.f, lane);
      }
    }
  }
}

// Adds `splits` float32 partial matrices of n elements in order and rounds once to bf16.  8 elements per thread.
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ part, int splits, long long n,
                                                           bf16* __restrict__ out) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const long long e = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (e >= n) return;
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
  for (int s = 0; s < splits; ++s) {
    const f32x4* p = reinterpret_cast<const f32x4*>(part + (long long)s * n + e);
    s0 += p[0];
    s1 += p[1];
  }
  bf16x8 o;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    o[t] = (bf16)s0[t];
    o[4 + t] = (bf16)s1[t];
  }
  *reinterpret_cast<bf16x8*>(out + e) = o;
}

// Column sums of gy [R][F] over `chunks` row ranges: part[chunk][f] (float32).  A thread per column.
__global__ __launch_bounds__(256) void colsum_kernel(const bf16* __restrict__ gy, int R, int F, long long ld, int chunks,
                                                     float* __restrict__ part) {
  const int f = blockIdx.x * 256 + threadIdx.x, ch = blockIdx.y;
  if (f >= F) return;
  const int r0 = (int)((long long)ch * R / chunks), r1 = (int)((long long)(ch + 1) * R / chunks);
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += (float)gy[(long long)r * ld + f];
  part[(long long)ch * F + f] = s;
}

int dw_splits(int F, int K, int R) {
  const int tiles = ((F + kTI - 1) / kTI) * ((K + kTJ - 1) / kTJ);
  const int ntot = 2 * ((R + kBK - 1) / kBK);
  int s = (384 + tiles - 1) / tiles;
  s = s > 16 ? 16 : s;
  s = s > ntot ? ntot : s;
  return s < 1 ? 1 : s;
}
int bias_chunks(int R) {
  const int c = (R + 127) / 128;
  return c > 64 ? 64 : c;
}

}  // namespace

// Row pitches (elements) up to 2^20: a tile's per-lane byte offsets (row within the tile x pitch) stay inside 32 bits.
bool linear_supported(int R, int K, int F, long long ldx, long long ldy, int dtype) {
  return dtype == 1 && R >= 1 && K >= 32 && F >= 32 && K % 32 == 0 && F % 32 == 0 && ldx >= K && ldy >= F &&
         ldx % 8 == 0 && ldy % 8 == 0 && ldx <= (1ll << 20) && ldy <= (1ll << 20) && K <= (1 << 20) && F <= (1 << 20);
}

size_t linear_bwd_workspace_bytes(int R, int K, int F) {
  const size_t dw = (size_t)dw_splits(F, K, R) * F * K * sizeof(float);
  const size_t db = (size_t)bias_chunks(R) * F * sizeof(float);
  return ((dw + 255) & ~(size_t)255) + ((db + 255) & ~(size_t)255);
}

hipError_t launch_linear_fwd(int R, int K, int F, long long ldx, long long ldy, const void* x, const void* tx,
                             const void* w, const void* bias, void* y, void* ty, hipStream_t st) {
  GemmArgs g{};
  g.P[0] = (const bf16*)x;
  g.P[1] = (const bf16*)tx;
  g.Q[0] = g.Q[1] = (const bf16*)w;
  g.ldP = ldx;
  g.ldQ = K;
  g.I = R;
  g.J = F;
  g.C = K;
  g.csets = 1;
  g.out[0] = (bf16*)y;
  g.out[1] = (bf16*)ty;
  g.ldo = ldy;
  g.bias = (const bf16*)bias;
  const int grid = 2 * ((R + kTI - 1) / kTI) * ((F + kTJ - 1) / kTJ);
  hipLaunchKernelGGL((gemm_kernel<false, false, false>), dim3(grid), dim3(kNT), 0, st, g);
  return hipGetLastError();
}

hipError_t launch_linear_bwd(int R, int K, int F, long long ldx, long long ldy, const void* x, const void* tx,
                             const void* w, const void* gy, const void* gty, void* gx, void* gtx, void* gw, void* gbias,
                             void* workspace, hipStream_t st) {
  {  // gx = gy W, gtx = gty W: rows = tokens, contraction over f, W read transposed
    GemmArgs g{};
    g.P[0] = (const bf16*)gy;
    g.P[1] = (const bf16*)gty;
    g.Q[0] = g.Q[1] = (const bf16*)w;
    g.ldP = ldy;
    g.ldQ = K;
    g.I = R;
    g.J = K;
    g.C = F;
    g.csets = 1;
    g.out[0] = (bf16*)gx;
    g.out[1] = (bf16*)gtx;
    g.ldo = ldx;
    const int grid = 2 * ((R + kTI - 1) / kTI) * ((K + kTJ - 1) / kTJ);
    hipLaunchKernelGGL((gemm_kernel<false, true, false>), dim3(grid), dim3(kNT), 0, st, g);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int splits = dw_splits(F, K, R);
  float* part = static_cast<float*>(workspace);
  {  // gW = gy^T x + gty^T tx: contraction over the tokens of both sets, both operands read transposed
    GemmArgs g{};
    g.P[0] = (const bf16*)gy;
    g.P[1] = (const bf16*)gty;
    g.Q[0] = (const bf16*)x;
    g.Q[1] = (const bf16*)tx;
    g.ldP = ldy;
    g.ldQ = ldx;
    g.I = F;
    g.J = K;
    g.C = R;
    g.csets = 2;
    g.part = part;
    g.splits = splits;
    const int grid = splits * ((F + kTI - 1) / kTI) * ((K + kTJ - 1) / kTJ);
    hipLaunchKernelGGL((gemm_kernel<true, true, true>), dim3(grid), dim3(kNT), 0, st, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long n = (long long)F * K;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, st, part, splits, n,
                       (bf16*)gw);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (gbias != nullptr) {
    const size_t dw = ((size_t)splits * F * K * sizeof(float) + 255) & ~(size_t)255;
    float* bp = reinterpret_cast<float*>(static_cast<char*>(workspace) + dw);
    const int chunks = bias_chunks(R);
    hipLaunchKernelGGL(colsum_kernel, dim3((F + 255) / 256, chunks), dim3(256), 0, st, (const bf16*)gy, R, F, ldy, chunks, bp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((F / 8 + 255) / 256)), dim3(256), 0, st, bp, chunks, (long long)F,
                       (bf16*)gbias);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace tvm
