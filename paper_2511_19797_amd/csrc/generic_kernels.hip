// Plain-ALU kernels: one wavefront per query row (or per key row), float32
// arithmetic throughout.  They serve the float32 dtype and every bf16 shape the
// matrix-core kernels do not take (head dims that are not a multiple of 8 or
// exceed 128).  Formulas: App. C of the paper -- the equations under "Step 1"
// for S, Sdot, P, N; Steps 2-6 for the six gradients, with the row sums
// Sigma_1, Sigma_2 collapsed to row dot products (Sigma_1 = gTO.O,
// Sigma_2 = gTO.tO, since O = P V and tO = (P o N) V + P tV).
#include "tvm_common.h"

namespace tvm {
namespace {

constexpr int kRowsPerBlock = 4;  // one wave each
constexpr int kDMax = 256;
constexpr int kTile = 64;         // keys (or queries) handled per step, one per lane

// ---------------------------------------------------------------------------------------
// Forward: wave w of the block owns query row i.  Per 64-key tile, lane j forms the scaled
// scores z_ij, zt_ij by a dot product over d, the wave does one online-softmax update, and
// then all lanes (now indexing d) accumulate sum_j p_ij V_j and sum_j (p zt)_ij V_j + p_ij tV_j.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void fwd_generic_kernel(Shape s, const T* __restrict__ q, const T* __restrict__ k,
                                                         const T* __restrict__ v, const T* __restrict__ tq,
                                                         const T* __restrict__ tk, const T* __restrict__ tv,
                                                         T* __restrict__ o, T* __restrict__ to,
                                                         float* __restrict__ lse, float* __restrict__ stats) {
  __shared__ float qs[kRowsPerBlock][kDMax], tqs[kRowsPerBlock][kDMax];
  __shared__ float ps[kRowsPerBlock][kTile], pzs[kRowsPerBlock][kTile];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblk = (s.M + kRowsPerBlock - 1) / kRowsPerBlock;
  const int bh = blockIdx.x / nblk, b = bh / s.H, h = bh % s.H;
  const int i = (blockIdx.x % nblk) * kRowsPerBlock + w;
  const long long base = b * s.sb + h * s.sh, qbase = b * s.qsb + h * s.qsh;  // key side, query side
  const bool rowok = i < s.M;
  for (int c = lane; c < s.D; c += 64) {
    qs[w][c] = rowok ? ldf(q + qbase + i * s.qsn + c) : 0.f;
    tqs[w][c] = rowok ? ldf(tq + qbase + i * s.qsn + c) : 0.f;
  }
  __syncthreads();
  float m = -INFINITY, l = 0.f, cs = 0.f;
  float ao[kDMax / 64] = {}, at[kDMax / 64] = {};
  for (int j0 = 0; j0 < s.N; j0 += kTile) {
    const int j = j0 + lane;
    float z = -INFINITY, zt = 0.f;
    if (j < s.N) {
      const T* kr = k + base + j * s.sn;
      const T* tkr = tk + base + j * s.sn;
      float a0 = 0.f, a1 = 0.f;
      for (int c = 0; c < s.D; ++c) {
        const float kc = ldf(kr + c);
        a0 = fmaf(qs[w][c], kc, a0);
        a1 = fmaf(tqs[w][c], kc, a1);
        a1 = fmaf(qs[w][c], ldf(tkr + c), a1);
      }
      z = a0 * s.alpha;
      zt = a1 * s.alpha;
    }
    const float mn = fmaxf(m, wave_max(z));
    const float f = __expf(m - mn);  // m = -inf on the first tile gives 0
    const float p = (j < s.N) ? __expf(z - mn) : 0.f;
    const float pz = p * zt;
    l = l * f + wave_sum(p);
    cs = cs * f + wave_sum(pz);
    m = mn;
    ps[w][lane] = p;
    pzs[w][lane] = pz;
    __syncthreads();
    const int jn = min(kTile, s.N - j0);
#pragma unroll
    for (int t = 0; t < kDMax / 64; ++t) {
      ao[t] *= f;
      at[t] *= f;
    }
    for (int jj = 0; jj < jn; ++jj) {
      const float pj = ps[w][jj], pzj = pzs[w][jj];
      const long long ro = base + (long long)(j0 + jj) * s.sn;
#pragma unroll
      for (int t = 0; t < kDMax / 64; ++t) {
        const int c = lane + 64 * t;
        if (c < s.D) {
          const float vv = ldf(v + ro + c), tvv = ldf(tv + ro + c);
          ao[t] = fmaf(pj, vv, ao[t]);
          at[t] = fmaf(pzj, vv, at[t]);
          at[t] = fmaf(pj, tvv, at[t]);
        }
      }
    }
    __syncthreads();
  }
  if (!rowok) return;
  const float inv = 1.f / l;
  const float mubar = cs * inv;
#pragma unroll
  for (int t = 0; t < kDMax / 64; ++t) {
    const int c = lane + 64 * t;
    if (c < s.D) {
      const float oc = ao[t] * inv;
      stf(o + qbase + i * s.qsn + c, oc);
      stf(to + qbase + i * s.qsn + c, at[t] * inv - mubar * oc);
    }
  }
  if (lane == 0) {
    const long long r = (long long)bh * s.M + i;
    if (lse) lse[r] = m + __logf(l);
    if (stats) stats[r] = mubar;
  }
}

// A tensor that one-sided calls leave out (null) reads as zero.
template <typename T>
__device__ __forceinline__ float ldz(const T* p, long long i) {
  return p ? ldf(p + i) : 0.f;
}

// ---------------------------------------------------------------------------------------
// Step 1 (row scalars).  dsig_i = gO_i.O_i + gTO_i.tO_i  (delta + Sigma_2);  sig1_i = gTO_i.O_i.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bwd_pre_kernel(Shape s, const T* __restrict__ o, const T* __restrict__ to,
                                                     const T* __restrict__ gO, const T* __restrict__ gTO,
                                                     float* __restrict__ dsig, float* __restrict__ sig1) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblk = (s.M + kRowsPerBlock - 1) / kRowsPerBlock;
  const int bh = blockIdx.x / nblk, b = bh / s.H, h = bh % s.H;
  const int i = (blockIdx.x % nblk) * kRowsPerBlock + w;
  if (i >= s.M) return;
  const long long ro = b * s.qsb + h * s.qsh + (long long)i * s.qsn;
  float a = 0.f, c1 = 0.f;
  for (int c = lane; c < s.D; c += 64) {
    const float oc = ldf(o + ro + c), toc = ldz(to, ro + c);
    const float g = ldz(gO, ro + c), gt = ldz(gTO, ro + c);
    a = fmaf(g, oc, a);
    a = fmaf(gt, toc, a);
    c1 = fmaf(gt, oc, c1);
  }
  a = wave_sum(a);
  c1 = wave_sum(c1);
  if (lane == 0) {
    const long long r = (long long)bh * s.M + i;
    dsig[r] = a;
    sig1[r] = c1;
  }
}

// ---------------------------------------------------------------------------------------
// Query side (Steps 3 and 5): wave per query row i; lane j rebuilds the tile column
// (P, N, gZt = P (E - Sigma_1), gZ = P (DF - delta - Sigma_2) + gZt N), then lanes index d.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bwd_row_generic_kernel(Shape s, const T* __restrict__ q, const T* __restrict__ k,
                                                             const T* __restrict__ v, const T* __restrict__ tq,
                                                             const T* __restrict__ tk, const T* __restrict__ tv,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ stats,
                                                             const T* __restrict__ gO, const T* __restrict__ gTO,
                                                             const float* __restrict__ dsig,
                                                             const float* __restrict__ sig1, T* __restrict__ dq,
                                                             T* __restrict__ dtq) {
  __shared__ float qs[kRowsPerBlock][kDMax], tqs[kRowsPerBlock][kDMax];
  __shared__ float gs[kRowsPerBlock][kDMax], tgs[kRowsPerBlock][kDMax];
  __shared__ float gzs[kRowsPerBlock][kTile], gzts[kRowsPerBlock][kTile];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblk = (s.M + kRowsPerBlock - 1) / kRowsPerBlock;
  const int bh = blockIdx.x / nblk, b = bh / s.H, h = bh % s.H;
  const int i = (blockIdx.x % nblk) * kRowsPerBlock + w;
  const long long base = b * s.sb + h * s.sh, qbase = b * s.qsb + h * s.qsh;  // key side, query side
  const bool rowok = i < s.M;
  for (int c = lane; c < s.D; c += 64) {
    const long long a = qbase + (long long)i * s.qsn + c;
    qs[w][c] = rowok ? ldf(q + a) : 0.f;
    tqs[w][c] = rowok ? ldz(tq, a) : 0.f;
    gs[w][c] = rowok ? ldz(gO, a) : 0.f;
    tgs[w][c] = rowok ? ldz(gTO, a) : 0.f;
  }
  const long long r = (long long)bh * s.M + (rowok ? i : 0);
  const float lse_i = lse[r], mubar_i = stats ? stats[r] : 0.f, dsig_i = dsig[r], sig1_i = sig1[r];
  __syncthreads();
  float aq[kDMax / 64] = {}, atq[kDMax / 64] = {};
  for (int j0 = 0; j0 < s.N; j0 += kTile) {
    const int j = j0 + lane;
    float gz = 0.f, gzt = 0.f;
    if (j < s.N) {
      const long long ro = base + (long long)j * s.sn;
      float a0 = 0.f, a1 = 0.f, df = 0.f, e = 0.f;
      for (int c = 0; c < s.D; ++c) {
        const float kc = ldf(k + ro + c), tkc = ldz(tk, ro + c);
        const float vc = ldf(v + ro + c), tvc = ldz(tv, ro + c);
        a0 = fmaf(qs[w][c], kc, a0);
        a1 = fmaf(tqs[w][c], kc, a1);
        a1 = fmaf(qs[w][c], tkc, a1);
        df = fmaf(gs[w][c], vc, df);
        df = fmaf(tgs[w][c], tvc, df);
        e = fmaf(tgs[w][c], vc, e);
      }
      const float p = __expf(a0 * s.alpha - lse_i);
      const float n = a1 * s.alpha - mubar_i;
      gzt = p * (e - sig1_i);
      gz = fmaf(gzt, n, p * (df - dsig_i));
    }
    gzs[w][lane] = gz;
    gzts[w][lane] = gzt;
    __syncthreads();
    const int jn = min(kTile, s.N - j0);
    for (int jj = 0; jj < jn; ++jj) {
      const float a = gzs[w][jj], bt = gzts[w][jj];
      const long long ro = base + (long long)(j0 + jj) * s.sn;
#pragma unroll
      for (int t = 0; t < kDMax / 64; ++t) {
        const int c = lane + 64 * t;
        if (c < s.D) {
          const float kc = ldf(k + ro + c), tkc = ldz(tk, ro + c);
          aq[t] = fmaf(a, kc, aq[t]);
          aq[t] = fmaf(bt, tkc, aq[t]);
          atq[t] = fmaf(bt, kc, atq[t]);
        }
      }
    }
    __syncthreads();
  }
  if (!rowok) return;
#pragma unroll
  for (int t = 0; t < kDMax / 64; ++t) {
    const int c = lane + 64 * t;
    if (c < s.D) {
      stf(dq + qbase + (long long)i * s.qsn + c, aq[t] * s.alpha);
      if (dtq) stf(dtq + qbase + (long long)i * s.qsn + c, atq[t] * s.alpha);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Key side (Steps 2, 4 and 6): wave per key row j; lane i rebuilds the tile row.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bwd_col_generic_kernel(Shape s, const T* __restrict__ q, const T* __restrict__ k,
                                                             const T* __restrict__ v, const T* __restrict__ tq,
                                                             const T* __restrict__ tk, const T* __restrict__ tv,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ stats,
                                                             const T* __restrict__ gO, const T* __restrict__ gTO,
                                                             const float* __restrict__ dsig,
                                                             const float* __restrict__ sig1, T* __restrict__ dk,
                                                             T* __restrict__ dtk, T* __restrict__ dv,
                                                             T* __restrict__ dtv) {
  __shared__ float ks[kRowsPerBlock][kDMax], tks[kRowsPerBlock][kDMax];
  __shared__ float vs[kRowsPerBlock][kDMax], tvs[kRowsPerBlock][kDMax];
  __shared__ float pp[kRowsPerBlock][kTile], ppd[kRowsPerBlock][kTile];
  __shared__ float gzs[kRowsPerBlock][kTile], gzts[kRowsPerBlock][kTile];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblk = (s.N + kRowsPerBlock - 1) / kRowsPerBlock;
  const int bh = blockIdx.x / nblk, b = bh / s.H, h = bh % s.H;
  const int j = (blockIdx.x % nblk) * kRowsPerBlock + w;
  const long long base = b * s.sb + h * s.sh, qbase = b * s.qsb + h * s.qsh;  // key side, query side
  const bool rowok = j < s.N;
  for (int c = lane; c < s.D; c += 64) {
    const long long a = base + (long long)j * s.sn + c;
    ks[w][c] = rowok ? ldf(k + a) : 0.f;
    tks[w][c] = rowok ? ldz(tk, a) : 0.f;
    vs[w][c] = rowok ? ldf(v + a) : 0.f;
    tvs[w][c] = rowok ? ldz(tv, a) : 0.f;
  }
  __syncthreads();
  float ak[kDMax / 64] = {}, atk[kDMax / 64] = {}, av[kDMax / 64] = {}, atv[kDMax / 64] = {};
  for (int i0 = 0; i0 < s.M; i0 += kTile) {
    const int i = i0 + lane;
    float p = 0.f, pd = 0.f, gz = 0.f, gzt = 0.f;
    if (i < s.M) {
      const long long ro = qbase + (long long)i * s.qsn;
      float a0 = 0.f, a1 = 0.f, df = 0.f, e = 0.f;
      for (int c = 0; c < s.D; ++c) {
        const float qc = ldf(q + ro + c), tqc = ldz(tq, ro + c);
        const float gc = ldz(gO, ro + c), tgc = ldz(gTO, ro + c);
        a0 = fmaf(qc, ks[w][c], a0);
        a1 = fmaf(tqc, ks[w][c], a1);
        a1 = fmaf(qc, tks[w][c], a1);
        df = fmaf(gc, vs[w][c], df);
        df = fmaf(tgc, tvs[w][c], df);
        e = fmaf(tgc, vs[w][c], e);
      }
      const long long r = (long long)bh * s.M + i;
      p = __expf(a0 * s.alpha - lse[r]);
      const float n = a1 * s.alpha - (stats ? stats[r] : 0.f);
      gzt = p * (e - sig1[r]);
      gz = fmaf(gzt, n, p * (df - dsig[r]));
      pd = p * n;
    }
    pp[w][lane] = p;
    ppd[w][lane] = pd;
    gzs[w][lane] = gz;
    gzts[w][lane] = gzt;
    __syncthreads();
    const int in = min(kTile, s.M - i0);
    for (int ii = 0; ii < in; ++ii) {
      const float p_ = pp[w][ii], pd_ = ppd[w][ii], gz_ = gzs[w][ii], gzt_ = gzts[w][ii];
      const long long ro = qbase + (long long)(i0 + ii) * s.qsn;
#pragma unroll
      for (int t = 0; t < kDMax / 64; ++t) {
        const int c = lane + 64 * t;
        if (c < s.D) {
          const float qc = ldf(q + ro + c), tqc = ldz(tq, ro + c);
          const float gc = ldz(gO, ro + c), tgc = ldz(gTO, ro + c);
          av[t] = fmaf(p_, gc, av[t]);
          av[t] = fmaf(pd_, tgc, av[t]);
          atv[t] = fmaf(p_, tgc, atv[t]);
          ak[t] = fmaf(gz_, qc, ak[t]);
          ak[t] = fmaf(gzt_, tqc, ak[t]);
          atk[t] = fmaf(gzt_, qc, atk[t]);
        }
      }
    }
    __syncthreads();
  }
  if (!rowok) return;
#pragma unroll
  for (int t = 0; t < kDMax / 64; ++t) {
    const int c = lane + 64 * t;
    if (c < s.D) {
      const long long a = base + (long long)j * s.sn + c;
      stf(dk + a, ak[t] * s.alpha);
      if (dtk) stf(dtk + a, atk[t] * s.alpha);
      stf(dv + a, av[t]);
      if (dtv) stf(dtv + a, atv[t]);
    }
  }
}

template <typename T>
hipError_t fwd_generic_t(const Shape& s, const FwdArgs& a, hipStream_t st) {
  dim3 grid(((s.M + kRowsPerBlock - 1) / kRowsPerBlock) * s.B * s.H);
  hipLaunchKernelGGL(fwd_generic_kernel<T>, grid, dim3(256), 0, st, s, (const T*)a.q, (const T*)a.k, (const T*)a.v,
                     (const T*)a.tq, (const T*)a.tk, (const T*)a.tv, (T*)a.o, (T*)a.to, a.lse, a.stats);
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_pre_t(const Shape& s, const BwdArgs& a, hipStream_t st) {
  dim3 grid(((s.M + kRowsPerBlock - 1) / kRowsPerBlock) * s.B * s.H);
  hipLaunchKernelGGL(bwd_pre_kernel<T>, grid, dim3(256), 0, st, s, (const T*)a.o, (const T*)a.to, (const T*)a.gO,
                     (const T*)a.gTO, a.dsig, a.sig1);
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_col_generic_t(const Shape& s, const BwdArgs& a, hipStream_t st) {
  dim3 grid(((s.N + kRowsPerBlock - 1) / kRowsPerBlock) * s.B * s.H);
  hipLaunchKernelGGL(bwd_col_generic_kernel<T>, grid, dim3(256), 0, st, s, (const T*)a.q, (const T*)a.k,
                     (const T*)a.v, (const T*)a.tq, (const T*)a.tk, (const T*)a.tv, a.lse, a.stats, (const T*)a.gO,
                     (const T*)a.gTO, a.dsig, a.sig1, (T*)a.dk, (T*)a.dtk, (T*)a.dv, (T*)a.dtv);
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_row_generic_t(const Shape& s, const BwdArgs& a, hipStream_t st) {
  dim3 grid(((s.M + kRowsPerBlock - 1) / kRowsPerBlock) * s.B * s.H);
  hipLaunchKernelGGL(bwd_row_generic_kernel<T>, grid, dim3(256), 0, st, s, (const T*)a.q, (const T*)a.k,
                     (const T*)a.v, (const T*)a.tq, (const T*)a.tk, (const T*)a.tv, a.lse, a.stats, (const T*)a.gO,
                     (const T*)a.gTO, a.dsig, a.sig1, (T*)a.dq, (T*)a.dtq);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_generic(const Shape& s, int dtype, const FwdArgs& a, hipStream_t st) {
  return dtype == 0 ? fwd_generic_t<float>(s, a, st) : fwd_generic_t<bf16>(s, a, st);
}
hipError_t launch_bwd_pre(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st) {
  return dtype == 0 ? bwd_pre_t<float>(s, a, st) : bwd_pre_t<bf16>(s, a, st);
}
hipError_t launch_bwd_col_generic(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st) {
  return dtype == 0 ? bwd_col_generic_t<float>(s, a, st) : bwd_col_generic_t<bf16>(s, a, st);
}
hipError_t launch_bwd_row_generic(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st) {
  return dtype == 0 ? bwd_row_generic_t<float>(s, a, st) : bwd_row_generic_t<bf16>(s, a, st);
}

}  // namespace tvm
