// Backward through both outputs on the bf16 matrix cores (gfx950), generic instruction order
// (the compiler schedules; used for head dims above 96, see bwd_row_pipe.hip and
// bwd_col_pipe.hip for the hand-scheduled kernels of the smaller head dims): a key-side kernel
// (dK, dtK, dV, dtV; Steps 2, 4, 6 of App. C plus the ordinary-attention terms of gO) and a
// query-side kernel (dQ, dtQ; Steps 3, 5), both recomputing the tile quantities from lse and
// stats ("Caching softmax statistics").  With G = gO, Gt = gTO and the row scalars of Step 1
// collapsed to dot products (dsig = G.O + Gt.tO, sig1 = Gt.O):
//
//   S = Q K^T             St = tQ K^T + Q tK^T        P = exp(alpha S - lse)
//   N = alpha St - stats  DF = G V^T + Gt tV^T        E = Gt V^T
//   gZt = P o (E - sig1)  gZ = P o (DF - dsig) + gZt o N        Pd = P o N
//
//   dV = P^T G + Pd^T Gt       dtV = P^T Gt
//   dK = alpha (gZ^T Q + gZt^T tQ)      dtK = alpha gZt^T Q
//   dQ = alpha (gZ K + gZt tK)          dtQ = alpha gZt K
//
// The query-side kernel runs first: it also computes the row scalars of Step 1 (two dot
// products per query row) and leaves them in the workspace for the key-side kernel.
//
// Both kernels share one skeleton.  A wave owns 32 rows of the "fixed" side (keys for the
// key-side kernel, queries for the query-side one) and keeps that side's four tensors as
// B-operand fragments in registers; the other side is streamed through LDS in tiles of 64
// rows (row-major, swizzled), read directly for the score products and through the
// transposing LDS read for the output products.  The next tile's global loads are issued into
// registers before the current tile is computed.  Score tiles are D[streamed][fixed]: a lane
// owns one fixed row, its 16 registers run over streamed rows, and the tile feeds the output
// products straight from registers.
// No atomics anywhere: every output element is produced by exactly one lane.
//
// MODE selects the upstream gradients that exist: 0 both; 1 gO only (gTO = 0: the ordinary
// attention backward, where E = gZt = 0, the tangent inputs drop out and only dQ, dK, dV are
// produced); 2 gTO only (the tangent path by itself, the paper's own split: the two products with
// gO drop out).  The one-sided modes serve every head dim; mode 0 only those above 96.
#pragma once
#include "mfma_tiles.h"

namespace tvm {
namespace {

constexpr int kFix = 128;  // fixed-side rows per workgroup (4 waves x 32)
constexpr int kNT = 256;
constexpr float kLog2e = 1.4426950408889634f;

template <int NDB>
__device__ __forceinline__ void zero_acc(f32x16 (&a)[NDB]) {
#pragma unroll
  for (int db = 0; db < NDB; ++db) a[db] = zero16();
}

// ------------------------------------------------------------------------------------------
// Key side.
// ------------------------------------------------------------------------------------------
template <int DK, int DV, int kTS, int MODE>
__global__ __launch_bounds__(kNT, MODE == 1 ? 2 : 1) void bwd_col_mfma_kernel(
    Shape s, const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ tq, const bf16* __restrict__ tk, const bf16* __restrict__ tv,
    const float* __restrict__ lse, const float* __restrict__ stats, const bf16* __restrict__ gO,
    const bf16* __restrict__ gTO, const float* __restrict__ dsig, const float* __restrict__ sig1,
    bf16* __restrict__ dk, bf16* __restrict__ dtk, bf16* __restrict__ dv, bf16* __restrict__ dtv) {
  using TX = Tile<kTS, DV / 8, kNT / 64>;  // read both ways: columns up to DV
  constexpr int ROWV = 4 * 256;                       // four float32 row vectors per stage (64 slots each)
  // one stage: Q, tQ, G, tG, row vectors; without gTO only Q and G (half the LDS: two workgroups per CU)
  constexpr int OFF_TQ = TX::BYTES, OFF_G = (MODE == 1 ? 1 : 2) * TX::BYTES, OFF_TG = 3 * TX::BYTES;
  constexpr int OFF_ROW = (MODE == 1 ? 2 : 4) * TX::BYTES;
  constexpr int BUF = OFF_ROW + ROWV;
  __shared__ __attribute__((aligned(16))) char lds[2 * BUF];
  constexpr int NKS = DK / 16, NDB = DV / 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int nfb = (s.N + kFix - 1) / kFix;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nfb, fb = wg - bh * nfb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;     // key side (fixed)
  const long long qbase = b * s.qsb + h * s.qsh;  // query side (streamed)
  const long long rbase = (long long)bh * s.M;
  const int j = fb * kFix + wave * 32 + ic;  // this lane's key
  const bool jok = j < s.N;

  const typename TX::Lane lx = TX::lane_setup(s.D, wave, lane);
  const unsigned pitch = (unsigned)(s.qsn * 2);  // row pitch of the streamed (query-side) tensors in bytes
  const unsigned lds0 = lds_addr_of(lds);
  // wave w also fetches row vector w (lse, stats, dsig, sig1) of the tile, one float per lane
  // (lanes past the tile or past the last row re-read the last row's value: masked rows, unused)
  const float* const rowsrc = (wave == 0 ? lse : wave == 1 ? stats : wave == 2 ? dsig : sig1) + rbase;
  auto issue = [&](int i0, unsigned buf) {  // i0 < N
    const long long ro = qbase + (long long)i0 * s.qsn;
    const int left = s.M - i0;
    TX::issue(lx, q + ro, pitch, left, buf, wave);
    if (MODE != 1) TX::issue(lx, tq + ro, pitch, left, buf + OFF_TQ, wave);
    if (MODE != 2) TX::issue(lx, gO + ro, pitch, left, buf + OFF_G, wave);
    if (MODE != 1) TX::issue(lx, gTO + ro, pitch, left, buf + OFF_TG, wave);
    if (MODE != 1 || (wave & 1) == 0)  // uniform: stats and sig1 are not needed without gTO
      dma_to_lds<4>(rowsrc + i0, (unsigned)min(lane, left - 1) * 4u, buf + OFF_ROW + wave * 256);
  };
  const typename TX::RAddr ra = TX::raddr(ic, hh);
  const typename TX::TAddr ta = TX::taddr(ic, hh);
  issue(0, lds0);

  bf16x8 kf[NKS], tkf[NKS], vf[NKS], tvf[NKS];
  gld_frags<NKS>(kf, k + base, s.sn, j, s.N, s.D, hh);
  gld_frags<NKS>(vf, v + base, s.sn, j, s.N, s.D, hh);
  if (MODE != 1) {
    gld_frags<NKS>(tkf, tk + base, s.sn, j, s.N, s.D, hh);
    gld_frags<NKS>(tvf, tv + base, s.sn, j, s.N, s.D, hh);
  }
  f32x16 aK[NDB], aTK[NDB], aV[NDB], aTV[NDB];
  zero_acc(aK);
  zero_acc(aTK);
  zero_acc(aV);
  zero_acc(aTV);
  const float c1 = s.alpha * kLog2e;

  pin_frags(kf);  // loaded before the wait for tile 0, not behind it
  pin_frags(vf);
  if (MODE != 1) {
    pin_frags(tkf);
    pin_frags(tvf);
  }
  dma_wait();
  __syncthreads();  // tile 0 has landed
  for (int i0 = 0, it = 0; i0 < s.M; i0 += kTS, ++it) {
    const char* lds_q = lds + (it & 1) * BUF;
    const char* lds_tq = lds_q + OFF_TQ;
    const char* lds_g = lds_q + OFF_G;
    const char* lds_tg = lds_q + OFF_TG;
    const float* row_lse = reinterpret_cast<const float*>(lds_q + OFF_ROW);
    const float* row_mub = row_lse + 64;
    const float* row_dsig = row_lse + 128;
    const float* row_sig1 = row_lse + 192;
    if (i0 + kTS < s.M) issue(i0 + kTS, lds0 + ((it + 1) & 1) * BUF);  // uniform: lands during this tile

#pragma unroll
    for (int ib = 0; ib < kTS / 32; ++ib) {
      if (i0 + ib * 32 >= s.M) break;  // uniform
      f32x16 sS = zero16(), sT = zero16();
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        const bf16x8 qf = TX::frag_row(lds_q, ra, ib, kk);
        sS = mfma(qf, kf[kk], sS);
        if (MODE != 1) {
          const bf16x8 tqf = TX::frag_row(lds_tq, ra, ib, kk);
          sT = mfma(tqf, kf[kk], sT);
          sT = mfma(qf, tkf[kk], sT);
        }
      }
      f32x16 sDF = zero16(), sE = zero16();
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        if (MODE != 2) {
          const bf16x8 gf = TX::frag_row(lds_g, ra, ib, kk);
          sDF = mfma(gf, vf[kk], sDF);
        }
        if (MODE != 1) {
          const bf16x8 tgf = TX::frag_row(lds_tg, ra, ib, kk);
          sE = mfma(tgf, vf[kk], sE);
          sDF = mfma(tgf, tvf[kk], sDF);
        }
      }
      if (i0 + ib * 32 + 32 > s.M) {  // uniform: ragged last block, queries >= M get probability 0
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (i0 + ib * 32 + drow(r, hh) >= s.M) sS[r] = -INFINITY;
      }
      bf16x8 pf[2], pdf[2], gzf[2], gztf[2];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int ro = ib * 32 + 8 * g4 + 4 * hh;
        const float4 l4 = *reinterpret_cast<const float4*>(row_lse + ro);
        const float4 d4 = *reinterpret_cast<const float4*>(row_dsig + ro);
        float4 m4 = make_float4(0.f, 0.f, 0.f, 0.f), s4 = m4;
        if (MODE != 1) {
          m4 = *reinterpret_cast<const float4*>(row_mub + ro);
          s4 = *reinterpret_cast<const float4*>(row_sig1 + ro);
        }
        const float la[4] = {l4.x, l4.y, l4.z, l4.w}, ma[4] = {m4.x, m4.y, m4.z, m4.w};
        const float da[4] = {d4.x, d4.y, d4.z, d4.w}, sa[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 4 * g4 + t;
          const float p = __builtin_amdgcn_exp2f(fmaf(sS[r], c1, -la[t] * kLog2e));
          pf[r >> 3][r & 7] = (bf16)p;
          if (MODE == 1) {
            gzf[r >> 3][r & 7] = (bf16)(p * (sDF[r] - da[t]));
          } else {
            const float n = fmaf(sT[r], s.alpha, -ma[t]);
            const float gzt = p * (sE[r] - sa[t]);
            const float gz = fmaf(gzt, n, p * (sDF[r] - da[t]));
            pdf[r >> 3][r & 7] = (bf16)(p * n);
            gzf[r >> 3][r & 7] = (bf16)gz;
            gztf[r >> 3][r & 7] = (bf16)gzt;
          }
        }
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          if (MODE != 2) {
            const bf16x8 gT = TX::frag_tr(lds_g, ta, 2 * ib + cc, db);
            aV[db] = mfma(gT, pf[cc], aV[db]);
          }
          const bf16x8 qT = TX::frag_tr(lds_q, ta, 2 * ib + cc, db);
          aK[db] = mfma(qT, gzf[cc], aK[db]);
          if (MODE != 1) {
            const bf16x8 tgT = TX::frag_tr(lds_tg, ta, 2 * ib + cc, db);
            aV[db] = mfma(tgT, pdf[cc], aV[db]);
            aTV[db] = mfma(tgT, pf[cc], aTV[db]);
            const bf16x8 tqT = TX::frag_tr(lds_tq, ta, 2 * ib + cc, db);
            aK[db] = mfma(tqT, gztf[cc], aK[db]);
            aTK[db] = mfma(qT, gztf[cc], aTK[db]);
          }
        }
    }
    dma_wait();
    __syncthreads();  // next tile landed; everyone is done with this one
  }
  if (!jok) return;
  const long long ro = base + (long long)j * s.sn;
  store_acc<NDB>(dk + ro, aK, s.alpha, s.D, hh);
  store_acc<NDB>(dv + ro, aV, 1.f, s.D, hh);
  if (MODE != 1) {
    store_acc<NDB>(dtk + ro, aTK, s.alpha, s.D, hh);
    store_acc<NDB>(dtv + ro, aTV, 1.f, s.D, hh);
  }
}

// ------------------------------------------------------------------------------------------
// Query side.
// ------------------------------------------------------------------------------------------
template <int DK, int DV, int kTS, int MODE>
__global__ __launch_bounds__(kNT, MODE == 1 ? 2 : 1) void bwd_row_mfma_kernel(
    Shape s, const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ tq, const bf16* __restrict__ tk, const bf16* __restrict__ tv,
    const bf16* __restrict__ o, const bf16* __restrict__ to, const float* __restrict__ lse,
    const float* __restrict__ stats, const bf16* __restrict__ gO, const bf16* __restrict__ gTO,
    float* __restrict__ dsig, float* __restrict__ sig1, bf16* __restrict__ dq, bf16* __restrict__ dtq,
    float* __restrict__ lse2w) {
  using TK = Tile<kTS, DV / 8, kNT / 64>;  // K, tK: read both ways
  using TV = Tile<kTS, DK / 8, kNT / 64>;  // V, tV: score products only
  // one stage: K, tK, V, tV; without gTO only K and V (half the LDS: two workgroups per CU)
  constexpr int OFF_TK = TK::BYTES, OFF_V = (MODE == 1 ? 1 : 2) * TK::BYTES, OFF_TV = 2 * TK::BYTES + TV::BYTES;
  constexpr int BUF = MODE == 1 ? TK::BYTES + TV::BYTES : 2 * TK::BYTES + 2 * TV::BYTES;
  __shared__ __attribute__((aligned(16))) char lds[2 * BUF];
  constexpr int NKS = DK / 16, NDB = DV / 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int nfb = (s.M + kFix - 1) / kFix;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nfb, fb = wg - bh * nfb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;     // key side (streamed)
  const long long qbase = b * s.qsb + h * s.qsh;  // query side (fixed)
  const int i = fb * kFix + wave * 32 + ic;  // this lane's query
  const bool iok = i < s.M;

  const typename TK::Lane lk = TK::lane_setup(s.D, wave, lane);
  const typename TV::Lane lv = TV::lane_setup(s.D, wave, lane);
  const unsigned pitch = (unsigned)(s.sn * 2);  // row pitch in bytes
  const unsigned lds0 = lds_addr_of(lds);
  auto issue = [&](int j0, unsigned buf) {  // j0 < N
    const long long ro = base + (long long)j0 * s.sn;
    const int left = s.N - j0;
    TK::issue(lk, k + ro, pitch, left, buf, wave);
    TV::issue(lv, v + ro, pitch, left, buf + OFF_V, wave);
    if (MODE != 1) {
      TK::issue(lk, tk + ro, pitch, left, buf + OFF_TK, wave);
      TV::issue(lv, tv + ro, pitch, left, buf + OFF_TV, wave);
    }
  };
  const typename TK::RAddr rk = TK::raddr(ic, hh);
  const typename TV::RAddr rv = TV::raddr(ic, hh);
  const typename TK::TAddr ta = TK::taddr(ic, hh);
  issue(0, lds0);

  bf16x8 qf[NKS], tqf[NKS], gf[NKS], tgf[NKS];
  gld_frags<NKS>(qf, q + qbase, s.qsn, i, s.M, s.D, hh);
  if (MODE != 1) gld_frags<NKS>(tqf, tq + qbase, s.qsn, i, s.M, s.D, hh);
  if (MODE != 2) gld_frags<NKS>(gf, gO + qbase, s.qsn, i, s.M, s.D, hh);
  if (MODE != 1) gld_frags<NKS>(tgf, gTO + qbase, s.qsn, i, s.M, s.D, hh);
  // Step 1 of App. C, fused: the row scalars delta + Sigma_2 = gO.O + gTO.tO and Sigma_1 = gTO.O of
  // this lane's query, from the same fragment layout (each half-wave holds half of the row);
  // they are also written out for the key-side kernel, which runs after this one.
  float ds = 0.f, s1 = 0.f;
  {
    bf16x8 of[NKS], tof[NKS];
    gld_frags<NKS>(of, o + qbase, s.qsn, i, s.M, s.D, hh);
    if (MODE != 1) gld_frags<NKS>(tof, to + qbase, s.qsn, i, s.M, s.D, hh);
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float oe = (float)of[kk][e];
        if (MODE != 2) ds = fmaf((float)gf[kk][e], oe, ds);
        if (MODE != 1) {
          const float gte = (float)tgf[kk][e];
          ds = fmaf(gte, (float)tof[kk][e], ds);
          s1 = fmaf(gte, oe, s1);
        }
      }
    ds += xhalf(ds);
    s1 += xhalf(s1);
  }
  // rows beyond N: zeros keep everything finite; nothing of theirs is stored
  const long long r = (long long)bh * s.M + (iok ? i : 0);
  const float lse2 = iok ? lse[r] * kLog2e : 0.f;
  const float mub = (MODE != 1 && iok) ? stats[r] : 0.f;
  if (iok && hh == 0) {
    if (lse2w != nullptr) {
      // for the hand-scheduled key-side passes (bwd_pass.hip): lse in log2 units, the two sums negated
      lse2w[r] = lse2;
      dsig[r] = -ds;
      sig1[r] = -s1;
    } else {
      dsig[r] = ds;
      if (MODE != 1) sig1[r] = s1;
    }
  }
  f32x16 aQ[NDB], aTQ[NDB];
  zero_acc(aQ);
  zero_acc(aTQ);
  const float c1 = s.alpha * kLog2e;

  pin_frags(qf);  // loaded before the wait for tile 0, not behind it
  if (MODE != 1) pin_frags(tqf);
  if (MODE != 2) pin_frags(gf);
  if (MODE != 1) pin_frags(tgf);
  dma_wait();
  __syncthreads();  // tile 0 has landed
  for (int j0 = 0, it = 0; j0 < s.N; j0 += kTS, ++it) {
    const char* lds_k = lds + (it & 1) * BUF;
    const char* lds_tk = lds_k + OFF_TK;
    const char* lds_v = lds_k + OFF_V;
    const char* lds_tv = lds_k + OFF_TV;
    if (j0 + kTS < s.N) issue(j0 + kTS, lds0 + ((it + 1) & 1) * BUF);  // uniform: lands during this tile

#pragma unroll
    for (int jb = 0; jb < kTS / 32; ++jb) {
      if (j0 + jb * 32 >= s.N) break;  // uniform
      // Fragments are fetched a whole phase ahead of the products that use them, so the LDS
      // latency of each phase hides behind the previous phase's matrix-core work.
      bf16x8 kfr[NKS], tkfr[NKS], vfr[NKS], tvfr[NKS];
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        kfr[kk] = TK::frag_row(lds_k, rk, jb, kk);
        if (MODE != 1) tkfr[kk] = TK::frag_row(lds_tk, rk, jb, kk);
      }
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        vfr[kk] = TV::frag_row(lds_v, rv, jb, kk);
        if (MODE != 1) tvfr[kk] = TV::frag_row(lds_tv, rv, jb, kk);
      }
      f32x16 sS = zero16(), sT = zero16();
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        sS = mfma(kfr[kk], qf[kk], sS);
        if (MODE != 1) {
          sT = mfma(kfr[kk], tqf[kk], sT);
          sT = mfma(tkfr[kk], qf[kk], sT);
        }
      }
      bf16x8 kT[2][NDB], tkT[2][NDB];
#pragma unroll
      for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          kT[cc][db] = TK::frag_tr(lds_k, ta, 2 * jb + cc, db);
          if (MODE != 1) tkT[cc][db] = TK::frag_tr(lds_tk, ta, 2 * jb + cc, db);
        }
      if (j0 + jb * 32 + 32 > s.N) {  // uniform: ragged last block, keys >= N get probability 0
#pragma unroll
        for (int rr = 0; rr < 16; ++rr)
          if (j0 + jb * 32 + drow(rr, hh) >= s.N) sS[rr] = -INFINITY;
      }
      // The E-type products run on the matrix cores while the VALU turns S, St into P and N,
      // one element per product (source order is the schedule: see the build flags).
      f32x16 sDF = zero16(), sE = zero16();
      float pp[16], nn[16];
      auto pw1 = [&](int rr) {
        if (rr < 16) {
          pp[rr] = __builtin_amdgcn_exp2f(fmaf(sS[rr], c1, -lse2));
          if (MODE != 1) nn[rr] = fmaf(sT[rr], s.alpha, -mub);
        }
      };
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        if (MODE != 1) sE = mfma(vfr[kk], tgf[kk], sE);
        pw1(3 * kk);
        if (MODE != 2) sDF = mfma(vfr[kk], gf[kk], sDF);
        pw1(3 * kk + 1);
        if (MODE != 1) sDF = mfma(tvfr[kk], tgf[kk], sDF);
        pw1(3 * kk + 2);
      }
#pragma unroll
      for (int rr = 3 * NKS; rr < 16; ++rr) pw1(rr);
      bf16x8 gzf[2], gztf[2];
#pragma unroll
      for (int rr = 0; rr < 16; ++rr) {
        if (MODE == 1) {
          gzf[rr >> 3][rr & 7] = (bf16)(pp[rr] * (sDF[rr] - ds));
        } else {
          const float gzt = pp[rr] * (sE[rr] - s1);
          const float gz = fmaf(gzt, nn[rr], pp[rr] * (sDF[rr] - ds));
          gzf[rr >> 3][rr & 7] = (bf16)gz;
          gztf[rr >> 3][rr & 7] = (bf16)gzt;
        }
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          aQ[db] = mfma(kT[cc][db], gzf[cc], aQ[db]);
          if (MODE != 1) {
            aQ[db] = mfma(tkT[cc][db], gztf[cc], aQ[db]);
            aTQ[db] = mfma(kT[cc][db], gztf[cc], aTQ[db]);
          }
        }
    }
    dma_wait();
    __syncthreads();  // next tile landed; everyone is done with this one
  }
  if (!iok) return;
  const long long ro = qbase + (long long)i * s.qsn;
  store_acc<NDB>(dq + ro, aQ, s.alpha, s.D, hh);
  if (MODE != 1) store_acc<NDB>(dtq + ro, aTQ, s.alpha, s.D, hh);
}

template <int DK, int DV, int MODE>
hipError_t launch_col(const Shape& s, const BwdArgs& a, hipStream_t st) {
  const int nfb = (s.N + kFix - 1) / kFix;
  hipLaunchKernelGGL((bwd_col_mfma_kernel<DK, DV, (DV > 96 ? 32 : 64), MODE>), dim3(nfb * s.B * s.H), dim3(kNT), 0, st, s,
                     (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk,
                     (const bf16*)a.tv, a.lse, a.stats, (const bf16*)a.gO, (const bf16*)a.gTO, a.dsig, a.sig1,
                     (bf16*)a.dk, (bf16*)a.dtk, (bf16*)a.dv, (bf16*)a.dtv);
  return hipGetLastError();
}

// pipe_ws: leave the row vectors in the workspace in the convention of the hand-scheduled key-side kernels
template <int DK, int DV, int MODE>
hipError_t launch_row(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws = false) {
  const int nfb = (s.M + kFix - 1) / kFix;
  hipLaunchKernelGGL((bwd_row_mfma_kernel<DK, DV, (DV > 96 ? 32 : 64), MODE>), dim3(nfb * s.B * s.H), dim3(kNT), 0, st, s,
                     (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk,
                     (const bf16*)a.tv, (const bf16*)a.o, (const bf16*)a.to, a.lse, a.stats, (const bf16*)a.gO,
                     (const bf16*)a.gTO, a.dsig, a.sig1, (bf16*)a.dq, (bf16*)a.dtq, pipe_ws ? a.lse2 : nullptr);
  return hipGetLastError();
}

}  // namespace
}  // namespace tvm
