// Backward for head dims in (96, 128] with the instruction stream laid out by hand: the key side (dK, dtK, dV, dtV;
// Steps 2, 4, 6 of App. C plus the ordinary-attention terms of gO) as TWO passes over the queries, and the query
// side (dQ, dtQ; Steps 1, 3, 5) as one pass over the keys with the code of pass K.
//
// At 128 columns the four accumulators of the one-pass kernel (bwd_col_pipe.hip) fill the AGPRs and the four
// fixed-side fragments the VGPRs.  Here each pass keeps two accumulators (128 AGPRs) and every fixed-side
// fragment it needs beside them in AGPRs, so that all 256 VGPRs serve the streamed side:
//
//   pass V:  dV += P^T G + Pd^T tG,  dtV += P^T tG          needs S, St (K, tK fixed)            48 products per block
//   pass K:  dK += gZ^T Q + gZt^T tQ,  dtK += gZt^T Q       needs S, St, E, DF (K, tK, V, tV)    72 products per block
//
// S and St are computed in both (120 products per block of 32 x 32 at d = 128 against 96 in one pass).  Same
// mathematics, data layout and row-scalar conventions as bwd_col_pipe.hip (lse in log2 units, sig1 and dsig
// negated, left in the workspace by the query-side kernel); a wave owns 32 keys and runs alone on its SIMD.
// Queries are streamed in tiles of ONE block of 32 (four tiles of 128 columns, three LDS stages of 49 KB), so
// every block ends with the workgroup barrier that frees its stage:
//
//   pass V   S | P, N, Pd of half 0 (nothing to hide behind) | OV(0) with P, N, Pd of half 1 | barrier | OV(1)
//   pass K   S | E (its products first, then those of DF) with P, N, then gZt | OK(0) (the products with gZt first) with gZ | barrier | OK(1)
//
// The tile after next is fetched behind the products of S and of the last phase, which carry no pointwise work.
//
// Pass Q is pass K with the two sides exchanged: a wave owns 32 queries (fragments of q, tq, gTO, gO fixed, dQ and dtQ
// accumulated) and streams K, tK, V, tV through the same LDS slots; E = V gTO^T and DF = V gO^T + tV gTO^T pair the
// same slots with the same fixed fragments as E = tG V^T, DF = tG tV^T + G V^T do in pass K, and dQ += gZ K + gZt tK,
// dtQ += gZt K are pass K's output products.  What differs: the row scalars belong to the lane (lse, stats from the
// forward, and Step 1's sums, formed here from the fragments and left in the workspace for the key side, which
// runs afterwards), and the masked entries of a ragged last tile are keys.
//
// HAS_G = false are the passes for a call without gO (the gradient of <gTO, tO> alone, Steps 1-6 of App. C by
// themselves): the products with G vanish (E phase: two per 16 head dims, DF = tG tV^T, in pass Q DF = tV gTO^T; OV:
// two per 32, dV += tG^T Pd, dtV += tG^T P), and the G tile is neither fetched nor read (pass Q: no fragments of gO).
//
// The translation unit is built with the machine scheduler off: source order is issue order.
#include "pipe_ops.h"

#include <type_traits>

namespace tvm {
namespace {

constexpr int kFix = 128;  // keys per workgroup (4 waves x 32)
constexpr int kNT = 256;

typedef __attribute__((ext_vector_type(4))) float f32x4;
__device__ __forceinline__ f32x4 lds_read_f4(unsigned addr, int imm) {
  typedef const f32x4 __attribute__((address_space(3))) * lp;
  return *(lp)(uintptr_t)(addr + (unsigned)imm);
}
__device__ __forceinline__ float f4(const f32x4& v, int t) { return v[t]; }
// landed() of pipe_ops.h for one tile
__device__ __forceinline__ void landed1(f32x16& a) { asm volatile("" : "+v"(a)); }

// PASS 1: dV, dtV into out0, out1;  PASS 2: dK, dtK;  PASS 3: dQ, dtQ.
//   f0..f3: the fixed side's tensors (passes V, K: k, tk, v, tv;  pass Q: q, tq, gTO, gO)
//   t0..t3: the streamed side's, in LDS slot order (passes V, K: q, tq, gTO, gO;  pass Q: k, tk, v, tv)
//   lse_in: passes V, K: lse in log2 units from the workspace;  pass Q: lse as the forward saved it
//   dsig, sig1: passes V, K: read (negated sums);  pass Q: written, with lse in log2 units to lse2w, for the key side:
//   negated and in log2 units if pipe_ws, else plain (the generic-order key-side kernel follows) and lse2w untouched
//   o, to: pass Q only (Step 1)
template <int DK, int DV, int PASS, bool HAS_G>
__global__ __launch_bounds__(kNT, 1) void bwd_pass_kernel(
    Shape s, const bf16* __restrict__ f0, const bf16* __restrict__ f1, const bf16* __restrict__ f2,
    const bf16* __restrict__ f3, const bf16* __restrict__ t0, const bf16* __restrict__ t1,
    const bf16* __restrict__ t2, const bf16* __restrict__ t3, const float* __restrict__ lse_in,
    const float* __restrict__ stats, float* __restrict__ dsig, float* __restrict__ sig1, float* __restrict__ lse2w,
    int pipe_ws, const bf16* __restrict__ o, const bf16* __restrict__ to, bf16* __restrict__ out0,
    bf16* __restrict__ out1) {
  static_assert(PASS >= 1 && PASS <= 3, "pass V, K or Q");
  constexpr bool PV = PASS == 1, PQ = PASS == 3;
  using TX = Tile<32, DV / 8, kNT / 64>;  // Q, tQ, G, tG: read both ways
  constexpr int OFF_TQ = TX::BYTES, OFF_G = 2 * TX::BYTES, OFF_TG = 3 * TX::BYTES, OFF_ROW = 4 * TX::BYTES;
  constexpr int BUF = 4 * TX::BYTES + 4 * 256;  // one stage: four tiles and four float32 row vectors (64 floats each, 32 used)
  static_assert(3 * BUF <= 160 * 1024, "three stages fit the LDS");
  __shared__ __attribute__((aligned(16))) char lds[3 * BUF];
  constexpr int NKS = DK / 16, NDB = DV / 32;
  constexpr int PG = HAS_G ? 3 : 2;          // products per step of the phases that G takes part in
  constexpr int NTG = HAS_G || PQ ? 2 : 1;   // streamed tiles in the gradient slots (tG and G, or tG alone; pass Q: V and tV)
  constexpr int NS = 3 * NKS;                // products of the S phase
  constexpr int NE = PG * NKS;               // products of the E phase
  constexpr int NH = (PV ? PG : 3) * NDB;    // products of half the output phase of this pass
  constexpr int FS = 4;                      // first pointwise slot of the E phase
  // pass V: pieces 24..47 of P, N, Pd (half 1) go behind the products of OV(0);  pass K: the 24 pieces of P, N behind
  // those of E from FS on, pieces 20..39 of gZ, gZt (half 1) behind those of OK(0)
  struct C {
    static constexpr int pwv(int u) { return (((u + 24) % 12) >> 1 == 1 || ((u + 24) % 12) >> 1 == 2) ? 12 : 8; }
    static constexpr int pwk(int u) { return (u % 6) >> 1 == 0 ? 8 : 12; }
    static constexpr int pw2(int) { return 8; }
    static constexpr int base_h(int v) { return 8 * share_count(v, (PV ? NTG : 2) * NDB, NH); }
    static constexpr int base_e(int v) { return 8 * share_count(v, 2 * NDB, NE) + (v < FS && !PQ ? 4 * share_count(v, 4, FS) : 0); }
  };
  static constexpr Deal<NH> kPwV = deal_out<NH>(24, 0, NH, 24, C::pwv, C::base_h);
  // Passes K, Q.  E phase: the NKS products of E come first, so that E has landed (four products on) while those of
  // DF still run: behind the products from FS to ES the 24 pieces of P, N, from ES on the 16 pieces of gZt = P o E
  // (both halves).  OK(0) starts with the 2 NDB products that take gZt alone; from its fifth product on (DF has
  // landed) the 12 pieces of gZ of half 0, done when its products with gZ begin, then the 12 of half 1.
  static constexpr int ES = NKS + 4 > FS + 2 * (NE - FS) / 3 ? NKS + 4 : FS + 2 * (NE - FS) / 3;
  static_assert(ES < NE, "room behind the products of DF for the pieces of gZt");
  struct CE {
    static constexpr int cost(int u) { return u < 24 ? C::pwk(u) : 8; }
    static constexpr Deal<NE> deal() {
      Deal<NE> d{};
      for (int i = 0; i <= NE; ++i) d.first[i] = i < FS ? 0 : 40;
      deal_range(d, 0, 24, FS, ES, cost, C::base_e);
      deal_range(d, 24, 40, ES, NE, cost, C::base_e);
      d.first[NE] = 40;
      return d;
    }
  };
  static constexpr Deal<NE> kPwE = CE::deal();
  static constexpr Deal<NH> kPwD = deal_out<NH>(24, 4, 2 * NDB, 12, C::pw2, C::base_h);
  constexpr int NTILE = 2 + NTG;              // tiles fetched per stage (passes V, K: the G tile's place stays empty without gO)
  constexpr int NDMA = NTILE * TX::IPW + (PQ ? 0 : 1);  // wave-loads per wave and tile (passes V, K: the last is a row vector)
  constexpr int NQB = NS + NH;                // products that carry tile loads: S and the last phase
  constexpr int NDMA_PRE = NS * NDMA / NQB;   // wave-loads issued before the barrier (behind the products of S)
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: what depends on it alone stays out of the VALU
  const int nfix = PQ ? s.M : s.N, nstr = PQ ? s.N : s.M;  // rows of the fixed side, of the streamed side
  const int nfb = (nfix + kFix - 1) / kFix;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nfb, fb = wg - bh * nfb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long kbase = b * s.sb + h * s.sh, qbase = b * s.qsb + h * s.qsh;  // key side, query side
  const long long base = PQ ? qbase : kbase;    // fixed side
  const long long tbase = PQ ? kbase : qbase;   // streamed side
  const long long fsn = PQ ? s.qsn : s.sn, tsn = PQ ? s.sn : s.qsn;
  const long long rbase = (long long)bh * s.M;
  const int j = fb * kFix + wave * 32 + ic;  // this lane's row of the fixed side (a key; pass Q: a query)

  const unsigned pitch = (unsigned)(tsn * 2);  // row pitch of the streamed tensors in bytes
  const unsigned lds0 = lds_addr_of(lds);
  const int nt = (nstr + 31) >> 5;  // tiles
  const int ilast = (nt - 1) * 32;  // first query of the last tile; loads "beyond" it fetch it again, unused
  // Per-lane byte offsets of this wave's loads within a tile, worked out once: for whole tiles, and for the last
  // tile, where rows past the end fetch its last row again (masked rows, unused).  Wave w also fetches row vector w
  // (lse in log2 units, stats, dsig, sig1) of the tile: one float per lane, lanes 32..63 the tile's last one again.
  typename TX::Offs of_full, of_last;
  unsigned rv_full, rv_last;
  {
    const typename TX::Lane lx = TX::lane_setup(s.D, wave, lane);
    of_full = TX::offsets(lx, pitch, 32);
    of_last = TX::offsets(lx, pitch, nstr - ilast);
    rv_full = (unsigned)min(lane, 31) * 4u;
    rv_last = (unsigned)min(lane, nstr - ilast - 1) * 4u;
  }
  const float* const rowsrc = (wave == 0 ? lse_in : wave == 1 ? stats : wave == 2 ? dsig : sig1) + rbase;  // (passes V, K)
  // wave-load number x (compile-time) of the tile whose first row is i0 (< nstr), into the stage at `buf`;
  // `last`: that tile is the last one
  auto dma = [&](int x, int i0, unsigned buf, bool last) {
    const long long ro = tbase + (long long)i0 * tsn;
    const int t = x % TX::IPW;
    const unsigned off = last ? of_last.o[t] : of_full.o[t];
    if (x < TX::IPW) TX::issue_at(off, t, t0 + ro, buf, wave);
    else if (x < 2 * TX::IPW) TX::issue_at(off, t, t1 + ro, buf + OFF_TQ, wave);
    else if (x < 3 * TX::IPW) TX::issue_at(off, t, t2 + ro, buf + OFF_TG, wave);
    else if (x < NTILE * TX::IPW) TX::issue_at(off, t, t3 + ro, buf + OFF_G, wave);
    else dma_to_lds<4>(rowsrc + i0, last ? rv_last : rv_full, buf + OFF_ROW + wave * 256);
  };
  const typename TX::RAddr ra = TX::raddr(ic, hh);
  const typename TX::TAddr ta = TX::taddr(ic, hh);
  // Start-up: tile 0 first, then the fixed-side fragments (scattered loads), then, once those have arrived, tile 1.
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, 0, lds0, nt == 1);
  bf16x8 kf[NKS], tkf[NKS], vf[NKS], tvf[NKS];  // passes V, K: of k, tk, v, tv;  pass Q: of q, tq, gTO, gO
  gld_frags<NKS>(kf, f0 + base, fsn, j, nfix, s.D, hh);
  gld_frags<NKS>(tkf, f1 + base, fsn, j, nfix, s.D, hh);
  if (!PV) {
    gld_frags<NKS>(vf, f2 + base, fsn, j, nfix, s.D, hh);
    if (HAS_G || !PQ) gld_frags<NKS>(tvf, f3 + base, fsn, j, nfix, s.D, hh);
  }
  // pass Q: the row scalars of this lane's query.  Step 1 of App. C, fused: delta + Sigma_2 = gO.O + gTO.tO and
  // Sigma_1 = gTO.O from the same fragment layout (each half-wave holds half of the row); they are also written out
  // for the key side, which runs after this kernel.
  float lse2 = 0.f, mub = 0.f, nds = 0.f, ns1 = 0.f;
  if (PQ) {
    const bool iok = j < s.M;
    float ds = 0.f, s1 = 0.f;
    {
      bf16x8 of[NKS], tof[NKS];
      gld_frags<NKS>(of, o + base, fsn, j, nfix, s.D, hh);
      gld_frags<NKS>(tof, to + base, fsn, j, nfix, s.D, hh);
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float oe = (float)of[kk][e], gte = (float)vf[kk][e];
          if (HAS_G) ds = fmaf((float)tvf[kk][e], oe, ds);
          ds = fmaf(gte, (float)tof[kk][e], ds);
          s1 = fmaf(gte, oe, s1);
        }
      ds += xhalf(ds);
      s1 += xhalf(s1);
    }
    // rows beyond M: zeros keep everything finite; nothing of theirs is stored
    const long long r = rbase + (iok ? j : 0);
    lse2 = iok ? lse_in[r] * 1.4426950408889634f : 0.f;
    mub = iok ? stats[r] : 0.f;
    nds = -ds;
    ns1 = -s1;
    if (iok && hh == 0) {
      if (pipe_ws) {
        lse2w[r] = lse2;
        dsig[r] = nds;
        sig1[r] = ns1;
      } else {
        dsig[r] = ds;
        sig1[r] = s1;
      }
    }
  }
  f32x16 a0[NDB], a1[NDB];  // pass V: dV, dtV;  pass K: dK, dtK;  pass Q: dQ, dtQ
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    a0[db] = zero16();
    a1[db] = zero16();
  }
  // wave-uniform scalars for the assembly blocks (SGPR operands)
  const float c1u = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha * 1.4426950408889634f)));
  const float alphau = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha)));

  dma_wait();  // tile 0 and this wave's fixed rows
  // tile 1 goes into the second stage now (any earlier and the wait for the fixed rows, which counts outstanding
  // loads, would also wait for it); it lands while tile 0 is computed
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, min(32, ilast), lds0 + BUF, nt <= 2);
  __syncthreads();  // tile 0 has landed
  bf16x8 rq[NKS], rtq[NKS];  // Q, tQ rows of the block whose S phase comes next
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    rq[kk] = lds_read16(lds0 + ((kk & 1) ? ra.o : ra.e), kk * 32);
    rtq[kk] = lds_read16(lds0 + ((kk & 1) ? ra.o : ra.e), OFF_TQ + kk * 32);
  }

  // One tile = one block of 32 queries.  RAG: queries beyond M exist in this tile (only ever the last one).
  //   sb / sbn / sbf: LDS address of this tile's stage / of the next tile's (landed when this tile's barrier is
  //   passed) / of the free one, into which the tile after next is fetched, one wave-load every few products;
  //   i0: first query;  in2: first query of the tile after next (clamped to the last tile);  in2last: that is the
  //   last tile.
  auto tile = [&](auto rag, unsigned sb, unsigned sbn, unsigned sbf, int i0, int in2, bool in2last, bool last) {
    constexpr bool RAG = decltype(rag)::value;
    const unsigned re = sb + ra.e, ro = sb + ra.o;        // rows of Q; tQ, G, tG at + OFF_*
    const unsigned tl = sb + ta.lo, th = sb + ta.hi;      // transposed
    const unsigned rv = sb + OFF_ROW + 16 * hh;           // row vectors: this half's four rows of each group of eight
    const unsigned nre = sbn + ra.e, nro = sbn + ra.o;    // the next tile's rows of Q
#define TVM_SHARE(x, m, CNT, N) for (int x = (m) * (CNT) / (N); x < ((m) + 1) * (CNT) / (N); ++x)
    bf16x8 rg[NKS], rtg[NKS];
    f32x16 sS, sT, sE, sDF;
    f32x4 la[4], ma[4], da[4], sa[4];  // row scalars of the block's queries, by group of eight
    float pp[16], nn[16];
    unsigned pk[8], pdk[8], gz[8], gzt[8];
    bf16x8 xT[NDB], txT[NDB], yT[NDB], tyT[NDB];  // transposed fragments of half 0 / of half 1
    float ta_[8], tb_[8], wa[8], wb[8];  // temporaries of element pair e, alive between its pieces

    // lse (log2 units) and stats of the query of element 2e + k2: by element in passes V, K, the lane's own in pass Q
    auto lse_of = [&](int e, int k2) { return PQ ? lse2 : f4(la[e >> 1], ((2 * e) & 3) + k2); };
    auto mu_of = [&](int e, int k2) { return PQ ? mub : f4(ma[e >> 1], ((2 * e) & 3) + k2); };
    // first step of a pair: its two scores in log2 units less lse (streamed rows beyond the end: probability 0)
    auto pw_scores = [&](int e) {
      float s0 = sS[2 * e], s1 = sS[2 * e + 1];
      if (RAG) {
        if (i0 + drow(2 * e, hh) >= nstr) s0 = -INFINITY;
        if (i0 + drow(2 * e + 1, hh) >= nstr) s1 = -INFINITY;
      }
      pw_fma2(ta_[e], tb_[e], s0, s1, c1u, lse_of(e, 0), lse_of(e, 1));
    };
    // pass V: P, N, Pd of the block as a stream of 8 x 6 pieces (pair e: elements 2e, 2e+1); two pairs take
    // turns, so that no piece reads what the piece right before it wrote
    auto pw1v_op = [&](int u) {
      const int e = 2 * (u / 12) + (u & 1), st = (u % 12) >> 1;
      if (st == 0) pw_scores(e);
      else if (st == 1) pw_exp_fma(pp[2 * e], ta_[e], nn[2 * e], sT[2 * e], alphau, mu_of(e, 0));
      else if (st == 2) pw_exp_fma(pp[2 * e + 1], tb_[e], nn[2 * e + 1], sT[2 * e + 1], alphau, mu_of(e, 1));
      else if (st == 3) pw_mul2(ta_[e], tb_[e], pp[2 * e], nn[2 * e], pp[2 * e + 1], nn[2 * e + 1]);
      else if (st == 4) pw_cvt(pk[e], pp[2 * e], pp[2 * e + 1]);
      else pw_cvt(pdk[e], ta_[e], tb_[e]);
    };
    // pass K: P, N alone (float32, for gZ and gZt) as 8 x 3 pieces
    auto pw1k_op = [&](int u) {
      const int e = 2 * (u / 6) + (u & 1), st = (u % 6) >> 1;
      if (st == 0) pw_scores(e);
      else if (st == 1) pw_exp_fma(pp[2 * e], ta_[e], nn[2 * e], sT[2 * e], alphau, mu_of(e, 0));
      else pw_exp_fma(pp[2 * e + 1], tb_[e], nn[2 * e + 1], sT[2 * e + 1], alphau, mu_of(e, 1));
    };
    // gZt = P o E of the block as a stream of 8 x 2 pieces, gZ = P o DF + gZt o N as one of 8 x 3 (E, DF come with
    // sig1, dsig already subtracted); two pairs take turns here too
    auto pw2e_op = [&](int u) {
      const int e = 2 * (u / 4) + (u & 1), st = (u % 4) >> 1;
      if (st == 0) pw_mul2(ta_[e], tb_[e], pp[2 * e], sE[2 * e], pp[2 * e + 1], sE[2 * e + 1]);
      else pw_cvt(gzt[e], ta_[e], tb_[e]);
    };
    auto pw2d_op = [&](int u) {
      const int e = 2 * (u / 6) + (u & 1), st = (u % 6) >> 1;
      if (st == 0) pw_mul2(wa[e], wb[e], pp[2 * e], sDF[2 * e], pp[2 * e + 1], sDF[2 * e + 1]);
      else if (st == 1) pw_fmac2(wa[e], wb[e], ta_[e], nn[2 * e], tb_[e], nn[2 * e + 1]);
      else pw_cvt(gz[e], wa[e], wb[e]);
    };
    auto tr_imm = [&](int cc, int db) { return cc * 16 * TX::PCH * 16 + db * 64; };

    // ---- S
#pragma unroll
    for (int m = 0; m < NS; ++m) {
      const int kk = m / 3, w = m - 3 * kk;
      if (w == 0) {
        if (kk == 0) mfma_fix0<RAG>(sS, rq[0], kf[0]);
        else mfma_fix<RAG>(sS, rq[kk], kf[kk]);
      } else if (w == 1) {
        if (kk == 0) mfma_fix0<RAG>(sT, rtq[0], kf[0]);
        else mfma_fix<RAG>(sT, rtq[kk], kf[kk]);
      } else {
        mfma_fix<RAG>(sT, rq[kk], tkf[kk]);
      }
      if (PV) {
#pragma unroll
        TVM_SHARE(x, m, NTG * NDB, NS) {  // tG^T, G^T of half 0
          const int db = x / NTG;
          if (x % NTG == 0) txT[db] = lds_read_tr(tl, th, OFF_TG + tr_imm(0, db));
          else xT[db] = lds_read_tr(tl, th, OFF_G + tr_imm(0, db));
        }
#pragma unroll
        TVM_SHARE(x, m, 8, NS) {  // lse, stats of the block
          if (x < 4) la[x] = lds_read_f4(rv, x * 32);
          else ma[x - 4] = lds_read_f4(rv, 256 + (x - 4) * 32);
        }
      } else {
#pragma unroll
        TVM_SHARE(x, m, NTG * NKS, NS) {  // tG, G rows
          const int k2 = x % NKS;
          if (x < NKS) rtg[k2] = lds_read16((k2 & 1) ? ro : re, OFF_TG + k2 * 32);
          else rg[k2] = lds_read16((k2 & 1) ? ro : re, OFF_G + k2 * 32);
        }
        if (!PQ) {
#pragma unroll
          TVM_SHARE(x, m, 12, NS) {  // -sig1 and -dsig of the block first (the first products of E start from them), then lse, stats of half 0
            if (x < 4) sa[x] = lds_read_f4(rv, 768 + x * 32);
            else if (x < 8) da[x - 4] = lds_read_f4(rv, 512 + (x - 4) * 32);
            else if (x < 10) la[x - 8] = lds_read_f4(rv, (x - 8) * 32);
            else ma[x - 10] = lds_read_f4(rv, 256 + (x - 10) * 32);
          }
        }
      }
#pragma unroll
      TVM_SHARE(x, m, NDMA, NQB) dma(x, in2, sbf, in2last);
    }
    if (PV) {
      // ---- P, N, Pd of half 0: nothing to hide behind
      mfma_settle();
      landed(sS, sT);
#pragma unroll
      for (int u = 0; u < 24; ++u) pw1v_op(u);
      // ---- OV(0), with P, N, Pd of half 1
#pragma unroll
      for (int m = 0; m < NH; ++m) {
        const int db = m / PG, w = m - PG * db;
        if (w == 0) { if (m == 0) mfma_acc<true>(a0[db], txT[db], frag_of(pdk, 0)); else mfma_acc<RAG>(a0[db], txT[db], frag_of(pdk, 0)); }
        else if (w == 1) mfma_acc<RAG>(a1[db], txT[db], frag_of(pk, 0));
        else mfma_acc<RAG>(a0[db], xT[db], frag_of(pk, 0));
#pragma unroll
        TVM_SHARE(x, m, NTG * NDB, NH) {  // tG^T, G^T of half 1
          const int d2 = x / NTG;
          if (x % NTG == 0) tyT[d2] = lds_read_tr(tl, th, OFF_TG + tr_imm(1, d2));
          else yT[d2] = lds_read_tr(tl, th, OFF_G + tr_imm(1, d2));
        }
#pragma unroll
        for (int u = kPwV.first[m]; u < kPwV.first[m + 1]; ++u) pw1v_op(24 + u);
      }
    } else {
      // ---- E, with P, N.  E and DF start from -sig1 and -dsig of their queries.
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          sE[4 * g4 + t] = PQ ? ns1 : sa[g4][t];
          sDF[4 * g4 + t] = PQ ? nds : da[g4][t];
        }
#pragma unroll
      for (int m = 0; m < NE; ++m) {
        // (the first product of either tile in the padded form: the copies of its start values may sit right in front)
        if (m == 0) {
          mfma_fix<true>(sE, rtg[0], vf[0]);
        } else if (m < NKS) {
          mfma_fix<RAG>(sE, rtg[m], vf[m]);
        } else {
          const int kk = (m - NKS) / (PG - 1), w = (m - NKS) - (PG - 1) * kk;
          if (w == 0 && (HAS_G || !PQ)) {
            if (m == NKS) mfma_fix<true>(sDF, rtg[kk], tvf[kk]);
            else mfma_fix<RAG>(sDF, rtg[kk], tvf[kk]);
          } else {  // (pass Q without gO: DF = tV gTO^T is this product alone)
            if (m == NKS) mfma_fix<true>(sDF, rg[kk], vf[kk]);
            else mfma_fix<RAG>(sDF, rg[kk], vf[kk]);
          }
        }
#pragma unroll
        TVM_SHARE(x, m, 2 * NDB, NE) {  // Q^T, tQ^T of half 0
          const int d2 = x >> 1;
          if ((x & 1) == 0) xT[d2] = lds_read_tr(tl, th, tr_imm(0, d2));
          else txT[d2] = lds_read_tr(tl, th, OFF_TQ + tr_imm(0, d2));
        }
        if (m < FS && !PQ) {
#pragma unroll
          TVM_SHARE(x, m, 4, FS) {  // lse, stats of half 1
            if (x < 2) la[2 + x] = lds_read_f4(rv, (2 + x) * 32);
            else ma[x] = lds_read_f4(rv, 256 + x * 32);
          }
        }
        if (m == FS) landed(sS, sT);
        if (m == ES) landed1(sE);  // (at least four products after the last one of E)
#pragma unroll
        for (int u = kPwE.first[m]; u < kPwE.first[m + 1]; ++u) {
          if (u < 24) pw1k_op(u);
          else pw2e_op(u - 24);
        }
      }
      // ---- OK(0): the products with gZt first; gZ of half 0 behind them, gZ of half 1 behind those with gZ of half 0
#pragma unroll
      for (int m = 0; m < NH; ++m) {
        if (m < 2 * NDB) {
          const int db = m >> 1;
          if ((m & 1) == 0) { if (m == 0) mfma_acc<true>(a0[db], txT[db], frag_of(gzt, 0)); else mfma_acc<RAG>(a0[db], txT[db], frag_of(gzt, 0)); }
          else mfma_acc<RAG>(a1[db], xT[db], frag_of(gzt, 0));
        } else {
          const int db = m - 2 * NDB;
          if (db == 0) mfma_acc<true>(a0[db], xT[db], frag_of(gz, 0));
          else mfma_acc<RAG>(a0[db], xT[db], frag_of(gz, 0));
        }
#pragma unroll
        TVM_SHARE(x, m, 2 * NDB, NH) {  // Q^T, tQ^T of half 1
          const int d2 = x >> 1;
          if ((x & 1) == 0) yT[d2] = lds_read_tr(tl, th, tr_imm(1, d2));
          else tyT[d2] = lds_read_tr(tl, th, OFF_TQ + tr_imm(1, d2));
        }
        if (m == 4) landed1(sDF);  // (four products after the last one of DF)
#pragma unroll
        for (int u = kPwD.first[m]; u < kPwD.first[m + 1]; ++u) pw2d_op(u);
      }
    }
    // every read of this stage has been issued; the next tile (fetched during the previous one) must have landed
    // before anyone goes on, the loads of the tile after next stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    dma_wait_keep<NDMA_PRE>();
    __syncthreads();
    // ---- second half of the output products; Q, tQ rows of the next block; tile loads
#pragma unroll
    for (int m = 0; m < NH; ++m) {
      const int db = m / (PV ? PG : 3), w = m - (PV ? PG : 3) * db;
      if (PV) {
        if (w == 0) { if (m == 0) mfma_acc<true>(a0[db], tyT[db], frag_of(pdk, 1)); else mfma_acc<RAG>(a0[db], tyT[db], frag_of(pdk, 1)); }
        else if (w == 1) mfma_acc<RAG>(a1[db], tyT[db], frag_of(pk, 1));
        else mfma_acc<RAG>(a0[db], yT[db], frag_of(pk, 1));
      } else {
        if (w == 0) { if (m == 0) mfma_acc<true>(a0[db], yT[db], frag_of(gz, 1)); else mfma_acc<RAG>(a0[db], yT[db], frag_of(gz, 1)); }
        else if (w == 1) mfma_acc<RAG>(a0[db], tyT[db], frag_of(gzt, 1));
        else mfma_acc<RAG>(a1[db], yT[db], frag_of(gzt, 1));
      }
#pragma unroll
      TVM_SHARE(x, NS + m, NDMA, NQB) dma(x, in2, sbf, in2last);
#pragma unroll
      TVM_SHARE(x, m, 2 * NKS, NH) {  // Q, tQ rows of the next block
        const int k2 = x % NKS;
        if (x < NKS) rq[k2] = lds_read16((k2 & 1) ? nro : nre, k2 * 32);
        else rtq[k2] = lds_read16((k2 & 1) ? nro : nre, OFF_TQ + k2 * 32);
      }
    }
#undef TVM_SHARE
    // behind the last tile the compiler may move the accumulators right away (a loop exit is where it
    // re-assigns registers): let the last products finish first
    if (last) mfma_settle();
  };

  // One copy of the whole-tile code serves every whole tile; tiles that do not exist are "fetched" as the last
  // tile again.
  const int nfull = nstr >> 5;  // tiles without rows beyond the end
  unsigned st0 = lds0, st1 = lds0 + BUF, st2 = lds0 + 2 * BUF;  // stage of this tile, of the next one, the free one
  for (int t = 0; t < nfull; ++t) {
    tile(std::false_type{}, st0, st1, st2, t * 32, min((t + 2) * 32, ilast), t + 3 >= nt, t + 1 == nt);
    const unsigned r0 = st0;
    st0 = st1;
    st1 = st2;
    st2 = r0;
  }
  if (nt > nfull) tile(std::true_type{}, st0, st1, st2, nfull * 32, ilast, true, true);
  dma_wait();       // the re-fetches of the last tile must be over before the buffers are reused below
  __syncthreads();
  mfma_settle();   // the last output products have landed before the accumulators are read
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    landed_acc(a0[db]);
    landed_acc(a1[db]);
  }
  {
    // nobody reads the tile buffers any more and no tile load is in flight: each wave stages its two output
    // tiles through a region of its own
    constexpr unsigned REG = 32 * (64 * NDB + 16);
    static_assert(4 * REG <= 3 * BUF, "the output staging fits the stages");
    const unsigned lw = lds0 + wave * REG;
    const int row0 = fb * kFix + wave * 32;
    const float scale = PV ? 1.f : s.alpha;
    store_tile_coalesced<NDB>(lw, out0 + base, fsn, row0, nfix, s.D, a0, scale, lane);
    store_tile_coalesced<NDB>(lw, out1 + base, fsn, row0, nfix, s.D, a1, scale, lane);
  }
}

template <int DK, int DV, bool HAS_G>
hipError_t launch_col(const Shape& s, const BwdArgs& a, hipStream_t st) {
  const int nfb = (s.N + kFix - 1) / kFix;
  const dim3 grid(nfb * s.B * s.H), block(kNT);
  // pass K first: it is the longer one
  hipLaunchKernelGGL((bwd_pass_kernel<DK, DV, 2, HAS_G>), grid, block, 0, st, s, (const bf16*)a.k, (const bf16*)a.tk,
                     (const bf16*)a.v, (const bf16*)a.tv, (const bf16*)a.q, (const bf16*)a.tq, (const bf16*)a.gTO,
                     (const bf16*)a.gO, a.lse2, a.stats, a.dsig, a.sig1, nullptr, 1, nullptr, nullptr, (bf16*)a.dk,
                     (bf16*)a.dtk);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((bwd_pass_kernel<DK, DV, 1, HAS_G>), grid, block, 0, st, s, (const bf16*)a.k, (const bf16*)a.tk,
                     (const bf16*)a.v, (const bf16*)a.tv, (const bf16*)a.q, (const bf16*)a.tq, (const bf16*)a.gTO,
                     (const bf16*)a.gO, a.lse2, a.stats, a.dsig, a.sig1, nullptr, 1, nullptr, nullptr, (bf16*)a.dv,
                     (bf16*)a.dtv);
  return hipGetLastError();
}

template <int DK, int DV, bool HAS_G>
hipError_t launch_row(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws) {
  const int nfb = (s.M + kFix - 1) / kFix;
  hipLaunchKernelGGL((bwd_pass_kernel<DK, DV, 3, HAS_G>), dim3(nfb * s.B * s.H), dim3(kNT), 0, st, s, (const bf16*)a.q,
                     (const bf16*)a.tq, (const bf16*)a.gTO, (const bf16*)a.gO, (const bf16*)a.k, (const bf16*)a.tk,
                     (const bf16*)a.v, (const bf16*)a.tv, a.lse, a.stats, a.dsig, a.sig1, a.lse2, pipe_ws ? 1 : 0,
                     (const bf16*)a.o, (const bf16*)a.to, (bf16*)a.dq, (bf16*)a.dtq);
  return hipGetLastError();
}

}  // namespace

// Key side, head dims 97..128, with both upstream gradients (a.mode 0) or with gTO alone (a.mode 2).  Needs the row
// vectors in the workspace in the convention of the hand-scheduled kernels (dsig, sig1 negated, lse in log2 units).
hipError_t launch_bwd_col_pass(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (a.mode == 1 || s.D <= 96 || s.D > 128) return hipErrorNotSupported;
  if (s.D <= 112) return a.mode == 0 ? launch_col<112, 128, true>(s, a, st) : launch_col<112, 128, false>(s, a, st);
  return a.mode == 0 ? launch_col<128, 128, true>(s, a, st) : launch_col<128, 128, false>(s, a, st);
}
// Query side, head dims 97..128, with both upstream gradients or with gTO alone.  pipe_ws: the row vectors go to the
// workspace in that convention (the passes above follow), else plain (the generic-order key-side kernel follows).
hipError_t launch_bwd_row_pass(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws) {
  if (a.mode == 1 || s.D <= 96 || s.D > 128) return hipErrorNotSupported;
  if (s.D <= 112) return a.mode == 0 ? launch_row<112, 128, true>(s, a, st, pipe_ws) : launch_row<112, 128, false>(s, a, st, pipe_ws);
  return a.mode == 0 ? launch_row<128, 128, true>(s, a, st, pipe_ws) : launch_row<128, 128, false>(s, a, st, pipe_ws);
}

}  // namespace tvm
