// Key-side backward kernel (dK, dtK, dV, dtV; Steps 2, 4, 6 of App. C plus the ordinary-attention
// terms of gO) for head dims up to 96, with the instruction stream laid out by hand.  Same
// mathematics and data layout as the generic-order kernel in bwd_mfma_kernels.h.
//
// A wave owns 32 keys (their K, tK, V, tV fragments stay in registers, four accumulators in
// AGPRs) and runs alone on its SIMD, so its VALU work, LDS reads and load issue are hidden only
// if they sit between its own matrix-core products.  Queries are streamed in tiles of 64 = two
// blocks of 32.  The output products of a block split by the contraction half cc (16 queries
// each), which is what lets the pointwise work trail the products by half a block:
//
//   phase     products (matrix cores)            in their shadow
//   S         S, St                              G, tG rows <- LDS;  lse, stats (half 0), -sig1, -dsig <- LDS;  tile loads
//   E         E, DF (from -sig1, -dsig)          P, N, Pd of half 0;  G^T, tG^T of half 0 <- LDS;  lse, stats (half 1) <- LDS
//   OV(0)     dV, dtV += (P, Pd of half 0) .     P, N, Pd of half 1;  G^T, tG^T of half 1 <- LDS
//   OV(1)     dV, dtV += (P, Pd of half 1) .     gZ, gZt of half 0;   Q^T, tQ^T of half 0 <- LDS
//   OK(0)     dK, dtK += (gZ, gZt of half 0) .   gZ, gZt of half 1;   Q^T, tQ^T of half 1 <- LDS
//   -- after the tile's second block: all reads of this buffer are done; the next tile must have landed, barrier --
//   OK(1)     dK, dtK += (gZ, gZt of half 1) .   Q, tQ rows of the next block <- LDS;  tile loads
//
// The pointwise work comes in pieces of one or two instructions, dealt out evenly over the products that
// can carry it (a lone wave has room for about 24 cycles of VALU work behind each product): P, N, Pd
// run from the fifth product of E to the end of OV(0), with half 0 complete when OV(0) starts.
// The row scalars come from the workspace as the hand-scheduled query-side kernel leaves them:
// lse in log2 units, and sig1, dsig negated, so that the E and DF tiles can start from them (the C
// operand of their first product) and gZt = P E, gZ = P DF + gZt N need no subtraction.
// Three LDS stages: tile t in use, tile t+1 landed (it was fetched during tile t-1), tile t+2 being
// fetched, one wave-load every few products and only in the phases without pointwise work.
//
// HAS_G = false is the kernel for a call without gO (the gradient of <gTO, tO> alone, Steps 1-6 of
// App. C by themselves): the products with G vanish, so the E phase has two products per 16 head dims
// instead of three (DF = tG tV^T), OV(0) and OV(1) two per 32 instead of three (dV += tG^T Pd,
// dtV += tG^T P), the G tile is neither fetched nor read, and the pointwise work is dealt out over the
// products that remain.
//
// The translation unit is built with the machine scheduler off: source order is issue order.
#if defined(TVM_PROFILE) && !defined(TVM_PIPE_TANGENT_ONLY) && !defined(TVM_PIPE_QKNORM)
#define TVM_PROF_READER tvmattn_debug_read_prof_col_pipe
#endif
#include "pipe_ops.h"

#include <type_traits>

namespace tvm {
namespace {

constexpr int kFix = 128;  // keys per workgroup (4 waves x 32)
constexpr int kNT = 256;
// One translation unit per variant (they compile side by side): with TVM_PIPE_TANGENT_ONLY defined this
// file yields the kernels for calls without gO and their launcher, else those for calls with both gradients.
#if defined(TVM_PIPE_TANGENT_ONLY)
constexpr bool kHasG = false;
constexpr bool kNorm = false;
#define TVM_PIPE_LAUNCHER launch_bwd_col_pipe_tangent
#elif defined(TVM_PIPE_QKNORM)  // ... and with the backward of the QK-norm of the keys in the epilogue
constexpr bool kHasG = true;
constexpr bool kNorm = true;
#define TVM_PIPE_LAUNCHER launch_bwd_col_pipe_qknorm
#else
constexpr bool kHasG = true;
constexpr bool kNorm = false;
#define TVM_PIPE_LAUNCHER launch_bwd_col_pipe
#endif

typedef __attribute__((ext_vector_type(4))) float f32x4;
__device__ __forceinline__ f32x4 lds_read_f4(unsigned addr, int imm) {
  typedef const f32x4 __attribute__((address_space(3))) * lp;
  return *(lp)(uintptr_t)(addr + (unsigned)imm);
}
__device__ __forceinline__ float f4(const f32x4& v, int t) { return v[t]; }

template <int DK, int DV, bool HAS_G, bool NORM>
__global__ __launch_bounds__(kNT, 1) void bwd_col_pipe_kernel(
    Shape s, const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ tq, const bf16* __restrict__ tk, const bf16* __restrict__ tv,
    const float* __restrict__ lse2w, const float* __restrict__ stats, const bf16* __restrict__ gO,
    const bf16* __restrict__ gTO, const float* __restrict__ dsig, const float* __restrict__ sig1,
    bf16* __restrict__ dk, bf16* __restrict__ dtk, bf16* __restrict__ dv, bf16* __restrict__ dtv,
    const bf16* __restrict__ nx, const bf16* __restrict__ ntx, const float* __restrict__ ngain, float neps,
    float* __restrict__ npart) {
  using TX = Tile<64, DV / 8, kNT / 64>;  // Q, tQ, G, tG: read both ways
  constexpr int OFF_TQ = TX::BYTES, OFF_G = 2 * TX::BYTES, OFF_TG = 3 * TX::BYTES, OFF_ROW = 4 * TX::BYTES;
  constexpr int BUF = 4 * TX::BYTES + 4 * 256;  // one stage: four tiles and four float32 row vectors (64 each)
  __shared__ __attribute__((aligned(16))) char lds[3 * BUF];  // three stages: in use, landed or landing, being filled
  constexpr int NKS = DK / 16, NDB = DV / 32;
  constexpr int NS = 3 * NKS;                      // products of the S phase
  constexpr int NH = 3 * NDB;                      // products of half the OK phase
  constexpr int PG = HAS_G ? 3 : 2;                // products per step of the phases that G takes part in
  constexpr int NE = PG * NKS;                     // products of the E phase
  constexpr int NHV = PG * NDB;                    // products of half the OV phase
  constexpr int NTG = HAS_G ? 2 : 1;               // transposed tiles read for OV (G^T and tG^T, or tG^T alone)
  constexpr int FS = NE > 4 ? 4 : NE - 1;          // first pointwise slot of the E phase
  // The 48 pieces of P, N, Pd of a block are dealt out by cost over the products of E (from FS on) and of
  // OV(0), half 0 (the first 24) complete when OV(0) starts; the 40 pieces of gZ, gZt over those of OV(1)
  // and OK(0), half 0 complete when OK(0) starts.  The transposing reads of those phases count as load.
  struct C {
    static constexpr int pw1(int u) { return ((u % 12) >> 1 == 1 || (u % 12) >> 1 == 2) ? 12 : 8; }
    static constexpr int pw2(int) { return 8; }
    static constexpr int base1(int v) {
      return v < NE ? 8 * share_count(v, NTG * NDB, NE) + (v < FS ? 4 * share_count(v, 4, FS) : 0)
                    : 8 * share_count(v - NE, NTG * NDB, NHV);
    }
    static constexpr int base2(int v) {
      return v < NHV ? 8 * share_count(v, 2 * NDB, NHV) : 8 * share_count(v - NHV, 2 * NDB, NH);
    }
  };
  static constexpr Deal<NE + NHV> kPw1 = deal_out<NE + NHV>(48, FS, NE, 24, C::pw1, C::base1);
  static constexpr Deal<NHV + NH> kPw2 = deal_out<NHV + NH>(40, 0, NHV, 20, C::pw2, C::base2);
  constexpr int NTILE = HAS_G ? 4 : 3;             // tiles fetched per stage (the G tile's place stays empty without gO)
  constexpr int NDMA = NTILE * TX::IPW + 1;        // wave-loads per wave and tile (the last: a row vector)
  // the tile after next is fetched behind the products of the phases that carry no pointwise work:
  // S and OK(1) of both blocks (the last of them behind the tile's barrier)
  constexpr int NQB = NS + NH;                     // such products per block
  constexpr int NDMA_PRE = (2 * NQB - NH) * NDMA / (2 * NQB);  // wave-loads issued before the barrier
  // register files: the accumulators fill 4*NDB*16 AGPRs; K, tK fragments always fit beside them,
  // V and tV fragments where there is room, else they stay in VGPRs
  constexpr bool V_IN_A = 64 * NDB + 12 * NKS <= 256, TV_IN_A = 64 * NDB + 16 * NKS <= 256;
  PROF_ENTRY;
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: what depends on it alone stays out of the VALU
  const int nfb = (s.N + kFix - 1) / kFix;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nfb, fb = wg - bh * nfb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;     // key side (fixed)
  const long long qbase = b * s.qsb + h * s.qsh;  // query side (streamed)
  const long long rbase = (long long)bh * s.M;
  const int j = fb * kFix + wave * 32 + ic;  // this lane's key

  const unsigned pitch = (unsigned)(s.qsn * 2);  // row pitch of the streamed (query-side) tensors in bytes
  const unsigned lds0 = lds_addr_of(lds);
  const int nt = (s.M + 63) >> 6;   // tiles
  const int ilast = (nt - 1) * 64;  // first query of the last tile; loads "beyond" it fetch it again, unused
  // Per-lane byte offsets of this wave's loads within a tile, worked out once: for whole tiles, and for
  // the last tile, where rows past the end fetch its last row again (masked rows, unused).  Wave w also
  // fetches row vector w (lse in log2 units, stats, dsig, sig1) of the tile, one float per lane.
  typename TX::Offs of_full, of_last;
  unsigned rv_full, rv_last;
  {
    const typename TX::Lane lx = TX::lane_setup(s.D, wave, lane);
    of_full = TX::offsets(lx, pitch, 64);
    of_last = TX::offsets(lx, pitch, s.M - ilast);
    rv_full = (unsigned)lane * 4u;
    rv_last = (unsigned)min(lane, s.M - ilast - 1) * 4u;
  }
  const float* const rowsrc = (wave == 0 ? lse2w : wave == 1 ? stats : wave == 2 ? dsig : sig1) + rbase;
  // wave-load number x (compile-time) of the tile whose first query is i0 (< N), into the stage at `buf`;
  // `last`: that tile is the last one
  auto dma = [&](int x, int i0, unsigned buf, bool last) {
    const long long ro = qbase + (long long)i0 * s.qsn;
    const int t = x % TX::IPW;
    const unsigned off = last ? of_last.o[t] : of_full.o[t];
    if (x < TX::IPW) TX::issue_at(off, t, q + ro, buf, wave);
    else if (x < 2 * TX::IPW) TX::issue_at(off, t, tq + ro, buf + OFF_TQ, wave);
    else if (x < 3 * TX::IPW) TX::issue_at(off, t, gTO + ro, buf + OFF_TG, wave);
    else if (x < NTILE * TX::IPW) TX::issue_at(off, t, gO + ro, buf + OFF_G, wave);
    else dma_to_lds<4>(rowsrc + i0, last ? rv_last : rv_full, buf + OFF_ROW + wave * 256);
  };
  const typename TX::RAddr ra = TX::raddr(ic, hh);
  const typename TX::TAddr ta = TX::taddr(ic, hh);
  // Start-up: tile 0 first (its loads are cheap to issue and everything waits for them at the first
  // barrier anyway), then the fixed-side fragments (scattered loads), then, once those have arrived, tile 1.
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, 0, lds0, nt == 1);
  bf16x8 kf[NKS], tkf[NKS], vf[NKS], tvf[NKS];
  gld_frags<NKS>(kf, k + base, s.sn, j, s.N, s.D, hh);
  gld_frags<NKS>(tkf, tk + base, s.sn, j, s.N, s.D, hh);
  gld_frags<NKS>(vf, v + base, s.sn, j, s.N, s.D, hh);
  gld_frags<NKS>(tvf, tv + base, s.sn, j, s.N, s.D, hh);
  PROF_P(11);
  f32x16 aK[NDB], aTK[NDB], aV[NDB], aTV[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    aK[db] = zero16();
    aTK[db] = zero16();
    aV[db] = zero16();
    aTV[db] = zero16();
  }
  // wave-uniform scalars for the assembly blocks (SGPR operands)
  const float c1u = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha * 1.4426950408889634f)));
  const float alphau = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha)));

  PROF_P(14);
  dma_wait();  // tile 0 and this wave's fixed rows
  PROF_P(12);
  // tile 1 goes into the second stage now (any earlier and the waits for the fixed rows, which count
  // outstanding loads, would also wait for it); it lands while tile 0 is computed
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, min(64, ilast), lds0 + BUF, nt <= 2);
  __syncthreads();  // tile 0 has landed
  PROF_P(15);
  bf16x8 rq[NKS], rtq[NKS];  // Q, tQ rows of the block whose S phase comes next
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    rq[kk] = lds_read16(lds0 + ((kk & 1) ? ra.o : ra.e), kk * 32);
    rtq[kk] = lds_read16(lds0 + ((kk & 1) ? ra.o : ra.e), OFF_TQ + kk * 32);
  }

  PROF_P(13);
  PROF_DECL;
  // One tile.  RAG: queries beyond N exist in this tile (only ever the last one).
  //   sb / sbn / sbf: LDS address of this tile's stage / of the next tile's (landed) / of the free one, into
  //   which the tile after next is fetched, one wave-load every few products;  i0: first query;
  //   in2: first query of the tile after next (clamped to the last tile);  in2last: that is the last tile.
  auto tile = [&](auto rag, unsigned sb, unsigned sbn, unsigned sbf, int i0, int in2, bool in2last, bool last) {
    constexpr bool RAG = decltype(rag)::value;
    const unsigned re = sb + ra.e, ro = sb + ra.o;        // rows of Q; tQ, G, tG at + OFF_*
    const unsigned tl = sb + ta.lo, th = sb + ta.hi;      // transposed
    const unsigned rv = sb + OFF_ROW + 16 * hh;           // row vectors: this half's four rows of each group of eight
    const unsigned nre = sbn + ra.e, nro = sbn + ra.o;    // the next tile's rows of Q
#define TVM_SHARE(x, m, CNT, N) for (int x = (m) * (CNT) / (N); x < ((m) + 1) * (CNT) / (N); ++x)

    auto block = [&](auto ibc) {
      constexpr int ib = decltype(ibc)::value;
      bf16x8 rg[NKS], rtg[NKS];
      f32x16 sS, sT, sE, sDF;
      f32x4 la[4], ma[4], da[4], sa[4];  // row scalars of the block's queries, by group of eight
      float pp[16], nn[16];
      unsigned pk[8], pdk[8], gz[8], gzt[8];
      bf16x8 xT[NDB], txT[NDB], yT[NDB], tyT[NDB];  // transposed fragments of the half in use / of the next half

      float ta[8], tb[8], wa[8], wb[8];  // temporaries of element pair e, alive between its pieces
      // P, N, Pd of the block as a stream of 8 x 6 pieces (pair e: elements 2e, 2e+1)
      auto pw1_op = [&](int u) {
        // two pairs take turns, so that no piece reads what the piece right before it wrote
        const int e = 2 * (u / 12) + (u & 1), st = (u % 12) >> 1, g4 = e >> 1, t = (2 * e) & 3;
        if (st == 0) {
          float s0 = sS[2 * e], s1 = sS[2 * e + 1];
          if (RAG) {  // queries beyond N: probability 0
            if (i0 + ib * 32 + drow(2 * e, hh) >= s.M) s0 = -INFINITY;
            if (i0 + ib * 32 + drow(2 * e + 1, hh) >= s.M) s1 = -INFINITY;
          }
          pw_fma2(ta[e], tb[e], s0, s1, c1u, f4(la[g4], t), f4(la[g4], t + 1));
        } else if (st == 1) {
          pw_exp_fma(pp[2 * e], ta[e], nn[2 * e], sT[2 * e], alphau, f4(ma[g4], t));
        } else if (st == 2) {
          pw_exp_fma(pp[2 * e + 1], tb[e], nn[2 * e + 1], sT[2 * e + 1], alphau, f4(ma[g4], t + 1));
        } else if (st == 3) {
          pw_mul2(ta[e], tb[e], pp[2 * e], nn[2 * e], pp[2 * e + 1], nn[2 * e + 1]);
        } else if (st == 4) {
          pw_cvt(pk[e], pp[2 * e], pp[2 * e + 1]);
        } else {
          pw_cvt(pdk[e], ta[e], tb[e]);
        }
      };
      // gZ, gZt of the block as a stream of 8 x 5 pieces (E, DF come with sig1, dsig already subtracted)
      auto pw2_op = [&](int u) {
        const int e = 2 * (u / 10) + (u & 1), st = (u % 10) >> 1;  // two pairs take turns here too
        if (st == 0) pw_mul2(ta[e], tb[e], pp[2 * e], sE[2 * e], pp[2 * e + 1], sE[2 * e + 1]);
        else if (st == 1) pw_mul2(wa[e], wb[e], pp[2 * e], sDF[2 * e], pp[2 * e + 1], sDF[2 * e + 1]);
        else if (st == 2) pw_fmac2(wa[e], wb[e], ta[e], nn[2 * e], tb[e], nn[2 * e + 1]);
        else if (st == 3) pw_cvt(gzt[e], ta[e], tb[e]);
        else pw_cvt(gz[e], wa[e], wb[e]);
      };
      auto tr_imm = [&](int cc, int db) { return (2 * ib + cc) * 16 * TX::PCH * 16 + db * 64; };

      PROF(7);
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
#pragma unroll
        TVM_SHARE(x, m, NTG * NKS, NS) {
          const int k2 = x % NKS;
          if (x < NKS) rtg[k2] = lds_read16((k2 & 1) ? ro : re, OFF_TG + ib * TX::kBlkBytes + k2 * 32);
          else rg[k2] = lds_read16((k2 & 1) ? ro : re, OFF_G + ib * TX::kBlkBytes + k2 * 32);
        }
#pragma unroll
        TVM_SHARE(x, m, 12, NS) {  // -sig1 and -dsig of the block first (the first products of E start from them), then lse, stats of half 0
          if (x < 4) sa[x] = lds_read_f4(rv, 768 + ib * 128 + x * 32);
          else if (x < 8) da[x - 4] = lds_read_f4(rv, 512 + ib * 128 + (x - 4) * 32);
          else if (x < 10) la[x - 8] = lds_read_f4(rv, ib * 128 + (x - 8) * 32);
          else ma[x - 10] = lds_read_f4(rv, 256 + ib * 128 + (x - 10) * 32);
        }
#pragma unroll
        TVM_SHARE(x, ib * NQB + m, NDMA, 2 * NQB) dma(x, in2, sbf, in2last);
      }
      PROF(0);
      // ---- E, with P, N, Pd of half 0.  E and DF start from -sig1 and -dsig of their rows (queries).
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          sE[4 * g4 + t] = sa[g4][t];
          sDF[4 * g4 + t] = da[g4][t];
        }
#pragma unroll
      for (int m = 0; m < NE; ++m) {
        const int kk = m / PG, w = m - PG * kk;
        if (w == 0) {
          if (V_IN_A) mfma_fix<RAG>(sE, rtg[kk], vf[kk]);
          else mfma_vv<RAG>(sE, rtg[kk], vf[kk]);
        } else if (w == 1) {
          if (TV_IN_A) mfma_fix<RAG>(sDF, rtg[kk], tvf[kk]);
          else mfma_vv<RAG>(sDF, rtg[kk], tvf[kk]);
        } else {
          if (V_IN_A) mfma_fix<RAG>(sDF, rg[kk], vf[kk]);
          else mfma_vv<RAG>(sDF, rg[kk], vf[kk]);
        }
#pragma unroll
        TVM_SHARE(x, m, NTG * NDB, NE) {  // tG^T, G^T of half 0
          const int db = x / NTG;
          if (x % NTG == 0) txT[db] = lds_read_tr(tl, th, OFF_TG + tr_imm(0, db));
          else xT[db] = lds_read_tr(tl, th, OFF_G + tr_imm(0, db));
        }
        if (m < FS) {
#pragma unroll
          TVM_SHARE(x, m, 4, FS) {  // lse, stats of half 1
            if (x < 2) la[2 + x] = lds_read_f4(rv, ib * 128 + (2 + x) * 32);
            else ma[x] = lds_read_f4(rv, 256 + ib * 128 + x * 32);
          }
        }
        if (m == FS) {
          if (NE < 6) mfma_settle();
          landed(sS, sT);
        }
        if (m >= FS) {
#pragma unroll
          for (int u = kPw1.first[m]; u < kPw1.first[m + 1]; ++u) pw1_op(u);
        }
      }
      PROF(1);
      // ---- OV(0), with P, N, Pd of half 1
#pragma unroll
      for (int m = 0; m < NHV; ++m) {
        const int db = m / PG, w = m - PG * db;
        if (w == 0) { if (m == 0) mfma_acc<true>(aV[db], txT[db], frag_of(pdk, 0)); else mfma_acc<RAG>(aV[db], txT[db], frag_of(pdk, 0)); }
        else if (w == 1) mfma_acc<RAG>(aTV[db], txT[db], frag_of(pk, 0));
        else mfma_acc<RAG>(aV[db], xT[db], frag_of(pk, 0));
#pragma unroll
        TVM_SHARE(x, m, NTG * NDB, NHV) {  // tG^T, G^T of half 1
          const int d2 = x / NTG;
          if (x % NTG == 0) tyT[d2] = lds_read_tr(tl, th, OFF_TG + tr_imm(1, d2));
          else yT[d2] = lds_read_tr(tl, th, OFF_G + tr_imm(1, d2));
        }
#pragma unroll
        for (int u = kPw1.first[NE + m]; u < kPw1.first[NE + m + 1]; ++u) pw1_op(u);
      }
      PROF(2);
      // ---- OV(1), with gZ, gZt of half 0
#pragma unroll
      for (int m = 0; m < NHV; ++m) {
        const int db = m / PG, w = m - PG * db;
        if (w == 0) { if (m == 0) mfma_acc<true>(aV[db], tyT[db], frag_of(pdk, 1)); else mfma_acc<RAG>(aV[db], tyT[db], frag_of(pdk, 1)); }
        else if (w == 1) mfma_acc<RAG>(aTV[db], tyT[db], frag_of(pk, 1));
        else mfma_acc<RAG>(aV[db], yT[db], frag_of(pk, 1));
#pragma unroll
        TVM_SHARE(x, m, 2 * NDB, NHV) {  // Q^T, tQ^T of half 0
          const int d2 = x >> 1;
          if ((x & 1) == 0) xT[d2] = lds_read_tr(tl, th, tr_imm(0, d2));
          else txT[d2] = lds_read_tr(tl, th, OFF_TQ + tr_imm(0, d2));
        }
        if (m == 0) landed(sE, sDF);  // at least four products after the last one of E
#pragma unroll
        for (int u = kPw2.first[m]; u < kPw2.first[m + 1]; ++u) pw2_op(u);
      }
      PROF(3);
      // ---- OK(0), with gZ, gZt of half 1
#pragma unroll
      for (int m = 0; m < NH; ++m) {
        const int db = m / 3, w = m - 3 * db;
        if (w == 0) { if (m == 0) mfma_acc<true>(aK[db], xT[db], frag_of(gz, 0)); else mfma_acc<RAG>(aK[db], xT[db], frag_of(gz, 0)); }
        else if (w == 1) mfma_acc<RAG>(aK[db], txT[db], frag_of(gzt, 0));
        else mfma_acc<RAG>(aTK[db], xT[db], frag_of(gzt, 0));
#pragma unroll
        TVM_SHARE(x, m, 2 * NDB, NH) {  // Q^T, tQ^T of half 1
          const int d2 = x >> 1;
          if ((x & 1) == 0) yT[d2] = lds_read_tr(tl, th, tr_imm(1, d2));
          else tyT[d2] = lds_read_tr(tl, th, OFF_TQ + tr_imm(1, d2));
        }
#pragma unroll
        for (int u = kPw2.first[NHV + m]; u < kPw2.first[NHV + m + 1]; ++u) pw2_op(u);
      }
      PROF(4);
      if (ib == 1) {
        // every read of this stage has been issued; the next tile (fetched during the previous one) must
        // have landed before anyone goes on, the loads of the tile after next stay in flight
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        dma_wait_keep<NDMA_PRE>();
        __syncthreads();
      }
      PROF(5);
      // ---- OK(1)
#pragma unroll
      for (int m = 0; m < NH; ++m) {
        const int db = m / 3, w = m - 3 * db;
        if (w == 0) { if (m == 0) mfma_acc<true>(aK[db], yT[db], frag_of(gz, 1)); else mfma_acc<RAG>(aK[db], yT[db], frag_of(gz, 1)); }
        else if (w == 1) mfma_acc<RAG>(aK[db], tyT[db], frag_of(gzt, 1));
        else mfma_acc<RAG>(aTK[db], yT[db], frag_of(gzt, 1));
#pragma unroll
        TVM_SHARE(x, ib * NQB + NS + m, NDMA, 2 * NQB) dma(x, in2, sbf, in2last);
#pragma unroll
        TVM_SHARE(x, m, 2 * NKS, NH) {  // Q, tQ rows of the next block
          const int k2 = x % NKS;
          const unsigned a0 = ib == 0 ? ((k2 & 1) ? ro : re) : ((k2 & 1) ? nro : nre);
          const int blk = ib == 0 ? TX::kBlkBytes : 0;
          if (x < NKS) rq[k2] = lds_read16(a0, blk + k2 * 32);
          else rtq[k2] = lds_read16(a0, OFF_TQ + blk + k2 * 32);
        }
      }
      PROF(6);
    };
    block(std::integral_constant<int, 0>{});
    block(std::integral_constant<int, 1>{});
#undef TVM_SHARE
    // behind the last tile the compiler may move the accumulators right away (a loop exit is where it
    // re-assigns registers): let the last products finish first
    if (last) mfma_settle();
  };

  // One copy of the whole-tile code serves every whole tile (it is the copy the compiler allocates
  // registers for best); tiles that do not exist are "fetched" as the last tile again.
  const int nfull = s.M >> 6;  // tiles without queries beyond M
  unsigned st0 = lds0, st1 = lds0 + BUF, st2 = lds0 + 2 * BUF;  // stage of this tile, of the next one, the free one
  for (int t = 0; t < nfull; ++t) {
    tile(std::false_type{}, st0, st1, st2, t * 64, min((t + 2) * 64, ilast), t + 3 >= nt, t + 1 == nt);
    const unsigned r0 = st0;
    st0 = st1;
    st1 = st2;
    st2 = r0;
  }
  if (nt > nfull) tile(std::true_type{}, st0, st1, st2, nfull * 64, ilast, true, true);
  dma_wait();       // the re-fetches of the last tile must be over before the buffers are reused below
  __syncthreads();
  PROF_DUMP;
  mfma_settle();   // the last output products have landed before the accumulators are read
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    landed_acc(aK[db]);
    landed_acc(aTK[db]);
    landed_acc(aV[db]);
    landed_acc(aTV[db]);
  }
  {
    // nobody reads the tile buffers any more and no tile load is in flight: each wave stages its
    // four output tiles through a region of its own
    constexpr unsigned REG = 32 * (64 * NDB + 16);
    const unsigned lw = lds0 + wave * (2 * REG);
    const int row0 = fb * kFix + wave * 32;
    if (!NORM) {
      store_tile_coalesced<NDB>(lw, dk + base, s.sn, row0, s.N, s.D, aK, s.alpha, lane);
      store_tile_coalesced<NDB>(lw, dtk + base, s.sn, row0, s.N, s.D, aTK, s.alpha, lane);
    } else {
      // k and tk were RMS-normalised with a gain before this attention (nx, ntx: the rows before that): the
      // accumulators hold the gradients with respect to the normalised rows; park both tiles and write the
      // gradients with respect to nx, ntx, and this workgroup's row of the gain gradient
      NormRows nr;
      norm_rows_fetch(nr, nx + base, ntx + base, s.sn, row0, s.N, s.D, lane);
      park_tile<NDB>(lw, aK, s.alpha, lane);
      park_tile<NDB>(lw + REG, aTK, s.alpha, lane);
      float gacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      store_tiles_through_norm<NDB>(lw, lw + REG, nr, ngain, neps, dk + base, dtk + base, s.sn, row0, s.N, s.D, lane, gacc);
      gain_partial_row(reinterpret_cast<float*>(lds + 4 * 2 * REG), gacc, npart + (long long)blockIdx.x * s.D, s.D, tid);
    }
    store_tile_coalesced<NDB>(lw, dv + base, s.sn, row0, s.N, s.D, aV, 1.f, lane);
    store_tile_coalesced<NDB>(lw, dtv + base, s.sn, row0, s.N, s.D, aTV, 1.f, lane);
  }
  PROF_EXIT;
}

template <int DK, int DV>
hipError_t launch(const Shape& s, const BwdArgs& a, hipStream_t st) {
  const int nfb = (s.N + kFix - 1) / kFix;
  hipLaunchKernelGGL((bwd_col_pipe_kernel<DK, DV, kHasG, kNorm>), dim3(nfb * s.B * s.H), dim3(kNT), 0, st, s, (const bf16*)a.q,
                     (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk, (const bf16*)a.tv,
                     a.lse2, a.stats, (const bf16*)a.gO, (const bf16*)a.gTO, a.dsig, a.sig1, (bf16*)a.dk,
                     (bf16*)a.dtk, (bf16*)a.dv, (bf16*)a.dtv, (const bf16*)a.nk, (const bf16*)a.ntk, a.ngk, a.neps, a.npart_k);
  return hipGetLastError();
}

}  // namespace

// Head dims up to 96.  Needs the row vectors the hand-scheduled query-side kernel leaves in the
// workspace (dsig, sig1 and lse in log2 units).
hipError_t TVM_PIPE_LAUNCHER(const Shape& s, const BwdArgs& a, hipStream_t st) {
  switch ((s.D + 15) / 16 * 16) {
    case 16: return launch<16, 32>(s, a, st);
    case 32: return launch<32, 32>(s, a, st);
    case 48: return launch<48, 64>(s, a, st);
    case 64: return launch<64, 64>(s, a, st);
    case 80: return launch<80, 96>(s, a, st);
    case 96: return launch<96, 96>(s, a, st);
    default: return hipErrorNotSupported;
  }
}

}  // namespace tvm
