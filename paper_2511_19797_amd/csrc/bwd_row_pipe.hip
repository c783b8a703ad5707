// Query-side backward kernel (dQ, dtQ; Steps 3 and 5 of App. C plus the ordinary-attention terms
// of gO, and the row scalars of Step 1) for head dims up to 96, with the instruction stream of a
// 64-key tile laid out by hand.  Same mathematics and data layout as the generic-order kernel
// in bwd_mfma_kernels.h; what differs is when things are issued.
//
// A wave runs alone on its SIMD (the register budget allows no second wave), so nothing hides
// its VALU work, LDS reads or load issue unless they sit between its own matrix-core products.
// A tile is two 32-key blocks; the products of one block are interleaved with the pointwise work
// of the other, and every memory instruction is issued between products, at least a phase
// before its data is needed:
//
//   phase        products (matrix cores)              in their shadow
//   S(0)         S, St of block 0                     E-fragments of block 0 <- LDS;  tile loads
//   E(0)         E, DF of block 0                     P, N of block 0;  S-fragments of block 1 <- LDS
//   S(1)         S, St of block 1                     gZ, gZt of block 0;  E-fragments of block 1 <- LDS
//   E(1)         E, DF of block 1                     P, N of block 1;  K^T, tK^T of block 0, half 0 <- LDS
//   O(0) half 0  dQ, dtQ += (gZ, gZt of block 0) .    K^T, tK^T of block 0, half 1 <- LDS;  tile loads;  from the
//                                                     fourth product on: gZ, gZt of block 1
//   O(0) half 1                                       gZ, gZt of block 1;  K^T, tK^T of block 1, half 0 <- LDS
//   O(1) half 0  dQ, dtQ += (gZ, gZt of block 1) .    K^T, tK^T of block 1, half 1 <- LDS;  tile loads
//   -- all reads of this tile's buffer are done: the next tile must have landed, workgroup barrier --
//   O(1) half 1                                       S-fragments of tile t+1 <- LDS;  tile loads
//
// The pointwise work comes in pieces of one or two instructions, dealt out evenly over the products of
// its phase: a lone wave has room for about 24 cycles of VALU work behind each product.
// "half" = contraction half of an output product (16 keys).  E and DF start from constant tiles
// holding -sig1 and -dsig of the lane's query, so gZt = P E, gZ = P DF + gZt N need no subtraction.
// Three LDS stages: tile t in use, tile t+1 landed (it was fetched during tile t-1), tile t+2 being
// fetched, one wave-load every few products and only in the phases without pointwise work.
//
// HAS_G = false is the kernel for a call without gO (the gradient of <gTO, tO> alone, Steps 1-6 of
// App. C by themselves): DF = tG tV^T and delta = 0, so an E phase has two products per 16 head dims
// instead of three, the fragments of gO are not loaded, and P, N are dealt out over the products left.
//
// The translation unit is built with the machine scheduler off: source order is issue order.
#if defined(TVM_PROFILE) && !defined(TVM_PIPE_TANGENT_ONLY) && !defined(TVM_PIPE_QKNORM)
#define TVM_PROF_READER tvmattn_debug_read_prof_row_pipe
#endif
#include "pipe_ops.h"

#include <type_traits>

namespace tvm {
namespace {

constexpr int kFix = 128;  // queries per workgroup (4 waves x 32)
constexpr int kNT = 256;
constexpr float kLog2e = 1.4426950408889634f;
// One translation unit per variant (they compile side by side): with TVM_PIPE_TANGENT_ONLY defined this
// file yields the kernels for calls without gO and their launcher, else those for calls with both gradients.
#if defined(TVM_PIPE_TANGENT_ONLY)
constexpr bool kHasG = false;
constexpr bool kNorm = false;
#define TVM_PIPE_LAUNCHER launch_bwd_row_pipe_tangent
#elif defined(TVM_PIPE_QKNORM)  // ... and with the backward of the QK-norm of the queries in the epilogue
constexpr bool kHasG = true;
constexpr bool kNorm = true;
#define TVM_PIPE_LAUNCHER launch_bwd_row_pipe_qknorm
#else
constexpr bool kHasG = true;
constexpr bool kNorm = false;
#define TVM_PIPE_LAUNCHER launch_bwd_row_pipe
#endif


template <int DK, int DV, bool HAS_G, bool NORM>
__global__ __launch_bounds__(kNT, 1) void bwd_row_pipe_kernel(
    Shape s, const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ tq, const bf16* __restrict__ tk, const bf16* __restrict__ tv,
    const bf16* __restrict__ o, const bf16* __restrict__ to, const float* __restrict__ lse,
    const float* __restrict__ stats, const bf16* __restrict__ gO, const bf16* __restrict__ gTO,
    float* __restrict__ dsig, float* __restrict__ sig1, float* __restrict__ lse2w, bf16* __restrict__ dq,
    bf16* __restrict__ dtq, const bf16* __restrict__ nx, const bf16* __restrict__ ntx, const float* __restrict__ ngain,
    float neps, float* __restrict__ npart) {
  using TK = Tile<64, DV / 8, kNT / 64>;  // K, tK: read both ways
  using TV = Tile<64, DK / 8, kNT / 64>;  // V, tV: score-type products only
  constexpr int OFF_TK = TK::BYTES, OFF_V = 2 * TK::BYTES, OFF_TV = 2 * TK::BYTES + TV::BYTES;
  constexpr int BUF = 2 * TK::BYTES + 2 * TV::BYTES;  // one stage: K, tK, V, tV
  __shared__ __attribute__((aligned(16))) char lds[3 * BUF];  // three stages: in use, landed or landing, being filled
  constexpr int NKS = DK / 16, NDB = DV / 32;
  constexpr int NS = 3 * NKS;                         // products of an S phase
  constexpr int PE = HAS_G ? 3 : 2;                   // products per 16 head dims of an E phase (without gO: DF = tG tV^T alone)
  constexpr int NE = PE * NKS;                        // products of an E phase
  constexpr int NH = 3 * NDB;                         // products of half an output phase
  constexpr int FS = NS > 4 ? 4 : NS - 1;             // first pointwise slot of an S phase
  constexpr int FE = NE > 4 ? 4 : NE - 1;             // ... of an E phase
  constexpr int P2S = NH > 3 ? 3 : NH;                // first product of O(0) behind which gZ, gZt of block 1 are made
  constexpr int NDMA = 2 * TK::IPW + 2 * TV::IPW;     // wave-loads per wave and tile
  // the tile after next is fetched behind the products of the phases that carry no pointwise work:
  // S(0), O(0) half 0, O(1) half 0 (before the barrier) and O(1) half 1 (behind it)
  constexpr int NQUIET = NS + 3 * NH;
  constexpr int NDMA_PRE = (NS + 2 * NH) * NDMA / NQUIET;  // wave-loads issued before the barrier
  PROF_ENTRY;
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: what depends on it alone stays out of the VALU
  const int nfb = (s.M + kFix - 1) / kFix;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nfb, fb = wg - bh * nfb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;     // key side (streamed)
  const long long qbase = b * s.qsb + h * s.qsh;  // query side (fixed)
  const int i = fb * kFix + wave * 32 + ic;  // this lane's query
  const bool iok = i < s.M;

  const unsigned pitch = (unsigned)(s.sn * 2);  // row pitch in bytes
  const unsigned lds0 = lds_addr_of(lds);
  const int nt = (s.N + 63) >> 6;      // tiles
  const int jlast = (nt - 1) * 64;     // first key of the last tile; loads "beyond" it fetch it again, unused
  // Per-lane byte offsets of this wave's loads within a tile, worked out once: for whole tiles, and for
  // the last tile, where rows past the end fetch its last row again (keys of probability 0)
  typename TK::Offs ok_full, ok_last;
  typename TV::Offs ov_full, ov_last;
  {
    const typename TK::Lane lk = TK::lane_setup(s.D, wave, lane);
    const typename TV::Lane lv = TV::lane_setup(s.D, wave, lane);
    ok_full = TK::offsets(lk, pitch, 64);
    ok_last = TK::offsets(lk, pitch, s.N - jlast);
    ov_full = TV::offsets(lv, pitch, 64);
    ov_last = TV::offsets(lv, pitch, s.N - jlast);
  }
  // wave-load number x (compile-time) of the tile whose first key is j0 (< N), into the stage at `buf`;
  // `last`: that tile is the last one
  auto dma = [&](int x, int j0, unsigned buf, bool last) {
    const long long ro = base + (long long)j0 * s.sn;
    if (x < 2 * TK::IPW) {
      const int t = x % TK::IPW;
      const unsigned off = last ? ok_last.o[t] : ok_full.o[t];
      if (x < TK::IPW) TK::issue_at(off, t, k + ro, buf, wave);
      else TK::issue_at(off, t, tk + ro, buf + OFF_TK, wave);
    } else {
      const int t = (x - 2 * TK::IPW) % TV::IPW;
      const unsigned off = last ? ov_last.o[t] : ov_full.o[t];
      if (x < 2 * TK::IPW + TV::IPW) TV::issue_at(off, t, v + ro, buf + OFF_V, wave);
      else TV::issue_at(off, t, tv + ro, buf + OFF_TV, wave);
    }
  };
  const typename TK::RAddr rk = TK::raddr(ic, hh);
  const typename TV::RAddr rv = TV::raddr(ic, hh);
  const typename TK::TAddr ta = TK::taddr(ic, hh);
  // Start-up: tile 0 first (its loads are cheap to issue and everything waits for them at the first
  // barrier anyway), then this lane's row scalars and fixed-side fragments (scattered loads), then, once those have arrived, tile 1.
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, 0, lds0, nt == 1);
  // rows beyond N: zeros keep everything finite; nothing of theirs is stored
  const long long r = (long long)bh * s.M + (iok ? i : 0);
  const float lse2 = iok ? lse[r] * kLog2e : 0.f;
  const float mub = iok ? stats[r] : 0.f;
  bf16x8 qf[NKS], tqf[NKS], gf[NKS], tgf[NKS], of[NKS], tof[NKS];
  if (HAS_G) gld_frags<NKS>(gf, gO + qbase, s.qsn, i, s.M, s.D, hh);
  gld_frags<NKS>(tgf, gTO + qbase, s.qsn, i, s.M, s.D, hh);
  gld_frags<NKS>(of, o + qbase, s.qsn, i, s.M, s.D, hh);
  gld_frags<NKS>(tof, to + qbase, s.qsn, i, s.M, s.D, hh);
  gld_frags<NKS>(qf, q + qbase, s.qsn, i, s.M, s.D, hh);
  gld_frags<NKS>(tqf, tq + qbase, s.qsn, i, s.M, s.D, hh);
  PROF_P(11);
  // Step 1 of App. C, fused: the row scalars delta + Sigma_2 = gO.O + gTO.tO and Sigma_1 = gTO.O of
  // this lane's query, from the same fragment layout (each half-wave holds half of the row), two
  // bf16 products per instruction, accumulated in float32; they are also written out for the
  // key-side kernel, which runs after this one.
  float ds = 0.f, s1 = 0.f;
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk)
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const bf16x2 tg2 = {tgf[kk][e], tgf[kk][e + 1]};
      const bf16x2 o2 = {of[kk][e], of[kk][e + 1]};
      const bf16x2 to2 = {tof[kk][e], tof[kk][e + 1]};
      if (HAS_G) {
        const bf16x2 g2 = {gf[kk][e], gf[kk][e + 1]};
        ds = __builtin_amdgcn_fdot2_f32_bf16(g2, o2, ds, false);
      }
      ds = __builtin_amdgcn_fdot2_f32_bf16(tg2, to2, ds, false);
      s1 = __builtin_amdgcn_fdot2_f32_bf16(tg2, o2, s1, false);
    }
  PROF_P(12);
  ds += xhalf(ds);
  s1 += xhalf(s1);
  PROF_P(13);
  // E and DF tiles start from -sig1 and -dsig of this lane's query (the same value in all 16
  // registers), which takes the subtractions out of the pointwise work
  f32x16 cE, cDF;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    cE[e] = -s1;
    cDF[e] = -ds;
  }
  asm volatile("" : "+v"(cE), "+v"(cDF));  // materialised here, once
  if (iok && hh == 0) {
    dsig[r] = -ds;  // negated: the key-side kernel starts its DF and E tiles from these
    sig1[r] = -s1;
    lse2w[r] = lse2;
  }
  f32x16 aQ[NDB], aTQ[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    aQ[db] = zero16();
    aTQ[db] = zero16();
  }
  // wave-uniform scalars for the assembly blocks (SGPR operands)
  const float c1u = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha * kLog2e)));
  const float alphau = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s.alpha)));

  PROF_P(14);
  dma_wait();  // tile 0 and this wave's fixed rows
  // tile 1 goes into the second stage now (any earlier and the waits for the fixed rows, which count
  // outstanding loads, would also wait for it); it lands while tile 0 is computed
#pragma unroll
  for (int x = 0; x < NDMA; ++x) dma(x, min(64, jlast), lds0 + BUF, nt <= 2);
  __syncthreads();  // tile 0 has landed
  PROF_P(15);
  bf16x8 ra[NKS], rb[NKS];  // S-fragments (K, tK rows) of the block whose S phase comes next
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    ra[kk] = lds_read16(lds0 + ((kk & 1) ? rk.o : rk.e), kk * 32);
    rb[kk] = lds_read16(lds0 + ((kk & 1) ? rk.o : rk.e), OFF_TK + kk * 32);
  }

  PROF_DECL;
  // One tile.  RAG: keys beyond N exist in this tile (only ever the last one).
  //   sb / sbn / sbf: LDS address of this tile's stage / of the next tile's (landed) / of the free one, into
  //   which the tile after next is fetched, one wave-load every few products;  j0: first key;
  //   jn2: first key of the tile after next (clamped to the last tile);  jn2last: that is the last tile.
  auto tile = [&](auto rag, unsigned sb, unsigned sbn, unsigned sbf, int j0, int jn2, bool jn2last, bool last) {
    constexpr bool RAG = decltype(rag)::value;
    const unsigned ke = sb + rk.e, ko = sb + rk.o;                   // K rows; tK at + OFF_TK
    const unsigned ve = sb + OFF_V + rv.e, vo = sb + OFF_V + rv.o;   // V rows; tV at + TV::BYTES
    const unsigned tl = sb + ta.lo, th = sb + ta.hi;                 // K transposed; tK at + OFF_TK
    const unsigned nke = sbn + rk.e, nko = sbn + rk.o;               // next tile's K rows
    bf16x8 rc[NKS], rd[NKS];
    f32x16 sS, sT, sE, sDF;
    float pp[16], nn[16];
    unsigned gz0[8], gzt0[8], gz1[8], gzt1[8];
    bf16x8 xT[NDB], txT[NDB], yT[NDB], tyT[NDB];  // transposed K, tK of the half in use / of the next half

    auto s_product = [&](int m) {  // m-th product of an S phase (operands ra, rb)
      const int kk = m / 3, w = m - 3 * kk;
      if (w == 0) {
        if (kk == 0) mfma_fix0<RAG>(sS, ra[0], qf[0]);
        else mfma_fix<RAG>(sS, ra[kk], qf[kk]);
      } else if (w == 1) {
        if (kk == 0) mfma_fix0<RAG>(sT, ra[0], tqf[0]);
        else mfma_fix<RAG>(sT, ra[kk], tqf[kk]);
      } else {
        mfma_fix<RAG>(sT, rb[kk], qf[kk]);
      }
    };
    auto e_product = [&](int m) {  // m-th product of an E phase (operands rc, rd)
      const int kk = m / PE, w = m - PE * kk;
      if (w == 0) {
        if (kk == 0) mfma_fixc<RAG>(sE, rc[0], tgf[0], cE);
        else mfma_fix<RAG>(sE, rc[kk], tgf[kk]);
      } else if (w == 1) {
        if (kk == 0) mfma_fixc<RAG>(sDF, rd[0], tgf[0], cDF);
        else mfma_fix<RAG>(sDF, rd[kk], tgf[kk]);
      } else {
        mfma_fix<RAG>(sDF, rc[kk], gf[kk]);
      }
    };
    // m-th product of half cc of an output phase (transposed fragments xT, txT of that half)
    auto o_product = [&](int m, int cc, const bf16x8 (&xT)[NDB], const bf16x8 (&txT)[NDB], const unsigned (&gz)[8],
                         const unsigned (&gzt)[8]) {
      const int db = m / 3, w = m - 3 * db;
      if (w == 0) {
        if (m == 0) mfma_acc<true>(aQ[db], xT[db], frag_of(gz, cc));  // gz, gzt may have been written just before
        else mfma_acc<RAG>(aQ[db], xT[db], frag_of(gz, cc));
      } else if (w == 1) {
        mfma_acc<RAG>(aQ[db], txT[db], frag_of(gzt, cc));
      } else {
        mfma_acc<RAG>(aTQ[db], xT[db], frag_of(gzt, cc));
      }
    };
    auto tr_imm = [&](int blk, int cc, int db) { return (2 * blk + cc) * 16 * TK::PCH * 16 + db * 64; };
    float ta[8], tb[8], wa[8], wb[8];  // temporaries, alive between the pieces of an element pair
    // P and N of a block as a stream of 8 x 3 pieces (pair e = u / 3: elements 2e, 2e+1)
    auto pw1_op = [&](int blk, int u) {
      const int e = u / 3, st = u - 3 * e;
      if (st == 0) {
        float s0 = sS[2 * e], s1 = sS[2 * e + 1];
        if (RAG) {  // keys beyond N: probability 0
          if (j0 + blk * 32 + drow(2 * e, hh) >= s.N) s0 = -INFINITY;
          if (j0 + blk * 32 + drow(2 * e + 1, hh) >= s.N) s1 = -INFINITY;
        }
        pw_fma2(ta[e], tb[e], s0, s1, c1u, lse2, lse2);
      } else if (st == 1) {
        pw_exp_fma(pp[2 * e], ta[e], nn[2 * e], sT[2 * e], alphau, mub);
      } else {
        pw_exp_fma(pp[2 * e + 1], tb[e], nn[2 * e + 1], sT[2 * e + 1], alphau, mub);
      }
    };
    // gZ, gZt of a block as a stream of 8 x 5 pieces (pair e = u / 5: elements 2e, 2e+1)
    auto pw2_op = [&](unsigned (&gz)[8], unsigned (&gzt)[8], int u) {
      const int e = u / 5, st = u - 5 * e;
      if (st == 0) pw_mul2(ta[e], tb[e], pp[2 * e], sE[2 * e], pp[2 * e + 1], sE[2 * e + 1]);
      else if (st == 1) pw_mul2(wa[e], wb[e], pp[2 * e], sDF[2 * e], pp[2 * e + 1], sDF[2 * e + 1]);
      else if (st == 2) pw_fmac2(wa[e], wb[e], ta[e], nn[2 * e], tb[e], nn[2 * e + 1]);
      else if (st == 3) pw_cvt(gzt[e], ta[e], tb[e]);
      else pw_cvt(gz[e], wa[e], wb[e]);
    };
    // share [m*CNT/N, (m+1)*CNT/N) of CNT side instructions goes after the m-th of N products
#define TVM_SHARE(x, m, CNT, N) for (int x = (m) * (CNT) / (N); x < ((m) + 1) * (CNT) / (N); ++x)

    PROF(7);
    // ---- S(0)
#pragma unroll
    for (int m = 0; m < NS; ++m) {
      s_product(m);
#pragma unroll
      TVM_SHARE(x, m, 2 * NKS, NS) {
        const int kk = x % NKS;
        if (x < NKS) rc[kk] = lds_read16((kk & 1) ? vo : ve, kk * 32);
        else rd[kk] = lds_read16((kk & 1) ? vo : ve, TV::BYTES + kk * 32);
      }
#pragma unroll
      TVM_SHARE(x, m, NDMA, NQUIET) dma(x, jn2, sbf, jn2last);
    }
    PROF(0);
    // ---- E(0), with P, N of block 0
#pragma unroll
    for (int m = 0; m < NE; ++m) {
      e_product(m);
#pragma unroll
      TVM_SHARE(x, m, 2 * NKS, NE) {  // S-fragments of block 1
        const int kk = x % NKS;
        if (x < NKS) ra[kk] = lds_read16((kk & 1) ? ko : ke, TK::kBlkBytes + kk * 32);
        else rb[kk] = lds_read16((kk & 1) ? ko : ke, OFF_TK + TK::kBlkBytes + kk * 32);
      }
      if (m == FE) {
        if (NE < 6) mfma_settle();
        landed(sS, sT);
      }
      if (m >= FE) {
#pragma unroll
        TVM_SHARE(u, m - FE, 24, NE - FE) pw1_op(0, u);
      }
    }
    PROF(1);
    // ---- S(1), with gZ, gZt of block 0
#pragma unroll
    for (int m = 0; m < NS; ++m) {
      s_product(m);
#pragma unroll
      TVM_SHARE(x, m, 2 * NKS, NS) {  // E-fragments of block 1
        const int kk = x % NKS;
        if (x < NKS) rc[kk] = lds_read16((kk & 1) ? vo : ve, TV::kBlkBytes + kk * 32);
        else rd[kk] = lds_read16((kk & 1) ? vo : ve, TV::BYTES + TV::kBlkBytes + kk * 32);
      }
      if (m == FS) {
        if (NS < 6) mfma_settle();
        landed(sE, sDF);
      }
      if (m >= FS) {
#pragma unroll
        TVM_SHARE(u, m - FS, 40, NS - FS) pw2_op(gz0, gzt0, u);
      }
    }
    PROF(2);
    // ---- E(1), with P, N of block 1
#pragma unroll
    for (int m = 0; m < NE; ++m) {
      e_product(m);
#pragma unroll
      TVM_SHARE(x, m, 2 * NDB, NE) {  // transposed K, tK of block 0, half 0
        const int db = x >> 1;
        if ((x & 1) == 0) xT[db] = lds_read_tr(tl, th, tr_imm(0, 0, db));
        else txT[db] = lds_read_tr(tl, th, OFF_TK + tr_imm(0, 0, db));
      }
      if (m == FE) {
        if (NE < 6) mfma_settle();
        landed(sS, sT);
      }
      if (m >= FE) {
#pragma unroll
        TVM_SHARE(u, m - FE, 24, NE - FE) pw1_op(1, u);
      }
    }
    PROF(3);
    // ---- O(0), with gZ, gZt of block 1 (spread over both halves)
#pragma unroll
    for (int m = 0; m < NH; ++m) {
      o_product(m, 0, xT, txT, gz0, gzt0);
#pragma unroll
      TVM_SHARE(x, NS + m, NDMA, NQUIET) dma(x, jn2, sbf, jn2last);
#pragma unroll
      TVM_SHARE(x, m, 2 * NDB, NH) {  // ... of block 0, half 1
        const int db = x >> 1;
        if ((x & 1) == 0) yT[db] = lds_read_tr(tl, th, tr_imm(0, 1, db));
        else tyT[db] = lds_read_tr(tl, th, OFF_TK + tr_imm(0, 1, db));
      }
      // gZ, gZt of block 1 start four products behind the last one of E(1) (where half 0 is that long) and
      // run to the end of half 1
      if (m == P2S) landed(sE, sDF);
      if (m >= P2S) {
#pragma unroll
        TVM_SHARE(u, m - P2S, 40, 2 * NH - P2S) pw2_op(gz1, gzt1, u);
      }
    }
#pragma unroll
    for (int m = 0; m < NH; ++m) {
      o_product(m, 1, yT, tyT, gz0, gzt0);
#pragma unroll
      TVM_SHARE(x, m, 2 * NDB, NH) {  // ... of block 1, half 0
        const int db = x >> 1;
        if ((x & 1) == 0) xT[db] = lds_read_tr(tl, th, tr_imm(1, 0, db));
        else txT[db] = lds_read_tr(tl, th, OFF_TK + tr_imm(1, 0, db));
      }
      if (P2S == NH && m == 0) landed(sE, sDF);  // NH + 1 >= 4 products behind the last one of E(1)
#pragma unroll
      TVM_SHARE(u, NH - P2S + m, 40, 2 * NH - P2S) pw2_op(gz1, gzt1, u);
    }
    PROF(4);
    // ---- O(1), half 0
#pragma unroll
    for (int m = 0; m < NH; ++m) {
      o_product(m, 0, xT, txT, gz1, gzt1);
#pragma unroll
      TVM_SHARE(x, NS + NH + m, NDMA, NQUIET) dma(x, jn2, sbf, jn2last);
#pragma unroll
      TVM_SHARE(x, m, 2 * NDB, NH) {  // ... of block 1, half 1
        const int db = x >> 1;
        if ((x & 1) == 0) yT[db] = lds_read_tr(tl, th, tr_imm(1, 1, db));
        else tyT[db] = lds_read_tr(tl, th, OFF_TK + tr_imm(1, 1, db));
      }
    }
    // every read of this stage has been issued; the next tile (fetched during the previous one) must have
    // landed before anyone goes on, the loads of the tile after next stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    dma_wait_keep<NDMA_PRE>();
    __syncthreads();
    PROF(5);
    // ---- O(1), half 1
#pragma unroll
    for (int m = 0; m < NH; ++m) {
      o_product(m, 1, yT, tyT, gz1, gzt1);
#pragma unroll
      TVM_SHARE(x, NS + 2 * NH + m, NDMA, NQUIET) dma(x, jn2, sbf, jn2last);
#pragma unroll
      TVM_SHARE(x, m, 2 * NKS, NH) {  // S-fragments of the next tile's block 0
        const int kk = x % NKS;
        if (x < NKS) ra[kk] = lds_read16((kk & 1) ? nko : nke, kk * 32);
        else rb[kk] = lds_read16((kk & 1) ? nko : nke, OFF_TK + kk * 32);
      }
    }
#undef TVM_SHARE
    PROF(6);
    // behind the last tile the compiler may move the accumulators right away (a loop exit is where it
    // re-assigns registers): let the last products finish first
    if (last) mfma_settle();
  };

  // the row scalars are first used inside the tile: make the compiler wait for their loads here,
  // not in the loop (where its wait would also cover the tile loads in flight)
  asm volatile("" ::"v"(lse2), "v"(mub));
  // One copy of the whole-tile code serves every whole tile (it is the copy the compiler allocates
  // registers for best); tiles that do not exist are "fetched" as the last tile again.
  const int nfull = s.N >> 6;  // tiles without keys beyond N
  unsigned st0 = lds0, st1 = lds0 + BUF, st2 = lds0 + 2 * BUF;  // stage of this tile, of the next one, the free one
  for (int t = 0; t < nfull; ++t) {
    tile(std::false_type{}, st0, st1, st2, t * 64, min((t + 2) * 64, jlast), t + 3 >= nt, t + 1 == nt);
    const unsigned r0 = st0;
    st0 = st1;
    st1 = st2;
    st2 = r0;
  }
  if (nt > nfull) tile(std::true_type{}, st0, st1, st2, nfull * 64, jlast, true, true);
  dma_wait();       // the re-fetches of the last tile must be over before the buffers are reused below
  __syncthreads();
  PROF_DUMP;
  mfma_settle();   // the last output products have landed before the accumulators are read
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    landed_acc(aQ[db]);
    landed_acc(aTQ[db]);
  }
  if (!NORM) {
    // nobody reads the tile buffers any more and no tile load is in flight: each wave stages its
    // two output tiles through a region of its own
    const unsigned lw = lds0 + wave * (32 * (64 * NDB + 16));
    const int row0 = fb * kFix + wave * 32;
    store_tile_coalesced<NDB>(lw, dq + qbase, s.qsn, row0, s.M, s.D, aQ, s.alpha, lane);
    store_tile_coalesced<NDB>(lw, dtq + qbase, s.qsn, row0, s.M, s.D, aTQ, s.alpha, lane);
  } else {
    // q and tq were RMS-normalised with a gain before this attention (nx, ntx: the rows before that): what is
    // in the accumulators are the gradients with respect to the normalised rows; park both tiles and write the
    // gradients with respect to nx, ntx, and this workgroup's row of the gain gradient
    constexpr unsigned REG = 32 * (64 * NDB + 16);
    const unsigned lw = lds0 + wave * (2 * REG);
    const int row0 = fb * kFix + wave * 32;
    NormRows nr;
    norm_rows_fetch(nr, nx + qbase, ntx + qbase, s.qsn, row0, s.M, s.D, lane);
    park_tile<NDB>(lw, aQ, s.alpha, lane);
    park_tile<NDB>(lw + REG, aTQ, s.alpha, lane);
    float gacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_tiles_through_norm<NDB>(lw, lw + REG, nr, ngain, neps, dq + qbase, dtq + qbase, s.qsn, row0, s.M, s.D, lane, gacc);
    gain_partial_row(reinterpret_cast<float*>(lds + 4 * 2 * REG), gacc, npart + (long long)blockIdx.x * s.D, s.D, tid);
  }
  PROF_EXIT;
}

template <int DK, int DV>
hipError_t launch(const Shape& s, const BwdArgs& a, hipStream_t st) {
  const int nfb = (s.M + kFix - 1) / kFix;
  hipLaunchKernelGGL((bwd_row_pipe_kernel<DK, DV, kHasG, kNorm>), dim3(nfb * s.B * s.H), dim3(kNT), 0, st, s, (const bf16*)a.q,
                     (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk, (const bf16*)a.tv,
                     (const bf16*)a.o, (const bf16*)a.to, a.lse, a.stats, (const bf16*)a.gO, (const bf16*)a.gTO,
                     a.dsig, a.sig1, a.lse2, (bf16*)a.dq, (bf16*)a.dtq, (const bf16*)a.nq, (const bf16*)a.ntq, a.ngq, a.neps,
                     a.npart_q);
  return hipGetLastError();
}

}  // namespace

// Head dims up to 96.
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
