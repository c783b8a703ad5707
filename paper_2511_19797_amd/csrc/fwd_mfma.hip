// Forward with tangent on the bf16 matrix cores (gfx950).
//
// One workgroup = NW waves, 32 query rows per wave, all of one (batch, head) (M queries, N keys); a wave keeps Q, tQ
// as B-operand fragments in registers for the whole kernel.  Keys are streamed in tiles of 64
// through LDS (row-major, swizzled): K, tK are read as score-product A operands, V, tV through
// the transposing LDS read as output-product A operands.  The next tile's global loads are
// issued into registers before the current tile is computed, so HBM/L2 latency hides behind
// the matrix-core work.
//
// Everything is computed transposed, S^T = K Q^T, so that a lane owns ONE query row (column ic
// of every D tile): row max / row sums are in-lane reductions plus one exchange between the two
// half-waves, the online-softmax rescale is a per-lane scalar, and the probabilities feed the
// next product from registers.
//
// Per 32-key block (the equations under "Step 1" of App. C, evaluated against a reference
// maximum m that is only raised when some row's maximum outgrows it by more than 2^8, so the
// accumulator rescale is rare; the final division by l makes the choice of m immaterial):
//   S^T  = K Q^T            St^T = K tQ^T + tK Q^T
//   p    = exp(alpha S - m)               (un-normalised)
//   l   += sum p ;  c += sum p * alpha St
//   accO += p V ;   accT += (p * alpha St) V + p tV
// Epilogue: O = accO / l,  stats = c / l,  tO = accT / l - stats * O,  lse = m + log l.
//
// Where the head dim leaves a spare column in the output tiles (D < DV, e.g. 72 in 96) the two
// row sums cost no VALU work: column D of the V tile is set to one and that of the tV tile to
// zero in LDS, so row D of accO is l and row D of accT is c, accumulated (and rescaled) by the
// matrix cores along with everything else, from the same bf16-rounded weights as the outputs.
#include "mfma_tiles.h"
#ifndef FWD_WIDE_FROM
#define FWD_WIDE_FROM 512  // keys from which a workgroup is eight waves instead of four (see launch)
#endif
#ifndef FWD_NW
#define FWD_NW 4   // waves per workgroup (two workgroups share a CU)
#define FWD_BN 32  // keys per LDS tile (one 32-key block)
#endif
// A second translation unit builds the same kernels with the query side's RMSNorm folded in (fwd_mfma_qnorm.hip):
// q, tq are then the rows before the normalisation, and each wave normalises its 32 rows where it loads them as
// fragments (RMSNorm with gain and its tangent: Sec. "Semi-Lipschitz control"; App. "Lipschitzness of RMSNorm"),
// writes the normalised rows out for the backward, and goes on as usual.
#ifndef TVM_FWD_QNORM
#define TVM_FWD_QNORM 0
#define TVM_FWD_LAUNCHER launch_fwd_mfma
#endif

namespace tvm {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleLog2 = 8.f;  // raise the reference maximum only beyond this growth (log2 units)

template <int DK, int DV, int NW, int kBN, bool SPARE>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void fwd_mfma_kernel(Shape s, const bf16* __restrict__ q,
                                                          const bf16* __restrict__ k, const bf16* __restrict__ v,
                                                          const bf16* __restrict__ tq, const bf16* __restrict__ tk,
                                                          const bf16* __restrict__ tv, bf16* __restrict__ o,
                                                          bf16* __restrict__ to, float* __restrict__ lse,
                                                          float* __restrict__ stats, const float* __restrict__ ngain,
                                                          float neps, bf16* __restrict__ qn, bf16* __restrict__ tqn) {
  constexpr bool QNORM = TVM_FWD_QNORM != 0;
  constexpr int NT = 64 * NW, BM = 32 * NW;
  using TK = Tile<kBN, DK / 8, NW>;
  using TV = Tile<kBN, DV / 8, NW>;
  constexpr int BUF = 2 * TK::BYTES + 2 * TV::BYTES;  // one stage: K, tK, V, tV
  __shared__ __attribute__((aligned(16))) char lds[2 * BUF];
  constexpr int NKS = DK / 16, NDB = DV / 32;
  static_assert(kBN == 32, "one block per tile: the spare-column rows are planted by 32 lanes");
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: what depends on it alone stays out of the VALU
  const int nmb = (s.M + BM - 1) / BM;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nmb, mb = wg - bh * nmb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;     // key side
  const long long qbase = b * s.qsb + h * s.qsh;  // query side
  const int i = mb * BM + wave * 32 + ic;  // this lane's query row
  const bool iok = i < s.M;

  const unsigned pitch = (unsigned)(s.sn * 2);  // row pitch in bytes
  const unsigned lds0 = lds_addr_of(lds);
  // per-lane byte offsets of this wave's loads within a tile, worked out once: for whole tiles, and for
  // the last tile, where rows past the end fetch its last row again (keys of probability 0)
  const int jlast = ((s.N - 1) / kBN) * kBN;
  typename TK::Offs ok_full, ok_last;
  typename TV::Offs ov_full, ov_last;
  {
    const typename TK::Lane lk = TK::lane_setup(s.D, wave, lane);
    const typename TV::Lane lv = TV::lane_setup(s.D, wave, lane);
    ok_full = TK::offsets(lk, pitch, kBN);
    ok_last = TK::offsets(lk, pitch, s.N - jlast);
    ov_full = TV::offsets(lv, pitch, kBN);
    ov_last = TV::offsets(lv, pitch, s.N - jlast);
  }
  auto issue = [&](int j0, unsigned buf) {  // j0 < N, a multiple of kBN
    const long long ro = base + (long long)j0 * s.sn;
    const bool last = j0 == jlast;
#pragma unroll
    for (int t = 0; t < TK::IPW; ++t) {
      const unsigned off = last ? ok_last.o[t] : ok_full.o[t];
      TK::issue_at(off, t, k + ro, buf, wave);
      TK::issue_at(off, t, tk + ro, buf + TK::BYTES, wave);
    }
#pragma unroll
    for (int t = 0; t < TV::IPW; ++t) {
      const unsigned off = last ? ov_last.o[t] : ov_full.o[t];
      TV::issue_at(off, t, v + ro, buf + 2 * TK::BYTES, wave);
      TV::issue_at(off, t, tv + ro, buf + 2 * TK::BYTES + TV::BYTES, wave);
    }
  };
  // SPARE: once a stage has landed, every wave sets column D of its V rows to one (lanes 0..31, row =
  // lane) and of its tV rows to zero (lanes 32..63) before it reads them; the loads had put a copy of
  // the row's first chunk there.  All waves write the same values, so they need not wait for each other.
  const int plant_off = (hh ? 2 * TK::BYTES + TV::BYTES : 2 * TK::BYTES) +
                        (ic * TV::PCH + ((s.D >> 3) ^ ((ic >> 2) & 3))) * 16;
  auto plant = [&](char* stage) {
    if (SPARE) *reinterpret_cast<uint4*>(stage + plant_off) = make_uint4(hh ? 0u : 0x3F80u, 0u, 0u, 0u);
  };
  const typename TK::RAddr rk = TK::raddr(ic, hh);
  const typename TV::TAddr tv_a = TV::taddr(ic, hh);
  issue(0, lds0);

  bf16x8 qf[NKS], tqf[NKS];
  {  // all loads in flight together, behind those of tile 0 and before the wait for it
    uint4 w0[NKS], w1[NKS];
    gld_frags_issue<NKS>(w0, q + qbase, s.qsn, i, s.M, s.D, hh);
    gld_frags_issue<NKS>(w1, tq + qbase, s.qsn, i, s.M, s.D, hh);
    gld_frags_finish<NKS>(qf, w0, i, s.M, s.D, hh);
    gld_frags_finish<NKS>(tqf, w1, i, s.M, s.D, hh);
  }
  if (QNORM) {
    // This lane holds half of row i (chunks 2kk + hh; zeros beyond D and beyond M), the lane 32 away the other half.
    // With r = 1/sqrt(mean(x^2) + eps) and mu = mean(x tx):  y = g x r,  ty = g (tx r - x r^3 mu), rounded to bf16
    // like the rows a separate normalisation would have stored; the rounded values are what the products use and
    // what is written out.
    float ss = 0.f, st = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = (float)qf[kk][e], t = (float)tqf[kk][e];
        ss = fmaf(x, x, ss);
        st = fmaf(x, t, st);
      }
    ss += xhalf(ss);
    st += xhalf(st);
    const float invd = 1.f / (float)s.D;
    const float r = 1.f / sqrtf(fmaf(ss, invd, neps));
    const float r3mu = r * r * r * (st * invd);
    const long long rowoff = qbase + (long long)(iok ? i : 0) * s.qsn;
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk) {
      const int c0 = kk * 16 + hh * 8;
      if (c0 < s.D) {  // (D is a multiple of 8: a chunk is in range as a whole)
        typedef __attribute__((ext_vector_type(4))) float f32x4;
        const f32x4 g0 = *reinterpret_cast<const f32x4*>(ngain + c0), g1 = *reinterpret_cast<const f32x4*>(ngain + c0 + 4);
        bf16x8 y, ty;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float g = e < 4 ? g0[e] : g1[e - 4];
          const float x = (float)qf[kk][e], t = (float)tqf[kk][e];
          y[e] = (bf16)(g * x * r);
          ty[e] = (bf16)(g * fmaf(t, r, -x * r3mu));
        }
        qf[kk] = y;
        tqf[kk] = ty;
        if (iok) {
          *reinterpret_cast<bf16x8*>(qn + rowoff + c0) = y;
          *reinterpret_cast<bf16x8*>(tqn + rowoff + c0) = ty;
        }
      }
    }
  }

  f32x16 accO[NDB], accT[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    accO[db] = zero16();
    accT[db] = zero16();
  }
  float m = -INFINITY, l = 0.f, cs = 0.f;
  const float c1 = s.alpha * kLog2e;  // scores are exponentiated in base 2

  pin_frags(qf);
  pin_frags(tqf);
  dma_wait();
  __syncthreads();  // tile 0 has landed
  plant(lds);
  // K, tK row fragments of the tile about to be computed: read one tile ahead, right behind the
  // barrier that says it has landed, so that their LDS latency hides behind the last output products
  bf16x8 kpre[NKS], tkpre[NKS];
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    kpre[kk] = TK::frag_row(lds, rk, 0, kk);
    tkpre[kk] = TK::frag_row(lds + TK::BYTES, rk, 0, kk);
  }
  for (int j0 = 0, it = 0; j0 < s.N; j0 += kBN, ++it) {
    const char* lds_k = lds + (it & 1) * BUF;
    const char* lds_v = lds_k + 2 * TK::BYTES;
    const char* lds_tv = lds_v + TV::BYTES;
    char* lds_next = lds + ((it + 1) & 1) * BUF;
    if (j0 + kBN < s.N) issue(j0 + kBN, lds0 + ((it + 1) & 1) * BUF);  // uniform: lands during this tile

    f32x16 sS = zero16(), sT = zero16();
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk) {
      sS = mfma(kpre[kk], qf[kk], sS);
      sT = mfma(kpre[kk], tqf[kk], sT);
      sT = mfma(tkpre[kk], qf[kk], sT);
    }
    if (j0 + 32 > s.N) {  // uniform: ragged last block, keys >= N get probability 0
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (j0 + drow(r, hh) >= s.N) sS[r] = -INFINITY;
    }
    float mx = sS[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sS[r]);
    mx = fmaxf(mx, xhalf(mx));  // finite: key 0 is never masked and lives in the first block
    if (__builtin_amdgcn_ballot_w64((mx - m) * c1 > kRescaleLog2) != 0) {  // uniform
      const float mn = fmaxf(m, mx);
      const float f = __builtin_amdgcn_exp2f((m - mn) * c1);  // m = -inf on the first block: 0
      m = mn;
      if (!SPARE) {
        l *= f;
        cs *= f;
      }
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          accO[db][r] *= f;
          accT[db][r] *= f;
        }
    }
    const float mc = m * c1;
    float ps = 0.f, pzs = 0.f;
    bf16x8 pf[2], pzf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(fmaf(sS[r], c1, -mc));
      const float pz = p * (sT[r] * s.alpha);
      if (!SPARE) {
        ps += p;
        pzs += pz;
      }
      pf[r >> 3][r & 7] = (bf16)p;
      pzf[r >> 3][r & 7] = (bf16)pz;
    }
    if (!SPARE) {
      l += ps;   // per-half partial sums; the halves are combined once, in the epilogue
      cs += pzs;
    }
    // output products of the first 16 keys, fragments straight from LDS
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const bf16x8 vf = TV::frag_tr(lds_v, tv_a, 0, db);
      const bf16x8 tvf = TV::frag_tr(lds_tv, tv_a, 0, db);
      accO[db] = mfma(vf, pf[0], accO[db]);
      accT[db] = mfma(vf, pzf[0], accT[db]);
      accT[db] = mfma(tvf, pf[0], accT[db]);
    }
    // the fragments of the other 16 keys go to registers: that is the last read of this tile's buffers
    bf16x8 vf1[NDB], tvf1[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      vf1[db] = TV::frag_tr(lds_v, tv_a, 1, db);
      tvf1[db] = TV::frag_tr(lds_tv, tv_a, 1, db);
    }
    dma_wait();
    __syncthreads();  // next tile landed; everyone is done with this one
    if (j0 + kBN < s.N) plant(lds_next);  // uniform; none behind the last tile: the buffers become the output staging
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk) {  // (behind the last tile: stale data, unused)
      kpre[kk] = TK::frag_row(lds_next, rk, 0, kk);
      tkpre[kk] = TK::frag_row(lds_next + TK::BYTES, rk, 0, kk);
    }
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      accO[db] = mfma(vf1[db], pf[1], accO[db]);
      accT[db] = mfma(vf1[db], pzf[1], accT[db]);
      accT[db] = mfma(tvf1[db], pf[1], accT[db]);
    }
  }
  // every wave is past the last barrier, but the staging below reuses the buffers that the reads just
  // issued (stale data of a tile that does not exist) still target: they are complete once their
  // registers are (which nothing uses); make that explicit
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();

  if (SPARE) {
    // row D of the accumulators (held by the lower half-wave) has the sums
    float lv = 0.f, cv = 0.f;
#pragma unroll
    for (int cand = DK - 8; cand <= DK; cand += 8)
      if (cand < DV && s.D == cand) {
        lv = accO[cand / 32][4 * ((cand % 32) / 8)];
        cv = accT[cand / 32][4 * ((cand % 32) / 8)];
      }
    const float lx = xhalf(lv), cx = xhalf(cv);
    l = hh ? lx : lv;
    cs = hh ? cx : cv;
  } else {
    l += xhalf(l);
    cs += xhalf(cs);
  }
  // rows beyond N hold garbage (possibly not finite) from here on; nothing of theirs is stored
  const float inv = 1.f / l;
  const float mubar = cs * inv;
  const float nmi = -mubar * inv;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) accT[db][r] = fmaf(nmi, accO[db][r], accT[db][r] * inv);
  {
    // the loop ended with a barrier and no tile load is in flight: each wave stages its two output
    // tiles through a region of the tile buffers of its own and stores whole rows
    const unsigned lw = lds0 + (unsigned)wave * (32 * (64 * NDB + 16));
    static_assert(NW * 32 * (64 * NDB + 16) <= 2 * BUF, "staging fits in the tile buffers");
    const int row0 = mb * BM + wave * 32;
    store_tile_coalesced<NDB>(lw, o + qbase, s.qsn, row0, s.M, s.D, accO, inv, lane);
    store_tile_coalesced<NDB>(lw, to + qbase, s.qsn, row0, s.M, s.D, accT, 1.f, lane);
  }
  if (iok && hh == 0) {
    const long long r = (long long)bh * s.M + i;
    if (lse) lse[r] = (m * c1 + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;  // (null: forward only, nothing saved)
    if (stats) stats[r] = mubar;
  }
}

template <int DK, int DV, int NW>
hipError_t launch_nw(const Shape& s, const FwdArgs& a, hipStream_t st) {
  constexpr int BN = FWD_BN;  // keys per LDS tile
  const int nmb = (s.M + 32 * NW - 1) / (32 * NW);
  const dim3 grid(nmb * s.B * s.H), block(64 * NW);
  const bf16 *q = (const bf16*)a.q, *k = (const bf16*)a.k, *v = (const bf16*)a.v, *tq = (const bf16*)a.tq,
             *tk = (const bf16*)a.tk, *tv = (const bf16*)a.tv;
  if (s.D < DV)  // a spare column in the output tiles carries the row sums
    hipLaunchKernelGGL((fwd_mfma_kernel<DK, DV, NW, BN, true>), grid, block, 0, st, s, q, k, v, tq, tk, tv, (bf16*)a.o,
                       (bf16*)a.to, a.lse, a.stats, a.ngq, a.neps, (bf16*)a.qn, (bf16*)a.tqn);
  else if constexpr (DK == DV)
    hipLaunchKernelGGL((fwd_mfma_kernel<DK, DV, NW, BN, false>), grid, block, 0, st, s, q, k, v, tq, tk, tv, (bf16*)a.o,
                       (bf16*)a.to, a.lse, a.stats, a.ngq, a.neps, (bf16*)a.qn, (bf16*)a.tqn);
  else
    return hipErrorNotSupported;  // D <= DK < DV: not reached
  return hipGetLastError();
}

// Waves per workgroup: four (two workgroups share a CU) for short key sequences, where a workgroup's start-up and
// epilogue overlap the other's loop; eight (one workgroup per CU, the same two waves per SIMD, every tile fetched
// once per CU instead of twice) from 512 keys on: 2 % faster at N = 1024 (250 against 256 us at C4, 236 against 241 us
// at d = 64), 3 % slower at N = 256.
template <int DK, int DV>
hipError_t launch(const Shape& s, const FwdArgs& a, hipStream_t st) {
  if constexpr (DV <= 96) {  // (above that a wave needs more than the 256 registers that two waves per SIMD leave it)
    if (s.N >= FWD_WIDE_FROM && s.M > 32 * FWD_NW) return launch_nw<DK, DV, 2 * FWD_NW>(s, a, st);
  }
  return launch_nw<DK, DV, FWD_NW>(s, a, st);
}

}  // namespace

hipError_t TVM_FWD_LAUNCHER(const Shape& s, const FwdArgs& a, hipStream_t st) {
  switch ((s.D + 15) / 16 * 16) {
    case 16: return launch<16, 32>(s, a, st);
    case 32: return launch<32, 32>(s, a, st);
    case 48: return launch<48, 64>(s, a, st);
    case 64: return launch<64, 64>(s, a, st);
    case 80: return launch<80, 96>(s, a, st);
    case 96: return launch<96, 96>(s, a, st);
    case 112: return launch<112, 128>(s, a, st);
    case 128: return launch<128, 128>(s, a, st);
    default: return hipErrorNotSupported;
  }
}

}  // namespace tvm
