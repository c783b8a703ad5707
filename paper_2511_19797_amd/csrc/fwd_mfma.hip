// Forward with tangent on the bf16 matrix cores (gfx950).
//
// One workgroup = NW waves, 32 query rows per wave, all of one (batch, head); a wave keeps Q, tQ
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
#include "mfma_tiles.h"
#ifndef FWD_NW
#define FWD_NW 4   // waves per workgroup (two workgroups share a CU)
#define FWD_BN 32  // keys per LDS tile
#endif

namespace tvm {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleLog2 = 8.f;  // raise the reference maximum only beyond this growth (log2 units)

template <int DK, int DV, int NW, int kBN>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void fwd_mfma_kernel(Shape s, const bf16* __restrict__ q,
                                                          const bf16* __restrict__ k, const bf16* __restrict__ v,
                                                          const bf16* __restrict__ tq, const bf16* __restrict__ tk,
                                                          const bf16* __restrict__ tv, bf16* __restrict__ o,
                                                          bf16* __restrict__ to, float* __restrict__ lse,
                                                          float* __restrict__ stats) {
  constexpr int NT = 64 * NW, BM = 32 * NW;
  using TK = Tile<kBN, DK / 8, NW>;
  using TV = Tile<kBN, DV / 8, NW>;
  constexpr int BUF = 2 * TK::BYTES + 2 * TV::BYTES;  // one stage: K, tK, V, tV
  __shared__ __attribute__((aligned(16))) char lds[2 * BUF];
  constexpr int NKS = DK / 16, NDB = DV / 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int nmb = (s.N + BM - 1) / BM;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);
  const int bh = wg / nmb, mb = wg - bh * nmb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;
  const int i = mb * BM + wave * 32 + ic;  // this lane's query row
  const bool iok = i < s.N;

  const typename TK::Lane lk = TK::lane_setup(s.D, wave, lane);
  const typename TV::Lane lv = TV::lane_setup(s.D, wave, lane);
  const unsigned pitch = (unsigned)(s.sn * 2);  // row pitch in bytes
  const unsigned lds0 = lds_addr_of(lds);
  auto issue = [&](int j0, unsigned buf) {  // j0 < N
    const long long ro = base + (long long)j0 * s.sn;
    const int left = s.N - j0;
    TK::issue(lk, k + ro, pitch, left, buf, wave);
    TK::issue(lk, tk + ro, pitch, left, buf + TK::BYTES, wave);
    TV::issue(lv, v + ro, pitch, left, buf + 2 * TK::BYTES, wave);
    TV::issue(lv, tv + ro, pitch, left, buf + 2 * TK::BYTES + TV::BYTES, wave);
  };
  const typename TK::RAddr rk = TK::raddr(ic, hh);
  const typename TV::TAddr tv_a = TV::taddr(ic, hh);
  issue(0, lds0);

  bf16x8 qf[NKS], tqf[NKS];
  gld_frags<NKS>(qf, q + base, s.sn, i, s.N, s.D, hh);
  gld_frags<NKS>(tqf, tq + base, s.sn, i, s.N, s.D, hh);

  f32x16 accO[NDB], accT[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    accO[db] = zero16();
    accT[db] = zero16();
  }
  float m = -INFINITY, l = 0.f, cs = 0.f;
  const float c1 = s.alpha * kLog2e;  // scores are exponentiated in base 2

  dma_wait();
  __syncthreads();  // tile 0 has landed
  for (int j0 = 0, it = 0; j0 < s.N; j0 += kBN, ++it) {
    const char* lds_k = lds + (it & 1) * BUF;
    const char* lds_tk = lds_k + TK::BYTES;
    const char* lds_v = lds_k + 2 * TK::BYTES;
    const char* lds_tv = lds_v + TV::BYTES;
    if (j0 + kBN < s.N) issue(j0 + kBN, lds0 + ((it + 1) & 1) * BUF);  // uniform: lands during this tile

#pragma unroll
    for (int jb = 0; jb < kBN / 32; ++jb) {
      if (j0 + jb * 32 >= s.N) break;  // uniform: the rest of the tile is beyond the last key
      f32x16 sS = zero16(), sT = zero16();
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        const bf16x8 kf = TK::frag_row(lds_k, rk, jb, kk);
        const bf16x8 tkf = TK::frag_row(lds_tk, rk, jb, kk);
        sS = mfma(kf, qf[kk], sS);
        sT = mfma(kf, tqf[kk], sT);
        sT = mfma(tkf, qf[kk], sT);
      }
      if (j0 + jb * 32 + 32 > s.N) {  // uniform: ragged last block, keys >= N get probability 0
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + jb * 32 + drow(r, hh) >= s.N) sS[r] = -INFINITY;
      }
      float mx = sS[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sS[r]);
      mx = fmaxf(mx, xhalf(mx));  // finite: key 0 is never masked and lives in the first block
      if (__builtin_amdgcn_ballot_w64((mx - m) * c1 > kRescaleLog2) != 0) {  // uniform
        const float mn = fmaxf(m, mx);
        const float f = __builtin_amdgcn_exp2f((m - mn) * c1);  // m = -inf on the first block: 0
        m = mn;
        l *= f;
        cs *= f;
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
        ps += p;
        pzs += pz;
        pf[r >> 3][r & 7] = (bf16)p;
        pzf[r >> 3][r & 7] = (bf16)pz;
      }
      l += ps;   // per-half partial sums; the halves are combined once, in the epilogue
      cs += pzs;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
          const bf16x8 vf = TV::frag_tr(lds_v, tv_a, 2 * jb + cc, db);
          const bf16x8 tvf = TV::frag_tr(lds_tv, tv_a, 2 * jb + cc, db);
          accO[db] = mfma(vf, pf[cc], accO[db]);
          accT[db] = mfma(vf, pzf[cc], accT[db]);
          accT[db] = mfma(tvf, pf[cc], accT[db]);
        }
    }
    dma_wait();
    __syncthreads();  // next tile landed; everyone is done with this one
  }

  l += xhalf(l);
  cs += xhalf(cs);
  if (!iok) return;
  const float inv = 1.f / l;
  const float mubar = cs * inv;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = db * 32 + 8 * g + 4 * hh;
      if (d0 < s.D) {
        bf16x4 vo, vt;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float oc = accO[db][4 * g + t] * inv;
          vo[t] = (bf16)oc;
          vt[t] = (bf16)fmaf(-mubar, oc, accT[db][4 * g + t] * inv);
        }
        *reinterpret_cast<bf16x4*>(o + base + (long long)i * s.sn + d0) = vo;
        *reinterpret_cast<bf16x4*>(to + base + (long long)i * s.sn + d0) = vt;
      }
    }
  if (hh == 0) {
    const long long r = (long long)bh * s.N + i;
    lse[r] = (m * c1 + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    stats[r] = mubar;
  }
}

template <int DK, int DV>
hipError_t launch(const Shape& s, const FwdArgs& a, hipStream_t st) {
  constexpr int NW = FWD_NW, BN = (DV > 96) ? 32 : FWD_BN;  // waves per workgroup, keys per LDS tile
  const int nmb = (s.N + 32 * NW - 1) / (32 * NW);
  hipLaunchKernelGGL((fwd_mfma_kernel<DK, DV, NW, BN>), dim3(nmb * s.B * s.H), dim3(64 * NW), 0, st, s,
                     (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk,
                     (const bf16*)a.tv, (bf16*)a.o, (bf16*)a.to, a.lse, a.stats);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_mfma(const Shape& s, const FwdArgs& a, hipStream_t st) {
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
