// Forward with tangent on the bf16 matrix cores (gfx950).
//
// One workgroup = 4 waves = 128 query rows of one (batch, head); wave w owns rows 32w..32w+31
// and keeps Q, tQ as B-operand fragments in registers for the whole kernel.  Keys are streamed
// in tiles of 64 through LDS: K, tK row-major (A operands of the score products), V, tV
// transposed in slot order (A operands of the output products).
//
// Everything is computed transposed, S^T = K Q^T, so that a lane owns ONE query row
// (column ic of every D tile): row max / row sums are in-lane reductions plus one exchange
// between the two half-waves, the online-softmax rescale is a per-lane scalar, and the
// probabilities feed the next product from registers.
//
// Per key tile (the equations under "Step 1" of App. C, evaluated with a running maximum):
//   S^T  = K Q^T            St^T = K tQ^T + tK Q^T
//   p    = exp(alpha S - m)               (un-normalised)
//   l   += sum p ;  c += sum p * alpha St
//   accO += p V ;   accT += (p * alpha St) V + p tV
// Epilogue: O = accO / l,  stats = c / l,  tO = accT / l - stats * O,  lse = m + log l.
#include "mfma_tiles.h"

namespace tvm {
namespace {

constexpr int kBM = 128;  // query rows per workgroup
constexpr int kBN = 64;   // keys per LDS tile
constexpr int kNT = 256;

template <int DK, int DV>
struct FwdLds {
  static constexpr int KP = DK + 8;   // row pitch (elements): 16-byte odd multiple -> conflict-free b128 reads
  static constexpr int JP = kBN + 8;
  bf16 k[kBN * KP];
  bf16 tk[kBN * KP];
  bf16 vt[DV * JP];
  bf16 tvt[DV * JP];
};

template <int DK, int DV>
__global__ __launch_bounds__(kNT, 2) void fwd_mfma_kernel(Shape s, const bf16* __restrict__ q,
                                                         const bf16* __restrict__ k, const bf16* __restrict__ v,
                                                         const bf16* __restrict__ tq, const bf16* __restrict__ tk,
                                                         const bf16* __restrict__ tv, bf16* __restrict__ o,
                                                         bf16* __restrict__ to, float* __restrict__ lse,
                                                         float* __restrict__ stats) {
  using L = FwdLds<DK, DV>;
  __shared__ __attribute__((aligned(16))) L sm;
  constexpr int NKS = DK / 16, NDB = DV / 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int nmb = (s.N + kBM - 1) / kBM;
  const int bh = blockIdx.x / nmb, mb = blockIdx.x - bh * nmb;
  const int b = bh / s.H, h = bh - b * s.H;
  const long long base = b * s.sb + h * s.sh;
  const int i = mb * kBM + wave * 32 + ic;  // this lane's query row
  const bool iok = i < s.N;

  bf16x8 qf[NKS], tqf[NKS];
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    const int c0 = kk * 16 + hh * 8;
    const bool ok = iok && c0 < s.D;
    qf[kk] = gld_frag(q + base + (long long)i * s.sn + c0, ok);
    tqf[kk] = gld_frag(tq + base + (long long)i * s.sn + c0, ok);
  }

  f32x16 accO[NDB], accT[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accO[db][r] = 0.f;
      accT[db][r] = 0.f;
    }
  float m = -INFINITY, l = 0.f, cs = 0.f;
  const float c1 = s.alpha * 1.4426950408889634f;  // scores are exponentiated in base 2

  for (int j0 = 0; j0 < s.N; j0 += kBN) {
    __syncthreads();
    load_rows<kBN, DK, L::KP, kNT>(sm.k, k + base, s.sn, j0, s.N, s.D, tid);
    load_rows<kBN, DK, L::KP, kNT>(sm.tk, tk + base, s.sn, j0, s.N, s.D, tid);
    load_transposed<kBN, DV, L::JP, kNT>(sm.vt, v + base, s.sn, j0, s.N, s.D, tid);
    load_transposed<kBN, DV, L::JP, kNT>(sm.tvt, tv + base, s.sn, j0, s.N, s.D, tid);
    __syncthreads();

#pragma unroll
    for (int jb = 0; jb < kBN / 32; ++jb) {
      if (j0 + jb * 32 >= s.N) break;  // uniform: the rest of the tile is beyond the last key
      f32x16 sS, sT;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        sS[r] = 0.f;
        sT[r] = 0.f;
      }
#pragma unroll
      for (int kk = 0; kk < NKS; ++kk) {
        const bf16x8 kf = lds_frag(sm.k + (jb * 32 + ic) * L::KP + kk * 16 + hh * 8);
        const bf16x8 tkf = lds_frag(sm.tk + (jb * 32 + ic) * L::KP + kk * 16 + hh * 8);
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
      mx = fmaxf(mx, xhalf(mx));
      const float mn = fmaxf(m, mx);  // finite: key 0 is never masked
      const float f = __builtin_amdgcn_exp2f((m - mn) * c1);
      m = mn;
      const float mc = mn * c1;
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
      ps += xhalf(ps);
      pzs += xhalf(pzs);
      l = fmaf(l, f, ps);
      cs = fmaf(cs, f, pzs);
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          accO[db][r] *= f;
          accT[db][r] *= f;
        }
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
          const bf16x8 vf = lds_frag(sm.vt + (db * 32 + ic) * L::JP + (2 * jb + cc) * 16 + hh * 8);
          const bf16x8 tvf = lds_frag(sm.tvt + (db * 32 + ic) * L::JP + (2 * jb + cc) * 16 + hh * 8);
          accO[db] = mfma(vf, pf[cc], accO[db]);
          accT[db] = mfma(vf, pzf[cc], accT[db]);
          accT[db] = mfma(tvf, pf[cc], accT[db]);
        }
    }
  }

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
  const int nmb = (s.N + kBM - 1) / kBM;
  hipLaunchKernelGGL((fwd_mfma_kernel<DK, DV>), dim3(nmb * s.B * s.H), dim3(kNT), 0, st, s, (const bf16*)a.q,
                     (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.tq, (const bf16*)a.tk, (const bf16*)a.tv,
                     (bf16*)a.o, (bf16*)a.to, a.lse, a.stats);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_mfma(const Shape& s, const FwdArgs& a, hipStream_t st) {
  const int dk = (s.D + 15) / 16 * 16;
  switch (dk) {
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
