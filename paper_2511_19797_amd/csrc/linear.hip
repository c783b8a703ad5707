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
// Workgroup: eight waves as 2 x 4 (two per SIMD), each with 4 x 2 blocks of 32 x 32 (128 accumulator registers): a
// 256 x 256 output tile (128 flop per byte staged: smaller tiles are bound by L2->LDS traffic), contraction in
// tiles of 64 through two LDS stages filled by asynchronous global->LDS loads (mfma_tiles.h: the same swizzled
// row-major tiles as the attention kernels; "row" fragments are 16-byte reads, "transposed" ones the transposing LDS
// read, here with the contraction index in natural order so that both kinds pair up).  Per contraction step of 16
// a wave reads 4 + 2 fragments for 8 products, a step ahead of the products that use them.  Workgroups are
// persistent, one per CU: each walks a list of output tiles in an order that keeps an XCD's workgroups on one patch
// of tiles, requests the next tile's first operands during the last contraction tile of the current one, and writes
// a tile's results while those land.
//
// grad W contracts over all tokens of both sets (32K rows at DiT-XL/2 512 px) for few output tiles, so the token
// range is split over several workgroups per tile; each leaves a float32 partial tile in the workspace and a second
// small kernel adds them in a fixed order (no atomics) and rounds once.  gb is a column sum of gy: partial sums over
// row ranges, then one kernel that adds those.
#include <type_traits>

#include "mfma_tiles.h"

namespace tvm {
namespace {

// Shape of a workgroup: NWI x NWJ waves, each with WI x WJ blocks of 32 x 32; NST LDS stages; OCC workgroups per CU.
template <int NWI_, int NWJ_, int WI_, int WJ_, int NST_, int OCC_>
struct Cfg {
  static constexpr int NWI = NWI_, NWJ = NWJ_, WI = WI_, WJ = WJ_, NST = NST_, OCC = OCC_;
  static constexpr int NW = NWI_ * NWJ_, NT = 64 * NW;
  static constexpr int TI = NWI_ * WI_ * 32;  // output rows per workgroup
  static constexpr int TJ = NWJ_ * WJ_ * 32;  // output columns per workgroup
};
constexpr int kBK = 64;                      // contraction per LDS tile
constexpr int kGI = 8;                       // tile rows per group in the order the tiles are handed out

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
  int nz;             // row sets (forward, grad x: 2) or splits (grad W)
};

template <bool PTR, bool QTR, bool PARTIAL, class C>
__global__ __launch_bounds__(C::NT, C::OCC) void gemm_kernel(GemmArgs g) {
  constexpr int kNW = C::NW, kWI = C::WI, kWJ = C::WJ, kTI = C::TI, kTJ = C::TJ, NST = C::NST;
  // tiles: "transposed" access [kBK][columns of the stored matrix]; "row" access [rows of the operand][32], two of
  // them back to back for the kBK = 64 entries of a contraction tile (rows of 64 bytes are dense in LDS and free of
  // bank conflicts; rows of 128 bytes would need padding)
  static_assert(kBK == 64, "a row-access operand is staged as two tiles of 32");
  using TP = typename std::conditional<PTR, Tile<kBK, kTI / 8, kNW>, Tile<kTI, 4, kNW>>::type;
  using TQ = typename std::conditional<QTR, Tile<kBK, kTJ / 8, kNW>, Tile<kTJ, 4, kNW>>::type;
  constexpr int P_BYTES = PTR ? TP::BYTES : 2 * TP::BYTES, Q_BYTES = QTR ? TQ::BYTES : 2 * TQ::BYTES;
  constexpr int BUF = P_BYTES + Q_BYTES;
  constexpr int STAGE_BYTES = NST * BUF;  // NST stages: tile t in use, tiles t+1 .. t+NST-2 landed or landing, one being refilled
  constexpr int LOADS = (PTR ? 1 : 2) * TP::IPW + (QTR ? 1 : 2) * TQ::IPW;  // wave-loads per wave and tile
  constexpr int OUT_REGION = 32 * (64 * kWJ + 16);  // per wave, for store_tile_coalesced
  constexpr int LDS_BYTES = STAGE_BYTES > kNW * OUT_REGION ? STAGE_BYTES : kNW * OUT_REGION;
  __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, ic = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave % C::NWI, wj = wave / C::NWI;
  const int nI = (g.I + kTI - 1) / kTI, nJ = (g.J + kTJ - 1) / kTJ;
  const int nct = (g.C + kBK - 1) / kBK;  // contraction tiles per set
  const int ntot = g.csets * nct;
  const unsigned lds0 = lds_addr_of(lds);
  const typename TP::RAddr rp = TP::raddr(ic, hh);
  const typename TQ::RAddr rq = TQ::raddr(ic, hh);
  const TrNat<TP> tp = TrNat<TP>::make(ic, hh);
  const TrNat<TQ> tq = TrNat<TQ>::make(ic, hh);
  f32x16 acc[kWI][kWJ];
  bf16x8 pf[2][kWI], qf[2][kWJ];
  static_assert(NST == 2, "two stages");
  static_assert(kNW * OUT_REGION <= BUF, "the output staging fits in one stage");

  // Writes out the accumulators of output tile (i0, j0) of row set / split zz.  Runs while the first loads of the
  // workgroup's next tile are on their way into one stage: bf16 results are staged through the other one, `stage`.
  auto write_out = [&](int i0, int j0, int zz, int stage) {
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
      const unsigned lw = lds0 + (unsigned)stage * BUF + (unsigned)wave * OUT_REGION;  // each wave stages its rows through a region of its own
      if (jw < g.J) {
#pragma unroll
        for (int a = 0; a < kWI; ++a) {
          const int row0 = i0 + (wi * kWI + a) * 32;
          store_tile_coalesced<kWJ>(lw, g.out[zz] + jw, g.ldo, row0, g.I, g.J - jw, acc[a], 1.f, lane);
        }
      }
    }
  };

  // Persistent workgroups, one per CU, each working through a list of output tiles: the next tile's first operands
  // are requested during the last contraction tile of the current one, and a tile's results are written while they
  // land (and drain to HBM while the next tile is computed).  Hardware
  // workgroup ids go round-robin over the 8 XCDs, each with an L2 of its own: XCD x owns the x-th eighth of the
  // logical tile ids, which its workgroups take in turn; logical ids walk the tiles of a row set (or split) in groups
  // of kGI tile rows, down the group first.  The ~32 workgroups of an XCD are then on a patch of about 8 x 4 tiles at
  // any one time and march through the contraction together: an operand panel comes from HBM once for the tiles of
  // the patch that share it.
  const bool late = !PARTIAL && wave >= kNW / 2;  // (uniform; waves w and w + 4 share a SIMD; grad W has no registers to spare for it)
  const int total = g.nz * nI * nJ;
  const int per_xcd = (total + 7) >> 3, wg_per_xcd = (int)(gridDim.x >> 3);
  const int id_end = min(total, ((int)(blockIdx.x & 7) + 1) * per_xcd);

  // An output tile: where it is, its range of contraction tiles, and the per-lane byte offsets of this wave's loads
  // within an operand tile (whole tiles / a set's last tile)
  struct Ctx {
    int i0, j0, zz, t_begin, t_end, pset;
    typename TP::Offs op_full, op_last;
    typename TQ::Offs oq_full, oq_last;
  };
  auto locate = [&](int wg) {
    Ctx c;
    c.zz = wg / (nI * nJ);  // row set (forward, grad x) or split (grad W)
    const int id = wg - c.zz * (nI * nJ);
    const int grp = id / (kGI * nJ), it_first = grp * kGI, gs = min(nI - it_first, kGI);
    const int rem = id - grp * (kGI * nJ);
    const int jt = rem / gs, it = it_first + (rem - jt * gs);
    c.i0 = it * kTI;
    c.j0 = jt * kTJ;
    c.t_begin = PARTIAL ? (int)((long long)c.zz * ntot / g.splits) : 0;
    c.t_end = PARTIAL ? (int)((long long)(c.zz + 1) * ntot / g.splits) : ntot;
    c.pset = PARTIAL ? 0 : c.zz;
    const unsigned pitchP = (unsigned)(g.ldP * 2), pitchQ = (unsigned)(g.ldQ * 2);
    const int clast = g.C - (nct - 1) * kBK;  // contraction entries in a set's last tile
    if (PTR) {
      const typename TP::Lane l = TP::lane_setup(min(g.I - c.i0, kTI), wave, lane);  // columns of the stored matrix = output rows
      c.op_full = TP::offsets(l, pitchP, kBK);
      c.op_last = TP::offsets(l, pitchP, clast);
    } else {
      c.op_full = c.op_last = TP::offsets(TP::lane_setup(32, wave, lane), pitchP, g.I - c.i0);
    }
    if (QTR) {
      const typename TQ::Lane l = TQ::lane_setup(min(g.J - c.j0, kTJ), wave, lane);
      c.oq_full = TQ::offsets(l, pitchQ, kBK);
      c.oq_last = TQ::offsets(l, pitchQ, clast);
    } else {
      c.oq_full = c.oq_last = TQ::offsets(TQ::lane_setup(32, wave, lane), pitchQ, g.J - c.j0);
    }
    return c;
  };
  // wave-load number x (compile-time, 0 .. LOADS-1) of contraction tile t of output tile c into the stage at `buf`
  auto issue = [&](const Ctx& c, int t, unsigned buf, int x) {
    const int set = t / nct, ct = t - set * nct;
    const long long c0 = (long long)ct * kBK;
    const bool last = ct == nct - 1;
    const bf16* pb = g.P[PARTIAL ? set : c.pset] + (PTR ? c0 * g.ldP + c.i0 : (long long)c.i0 * g.ldP + c0);
    const bf16* qb = g.Q[PARTIAL ? set : 0] + (QTR ? c0 * g.ldQ + c.j0 : (long long)c.j0 * g.ldQ + c0);
    // (row access: the contraction length is a multiple of 32, so the second half of a set's last tile is either
    // whole or absent; an absent half fetches the first half again, and its fragments are zeroed on the P side)
    const int half2 = (last && g.C - (int)c0 <= 32) ? 0 : 32;
    constexpr int NP = (PTR ? 1 : 2) * TP::IPW;
    if (x < NP) {
      if (PTR) TP::issue_at(last ? c.op_last.o[x] : c.op_full.o[x], x, pb, buf, wave);
      else if (x < TP::IPW) TP::issue_at(c.op_full.o[x], x, pb, buf, wave);
      else TP::issue_at(c.op_full.o[x - TP::IPW], x - TP::IPW, pb + half2, buf + TP::BYTES, wave);
    } else {
      const int y = x - NP;
      if (QTR) TQ::issue_at(last ? c.oq_last.o[y] : c.oq_full.o[y], y, qb, buf + P_BYTES, wave);
      else if (y < TQ::IPW) TQ::issue_at(c.oq_full.o[y], y, qb, buf + P_BYTES, wave);
      else TQ::issue_at(c.oq_full.o[y - TQ::IPW], y - TQ::IPW, qb + half2, buf + P_BYTES + TQ::BYTES, wave);
    }
  };
  // A ragged last contraction tile of a set: entries beyond the set's end were fetched as copies of valid ones (the
  // set's last row, or the first half of the tile); on the P side each wave overwrites with zeros what it fetched of
  // them (call this once its own loads have landed), so that those entries contribute nothing.
  auto fix_ragged = [&](int t, int n) {
    const int ct = t % nct;
    const int cvalid = ct == nct - 1 ? g.C - ct * kBK : kBK;
    if (cvalid < kBK) {
      char* pt = lds + n * BUF;
#pragma unroll
      for (int x = 0; x < TP::IPW; ++x) {
        const int pos = (wave + x * kNW) * 64 + lane;  // chunk of the tile this lane fetched with wave-load x
        if (PTR) {
          if (pos / TP::PCH >= cvalid) *reinterpret_cast<uint4*>(pt + pos * 16) = make_uint4(0u, 0u, 0u, 0u);
        } else if (cvalid <= 32) {
          *reinterpret_cast<uint4*>(pt + TP::BYTES + pos * 16) = make_uint4(0u, 0u, 0u, 0u);
        }
      }
    }
  };

  int wg = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (wg >= id_end) return;  // (the grid is never larger than the tiles need, but an XCD's share may be short)
  Ctx cur = locate(wg);
  int n0 = 0;  // the stage that holds (or is receiving) the first contraction tile of `cur`
#pragma unroll
  for (int x = 0; x < LOADS; ++x) issue(cur, cur.t_begin, lds0, x);
  int prev_i0 = 0, prev_j0 = 0, prev_zz = -1;  // the tile whose results are still in the accumulators (zz < 0: none)
  for (;;) {
    // The first contraction tile of `cur` is on its way into stage n0 (requested during the last contraction tile of
    // the output tile before, or just now for the workgroup's first one); the other stage is free.  In this order: the
    // bias values are requested; the wait for the loads in flight; the results of the tile before leave through the
    // free stage (their stores are not waited for here: the next wait comes a contraction tile later); the
    // accumulators start from the bias (row set 0; the tangent has none) or from zero.
    float bv[kWJ][16];
    {
      const bool with_bias = !PARTIAL && g.bias != nullptr && cur.pset == 0;
      const int jw = cur.j0 + wj * (kWJ * 32);
#pragma unroll
      for (int b = 0; b < kWJ; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jw + b * 32 + drow(r, hh);
          bv[b][r] = with_bias && j < g.J ? (float)g.bias[j] : 0.f;
        }
    }
    dma_wait();
    fix_ragged(cur.t_begin, n0);
    if (prev_zz >= 0) write_out(prev_i0, prev_j0, prev_zz, n0 ^ 1);
    prev_i0 = cur.i0;
    prev_j0 = cur.j0;
    prev_zz = cur.zz;
#pragma unroll
    for (int b = 0; b < kWJ; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int a = 0; a < kWI; ++a) acc[a][b][r] = bv[b][r];
    __syncthreads();  // the first contraction tile is there for everyone; everyone's staging reads are over
    const bool has_next = wg + wg_per_xcd < id_end;  // uniform
    const int t_begin = cur.t_begin, t_end = cur.t_end;
    int n = n0;
    for (int t = t_begin; t < t_end; ++t, n ^= 1) {
      // tile t is there for everyone and everyone is done with tile t-1, whose stage is refilled now
      const bool more = t + 1 < t_end;  // uniform
      const char* sp = lds + n * BUF;
      const char* sq = sp + P_BYTES;
      // fragments of contraction step kk into register set `set`
      auto fetch = [&](int set, int kk) {
#pragma unroll
        for (int a = 0; a < kWI; ++a)
          pf[set][a] = PTR ? tp.frag(sp, kk, wi * kWI + a) : TP::frag_row(sp + (kk >> 1) * TP::BYTES, rp, wi * kWI + a, kk & 1);
#pragma unroll
        for (int b = 0; b < kWJ; ++b)
          qf[set][b] = QTR ? tq.frag(sq, kk, wj * kWJ + b) : TQ::frag_row(sq + (kk >> 1) * TQ::BYTES, rq, wj * kWJ + b, kk & 1);
      };
      auto products = [&](int set) {
#pragma unroll
        for (int a = 0; a < kWI; ++a)
#pragma unroll
          for (int b = 0; b < kWJ; ++b) acc[a][b] = mfma(qf[set][b], pf[set][a], acc[a][b]);
      };
      // Two register sets take turns: the LDS reads of step kk+1 are issued ahead of the products of step kk (the
      // scheduling barriers keep the compiler from sinking them back to their first use), and the next tile's loads
      // are issued while the first fragments are on their way from LDS.  The two waves that share a SIMD meet the
      // per-tile barrier one contraction step apart: the second one (`late`) arrives before its last step, whose
      // fragments it already holds, so that right behind the barrier the matrix pipe has that step's products to
      // run while both waves wait for their first fragments of the new tile.
      static_assert(kBK / 16 == 4, "four contraction steps per tile");
      auto sync = [&]() {
        if (more) {
          dma_wait();  // the next tile has landed
          fix_ragged(t + 1, n ^ 1);
        }  // (behind an output tile's last contraction tile the loads in flight are the next output tile's: not waited for here)
        __syncthreads();  // it is there for everyone, and nobody reads this tile from LDS any more
      };
      fetch(0, 0);
      fetch(1, 1);
      __builtin_amdgcn_sched_barrier(0);
      if (more) {
#pragma unroll
        for (int x = 0; x < LOADS; ++x) issue(cur, t + 1, lds0 + (n ^ 1) * BUF, x);
      } else if (has_next) {
        // the workgroup's next output tile: its first operands are requested now, a contraction tile ahead of the
        // results of this one, into the stage that this tile no longer uses
        const Ctx nx = locate(wg + wg_per_xcd);
#pragma unroll
        for (int x = 0; x < LOADS; ++x) issue(nx, nx.t_begin, lds0 + (n ^ 1) * BUF, x);
      }
      __builtin_amdgcn_sched_barrier(0);
      products(0);
      __builtin_amdgcn_sched_barrier(0);
      fetch(0, 2);
      __builtin_amdgcn_sched_barrier(0);
      products(1);
      __builtin_amdgcn_sched_barrier(0);
      fetch(1, 3);
      __builtin_amdgcn_sched_barrier(0);
      products(0);
      __builtin_amdgcn_sched_barrier(0);
      if (late) sync();
      __builtin_amdgcn_sched_barrier(0);
      products(1);
      __builtin_amdgcn_sched_barrier(0);
      if (!late) sync();
    }
    // n: the stage behind the one computed from last, i.e. where the next output tile's first operands are landing
    if (!has_next) {
      write_out(prev_i0, prev_j0, prev_zz, n ^ 1);
      break;
    }
    wg += wg_per_xcd;
    cur = locate(wg);  // (worked out again rather than kept in registers through the loop)
    n0 = n;
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

// Column sums of gy [R][F] over `chunks` row ranges: part[chunk][f] (float32).  A lane takes 8 columns (16-byte
// loads, a wave 512 columns of a row), the four waves of a workgroup every fourth row of the chunk each; their sums
// meet in LDS, in a fixed order.
__global__ __launch_bounds__(256) void colsum_kernel(const bf16* __restrict__ gy, int R, int F, long long ld, int chunks,
                                                     float* __restrict__ part) {
  __shared__ float red[4][64][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ch = blockIdx.y;
  const int f = (blockIdx.x * 64 + lane) * 8;  // (F is a multiple of 8: eight columns are in range together)
  const int r0 = (int)((long long)ch * R / chunks), r1 = (int)((long long)(ch + 1) * R / chunks);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (f < F) {
    const bf16* col = gy + f;
    int r = r0 + wave;
    for (; r + 12 < r1; r += 16) {  // four rows in flight
      bf16x8 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const bf16x8*>(col + (long long)(r + 4 * u) * ld);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += (float)v[u][e];
    }
    for (; r < r1; r += 4) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(col + (long long)r * ld);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += (float)v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[wave][lane][e] = acc[e];
  __syncthreads();
  if (wave == 0 && f < F) {
#pragma unroll
    for (int e = 0; e < 8; ++e) part[(long long)ch * F + f + e] = (red[0][lane][e] + red[1][lane][e]) + (red[2][lane][e] + red[3][lane][e]);
  }
}

// Adds the `chunks` partial rows of the column sums, part[chunk][f], and rounds once to bf16.  A workgroup of 16
// waves takes 64 columns: wave w adds rows w, w + 16, ... (16 loads in flight), and the 16 sums meet in LDS, in a
// fixed order.  (Few output elements and many rows: with a thread per column walking all rows in turn, one or two
// workgroups spent 70 us on 256 rows of dependent latencies.)
__global__ __launch_bounds__(1024) void bias_sum_kernel(const float* __restrict__ part, int chunks, int F,
                                                        bf16* __restrict__ out) {
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int f = blockIdx.x * 64 + lane;
  float acc = 0.f;
  if (f < F) {
    for (int c0 = wave; c0 < chunks; c0 += 256) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int c = c0 + 16 * u;
        v[u] = c < chunks ? part[(long long)c * F + f] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) acc += v[u];
    }
  }
  red[wave][lane] = acc;
  __syncthreads();
  if (wave == 0 && f < F) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) t += red[w][lane];
    out[f] = (bf16)t;
  }
}

// The shapes in use: forward and grad x, grad W
using CfgF = Cfg<2, 4, 4, 2, 2, 1>;
using CfgX = Cfg<2, 4, 4, 2, 2, 1>;
using CfgW = Cfg<2, 4, 4, 2, 2, 1>;

int dw_splits(int F, int K, int R) {
  const int tiles = ((F + CfgW::TI - 1) / CfgW::TI) * ((K + CfgW::TJ - 1) / CfgW::TJ);
  const int ntot = 2 * ((R + kBK - 1) / kBK);
  // The fewest rounds of workgroups over the chip's 256 CUs (one workgroup each), each round costing its share of
  // the contraction plus a fixed part (start-up, the float32 partial tile); ties go to fewer splits.
  int best = 1;
  long long best_cost = -1;
  for (int s = 1; s <= 32 && s <= ntot; ++s) {
    const long long rounds = ((long long)s * tiles + 255) / 256;
    const long long cost = rounds * ((ntot + s - 1) / s + 64);
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = s;
    }
  }
  return best;
}
// Persistent workgroups: 8 XCDs x at most 32 CUs, fewer where an XCD's share of the tiles is smaller.
int persistent_grid(int tiles) {
  const int per = (tiles + 7) / 8;
  return 8 * (per < 32 ? per : 32);
}
int bias_chunks(int R) {
  const int c = (R + 63) / 64;
  return c > 256 ? 256 : c;
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
  g.nz = 2;
  const int grid = persistent_grid(2 * ((R + CfgF::TI - 1) / CfgF::TI) * ((F + CfgF::TJ - 1) / CfgF::TJ));
  hipLaunchKernelGGL((gemm_kernel<false, false, false, CfgF>), dim3(grid), dim3(CfgF::NT), 0, st, g);
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
    g.nz = 2;
    const int grid = persistent_grid(2 * ((R + CfgX::TI - 1) / CfgX::TI) * ((K + CfgX::TJ - 1) / CfgX::TJ));
    hipLaunchKernelGGL((gemm_kernel<false, true, false, CfgX>), dim3(grid), dim3(CfgX::NT), 0, st, g);
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
    g.nz = splits;
    const int grid = persistent_grid(splits * ((F + CfgW::TI - 1) / CfgW::TI) * ((K + CfgW::TJ - 1) / CfgW::TJ));
    hipLaunchKernelGGL((gemm_kernel<true, true, true, CfgW>), dim3(grid), dim3(CfgW::NT), 0, st, g);
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
    hipLaunchKernelGGL(colsum_kernel, dim3((F + 511) / 512, chunks), dim3(256), 0, st, (const bf16*)gy, R, F, ldy, chunks, bp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bias_sum_kernel, dim3((unsigned)((F + 63) / 64)), dim3(1024), 0, st, bp, chunks, F, (bf16*)gbias);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace tvm
