// bf16 matrix-core building blocks shared by the forward and backward kernels (gfx950).
//
// One MFMA is used throughout: v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] B[16x32].
// Operand layout per lane (lane = 32*hh + ic):
//   A: row ic of A, eight consecutive k starting at 8*hh          (8 bf16 = 16 bytes)
//   B: column ic of B, the same eight k
//   D: column ic of D, rows 8*(r/4) + 4*hh + (r%4) for register r = 0..15
// Since A and B index k the same way, any fixed permutation of k applied to both operands
// leaves the product unchanged.  That is used to feed a D-layout tile straight back in as the
// B operand of the next product: registers 8c..8c+7 of a D tile are, for this lane, the eight
// rows 16c + {0,1,2,3, 8,9,10,11} + 4*hh ("slot order"), so the A operand of that product is
// fetched from LDS with its contraction index in the same order.
//
// LDS tiles are row-major [rows][D] in 16-byte chunks with a swizzle: element (s, col) lives in
// physical chunk  s*PCH + ((col/8) ^ ((s>>2)&3)),  PCH = 4 (mod 8) chunks per row.  Two access
// patterns hit every bank exactly once per pass with this layout:
//   (R) ds_read_b128, lanes = 16 consecutive rows, same logical chunk      (score products)
//   (T) ds_read_b64_tr_b16, a 32-lane half = 4 consecutive rows x 64 bytes  (output products)
// The transposing read hands lane i of a 16-lane group the i-th column of the 4 x 16 block whose
// row e is supplied by lanes 4e..4e+3 (four elements each); two of them build one A fragment of
// X^T in slot order, with no transposed copy in LDS and no data movement through the VALU.
#pragma once
#include "tvm_common.h"

namespace tvm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The same product with the register file of every operand spelled out, for kernels whose
// instruction order is laid out by hand (their translation unit is built with the machine
// scheduler off, so source order is issue order).  The compiler treats these as ordinary
// instructions: it knows neither that the result lands some 40-50 cycles after issue nor that a
// VALU read before then would see stale data.  The caller keeps at least four further
// matrix-core products (or mfma_settle) between a product and the first non-matrix read of its
// result; feeding the result to the next product as C needs no distance.
//   mfma_acc : accumulator in AGPRs, both operands in VGPRs        (output products)
//   mfma_fix : result in VGPRs, B = a fixed-side fragment in AGPRs  (score-type products)
//   mfma_fix0: the same with C = 0 (starts a tile)
//   mfma_fixc: as mfma_fix0 with a tile of start values instead of 0
//   mfma_vv, mfma_vv0: as mfma_fix, mfma_fix0 with B in VGPRs too
// PAD puts two idle issue slots in front of the product: a matrix-core instruction must not read a
// register that a VALU instruction (a register copy the compiler placed there, say) wrote in
// one of the two slots before it.
#define TVM_MFMA_PAD "s_nop 1\n\t"
template <bool PAD = false>
__device__ __forceinline__ void mfma_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
template <bool PAD = false>
__device__ __forceinline__ void mfma_fix(f32x16& sc, bf16x8 a, bf16x8 fixed_b) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sc) : "v"(a), "a"(fixed_b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sc) : "v"(a), "a"(fixed_b));
}
template <bool PAD = false>
__device__ __forceinline__ void mfma_fix0(f32x16& sc, bf16x8 a, bf16x8 fixed_b) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sc) : "v"(a), "a"(fixed_b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sc) : "v"(a), "a"(fixed_b));
}
// result in VGPRs, B = a fixed-side fragment in AGPRs, C = a separate tile in VGPRs (starts a tile from it)
template <bool PAD = false>
__device__ __forceinline__ void mfma_fixc(f32x16& sc, bf16x8 a, bf16x8 fixed_b, const f32x16& c) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(sc) : "v"(a), "a"(fixed_b), "v"(c));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(sc) : "v"(a), "a"(fixed_b), "v"(c));
}
// result in VGPRs, both operands in VGPRs
template <bool PAD = false>
__device__ __forceinline__ void mfma_vv(f32x16& sc, bf16x8 a, bf16x8 b) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sc) : "v"(a), "v"(b));
}
template <bool PAD = false>
__device__ __forceinline__ void mfma_vv0(f32x16& sc, bf16x8 a, bf16x8 b) {
  if (PAD) asm volatile(TVM_MFMA_PAD "v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sc) : "v"(a), "v"(b));
}
#undef TVM_MFMA_PAD
// Idles long enough for every product issued so far to have written its result.
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// Row (M index) held in register r of a D tile by a lane of half hh.
__device__ __forceinline__ int drow(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// Chunks (16 B) per LDS row for a tile whose widest access covers `cols` columns.
constexpr int pitch_chunks(int cols) {
  int p = (cols / 8 + 3) / 4 * 4;
  return (p % 8 == 0) ? p + 4 : p;
}

// Byte offset of logical chunk c of row s.
template <int PCH>
__device__ __forceinline__ int chunk_off(int s, int c) {
  return (s * PCH + (c ^ ((s >> 2) & 3))) * 16;
}

// Asynchronous global -> LDS copy: every lane fetches `BYTES` (16 or 4) from `base + off`
// (wave-uniform 64-bit base, per-lane unsigned 32-bit byte offset) and the wave writes them to
// LDS at address lds_addr + lane * BYTES (lds_addr wave-uniform).  Written as inline assembly so
// that the compiler does not serialise later LDS reads of OTHER buffers behind these loads; the
// kernels wait for them explicitly (dma_wait) before the barrier that publishes a tile.
template <int BYTES>
__device__ __forceinline__ void dma_to_lds(const void* base, unsigned off, unsigned lds_addr) {
  static_assert(BYTES == 16 || BYTES == 4, "dword or dwordx4");
  const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
  const unsigned long long b = (unsigned long long)(uintptr_t)base;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b), hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
  const unsigned long long bu = ((unsigned long long)hi << 32) | lo;  // provably uniform: lives in an SGPR pair
  // (one idle slot between the write of M0 and the load that takes its LDS address from it: the wait state
  // the ISA asks for after a scalar write of M0, which the compiler cannot insert inside an assembly statement)
  if (BYTES == 16)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m), "v"(off), "s"(bu) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(m), "v"(off), "s"(bu) : "memory", "m0");
}
// Waits until all of this wave's outstanding global loads (including dma_to_lds) have completed.
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Waits until at most KEEP of them are outstanding (they complete in issue order).
template <int KEEP>
__device__ __forceinline__ void dma_wait_keep() {
  static_assert(KEEP >= 0 && KEEP < 64, "vmcnt is six bits");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KEEP) : "memory");
}

// LDS address (the 32-bit value LDS instructions and M0 use) of a __shared__ object.
__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// A streamed tile: ROWS rows, logical chunks [0, NCH) (columns [0, 8*NCH)), filled by NW waves
// with asynchronous global->LDS loads (global_load_lds_dwordx4: each wave instruction fills 64
// consecutive physical chunks, every lane fetching the global chunk that the swizzle puts at
// its position).  No staging registers, no branches: every lane of every wave-load always
// fetches something valid.
//   - columns beyond D and pad positions: chunk 0 of the row (finite data; whatever multiplies
//     it is zero, or lands in output rows beyond D that are never stored);
//   - rows beyond the last one: the last row again (the kernels give such rows weight exactly 0);
//   - positions past the tile (when the tile is not a whole number of wave-loads per wave):
//     slack space after the tile, never read.
// The loads complete in the background and are waited for (dma_wait) just before the workgroup
// barrier that ends the computation on the other buffer.
template <int ROWS_, int NCH_, int NW_>
struct Tile {
  static constexpr int ROWS = ROWS_, NCH = NCH_, NW = NW_;
  static constexpr int PCH = pitch_chunks(NCH_ * 8);
  static constexpr int NINST = (ROWS_ * PCH + 63) / 64;  // wave-wide load instructions per tile
  static constexpr int IPW = (NINST + NW_ - 1) / NW_;    // of which each wave issues this many
  static constexpr int BYTES = IPW * NW_ * 1024;         // LDS footprint (tile + slack)

  // Per-lane constants: tile row and byte offset within the row of each chunk this lane fetches.
  struct Lane {
    unsigned col[IPW];
    int srow[IPW];
  };
  __device__ __forceinline__ static Lane lane_setup(int D, int wave, int lane) {
    Lane L;
#pragma unroll
    for (int t = 0; t < IPW; ++t) {
      const int P = (wave + t * NW) * 64 + lane;
      const int s = P / PCH;
      const int c = (P - s * PCH) ^ ((s >> 2) & 3);
      L.col[t] = (unsigned)((c * 8 < D ? c * 8 : 0) * 2);
      L.srow[t] = s;
    }
    return L;
  }
  // t-th wave-load of the tile whose first row is at `tile` (row pitch `pitch` bytes); rows_left >= 1
  // rows exist from there on.  `lds` is the LDS address of the tile buffer.
  __device__ __forceinline__ static void issue_one(const Lane& L, int t, const bf16* __restrict__ tile, unsigned pitch,
                                                   int rows_left, unsigned lds, int wave) {
    const unsigned r = (unsigned)min(L.srow[t], rows_left - 1);
    dma_to_lds<16>(tile, r * pitch + L.col[t], lds + (unsigned)(wave + t * NW) * 1024u);
  }
  __device__ __forceinline__ static void issue(const Lane& L, const bf16* __restrict__ tile, unsigned pitch,
                                               int rows_left, unsigned lds, int wave) {
#pragma unroll
    for (int t = 0; t < IPW; ++t) issue_one(L, t, tile, pitch, rows_left, lds, wave);
  }
  // The same with the per-lane byte offsets worked out once: `rows` = rows that exist from the
  // tile's first row on (64 or more for a whole tile; the last tile's count for the last one).
  struct Offs {
    unsigned o[IPW];
  };
  __device__ __forceinline__ static Offs offsets(const Lane& L, unsigned pitch, int rows) {
    Offs f;
#pragma unroll
    for (int t = 0; t < IPW; ++t) f.o[t] = (unsigned)min(L.srow[t], rows - 1) * pitch + L.col[t];
    return f;
  }
  // t-th wave-load with a ready offset; `wave` must be wave-uniform in the compiler's eyes (read
  // through readfirstlane) so that the LDS address is scalar arithmetic
  __device__ __forceinline__ static void issue_at(unsigned off, int t, const bf16* __restrict__ tile, unsigned lds,
                                                  int wave) {
    dma_to_lds<16>(tile, off, lds + (unsigned)(wave + t * NW) * 1024u);
  }
  // Read addressing.  All swizzle arithmetic is folded into a few per-lane constants so that
  // every fragment read is  lane constant + compile-time immediate.
  //
  // (R) fragment kk of row (32*blk + ic): logical chunk 2kk+hh, XORed with x = (ic>>2)&3.
  //     (2kk+hh)^x = 2kk + (hh^(x&1)) + (x&2 ? (kk even ? +2 : -2) : 0): one constant for even kk, one for odd.
  struct RAddr {
    int e, o;
  };
  __device__ __forceinline__ static RAddr raddr(int ic, int hh) {
    const int x = (ic >> 2) & 3;
    const int base = (ic * PCH + (hh ^ (x & 1))) * 16;
    const int d = (x & 2) ? 32 : 0;
    return RAddr{base + d, base - d};
  }
  static constexpr int kBlkBytes = 32 * PCH * 16;  // 32 rows
  // `p` = tensor base within the stage; blk and kk are compile-time after unrolling
  __device__ __forceinline__ static bf16x8 frag_row(const char* p, RAddr a, int blk, int kk) {
    return *reinterpret_cast<const bf16x8*>(p + ((kk & 1) ? a.o : a.e) + blk * kBlkBytes + kk * 32);
  }
  // (T) A fragment of X^T: row (32*db + ic) of X^T, contraction index = rows 16*cc.. of X in slot
  //     order.  Lane (16*bq + i, hh) supplies rows 4hh + (i>>2) (+8 for the second read), logical
  //     chunk 4db + y with y = 2bq + ((i&3)>>1), XORed with (row>>2)&3 = hh (resp. hh+2).
  struct TAddr {
    int lo, hi;
  };
  __device__ __forceinline__ static TAddr taddr(int ic, int hh) {
    const int i = ic & 15, bq = ic >> 4;
    const int y = 2 * bq + ((i & 3) >> 1);
    const int row = 4 * hh + (i >> 2);
    const int sub = (i & 1) * 8;
    return TAddr{(row * PCH + (y ^ hh)) * 16 + sub, ((row + 8) * PCH + (y ^ (hh + 2))) * 16 + sub};
  }
  __device__ __forceinline__ static bf16x8 frag_tr(const char* p, TAddr a, int cc, int db) {
    typedef bf16x4 __attribute__((address_space(3))) * lp;
    const int imm = cc * 16 * PCH * 16 + db * 64;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(p + a.lo + imm));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(p + a.hi + imm));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};

// Zero-fills `bytes` (a multiple of 16) of LDS with all NT threads of the workgroup.
template <int NT>
__device__ __forceinline__ void lds_zero(char* lds, int bytes, int tid) {
  for (int o = tid * 16; o < bytes; o += NT * 16) *reinterpret_cast<uint4*>(lds + o) = make_uint4(0, 0, 0, 0);
}

// Fixed-side fragments: chunks 2kk+hh (kk < NKS) of row `row` of a [N,D] matrix, zero where the row
// or the chunk is out of range.  The loads are unconditional (from a clamped, always valid
// address) and the zeroing is a select on the loaded value, so all of them are in flight together.
// In two steps, so that a kernel that needs several fragments can issue the loads of all of them before it
// touches the first value (each select waits for its load; one fragment after the other would pay one
// memory round trip per fragment).
template <int NKS>
__device__ __forceinline__ void gld_frags_issue(uint4 (&raw)[NKS], const bf16* __restrict__ head, long long sn, int row,
                                                int N, int D, int hh) {
  const bf16* p = head + (long long)min(row, N - 1) * sn;
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    const int c0 = kk * 16 + hh * 8;
    raw[kk] = *reinterpret_cast<const uint4*>(p + (c0 < D ? c0 : 0));
  }
}
template <int NKS>
__device__ __forceinline__ void gld_frags_finish(bf16x8 (&f)[NKS], const uint4 (&raw)[NKS], int row, int N, int D, int hh) {
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) {
    const bool ok = row < N && kk * 16 + hh * 8 < D;
    uint4 v = raw[kk];
    v.x = ok ? v.x : 0u;
    v.y = ok ? v.y : 0u;
    v.z = ok ? v.z : 0u;
    v.w = ok ? v.w : 0u;
    f[kk] = __builtin_bit_cast(bf16x8, v);
  }
}
template <int NKS>
__device__ __forceinline__ void gld_frags(bf16x8 (&f)[NKS], const bf16* __restrict__ head, long long sn, int row, int N,
                                          int D, int hh) {
  uint4 raw[NKS];
  gld_frags_issue<NKS>(raw, head, sn, row, N, D, hh);
  gld_frags_finish<NKS>(f, raw, row, N, D, hh);
}

// Makes the fragments exist here: placed before a wait or a barrier it keeps the compiler from sinking their
// loads below it (it would: they read memory nobody writes), which would turn one memory round trip into two.
template <int NKS>
__device__ __forceinline__ void pin_frags(bf16x8 (&f)[NKS]) {
#pragma unroll
  for (int kk = 0; kk < NKS; ++kk) asm volatile("" : "+v"(f[kk]));
}

__device__ __forceinline__ bf16x8 zero_unless(bf16x8 f, bool keep) {
  uint4 v = __builtin_bit_cast(uint4, f);
  v.x = keep ? v.x : 0u;
  v.y = keep ? v.y : 0u;
  v.z = keep ? v.z : 0u;
  v.w = keep ? v.w : 0u;
  return __builtin_bit_cast(bf16x8, v);
}

// The value the lane 32 away holds (one VALU swap of the two half-waves, no trip through LDS).
__device__ __forceinline__ float xhalf(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // r[0] = {lo, lo}, r[1] = {hi, hi}
  return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  This maps the
// hardware id to a logical id such that consecutive logical ids (the blocks of one head, which
// stream the same tensors) run on the same XCD.
__device__ __forceinline__ int xcd_remap(int wg, int nwg) {
  const int per = nwg >> 3;
  if ((nwg & 7) != 0) return wg;
  return (wg & 7) * per + (wg >> 3);
}

// Stores a transposed accumulator (rows = d, column = this lane's row of the output) as bf16, scaled.
template <int NDB>
__device__ __forceinline__ void store_acc(bf16* __restrict__ dst, const f32x16 (&a)[NDB], float scale, int D, int hh) {
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = db * 32 + 8 * g + 4 * hh;
      if (d0 < D) {
        bf16x4 o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (bf16)(a[db][4 * g + t] * scale);
        *reinterpret_cast<bf16x4*>(dst + d0) = o;
      }
    }
}

// Coalesced store of one wave's [32 x D] output tile held as transposed accumulators (rows = d,
// column = this lane's output row): the wave parks the tile in its own LDS region as bf16, row by
// row, then writes it out in 16-byte chunks with consecutive lanes on consecutive chunks, so a
// wave store covers whole rows instead of 32 scattered 8-byte pieces (which cost about four
// times as much per byte).  Only wave-local ordering is needed: a wave reads back what it wrote
// itself, and the LDS executes one wave's instructions in order.
//   lds_wave: LDS address of this wave's region, 32 * (64*NDB + 16) bytes, not in use by anyone else.
//   head: the tensor's (batch, head) base;  row0: first of the wave's 32 rows;  rows >= N are skipped.
template <int NDB>
__device__ __forceinline__ void store_tile_coalesced(unsigned lds_wave, bf16* __restrict__ head, long long sn, int row0,
                                                     int N, int D, const f32x16 (&a)[NDB], float scale, int lane) {
  constexpr int PB = 64 * NDB + 16;  // row pitch: 16-byte aligned, and 8-byte writes of 32 lanes hit 64 distinct banks
  constexpr int NCH = 4 * NDB;       // 16-byte chunks per (padded) row
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  typedef u32x2 __attribute__((address_space(3))) * wp;
  typedef const u32x4 __attribute__((address_space(3))) * rp;
  const int ic = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 o;
#pragma unroll
      for (int t = 0; t < 4; ++t) o[t] = (bf16)(a[db][4 * g + t] * scale);
      *(wp)(uintptr_t)(lds_wave + (unsigned)(ic * PB + (db * 32 + 8 * g + 4 * hh) * 2)) = __builtin_bit_cast(u32x2, o);
    }
#pragma unroll
  for (int it = 0; it < (32 * NCH + 63) / 64; ++it) {
    const int idx = it * 64 + lane;
    const int r = idx / NCH, c = idx - r * NCH;
    if (idx < 32 * NCH && c * 8 < D && row0 + r < N) {
      const u32x4 v = *(rp)(uintptr_t)(lds_wave + (unsigned)(r * PB + c * 16));
      *reinterpret_cast<u32x4*>(head + (long long)(row0 + r) * sn + c * 8) = v;
    }
  }
}


// ---- Backward through an RMSNorm with gain that normalised the rows before the attention, in the epilogue.
// Sum over the 16 lanes of a row group (lanes 16k .. 16k+15), the same bits in all of them: a butterfly of four
// data-parallel-primitive moves, no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_move16(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float sum16(float x) {
  x += dpp_move16<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_move16<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_move16<0x141>(x);  // row_half_mirror
  x += dpp_move16<0x140>(x);  // row_mirror
  return x;
}
// Parks one wave's [32 x D] tile (transposed accumulators, scaled) in its LDS region as bf16, row by row: the
// first half of store_tile_coalesced.  Region: 32 * (64*NDB + 16) bytes.
template <int NDB>
__device__ __forceinline__ void park_tile(unsigned lds_wave, const f32x16 (&a)[NDB], float scale, int lane) {
  constexpr int PB = 64 * NDB + 16;
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
  typedef u32x2 __attribute__((address_space(3))) * wp;
  const int ic = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 o;
#pragma unroll
      for (int t = 0; t < 4; ++t) o[t] = (bf16)(a[db][4 * g + t] * scale);
      *(wp)(uintptr_t)(lds_wave + (unsigned)(ic * PB + (db * 32 + 8 * g + 4 * hh) * 2)) = __builtin_bit_cast(u32x2, o);
    }
}
// The wave's 32 rows were y = g o x r, ty = g o (tx r - x r^3 m) with r = 1 / sqrt(mean(x^2) + eps), m = mean(x tx)
// (RMSNorm with gain as QK-norm and its tangent; Sec. "Semi-Lipschitz control", App. "Lipschitzness of RMSNorm")
// before they entered the attention.  With the gradients gy, gty of the attention with respect to y, ty parked at
// lds_gy, lds_gty (park_tile), this reads x, tx, writes the gradients with respect to them,
//     gtx = r w - (r^3 Bw / d) x,   gx = r u - r^3 m w - (r^3 Bw / d) tx + x (3 r^5 m Bw - r^3 (A + C)) / d
//     (u = g o gy, w = g o gty, A = <u,x>, Bw = <w,x>, C = <w,tx>),
// 16 lanes to a row and 16 bytes per lane, four rows at a time, and adds this wave's part of the gain gradient,
// gy o x r + gty o (tx r - x r^3 m), for the lane's eight columns into gacc.  Needs D <= 128.
// The rows of x and tx are fetched first, all of them (norm_rows_fetch: call it before the tiles are parked, so
// that one memory round trip covers the wave's 32 rows), then worked on.
struct NormRows {
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  u32x4 x[8], t[8];
};
__device__ __forceinline__ void norm_rows_fetch(NormRows& nr, const bf16* __restrict__ x_head, const bf16* __restrict__ tx_head,
                                                long long sn, int row0, int N, int D, int lane) {
  const int lr = lane & 15, slot = lane >> 4;
  const int c8 = lr * 8 < D ? lr * 8 : 0;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const long long off = (long long)min(row0 + it * 4 + slot, N - 1) * sn + c8;
    nr.x[it] = *reinterpret_cast<const NormRows::u32x4*>(x_head + off);
    nr.t[it] = *reinterpret_cast<const NormRows::u32x4*>(tx_head + off);
  }
}
template <int NDB>
__device__ __forceinline__ void store_tiles_through_norm(unsigned lds_gy, unsigned lds_gty, const NormRows& nr,
                                                         const float* __restrict__ gain, float eps,
                                                         bf16* __restrict__ gx_head, bf16* __restrict__ gtx_head,
                                                         long long sn, int row0, int N, int D, int lane, float (&gacc)[8]) {
  constexpr int PB = 64 * NDB + 16;
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  typedef const u32x4 __attribute__((address_space(3))) * rp;
  const int lr = lane & 15, slot = lane >> 4;
  const bool live = lr * 8 < D;   // (D is a multiple of 8 on this path)
  const int c8 = live ? lr * 8 : 0;
  const float invd = 1.0f / (float)D;
  float g[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] = live ? gain[c8 + e] : 0.f;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = it * 4 + slot;
    const bool valid = row0 + r < N;
    const long long off = (long long)min(row0 + r, N - 1) * sn + c8;
    u32x4 rx = nr.x[it];
    u32x4 rt = nr.t[it];
    u32x4 ry = *(rp)(uintptr_t)(lds_gy + (unsigned)(r * PB + c8 * 2));
    u32x4 rz = *(rp)(uintptr_t)(lds_gty + (unsigned)(r * PB + c8 * 2));
    if (!live) rx = rt = ry = rz = u32x4{0u, 0u, 0u, 0u};
    const bf16x8 xb = __builtin_bit_cast(bf16x8, rx), tb = __builtin_bit_cast(bf16x8, rt);
    const bf16x8 yb = __builtin_bit_cast(bf16x8, ry), zb = __builtin_bit_cast(bf16x8, rz);
    float x[8], t[8], u[8], w[8];
    float sxx = 0.f, sxt = 0.f, sA = 0.f, sB = 0.f, sC = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x[e] = (float)xb[e];
      t[e] = (float)tb[e];
      u[e] = g[e] * (float)yb[e];
      w[e] = g[e] * (float)zb[e];
      sxx = fmaf(x[e], x[e], sxx);
      sxt = fmaf(x[e], t[e], sxt);
      sA = fmaf(u[e], x[e], sA);
      sB = fmaf(w[e], x[e], sB);
      sC = fmaf(w[e], t[e], sC);
    }
    sxx = sum16(sxx);
    sxt = sum16(sxt);
    sA = sum16(sA);
    sB = sum16(sB);
    sC = sum16(sC);
    const float rr = 1.0f / sqrtf(sxx * invd + eps);
    const float r3 = rr * rr * rr, m = sxt * invd;
    const float r3m = r3 * m, kB = r3 * sB * invd;
    const float kx = (3.0f * r3 * rr * rr * m * sB - r3 * (sA + sC)) * invd;
    bf16x8 ox, ot;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      ot[e] = (bf16)(rr * w[e] - kB * x[e]);
      ox[e] = (bf16)(rr * u[e] - r3m * w[e] - kB * t[e] + kx * x[e]);
      const float term = (float)yb[e] * (x[e] * rr) + (float)zb[e] * (t[e] * rr - x[e] * r3m);
      gacc[e] += valid ? term : 0.f;
    }
    if (live && valid) {
      *reinterpret_cast<u32x4*>(gx_head + off) = __builtin_bit_cast(u32x4, ox);
      *reinterpret_cast<u32x4*>(gtx_head + off) = __builtin_bit_cast(u32x4, ot);
    }
  }
}
// One row of gain-gradient column sums per workgroup: the 4 waves x 4 row slots add their gacc in a fixed order
// through `red` (LDS, 16 x 128 floats, free to use) and the row goes to part[0 .. D).  Call with all threads.
__device__ __forceinline__ void gain_partial_row(float* red, const float (&gacc)[8], float* __restrict__ part, int D, int tid) {
  const int lane = tid & 63, wave = tid >> 6, lr = lane & 15, slot = lane >> 4;
#pragma unroll
  for (int e = 0; e < 8; ++e) red[(wave * 4 + slot) * 128 + lr * 8 + e] = gacc[e];
  __syncthreads();
  for (int col = tid; col < D; col += 256) {
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) sum += red[k * 128 + col];
    part[col] = sum;
  }
}

}  // namespace tvm
