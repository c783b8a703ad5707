// Building blocks of the hand-scheduled backward kernels (bwd_row_pipe.hip, bwd_col_pipe.hip): LDS
// reads from integer addresses (lane constant + immediate), the pointwise work as inline assembly,
// and the markers that tell the compiler when a matrix-core result may be read.
//
// Rules these kernels follow (their translation units are built with the machine scheduler off,
// so source order is issue order, and tests/test_isa_hazards.py checks the generated assembly):
//   - a matrix-core result is first read by anything else behind a landed() marker, which sits at
//     least four matrix-core products after the one that wrote it;
//   - a register written by a VALU instruction is not read by a matrix-core instruction in the
//     next two issue slots (the PAD form of the product puts two idle slots in front).
#pragma once
#include "mfma_tiles.h"
#include "pipe_prof.h"  // PROF_* cycle stamps: empty unless this is a diagnostic build (-DTVM_PROFILE)

namespace tvm {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ bf16x8 lds_read16(unsigned addr, int imm) {
  typedef const bf16x8 __attribute__((address_space(3))) * lp;
  return *(lp)(uintptr_t)(addr + (unsigned)imm);
}
__device__ __forceinline__ bf16x8 lds_read_tr(unsigned lo, unsigned hi, int imm) {
  typedef bf16x4 __attribute__((address_space(3))) * lp;
  const bf16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(uintptr_t)(lo + (unsigned)imm));
  const bf16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lp)(uintptr_t)(hi + (unsigned)imm));
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}
// The pointwise work is inline assembly too, so that it stays in the slot it is written in (the
// optimizer moves plain arithmetic freely between the matrix-core instructions otherwise).  It comes
// in pieces of one or two instructions (about 8 cycles each: v_exp_f32 and
// v_cvt_pk_bf16_f32 take the VALU for two issue slots), so that it can be dealt out evenly: behind one
// matrix-core product a lone wave has room for about 24 cycles of other VALU work (measured: six
// plain instructions, or three of the slow ones), whatever is issued beyond that delays the next
// product.  Dependent instructions closer than three apart also cost extra cycles.
//   a = x0 c - y0,  b = x1 c - y1      (c wave-uniform)
__device__ __forceinline__ void pw_fma2(float& a, float& b, float x0, float x1, float c, float y0, float y1) {
  asm volatile(
      "v_fma_f32 %0, %2, %4, -%5\n\t"
      "v_fma_f32 %1, %3, %4, -%6"
      : "=&v"(a), "=&v"(b)
      : "v"(x0), "v"(x1), "s"(c), "v"(y0), "v"(y1));
}
//   p = exp2(t),  n = x c - y          (c wave-uniform).  The exponential never ends a piece: the VALU
//   instruction right behind a transcendental one must not read its result (no interlock), and what
//   follows a piece may be a register copy of the compiler's.
__device__ __forceinline__ void pw_exp_fma(float& p, float t, float& n, float x, float c, float y) {
  asm volatile(
      "v_exp_f32 %0, %2\n\t"
      "v_fma_f32 %1, %3, %4, -%5"
      : "=&v"(p), "=&v"(n)
      : "v"(t), "v"(x), "s"(c), "v"(y));
}
//   a = x0 y0,  b = x1 y1
__device__ __forceinline__ void pw_mul2(float& a, float& b, float x0, float y0, float x1, float y1) {
  asm volatile(
      "v_mul_f32 %0, %2, %3\n\t"
      "v_mul_f32 %1, %4, %5"
      : "=&v"(a), "=&v"(b)
      : "v"(x0), "v"(y0), "v"(x1), "v"(y1));
}
//   a += x0 y0,  b += x1 y1
__device__ __forceinline__ void pw_fmac2(float& a, float& b, float x0, float y0, float x1, float y1) {
  asm volatile(
      "v_fmac_f32 %0, %2, %3\n\t"
      "v_fmac_f32 %1, %4, %5"
      : "+v"(a), "+v"(b)
      : "v"(x0), "v"(y0), "v"(x1), "v"(y1));
}
//   r = (bf16(lo), bf16(hi)), round to nearest even
__device__ __forceinline__ void pw_cvt(unsigned& r, float lo, float hi) {
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
}
// Dealing side operations out over the products of a phase by cost.  Operation u (issued in order) costs
// cost(u) cycles, slot s (the gap behind product s) already carries base(s) cycles of other side
// instructions; slots before s0 take none.  Greedy: every slot takes operations while that brings it closer
// to the average load of the slots that are left.  At least k_ops operations are placed before slot k_slot
// (a deadline: the products from k_slot on read their results).  Operations [first[s], first[s+1]) go
// behind product s.
template <int NSLOT>
struct Deal {
  int first[NSLOT + 1];
};
__host__ __device__ constexpr int share_count(int m, int cnt, int n) { return (m + 1) * cnt / n - m * cnt / n; }
template <int NSLOT, typename Cost, typename Base>
__host__ __device__ constexpr void deal_range(Deal<NSLOT>& d, int u0, int u1, int sa, int sb, Cost cost, Base base) {
  int total = 0;
  for (int u = u0; u < u1; ++u) total += cost(u);
  for (int s = sa; s < sb; ++s) total += base(s);
  int u = u0;
  for (int s = sa; s < sb; ++s) {
    d.first[s] = u;
    const int left = sb - s;
    const int target = (total + left - 1) / left;
    int load = base(s);
    if (s == sb - 1) {
      while (u < u1) load += cost(u++);
    } else {
      while (u < u1 && load + cost(u) / 2 < target) load += cost(u++);
    }
    total -= load;
  }
}
template <int NSLOT, typename Cost, typename Base>
__host__ __device__ constexpr Deal<NSLOT> deal_out(int nops, int s0, int k_slot, int k_ops, Cost cost, Base base) {
  Deal<NSLOT> d{};
  for (int s = 0; s <= NSLOT; ++s) d.first[s] = s < s0 ? 0 : nops;
  if (s0 >= NSLOT) return d;
  deal_range(d, 0, nops, s0, NSLOT, cost, base);
  if (k_slot > s0 && k_slot < NSLOT && d.first[k_slot] < k_ops) {
    deal_range(d, 0, k_ops, s0, k_slot, cost, base);
    deal_range(d, k_ops, nops, k_slot, NSLOT, cost, base);
  }
  d.first[NSLOT] = nops;
  return d;
}

// From here on the compiler may read the tiles: every use below this point depends on it.  Placed
// after enough further products that the ones writing the tiles have finished.
__device__ __forceinline__ void landed(f32x16& a, f32x16& b) { asm volatile("" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void landed_acc(f32x16& a) { asm volatile("" : "+a"(a)); }
__device__ __forceinline__ bf16x8 frag_of(const unsigned (&w)[8], int cc) {
  const uint4 v = make_uint4(w[4 * cc], w[4 * cc + 1], w[4 * cc + 2], w[4 * cc + 3]);
  return __builtin_bit_cast(bf16x8, v);
}


}  // namespace tvm
