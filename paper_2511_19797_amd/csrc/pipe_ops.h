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

namespace tvm {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// Optional cycle stamps per phase (build with -DTVM_PROFILE; each translation unit has its own counters and exports its own reader).
#if defined(TVM_PROFILE)
static __device__ long long g_prof_pipe[16];
#define PROF_ENTRY const long long pe_ = clock64(); long long pp_[16]
#define PROF_P(i) pp_[i] = clock64() - pe_
#define PROF_DECL long long pt_ = clock64(), pa_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; const long long pl_ = pt_
#define PROF(i)                        \
  do {                                 \
    const long long n_ = clock64();    \
    pa_[i] += n_ - pt_;                \
    pt_ = n_;                          \
  } while (0)
#define PROF_DUMP                                  \
  const long long px_ = clock64();                 \
  if (blockIdx.x == 3 && threadIdx.x == 0)         \
    for (int i_ = 0; i_ < 8; ++i_) g_prof_pipe[i_] = pa_[i_]
#define PROF_EXIT                                                      \
  if (blockIdx.x == 3 && threadIdx.x == 0) {                           \
    g_prof_pipe[8] = pl_ - pe_;                                        \
    g_prof_pipe[9] = px_ - pl_;                                        \
    g_prof_pipe[10] = clock64() - px_;                                 \
    for (int i_ = 11; i_ < 16; ++i_) g_prof_pipe[i_] = pp_[i_];        \
  }
#else
#define PROF_ENTRY
#define PROF_P(i)
#define PROF_DECL
#define PROF(i)
#define PROF_DUMP
#define PROF_EXIT
#endif

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
// optimizer moves plain arithmetic freely between the matrix-core instructions otherwise).
//   P = exp2(S c1 - lse2),  N = St alpha - mub
__device__ __forceinline__ void pw1_asm(float& p, float& n, float sv, float st, float c1, float lse2, float alpha,
                                        float mub) {
  float t;
  asm volatile(
      "v_fma_f32 %2, %3, %5, -%6\n\t"
      "v_fma_f32 %1, %4, %7, -%8\n\t"
      "v_exp_f32 %0, %2"
      : "=v"(p), "=v"(n), "=&v"(t)
      : "v"(sv), "v"(st), "s"(c1), "v"(lse2), "s"(alpha), "v"(mub));
}
//   gZt = P (E - sig1),  gZ = P (DF - dsig) + gZt N, for two neighbouring elements, rounded to bf16 and packed
__device__ __forceinline__ void pw2_asm(unsigned& gz, unsigned& gzt, float e0, float e1, float f0, float f1, float p0,
                                        float p1, float n0, float n1, float s1, float ds) {
  float t0, t1, w0, w1;
  asm volatile(
      "v_sub_f32 %2, %6, %14\n\t"
      "v_sub_f32 %3, %7, %14\n\t"
      "v_sub_f32 %4, %8, %15\n\t"
      "v_sub_f32 %5, %9, %15\n\t"
      "v_mul_f32 %2, %10, %2\n\t"
      "v_mul_f32 %3, %11, %3\n\t"
      "v_mul_f32 %4, %10, %4\n\t"
      "v_mul_f32 %5, %11, %5\n\t"
      "v_fmac_f32 %4, %2, %12\n\t"
      "v_fmac_f32 %5, %3, %13\n\t"
      "v_cvt_pk_bf16_f32 %0, %4, %5\n\t"
      "v_cvt_pk_bf16_f32 %1, %2, %3"
      : "=&v"(gz), "=&v"(gzt), "=&v"(t0), "=&v"(t1), "=&v"(w0), "=&v"(w1)
      : "v"(e0), "v"(e1), "v"(f0), "v"(f1), "v"(p0), "v"(p1), "v"(n0), "v"(n1), "v"(s1), "v"(ds));
}
//   The same with sig1 and dsig per element (the key-side kernel: its elements are different queries).
__device__ __forceinline__ void pw2_pair_asm(unsigned& gz, unsigned& gzt, float e0, float e1, float f0, float f1,
                                             float p0, float p1, float n0, float n1, float sa0, float sa1, float da0,
                                             float da1) {
  float t0, t1, w0, w1;
  asm volatile(
      "v_sub_f32 %2, %6, %14\n\t"
      "v_sub_f32 %3, %7, %15\n\t"
      "v_sub_f32 %4, %8, %16\n\t"
      "v_sub_f32 %5, %9, %17\n\t"
      "v_mul_f32 %2, %10, %2\n\t"
      "v_mul_f32 %3, %11, %3\n\t"
      "v_mul_f32 %4, %10, %4\n\t"
      "v_mul_f32 %5, %11, %5\n\t"
      "v_fmac_f32 %4, %2, %12\n\t"
      "v_fmac_f32 %5, %3, %13\n\t"
      "v_cvt_pk_bf16_f32 %0, %4, %5\n\t"
      "v_cvt_pk_bf16_f32 %1, %2, %3"
      : "=&v"(gz), "=&v"(gzt), "=&v"(t0), "=&v"(t1), "=&v"(w0), "=&v"(w1)
      : "v"(e0), "v"(e1), "v"(f0), "v"(f1), "v"(p0), "v"(p1), "v"(n0), "v"(n1), "v"(sa0), "v"(sa1), "v"(da0),
        "v"(da1));
}
//   The key-side kernel's second step when E and DF already have sig1 and dsig subtracted (their
//   tiles start from -sig1, -dsig instead of 0):  gZt = P E',  gZ = P DF' + gZt N.
__device__ __forceinline__ void pw2_shifted_pair_asm(unsigned& gz, unsigned& gzt, float e0, float e1, float f0, float f1,
                                                     float p0, float p1, float n0, float n1) {
  float t0, t1, w0, w1;
  asm volatile(
      "v_mul_f32 %2, %10, %6\n\t"
      "v_mul_f32 %3, %11, %7\n\t"
      "v_mul_f32 %4, %10, %8\n\t"
      "v_mul_f32 %5, %11, %9\n\t"
      "v_fmac_f32 %4, %2, %12\n\t"
      "v_fmac_f32 %5, %3, %13\n\t"
      "v_cvt_pk_bf16_f32 %0, %4, %5\n\t"
      "v_cvt_pk_bf16_f32 %1, %2, %3"
      : "=&v"(gz), "=&v"(gzt), "=&v"(t0), "=&v"(t1), "=&v"(w0), "=&v"(w1)
      : "v"(e0), "v"(e1), "v"(f0), "v"(f1), "v"(p0), "v"(p1), "v"(n0), "v"(n1));
}
//   The key-side kernel's form of the first step, for two neighbouring elements: P and N as above
//   (lse2, mub per element), plus Pd = P N, with P and Pd rounded to bf16 and packed.
__device__ __forceinline__ void pw1_pair_asm(float& p0, float& p1, float& n0, float& n1, unsigned& pk, unsigned& pdk,
                                             float s0, float s1, float st0, float st1, float c1, float l0, float l1,
                                             float alpha, float m0, float m1) {
  float t0, t1;
  asm volatile(
      "v_fma_f32 %6, %8, %12, -%13\n\t"
      "v_fma_f32 %7, %9, %12, -%14\n\t"
      "v_exp_f32 %0, %6\n\t"
      "v_exp_f32 %1, %7\n\t"
      "v_fma_f32 %2, %10, %15, -%16\n\t"
      "v_fma_f32 %3, %11, %15, -%17\n\t"
      "v_mul_f32 %6, %0, %2\n\t"
      "v_mul_f32 %7, %1, %3\n\t"
      "v_cvt_pk_bf16_f32 %4, %0, %1\n\t"
      "v_cvt_pk_bf16_f32 %5, %6, %7"
      : "=&v"(p0), "=&v"(p1), "=&v"(n0), "=&v"(n1), "=&v"(pk), "=&v"(pdk), "=&v"(t0), "=&v"(t1)
      : "v"(s0), "v"(s1), "v"(st0), "v"(st1), "s"(c1), "v"(l0), "v"(l1), "s"(alpha), "v"(m0), "v"(m1));
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
