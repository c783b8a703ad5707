// Diagnostic builds only (-DTVM_PROFILE): cycle stamps per phase of the hand-scheduled backward kernels, kept for one
// workgroup in a device array of the translation unit, and the reader that copies them out.  In a product build
// every PROF_* macro is empty and nothing of this header reaches the library.
#pragma once
#if defined(TVM_PROFILE)
#include <hip/hip_runtime.h>
#if !defined(TVM_PROF_BLOCK)
#define TVM_PROF_BLOCK 3  // hardware id of the workgroup whose stamps are kept
#endif
namespace tvm {
static __device__ long long g_prof_pipe[16];
}
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
  if (blockIdx.x == TVM_PROF_BLOCK && threadIdx.x == 0)         \
    for (int i_ = 0; i_ < 8; ++i_) g_prof_pipe[i_] = pa_[i_]
#define PROF_EXIT                                                      \
  if (blockIdx.x == TVM_PROF_BLOCK && threadIdx.x == 0) {                           \
    g_prof_pipe[8] = pl_ - pe_;                                        \
    g_prof_pipe[9] = px_ - pl_;                                        \
    g_prof_pipe[10] = clock64() - px_;                                 \
    for (int i_ = 11; i_ < 16; ++i_) g_prof_pipe[i_] = pp_[i_];        \
  }
// One reader per translation unit that asks for it (TVM_PROF_READER names it).
#if defined(TVM_PROF_READER)
extern "C" int TVM_PROF_READER(long long* out16) {
  return (int)hipMemcpyFromSymbol(out16, HIP_SYMBOL(tvm::g_prof_pipe), sizeof(long long) * 16);
}
#endif
#else
#define PROF_ENTRY
#define PROF_P(i)
#define PROF_DECL
#define PROF(i)
#define PROF_DUMP
#define PROF_EXIT
#endif
