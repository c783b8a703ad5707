// Backward launchers for one upstream gradient (gTO only: the tangent path by itself), every head dim the matrix-core
// path takes (see bwd_mfma_kernels.h for the kernels).
#include "bwd_mfma_kernels.h"

namespace tvm {

#define TVM_BY_HEAD_DIM(fn)                          \
  switch ((s.D + 15) / 16 * 16) {                    \
    case 16: return fn<16, 32, 2>(s, a, st);          \
    case 32: return fn<32, 32, 2>(s, a, st);          \
    case 48: return fn<48, 64, 2>(s, a, st);          \
    case 64: return fn<64, 64, 2>(s, a, st);          \
    case 80: return fn<80, 96, 2>(s, a, st);          \
    case 96: return fn<96, 96, 2>(s, a, st);          \
    case 112: return fn<112, 128, 2>(s, a, st);       \
    case 128: return fn<128, 128, 2>(s, a, st);       \
    default: return hipErrorNotSupported;            \
  }

hipError_t launch_bwd_col_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st) { TVM_BY_HEAD_DIM(launch_col) }
hipError_t launch_bwd_row_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st) { TVM_BY_HEAD_DIM(launch_row) }

}  // namespace tvm
