// Backward launchers for one upstream gradient (gTO only: the tangent path by itself) at head dims above 96, where
// the hand-scheduled kernels do not go (see bwd_mfma_kernels.h for the kernels; up to 96 it is bwd_*_pipe_tangent.hip).
#include "bwd_mfma_kernels.h"

namespace tvm {

#define TVM_BY_HEAD_DIM(fn)                          \
  switch ((s.D + 15) / 16 * 16) {                    \
    case 112: return fn<112, 128, 2>(s, a, st);       \
    case 128: return fn<128, 128, 2>(s, a, st);       \
    default: return hipErrorNotSupported;            \
  }

hipError_t launch_bwd_col_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st) { TVM_BY_HEAD_DIM(launch_col) }
hipError_t launch_bwd_row_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st) { TVM_BY_HEAD_DIM(launch_row) }

}  // namespace tvm
