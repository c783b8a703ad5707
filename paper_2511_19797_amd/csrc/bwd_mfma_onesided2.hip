// Backward launchers for one upstream gradient (gTO only: the tangent path by itself) at head dims above 96 on the
// generic-order kernels (bwd_mfma_kernels.h): the query side always, the key side for few queries (otherwise it runs
// as the hand-scheduled passes of bwd_pass.hip; up to 96 it is bwd_*_pipe_tangent.hip).
#include "bwd_mfma_kernels.h"

namespace tvm {

hipError_t launch_bwd_col_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st) {
  switch ((s.D + 15) / 16 * 16) {
    case 112: return launch_col<112, 128, 2>(s, a, st);
    case 128: return launch_col<128, 128, 2>(s, a, st);
    default: return hipErrorNotSupported;
  }
}
// pipe_ws: the row vectors go to the workspace as the hand-scheduled key-side passes read them
hipError_t launch_bwd_row_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws) {
  switch ((s.D + 15) / 16 * 16) {
    case 112: return launch_row<112, 128, 2>(s, a, st, pipe_ws);
    case 128: return launch_row<128, 128, 2>(s, a, st, pipe_ws);
    default: return hipErrorNotSupported;
  }
}

}  // namespace tvm
