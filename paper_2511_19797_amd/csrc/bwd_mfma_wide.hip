// Backward launchers, head dims 97..128 (see bwd_mfma_kernels.h for the kernels).
#include "bwd_mfma_kernels.h"

namespace tvm {

hipError_t launch_bwd_col_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (s.D <= 112) return launch_col<112, 128, 0>(s, a, st);
  if (s.D <= 128) return launch_col<128, 128, 0>(s, a, st);
  return hipErrorNotSupported;
}
hipError_t launch_bwd_row_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws) {
  if (s.D <= 112) return launch_row<112, 128, 0>(s, a, st, pipe_ws);
  if (s.D <= 128) return launch_row<128, 128, 0>(s, a, st, pipe_ws);
  return hipErrorNotSupported;
}

}  // namespace tvm
