// The forward kernels of fwd_mfma.hip with the query side's RMSNorm (with gain, and its tangent) folded into the
// load of the query fragments: one translation unit per variant, so that they compile side by side.
#define TVM_FWD_QNORM 1
#define TVM_FWD_LAUNCHER launch_fwd_mfma_qnorm
#include "fwd_mfma.hip"
