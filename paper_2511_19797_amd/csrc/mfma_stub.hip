#include "tvm_common.h"
namespace tvm {
bool mfma_supported(const Shape&, int) { return false; }
hipError_t launch_fwd_mfma(const Shape&, const FwdArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_mfma(const Shape&, const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}
