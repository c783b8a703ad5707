#include "tvm_common.h"
namespace tvm {
bool mfma_supported(const Shape& s, int dtype) { return dtype == 1 && s.D % 8 == 0 && s.D <= 128; }
hipError_t launch_bwd_mfma(const Shape& s, const BwdArgs& a, hipStream_t st) { return launch_bwd_generic(s, 1, a, st); }
}
