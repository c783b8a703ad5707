// Stand-ins for the kernel launchers, so that the C-ABI's host code (argument validation, workspace layout,
// dispatch) can run under AddressSanitizer and UndefinedBehaviorSanitizer on a machine without a GPU: every
// launcher records that it was reached and returns success without touching the device.
#include "../../paper_2511_19797_amd/csrc/tvm_common.h"

int g_stub_launches = 0;

namespace tvm {
#define STUB(sig) hipError_t sig { ++g_stub_launches; return hipSuccess; }
STUB(launch_fwd_generic(const Shape&, int, const FwdArgs&, hipStream_t))
STUB(launch_bwd_pre(const Shape&, int, const BwdArgs&, hipStream_t))
STUB(launch_bwd_col_generic(const Shape&, int, const BwdArgs&, hipStream_t))
STUB(launch_bwd_row_generic(const Shape&, int, const BwdArgs&, hipStream_t))
STUB(launch_fwd_mfma(const Shape&, const FwdArgs&, hipStream_t))
STUB(launch_fwd_mfma_qnorm(const Shape&, const FwdArgs&, hipStream_t))
STUB(launch_bwd_col_mfma(const Shape&, const BwdArgs&, hipStream_t))
STUB(launch_bwd_row_mfma(const Shape&, const BwdArgs&, hipStream_t))
STUB(launch_bwd_row_pipe_qknorm(const Shape&, const BwdArgs&, hipStream_t))
STUB(launch_bwd_col_pipe_qknorm(const Shape&, const BwdArgs&, hipStream_t))
STUB(launch_gain_grad_sum(const float*, int, float*, const float*, int, float*, int, hipStream_t))
STUB(launch_qknorm_fwd(const NormArgs&, int, hipStream_t))
STUB(launch_qknorm_bwd(const NormArgs&, int, hipStream_t))
STUB(launch_gate_fwd(const GateArgs&, int, hipStream_t))
STUB(launch_gate_bwd(const GateArgs&, int, hipStream_t))
STUB(launch_gelu_fwd(long long, int, const void*, const void*, void*, void*, hipStream_t))
STUB(launch_gelu_bwd(long long, int, const void*, const void*, const void*, const void*, void*, void*, hipStream_t))
STUB(launch_adaln_fwd(const AdalnArgs&, int, hipStream_t))
STUB(launch_adaln_bwd(const AdalnArgs&, int, hipStream_t))
STUB(launch_linear_fwd(int, int, int, long long, long long, const void*, const void*, const void*, const void*, void*, void*,
                       hipStream_t))
STUB(launch_linear_bwd(int, int, int, long long, long long, const void*, const void*, const void*, const void*, const void*,
                       void*, void*, void*, void*, void*, hipStream_t))
#undef STUB
bool mfma_supported(const Shape& s, int dtype) { return dtype == 1 && s.D % 8 == 0 && s.D <= 128; }
bool adaln_supported(int C, int dtype) {
  const int per = dtype == 1 ? 8 : 4;
  return C % per == 0 && C / per <= 256;
}
int adaln_wgs(int, int T, bool, bool) { return T < 64 ? 1 : 16; }
bool linear_supported(int R, int K, int F, long long ldx, long long ldy, int dtype) {
  return dtype == 1 && R >= 1 && K % 32 == 0 && F % 32 == 0 && ldx % 8 == 0 && ldy % 8 == 0;
}
size_t linear_bwd_workspace_bytes(int, int K, int F) { return (size_t)4 * F * K * 4 + (size_t)64 * F * 4; }
}  // namespace tvm
