// Backward launchers, head dims up to 96 (see bwd_mfma_kernels.h for the kernels).
#include "bwd_mfma_kernels.h"

namespace tvm {

// d > 96 is instantiated in bwd_mfma_wide.hip (built with different code-generation flags)
hipError_t launch_bwd_col_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st);

bool mfma_supported(const Shape& s, int dtype) {
  // bf16, 16-byte chunks, and row pitches whose tile offsets fit the 32-bit lane offsets of the LDS loads
  return dtype == 1 && s.D % 8 == 0 && s.D <= 128 && s.sn < (1ll << 22);
}

#define TVM_DISPATCH_D(FN, WIDE)                  \
  switch ((s.D + 15) / 16 * 16) {                 \
    case 16: return FN<16, 32>(s, a, st);         \
    case 32: return FN<32, 32>(s, a, st);         \
    case 48: return FN<48, 64>(s, a, st);         \
    case 64: return FN<64, 64>(s, a, st);         \
    case 80: return FN<80, 96>(s, a, st);         \
    case 96: return FN<96, 96>(s, a, st);         \
    default: return WIDE(s, a, st);               \
  }

hipError_t launch_bwd_col_mfma(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (s.D <= 96) return launch_bwd_col_pipe(s, a, st);  // hand-scheduled variant (bwd_col_pipe.hip)
  return launch_bwd_col_mfma_wide(s, a, st);
}
hipError_t launch_bwd_row_mfma(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (s.D <= 96) return launch_bwd_row_pipe(s, a, st);  // hand-scheduled variant (bwd_row_pipe.hip)
  return launch_bwd_row_mfma_wide(s, a, st);
}

#if defined(TVM_PROFILE)
extern "C" int tvmattn_debug_read_prof(long long* out16) {
  return (int)hipMemcpyFromSymbol(out16, HIP_SYMBOL(g_prof), sizeof(long long) * 16);
}
#endif

}  // namespace tvm
