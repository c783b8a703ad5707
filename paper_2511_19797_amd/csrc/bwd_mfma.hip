// Backward dispatch on the bf16 matrix cores: hand-scheduled kernels for head dims up to 96 with both
// upstream gradients (bwd_row_pipe.hip, bwd_col_pipe.hip) or with gTO alone (the same two sources built
// without the products of gO: bwd_*_pipe_tangent.hip); above 96 the hand-scheduled passes of bwd_pass.hip (one over
// the keys for the query side, two over the queries for the key side), or for short sequences the generic-order
// kernels (bwd_mfma_wide.hip); generic-order kernels for the query side with gTO alone above 96
// (bwd_mfma_onesided2.hip) and for calls with gO alone (bwd_mfma_onesided1.hip).
#include "tvm_common.h"

namespace tvm {

hipError_t launch_bwd_col_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_mfma_wide(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws);
hipError_t launch_bwd_col_pass(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_pass(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws);
hipError_t launch_bwd_col_pipe_tangent(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_pipe_tangent(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_col_onesided1(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_onesided1(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_col_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_onesided2(const Shape& s, const BwdArgs& a, hipStream_t st, bool pipe_ws);

bool mfma_supported(const Shape& s, int dtype) {
  // bf16, 16-byte chunks, and row pitches whose tile offsets fit the 32-bit lane offsets of the LDS loads
  return dtype == 1 && s.D % 8 == 0 && s.D <= 128 && s.sn < (1ll << 22) && s.qsn < (1ll << 22);
}

// Head dims above 96 with both gradients or with gTO alone: the key side runs as the two hand-scheduled passes unless
// there are so few queries (two tiles of 32 at most) that a second launch costs more than the passes save (measured:
// 64 queries 56 against 51 us, from 128 queries on the passes are ahead, 2.40 against 3.18 ms at 4096).  The query
// side runs as the hand-scheduled pass over the keys on the same terms (64 keys: 40 against 35 us,
// 128: the same, 256: 105 against 115 us, 4096: 1.43 against 1.80 ms); so does the query side of a call with gTO alone.
static bool key_side_in_two_passes(const Shape& s) { return s.D > 96 && s.M > 64; }
static bool query_side_as_pass(const Shape& s) { return s.D > 96 && s.N > 64; }

// The query-side kernel runs first in both families: it leaves the row scalars of Step 1 of
// App. C in the workspace for the key-side kernel (the hand-scheduled pair also lse in log2 units).
hipError_t launch_bwd_col_mfma(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (a.mode == 2 && s.D <= 96) return launch_bwd_col_pipe_tangent(s, a, st);
  if (a.mode == 2 && key_side_in_two_passes(s)) return launch_bwd_col_pass(s, a, st);
  if (a.mode != 0) return launch_bwd_col_onesided(s, a, st);
  if (s.D <= 96) return launch_bwd_col_pipe(s, a, st);
  return key_side_in_two_passes(s) ? launch_bwd_col_pass(s, a, st) : launch_bwd_col_mfma_wide(s, a, st);
}
hipError_t launch_bwd_row_mfma(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (a.mode == 2 && s.D <= 96) return launch_bwd_row_pipe_tangent(s, a, st);
  if (a.mode == 2 && query_side_as_pass(s)) return launch_bwd_row_pass(s, a, st, key_side_in_two_passes(s));
  if (a.mode != 0) return launch_bwd_row_onesided(s, a, st);
  if (s.D <= 96) return launch_bwd_row_pipe(s, a, st);
  // (either kernel leaves the row vectors in the workspace as the key side that follows reads them)
  return query_side_as_pass(s) ? launch_bwd_row_pass(s, a, st, key_side_in_two_passes(s))
                               : launch_bwd_row_mfma_wide(s, a, st, key_side_in_two_passes(s));
}
// One upstream gradient only (generic-order kernels that leave out what vanishes with the other).
hipError_t launch_bwd_col_onesided(const Shape& s, const BwdArgs& a, hipStream_t st) {
  return a.mode == 1 ? launch_bwd_col_onesided1(s, a, st) : launch_bwd_col_onesided2(s, a, st);
}
hipError_t launch_bwd_row_onesided(const Shape& s, const BwdArgs& a, hipStream_t st) {
  return a.mode == 1 ? launch_bwd_row_onesided1(s, a, st) : launch_bwd_row_onesided2(s, a, st, key_side_in_two_passes(s));
}

}  // namespace tvm
