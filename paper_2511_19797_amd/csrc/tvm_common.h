// Shared device-side types for the tvmattn kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tvm {

typedef __bf16 bf16;

// Logical problem: M queries and N keys per (batch, head), head dim D.  Key-side tensors (k, v, tk, tv and their
// gradients) are [B,H,N,D] with element strides sb, sh, sn; query-side tensors (q, tq, o, to, gO, gTO, dq,
// dtq) are [B,H,M,D] with qsb, qsh, qsn; lse, stats and the workspace row vectors are [B,H,M] contiguous.
struct Shape {
  int B, H, N, D;
  float alpha;          // softmax scale actually used (already resolved from desc.scale)
  long long sb, sh, sn; // element strides, key side
  int M;                // queries (= N for self-attention)
  long long qsb, qsh, qsn;  // element strides, query side
};

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16* p) { return (float)*p; }
__device__ __forceinline__ void stf(float* p, float x) { *p = x; }
__device__ __forceinline__ void stf(bf16* p, float x) { *p = (bf16)x; }  // round-to-nearest-even

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Host-side launchers (defined in the kernel translation units; all return hipGetLastError()).
struct FwdArgs {
  const void *q, *k, *v, *tq, *tk, *tv;
  void *o, *to;
  float *lse, *stats;
  // forward with the query side's normalisation folded in (launch_fwd_mfma_qnorm only): q, tq are the rows before the
  // norm; the gain, eps, and where the normalised rows go
  const float* ngq = nullptr;
  float neps = 0.f;
  void *qn = nullptr, *tqn = nullptr;
};
struct BwdArgs {
  const void *q, *k, *v, *tq, *tk, *tv, *o, *to;
  const float *lse, *stats;
  const void *gO, *gTO;
  void *dq, *dk, *dv, *dtq, *dtk, *dtv;
  float *dsig;  // workspace: delta + Sigma_2 per row
  float *sig1;  // workspace: Sigma_1 per row
  float *lse2;  // workspace: lse in log2 units per row (written and read by the hand-scheduled kernels only)
  int mode;     // upstream gradients that exist: 0 both, 1 gO only (gTO null), 2 gTO only (gO null)
  // backward through the QK-norm in the epilogues (launch_bwd_*_pipe_qknorm only): the rows before the
  // normalisation, the gains, eps, and one partial gain-gradient row per workgroup of the two kernels
  const void *nq = nullptr, *ntq = nullptr, *nk = nullptr, *ntk = nullptr;
  const float *ngq = nullptr, *ngk = nullptr;
  float neps = 0.f;
  float *npart_q = nullptr, *npart_k = nullptr;
};

hipError_t launch_fwd_generic(const Shape& s, int dtype, const FwdArgs& a, hipStream_t st);
hipError_t launch_bwd_pre(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_col_generic(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_generic(const Shape& s, int dtype, const BwdArgs& a, hipStream_t st);

// bf16 matrix-core paths; `supported` says whether the shape is one they take.
bool mfma_supported(const Shape& s, int dtype);
hipError_t launch_fwd_mfma(const Shape& s, const FwdArgs& a, hipStream_t st);
hipError_t launch_fwd_mfma_qnorm(const Shape& s, const FwdArgs& a, hipStream_t st);
hipError_t launch_bwd_col_mfma(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_mfma(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_col_onesided(const Shape& s, const BwdArgs& a, hipStream_t st);  // a.mode 1 or 2, any head dim
hipError_t launch_bwd_row_onesided(const Shape& s, const BwdArgs& a, hipStream_t st);
hipError_t launch_bwd_row_pipe(const Shape& s, const BwdArgs& a, hipStream_t st);  // head dims up to 96
hipError_t launch_bwd_col_pipe(const Shape& s, const BwdArgs& a, hipStream_t st);  // head dims up to 96, after the former
hipError_t launch_bwd_row_pipe_qknorm(const Shape& s, const BwdArgs& a, hipStream_t st);  // the same two with the QK-norm's
hipError_t launch_bwd_col_pipe_qknorm(const Shape& s, const BwdArgs& a, hipStream_t st);  // backward in their epilogues
hipError_t launch_gain_grad_sum(const float* part_q, int rows_q, float* gg_q, const float* part_k, int rows_k, float* gg_k,
                                int D, hipStream_t st);  // adds partial gain-gradient rows in order (qknorm.hip)


// RMSNorm with gain as QK-norm, with tangent (qknorm.hip).  One side = the rows of q (and tq) or of k (and tk).
struct NormSide {
  const void *x, *tx;      // inputs [B,H,n,D]
  const float* g;          // gain [D]
  const void *gy, *gty;    // backward: upstream gradients of the normalised tensor and of its tangent
  void *y, *ty;            // forward: outputs; backward: gradients of x and tx
  float* part;             // backward: per-workgroup partial sums of the gain gradient [nwg][D]
  float* gg;               // backward: gain gradient [D]
  int n;                   // rows per (batch, head)
  long long sb, sh, sn;    // element strides
  int nwg;                 // workgroups that work on this side
};
struct NormArgs {
  NormSide side[2];
  int B, H, D;
  float eps;
};
constexpr int kNormRowsPerWg = 16;   // rows a workgroup works on at a time (16 lanes each)
constexpr int kNormMaxWg = 1024;     // workgroups per side at most (they stride over the rows; two sides fill the chip)
hipError_t launch_qknorm_fwd(const NormArgs& a, int dtype, hipStream_t st);
hipError_t launch_qknorm_bwd(const NormArgs& a, int dtype, hipStream_t st);


// Normalised adaptive-layer-norm modulation with tangent (adaln.hip).
struct AdalnArgs {
  const void *x, *tx, *gy, *gty;    // [B,T,C] dtype, contiguous (gy, gty: backward only)
  const void *gres = nullptr, *gtres = nullptr;  // backward, optional (both or neither): added to the gradients of x, tx
  const float *a, *ta, *b, *tb;     // [B,C] float32
  void *y, *ty;                     // forward: outputs; backward: gradients of x and tx
  float* part;                      // backward workspace [B][nwg][4][C]: per-workgroup sums over tokens
  float *ga, *gta, *gb, *gtb;       // backward: gradients of a, ta, b, tb
  int B, T, C, nwg;                 // nwg: workgroups per batch element
  float eps;
};
// Normalised gate of a residual branch: z = x + RMSNorm^-(c) o h with tangent, and its backward.
struct GateArgs {
  const void *x, *tx, *h, *th;      // [B,T,C] dtype, contiguous (x, tx: forward only)
  const void *gz, *gtz;             // backward: upstream gradients, [B,T,C] dtype
  const float *c, *tc;              // [B,C] float32
  void *z, *tz;                     // forward: outputs; backward: gradients of h and th
  float* part;                      // backward workspace [B][nwg][2][C]: per-workgroup sums over tokens
  float *gc, *gtc;                  // backward: gradients of c, tc
  int B, T, C, nwg;
  float eps;
};
hipError_t launch_gate_fwd(const GateArgs& a, int dtype, hipStream_t st);
hipError_t launch_gate_bwd(const GateArgs& a, int dtype, hipStream_t st);
bool adaln_supported(int C, int dtype);
// The MLP's activation with tangent (n elements per tensor, a whole number of 16-byte chunks).
hipError_t launch_gelu_fwd(long long n, int dtype, const void* u, const void* tu, void* a, void* ta, hipStream_t st);
hipError_t launch_gelu_bwd(long long n, int dtype, const void* u, const void* tu, const void* ga, const void* gta,
                           void* gu, void* gtu, hipStream_t st);
// Linear layer on a token and its tangent (linear.hip): bf16 only, K and F multiples of 32.
// ldx, ldy: row pitch in elements of the [R,K] tensors (x, tx, gx, gtx) and of the [R,F] tensors (y, ty, gy, gty).
bool linear_supported(int R, int K, int F, long long ldx, long long ldy, int dtype);
size_t linear_bwd_workspace_bytes(int R, int K, int F);
hipError_t launch_linear_fwd(int R, int K, int F, long long ldx, long long ldy, const void* x, const void* tx,
                             const void* w, const void* bias, void* y, void* ty, hipStream_t st);
hipError_t launch_linear_bwd(int R, int K, int F, long long ldx, long long ldy, const void* x, const void* tx,
                             const void* w, const void* gy, const void* gty, void* gx, void* gtx, void* gw, void* gbias,
                             void* workspace, hipStream_t st);
int adaln_wgs(int B, int T, bool backward, bool gate);  // workgroups per batch element of a token kernel
hipError_t launch_adaln_fwd(const AdalnArgs& a, int dtype, hipStream_t st);
hipError_t launch_adaln_bwd(const AdalnArgs& a, int dtype, hipStream_t st);

}  // namespace tvm
