/*
 * tvmattn -- fused multi-head softmax attention with a JVP tangent, and its
 * backward through both outputs, for AMD MI355X (gfx950).
 *
 * Operation (Terminal Velocity Matching, App. C "Flash Attention JVP with
 * Backward Pass"; eq. (sdpa), the "Background" paragraph and the equations
 * under "Step 1").  Per batch b and head h, with Q, tQ [M,D] (queries), K, V,
 * tK, tV [N,D] (keys; the paper's Background allows M != N, self-attention has
 * M = N) and alpha = scale:
 *
 *     z  = alpha Q K^T                       zt = alpha (tQ K^T + Q tK^T)
 *     P  = softmax_rows(z)                   lse_i   = log sum_j exp(z_ij)
 *     stats_i = sum_j P_ij zt_ij             (the paper's mu_i / l_i)
 *     O  = P V                               tO = (P o (zt - stats 1^T)) V + P tV
 *
 * tO is the directional derivative of O along (tQ,tK,tV).  No N x N matrix is
 * ever stored ("Caching softmax statistics": only lse and stats are kept).
 *
 * The backward returns the gradient of  <gO,O> + <gTO,tO>  with respect to all
 * six inputs (Steps 1-6 of App. C give the gTO part; the gO part is ordinary
 * attention backward; the library returns their sum).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device.  The
 *     caller owns every buffer; the library never allocates, frees or
 *     synchronises.  All work is enqueued on `hip_stream` (a hipStream_t cast
 *     to void*; NULL is the default stream).
 *   - Big tensors have element type `dtype` and innermost stride 1.  Key-side
 *     tensors (k, v, tk, tv and their gradients) have logical shape [B,H,N,D]
 *     and the element strides stride_b, stride_h, stride_n of the descriptor;
 *     query-side tensors (q, tq, o, to, gO, gTO, dq, dtq) have [B,H,M,D] and
 *     qstride_b, qstride_h, qstride_n.  All three strides of a side 0 means
 *     contiguous (for the query side with M = 0 or M = N: the key side's
 *     strides).  Base pointers must be 16-byte aligned and all strides
 *     multiples of 16 bytes.
 *   - Row vectors (lse, stats) are contiguous [B,H,M] float32.
 *   - Arithmetic: products of dtype elements accumulate in float32; softmax and
 *     all row statistics are float32; outputs are rounded once to dtype.
 *   - Return value: TVMATTN_OK (0) or a negative tvmattn_status.  Arguments are
 *     validated before the first launch: on INVALID_ARG, UNSUPPORTED or
 *     WORKSPACE_TOO_SMALL nothing has been enqueued.  No C++ exception crosses
 *     this boundary.
 *   - No output may overlap an input, another output or the workspace: checked element-exactly for tensors of
 *     one layout (slices of one fused buffer that interleave without sharing an element are fine), by address
 *     range otherwise.  Calls on the same stream are ordered; calls on different streams may overlap if their
 *     buffers are disjoint.  The library keeps no state between calls (tvmattn_jvp_bwd_static's scratch aside).
 */
#ifndef TVMATTN_H
#define TVMATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TVMATTN_F32 = 0,  /* float32 storage; float32 arithmetic */
  TVMATTN_BF16 = 1  /* bfloat16 storage; bf16 x bf16 -> float32 matrix-core products */
} tvmattn_dtype;

typedef enum {
  TVMATTN_OK = 0,
  TVMATTN_INVALID_ARG = -1,         /* null pointer, bad shape, misaligned pointer or stride */
  TVMATTN_UNSUPPORTED = -2,         /* dtype unknown, D > 256, sizes beyond 2^31 rows */
  TVMATTN_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < tvmattn_jvp_bwd_workspace_bytes() */
  TVMATTN_LAUNCH_FAILED = -4,       /* hipGetLastError() after a launch was not hipSuccess */
  TVMATTN_SCRATCH_TOO_SMALL = -5    /* tvmattn_jvp_bwd_static: more than TVMATTN_STATIC_MAX_ROWS query rows */
} tvmattn_status;

/* Per-call switches, OR-ed into tvmattn_desc.flags.  Unknown bits are TVMATTN_INVALID_ARG. */
enum {
  /* Diagnostic: serve this call with the plain-ALU kernels even where the matrix-core kernels would take it
   * (bf16 with D a multiple of 8 and D <= 128).  Both families compute the operation stated above. */
  TVMATTN_FLAG_PLAIN_ALU = 1
};

typedef struct {
  int32_t B;        /* batch                       >= 1 */
  int32_t H;        /* heads                       >= 1 */
  int32_t N;        /* keys (and queries, unless M is set)  >= 1 */
  int32_t D;        /* head dimension              1..256 */
  int32_t dtype;    /* tvmattn_dtype */
  float scale;      /* alpha; 0 selects 1/sqrt(D) (the true D, never a padded one) */
  int64_t stride_b; /* element strides of the key-side [B,H,N,D] tensors; all zero = contiguous */
  int64_t stride_h;
  int64_t stride_n;
  int32_t M;        /* queries; 0 = N (self-attention) */
  int32_t flags;    /* 0, or TVMATTN_FLAG_* bits */
  int64_t qstride_b; /* element strides of the query-side [B,H,M,D] tensors; all zero = contiguous, */
  int64_t qstride_h; /* or the key side's strides where M is 0 or N */
  int64_t qstride_n;
} tvmattn_desc;

/* Library version, major*10000 + minor*100 + patch. */
int tvmattn_version(void);

/* Static, never-NULL description of a status code. */
const char* tvmattn_strerror(int status);

/*
 * Forward with tangent (one online-softmax pass over the keys).
 *   in : q, tq            [B,H,M,D] dtype (query side)
 *        k, v, tk, tv     [B,H,N,D] dtype (key side)
 *   out: o, to            [B,H,M,D] dtype
 *        lse, stats       [B,H,M]   float32 (natural log of the row sum of exp(z); mu/l)
 * lse and stats may both be NULL: a forward whose backward will not be taken saves nothing
 * (the "detached" use of the tangent; one of the two alone is TVMATTN_INVALID_ARG).
 */
int tvmattn_jvp_fwd(const tvmattn_desc* desc,
                    const void* q, const void* k, const void* v,
                    const void* tq, const void* tk, const void* tv,
                    void* o, void* to, float* lse, float* stats,
                    void* hip_stream);

/* Bytes of device scratch tvmattn_jvp_bwd needs for this descriptor (0 on a bad descriptor). */
size_t tvmattn_jvp_bwd_workspace_bytes(const tvmattn_desc* desc);

/*
 * Backward through both outputs.
 *   in : q,k,v,tq,tk,tv   as given to the forward
 *        o,to,lse,stats   as written by the forward
 *        gO, gTO          [B,H,M,D] dtype, upstream gradients of o and to
 *   out: dq, dtq          [B,H,M,D] dtype;  dk, dv, dtk, dtv  [B,H,N,D] dtype; each element written exactly once
 *   workspace: device memory, 16-byte aligned, at least
 *        tvmattn_jvp_bwd_workspace_bytes(desc) bytes; contents need not be initialised
 *        and are undefined afterwards.
 * Launches on the stream: a query-side pass (dq,dtq; Steps 3,5) that also forms the row
 * scalars of Step 1 (delta = gO.O, Sigma_1 = gTO.O, Sigma_2 = gTO.tO per row; a separate
 * launch on the plain-ALU path), then a key-side pass (dk,dtk,dv,dtv; Steps 2,4,6).
 * No atomics: results are bitwise reproducible.
 *
 * One upstream gradient only (both NULL is TVMATTN_INVALID_ARG):
 *   gTO == NULL  the gradient of <gO, O> alone, i.e. the ordinary attention backward (the part
 *                the paper leaves to a standard kernel, App. C).  The tangent path drops out:
 *                tq, tk, tv, to and stats are not read, dtq, dtk, dtv are not written, and any of
 *                these eight may be NULL.
 *   gO == NULL   the gradient of <gTO, tO> alone (the paper's Steps 1-6 by themselves); all
 *                six outputs are written.
 * Both are served by kernels that leave out the products that vanish, not by zero-filled inputs.
 */
int tvmattn_jvp_bwd(const tvmattn_desc* desc,
                    const void* q, const void* k, const void* v,
                    const void* tq, const void* tk, const void* tv,
                    const void* o, const void* to, const float* lse, const float* stats,
                    const void* gO, const void* gTO,
                    void* dq, void* dk, void* dv, void* dtq, void* dtk, void* dtv,
                    void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/*
 * tvmattn_jvp_bwd with a timing hook, for benchmarks: `events` points to four hipEvent_t handles created by the
 * caller with timing enabled; the call records, on its stream, events[0] before its first launch, events[1] after
 * the row-scalar kernel (a separate launch only on the plain-ALU path), events[2] after the query-side kernel and
 * events[3] after the key-side kernel.  A NULL handle among the four skips that record; events == NULL is
 * tvmattn_jvp_bwd itself.  Nothing is kept between calls.
 */
int tvmattn_jvp_bwd_timed(const tvmattn_desc* desc,
                          const void* q, const void* k, const void* v,
                          const void* tq, const void* tk, const void* tv,
                          const void* o, const void* to, const float* lse, const float* stats,
                          const void* gO, const void* gTO,
                          void* dq, void* dk, void* dv, void* dtq, void* dtk, void* dtv,
                          void* workspace, size_t workspace_bytes,
                          void* const* events, void* hip_stream);

/*
 * tvmattn_jvp_bwd for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same
 * kernels, same results bit for bit.  The three float32 row vectors that the workspace otherwise holds live in a
 * static device array of 3 * TVMATTN_STATIC_MAX_ROWS floats (12 MiB on every GPU the library runs on, held until
 * the process ends).  The call allocates nothing and frees nothing.
 *   - B*H*M (query rows) above TVMATTN_STATIC_MAX_ROWS: TVMATTN_SCRATCH_TOO_SMALL, nothing enqueued.
 *   - The device that is current at the call must be the one hip_stream belongs to; each GPU has its own array.
 *   - Every call on a GPU shares that GPU's array: calls that may overlap in time on one GPU (different streams,
 *     or different host threads without an order between their streams) race on it.  Calls on one stream are safe.
 *   - Nothing in the array has to start at zero and nothing of a previous call is read: every entry a call reads
 *     it has written before.
 */
#define TVMATTN_STATIC_MAX_ROWS (1 << 20)
int tvmattn_jvp_bwd_static(const tvmattn_desc* desc,
                           const void* q, const void* k, const void* v,
                           const void* tq, const void* tk, const void* tv,
                           const void* o, const void* to, const float* lse, const float* stats,
                           const void* gO, const void* gTO,
                           void* dq, void* dk, void* dv, void* dtq, void* dtk, void* dtv,
                           void* hip_stream);

/*
 * RMSNorm with a learnable gain as QK-norm, with tangent: the operation that normalises queries and keys
 * right before attention in the paper's network (Sec. "Semi-Lipschitz control"; definition and Jacobian in
 * App. "Lipschitzness of RMSNorm").  Per row x of q or of k (D elements), with its tangent tx:
 *
 *     r = 1 / sqrt( (1/D) sum_i x_i^2 + eps )        (the mean of squares: what the printed Jacobian belongs to)
 *     y = g o x r                                    ty = g o ( tx r - x r^3 (1/D) sum_i x_i tx_i )
 *
 * ty is the directional derivative of y along tx; the gain g has no tangent.  One launch normalises both sides.
 *   in : q, tq            [B,H,M,D] dtype, query-side strides of the descriptor
 *        k, tk            [B,H,N,D] dtype, key-side strides
 *        gain_q, gain_k   [D] float32, contiguous, shared by all batches and heads
 *        eps              >= 0, finite
 *   out: qn, tqn, kn, tkn like their inputs; these are what tvmattn_jvp_fwd takes as q, tq, k, tk
 * desc->scale is not used.  Arithmetic is float32; outputs are rounded once to dtype.
 */
int tvmattn_qknorm_jvp_fwd(const tvmattn_desc* desc,
                           const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps,
                           void* qn, void* tqn, void* kn, void* tkn,
                           void* hip_stream);

/* Bytes of device scratch tvmattn_qknorm_jvp_bwd needs for this descriptor (0 on a bad descriptor). */
size_t tvmattn_qknorm_jvp_bwd_workspace_bytes(const tvmattn_desc* desc);

/*
 * Backward of the above: the gradient of  <gqn,qn> + <gtqn,tqn> + <gkn,kn> + <gtkn,tkn>.
 *   in : q, tq, k, tk, gain_q, gain_k, eps   as given to the forward (nothing is saved: r is recomputed)
 *        gqn, gtqn, gkn, gtkn                upstream gradients, like qn, tqn, kn, tkn (the dq, dtq, dk, dtk that
 *                                            tvmattn_jvp_bwd returns)
 *   out: dq, dtq, dk, dtk                    like q, tq, k, tk
 *        dgain_q, dgain_k                    [D] float32, summed over all rows of their side
 *   workspace: device memory, 16-byte aligned, at least tvmattn_qknorm_jvp_bwd_workspace_bytes(desc) bytes;
 *        contents need not be initialised and are undefined afterwards.
 * Two launches (rows, then the sum of per-workgroup partial gain gradients in a fixed order).  No atomics:
 * results are bitwise reproducible.
 */
int tvmattn_qknorm_jvp_bwd(const tvmattn_desc* desc,
                           const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps,
                           const void* gqn, const void* gtqn, const void* gkn, const void* gtkn,
                           void* dq, void* dtq, void* dk, void* dtk, float* dgain_q, float* dgain_k,
                           void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * tvmattn_qknorm_jvp_fwd and tvmattn_jvp_fwd in one call (Sec. "Semi-Lipschitz control": RMSNorm with a learnable
 * gain on q and k right before the attention; App. C for the attention and its tangent).  The key side goes through
 * the normalisation kernel; the query side is normalised inside the attention forward, where each wave loads its
 * query rows as fragments, so the forward reads the rows as they were before the norm and the normalised query rows
 * are only written, not read back.
 *   in : q, tq, k, tk, gain_q, gain_k, eps   as for tvmattn_qknorm_jvp_fwd
 *        v, tv                               as for tvmattn_jvp_fwd
 *   out: qn, tqn, kn, tkn                    the normalised rows and their tangents (the backward needs them:
 *                                            give them to tvmattn_jvp_bwd_qknorm or tvmattn_jvp_bwd)
 *        o, to, lse, stats                   as from tvmattn_jvp_fwd on (qn, kn, v, tqn, tkn, tv); lse and stats both
 *                                            NULL: nothing is saved
 * The normalised rows are rounded to dtype before the products use them, as when the two calls are made one after
 * the other; the results agree with those to rounding (the order of the float32 operations differs).
 * Served by the matrix-core forward only: bfloat16, D a multiple of 8, D <= 128; anything else returns
 * TVMATTN_UNSUPPORTED: make the two calls there.  Two launches, no workspace.
 */
int tvmattn_jvp_fwd_qknorm(const tvmattn_desc* desc,
                           const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps,
                           const void* v, const void* tv,
                           void* qn, void* tqn, void* kn, void* tkn,
                           void* o, void* to, float* lse, float* stats,
                           void* hip_stream);

/*
 * tvmattn_jvp_bwd and tvmattn_qknorm_jvp_bwd in one call, for attention whose q, tq, k, tk came out of
 * tvmattn_qknorm_jvp_fwd: the backward of the normalisation runs in the epilogues of the attention's two
 * backward kernels (each has the rows of one side in registers when it ends), so the gradients with respect to the
 * normalised tensors never reach device memory.
 *   in : q, tq, k, tk, gain_q, gain_k, eps   as given to tvmattn_qknorm_jvp_fwd
 *        qn, tqn, kn, tkn                    as it wrote them (and as given to tvmattn_jvp_fwd as q, tq, k, tk)
 *        v, tv, o, to, lse, stats, gO, gTO   as for tvmattn_jvp_bwd; both upstream gradients are required
 *   out: dq, dtq, dk, dtk                    gradients with respect to q, tq, k, tk (before the normalisation)
 *        dv, dtv                             as from tvmattn_jvp_bwd
 *        dgain_q, dgain_k                    [D] float32
 *   workspace: device memory, 16-byte aligned, at least tvmattn_jvp_bwd_qknorm_workspace_bytes(desc) bytes.
 * Served by the hand-scheduled kernels only: bfloat16, D a multiple of 8, D <= 96; anything else returns
 * TVMATTN_UNSUPPORTED (and the size query 0): call tvmattn_jvp_bwd and tvmattn_qknorm_jvp_bwd one after the other
 * there.  Three launches (query side, key side, the ordered sum of per-workgroup gain-gradient rows); no atomics.
 * The gradients with respect to the normalised rows are rounded to dtype between the two steps, as they are when
 * the two calls are made separately.
 */
size_t tvmattn_jvp_bwd_qknorm_workspace_bytes(const tvmattn_desc* desc);
int tvmattn_jvp_bwd_qknorm(const tvmattn_desc* desc,
                           const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps,
                           const void* qn, const void* tqn, const void* kn, const void* tkn,
                           const void* v, const void* tv,
                           const void* o, const void* to, const float* lse, const float* stats,
                           const void* gO, const void* gTO,
                           void* dq, void* dk, void* dv, void* dtq, void* dtk, void* dtv,
                           float* dgain_q, float* dgain_k,
                           void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Normalised adaptive-layer-norm modulation with tangent: the operand of ATTN and of MLP in the paper's block
 * (Sec. "Semi-Lipschitz control", the equation for AdaLN(x, t); App. "Full Description of Normalization of
 * Modulation").  With RMSNorm^- the RMSNorm without learnable parameters (v / sqrt(mean(v^2) + eps) over the C
 * entries of a vector v):
 *
 *     y  = RMSNorm^-(x) o RMSNorm^-(a) + RMSNorm^-(b)
 *     ty = its directional derivative along (tx, ta, tb)
 *
 *   in : x, tx           [B,T,C] dtype, contiguous: a token's features and their tangent
 *        a, ta, b, tb    [B,C] float32, contiguous: scale and shift of the token's batch element, and tangents
 *        eps             >= 0, finite
 *   out: y, ty           [B,T,C] dtype
 * C must be a multiple of 16 bytes' worth of elements and at most 256 such chunks (2048 for bfloat16, 1024 for
 * float32), B at most 65535; otherwise TVMATTN_UNSUPPORTED.  One launch, no workspace.  Arithmetic is float32.
 */
int tvmattn_adaln_jvp_fwd(int B, int T, int C, int dtype,
                          const void* x, const void* tx,
                          const float* a, const float* ta, const float* b, const float* tb, float eps,
                          void* y, void* ty, void* hip_stream);

/*
 * Backward of the above: the gradient of <gy,y> + <gty,ty> with respect to all six inputs.
 *   in : x, tx, a, ta, b, tb, eps as given to the forward (nothing is saved); gy, gty [B,T,C] dtype
 *   out: gx, gtx [B,T,C] dtype; ga, gta, gb, gtb [B,C] float32 (summed over the T tokens of their batch element)
 *   workspace: device memory, 16-byte aligned, at least tvmattn_adaln_jvp_bwd_workspace_bytes(...) bytes
 *              (0 = unsupported shape).
 * Two launches; the sums over tokens use no atomics and are bitwise reproducible.
 */
size_t tvmattn_adaln_jvp_bwd_workspace_bytes(int B, int T, int C, int dtype);
int tvmattn_adaln_jvp_bwd(int B, int T, int C, int dtype,
                          const void* x, const void* tx,
                          const float* a, const float* ta, const float* b, const float* tb, float eps,
                          const void* gy, const void* gty,
                          void* gx, void* gtx, float* ga, float* gta, float* gb, float* gtb,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same with the gradients that reach x and tx by another way added on the way out: in the block, x feeds the
 * modulation and also runs on along the residual connection, so its gradient is the stream's (gres, gtres) plus the
 * modulation's.  gres, gtres: [B,T,C] dtype, both given or both NULL (NULL: the call above); gx may not alias them.
 * Saves the pass over six tensors that a separate addition would take.
 */
int tvmattn_adaln_jvp_bwd_residual(int B, int T, int C, int dtype,
                                   const void* x, const void* tx,
                                   const float* a, const float* ta, const float* b, const float* tb, float eps,
                                   const void* gy, const void* gty, const void* gres, const void* gtres,
                                   void* gx, void* gtx, float* ga, float* gta, float* gb, float* gtb,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Normalised gate of a residual branch with tangent: how the output h of ATTN or of MLP re-enters the residual
 * stream in the paper's block (App. "Full Description of Normalization of Modulation", the two layer equations):
 *
 *     z  = x + RMSNorm^-(c) o h
 *     tz = its directional derivative along (tx, th, tc)
 *
 *   in : x, tx, h, th    [B,T,C] dtype, contiguous: the stream, the branch output, and their tangents
 *        c, tc           [B,C] float32, contiguous: the gate of the token's batch element and its tangent
 *        eps             >= 0, finite
 *   out: z, tz           [B,T,C] dtype; z may be x itself and tz may be tx itself (the stream updated in place);
 *                        no other aliasing of an input
 * Shape limits as for tvmattn_adaln_jvp_fwd.  One launch, no workspace.  Arithmetic is float32.
 */
int tvmattn_gate_jvp_fwd(int B, int T, int C, int dtype,
                         const void* x, const void* tx, const void* h, const void* th,
                         const float* c, const float* tc, float eps,
                         void* z, void* tz, void* hip_stream);

/*
 * Backward of the above: the gradient of <gz,z> + <gtz,tz>.  The gradients with respect to x and tx are gz and gtz
 * themselves and are not written.
 *   in : h, th, c, tc, eps as given to the forward (nothing is saved); gz, gtz [B,T,C] dtype
 *   out: gh, gth [B,T,C] dtype; gc, gtc [B,C] float32 (summed over the T tokens of their batch element)
 *   workspace: device memory, 16-byte aligned, at least tvmattn_gate_jvp_bwd_workspace_bytes(...) bytes
 *              (0 = unsupported shape).
 * Two launches; the sums over tokens use no atomics and are bitwise reproducible.
 */
size_t tvmattn_gate_jvp_bwd_workspace_bytes(int B, int T, int C, int dtype);
int tvmattn_gate_jvp_bwd(int B, int T, int C, int dtype,
                         const void* h, const void* th, const float* c, const float* tc, float eps,
                         const void* gz, const void* gtz,
                         void* gh, void* gth, float* gc, float* gtc,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The activation between the MLP's two linear layers, with tangent (the MLP branch of the paper's block, App. "Full
 * Description of Normalization of Modulation"; the JVP of Sec. 4 runs through it).  The paper does not name the
 * activation: DiT's is taken, the GELU in its tanh form, gelu(u) = u/2 (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3))):
 *
 *     a = gelu(u),   ta = gelu'(u) tu          (pointwise; the linear layers around it are plain matrix products)
 *
 *   in : u, tu   n elements of dtype each, contiguous, 16-byte aligned; n a whole number of 16-byte chunks
 *   out: a, ta   likewise; must not alias an input
 * One launch, no workspace.  Arithmetic is float32.
 */
int tvmattn_gelu_jvp_fwd(long long n, int dtype, const void* u, const void* tu, void* a, void* ta, void* hip_stream);

/*
 * Backward of the above: the gradient of <ga,a> + <gta,ta>:  gu = ga gelu'(u) + gta tu gelu''(u),  gtu = gta gelu'(u).
 *   in : u, tu as given to the forward (nothing is saved); ga, gta n elements of dtype
 *   out: gu, gtu
 */
int tvmattn_gelu_jvp_bwd(long long n, int dtype, const void* u, const void* tu, const void* ga, const void* gta,
                         void* gu, void* gtu, void* hip_stream);

/*
 * A linear layer applied to a token and to its tangent: the query/key/value and output projections around the
 * attention and the two layers of the MLP in the paper's block (App. "Full Description of Normalization of
 * Modulation", the two layer equations; the JVP of Sec. 4 runs through them along the network's inputs, so the
 * weights carry no tangent):
 *
 *     y = x W^T + b,   ty = tx W^T
 *
 *   in : x, tx   [R,K] dtype: R tokens of K features, rows ldx elements apart (0 = K: dense)
 *        w       [F,K] dtype, contiguous (row f holds the weights of output feature f)
 *        bias    [F] dtype, or NULL
 *   out: y, ty   [R,F] dtype, rows ldy elements apart (0 = F: dense)
 * Row pitches let a layer read from or write into a slice of a wider buffer (the q, k, v slices of a fused projection,
 * an attention output laid out like its queries) without a copy; they must be multiples of 8 elements.
 * Served for bfloat16 with K and F multiples of 32 (products on the matrix cores, float32 accumulation, outputs
 * rounded once); anything else returns TVMATTN_UNSUPPORTED.  One launch over the stacked rows [x; tx], no workspace.
 */
int tvmattn_linear_jvp_fwd(int R, int K, int F, int dtype,
                           const void* x, const void* tx, long long ldx, const void* w, const void* bias,
                           void* y, void* ty, long long ldy, void* hip_stream);

/*
 * Backward of the above: the gradient of <gy,y> + <gty,ty>:
 *     gx = gy W,   gtx = gty W,   gw = gy^T x + gty^T tx,   gbias = sum over the R tokens of gy.
 *   in : x, tx (pitch ldx), w as given to the forward; gy, gty [R,F] dtype (pitch ldy)
 *   out: gx, gtx [R,K] dtype (pitch ldx); gw [F,K] dtype, contiguous; gbias [F] dtype or NULL (not wanted)
 *   workspace: device memory, 16-byte aligned, at least tvmattn_linear_jvp_bwd_workspace_bytes(...) bytes (0 =
 *              unsupported shape): float32 partial sums of gw over ranges of tokens, and of gbias.
 * Launches: gx and gtx in one; gw as partial sums over token ranges and their sum in a fixed order (no atomics,
 * bitwise reproducible); gbias likewise.
 */
size_t tvmattn_linear_jvp_bwd_workspace_bytes(int R, int K, int F, int dtype);
int tvmattn_linear_jvp_bwd(int R, int K, int F, int dtype,
                           const void* x, const void* tx, long long ldx, const void* w,
                           const void* gy, const void* gty, long long ldy,
                           void* gx, void* gtx, void* gw, void* gbias,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TVMATTN_H */
