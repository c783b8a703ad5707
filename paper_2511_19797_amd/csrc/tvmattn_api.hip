// C-ABI entry points: argument validation and dispatch.  No allocation, no synchronisation.
#include "../../include/tvmattn.h"

#include <math.h>

#include "tvm_common.h"

namespace {

int g_path = 0;  // 0 = choose per shape, 1 = plain-ALU kernels only (diagnostic)
hipEvent_t g_ev[4];
bool g_ev_on = false;

inline void mark(int i, hipStream_t st) {
  if (g_ev_on && g_ev[i]) (void)hipEventRecord(g_ev[i], st);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One side's strides: all zero selects `dflt_*`; otherwise row pitch >= D and 16-byte multiples.
bool side_strides(long long esz, int D, long long& sb, long long& sh, long long& sn, long long dflt_b, long long dflt_h,
                  long long dflt_n) {
  if (sb == 0 && sh == 0 && sn == 0) {
    sb = dflt_b;
    sh = dflt_h;
    sn = dflt_n;
  }
  if (sn < D || sh < 1 || sb < 1) return false;
  return (sn * esz) % 16 == 0 && (sh * esz) % 16 == 0 && (sb * esz) % 16 == 0;
}

// Validates the descriptor and resolves sizes, strides and scale.
int resolve(const tvmattn_desc* d, tvm::Shape* s) {
  if (!d) return TVMATTN_INVALID_ARG;
  if (d->B < 1 || d->H < 1 || d->N < 1 || d->D < 1 || d->M < 0 || d->reserved != 0) return TVMATTN_INVALID_ARG;
  if (d->dtype != TVMATTN_F32 && d->dtype != TVMATTN_BF16) return TVMATTN_UNSUPPORTED;
  if (d->D > 256) return TVMATTN_UNSUPPORTED;
  if (!(d->scale >= 0.f) || isinf(d->scale)) return TVMATTN_INVALID_ARG;
  const long long esz = d->dtype == TVMATTN_F32 ? 4 : 2;
  const int M = d->M ? d->M : d->N;
  long long sb = d->stride_b, sh = d->stride_h, sn = d->stride_n;
  if (!side_strides(esz, d->D, sb, sh, sn, (long long)d->N * d->D * d->H, (long long)d->N * d->D, d->D))
    return TVMATTN_INVALID_ARG;
  long long qsb = d->qstride_b, qsh = d->qstride_h, qsn = d->qstride_n;
  const bool same = M == d->N;  // self-attention: the query side defaults to the key side's layout
  if (!side_strides(esz, d->D, qsb, qsh, qsn, same ? sb : (long long)M * d->D * d->H, same ? sh : (long long)M * d->D,
                    same ? sn : d->D))
    return TVMATTN_INVALID_ARG;
  if ((long long)d->B * d->H * d->N >= (1ll << 31) || (long long)d->B * d->H * M >= (1ll << 31)) return TVMATTN_UNSUPPORTED;
  s->B = d->B;
  s->H = d->H;
  s->N = d->N;
  s->D = d->D;
  s->alpha = d->scale == 0.f ? 1.0f / sqrtf((float)d->D) : d->scale;
  s->sb = sb;
  s->sh = sh;
  s->sn = sn;
  s->M = M;
  s->qsb = qsb;
  s->qsh = qsh;
  s->qsn = qsn;
  return TVMATTN_OK;
}

// Every listed pointer must be non-null and 16-byte aligned, no output may be an input or another
// output.  Entries that the call's mode does not use are passed as `skip` (a null there is fine,
// and the pointer takes no part in the aliasing check).
const void* const skip = reinterpret_cast<const void*>(uintptr_t(1));
template <size_t NI, size_t NO>
int check_ptrs(const void* const (&in)[NI], void* const (&out)[NO]) {
  for (size_t i = 0; i < NI; ++i)
    if (in[i] != skip && (!in[i] || !aligned16(in[i]))) return TVMATTN_INVALID_ARG;
  for (size_t o = 0; o < NO; ++o) {
    if (out[o] == skip) continue;
    if (!out[o] || !aligned16(out[o])) return TVMATTN_INVALID_ARG;
    for (size_t i = 0; i < NI; ++i)
      if (out[o] == in[i]) return TVMATTN_INVALID_ARG;
    for (size_t p = 0; p < o; ++p)
      if (out[o] == out[p]) return TVMATTN_INVALID_ARG;
  }
  return TVMATTN_OK;
}
inline const void* unless(bool unused, const void* p) { return unused ? skip : p; }
inline void* unless(bool unused, void* p) { return unused ? const_cast<void*>(skip) : p; }

}  // namespace

extern "C" {

int tvmattn_version(void) { return 500; }  // 0.5.0: AdaLN modulation, residual gate, MLP activation; 0.4.0: QK-norm entry points; 0.3.0: M != N (the descriptor grew); 0.2.0: one-sided backward, forward that saves nothing

const char* tvmattn_strerror(int status) {
  switch (status) {
    case TVMATTN_OK: return "ok";
    case TVMATTN_INVALID_ARG: return "invalid argument (null/misaligned pointer, bad shape, stride or scale, or aliasing)";
    case TVMATTN_UNSUPPORTED: return "unsupported (dtype, head dimension > 256, or too many rows)";
    case TVMATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TVMATTN_LAUNCH_FAILED: return "kernel launch failed";
    default: return "unknown status";
  }
}

int tvmattn_set_path(int path) {
  if (path != 0 && path != 1) return TVMATTN_INVALID_ARG;
  g_path = path;
  return TVMATTN_OK;
}

int tvmattn_set_bwd_events(void* const* events) {
  g_ev_on = events != nullptr;
  if (events)
    for (int i = 0; i < 4; ++i) g_ev[i] = static_cast<hipEvent_t>(events[i]);  // NULL: that record is skipped
  return TVMATTN_OK;
}

int tvmattn_jvp_fwd(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                    const void* tk, const void* tv, void* o, void* to, float* lse, float* stats, void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if ((lse == nullptr) != (stats == nullptr)) return TVMATTN_INVALID_ARG;  // saved together or not at all
  const bool nosave = lse == nullptr;
  const void* const in[] = {q, k, v, tq, tk, tv};
  void* const out[] = {o, to, unless(nosave, (void*)lse), unless(nosave, (void*)stats)};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  tvm::FwdArgs a{q, k, v, tq, tk, tv, o, to, lse, stats};
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (g_path == 0 && tvm::mfma_supported(s, desc->dtype))
    e = tvm::launch_fwd_mfma(s, a, st);
  else
    e = tvm::launch_fwd_generic(s, desc->dtype, a, st);
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}

size_t tvmattn_jvp_bwd_workspace_bytes(const tvmattn_desc* desc) {
  tvm::Shape s;
  if (resolve(desc, &s)) return 0;
  // three float32 row vectors (delta + Sigma_2, Sigma_1, lse in log2 units), one entry per query row, each
  // padded to a 256-byte multiple
  const size_t rows = (size_t)s.B * s.H * s.M;
  const size_t one = (rows * sizeof(float) + 255) & ~(size_t)255;
  return 3 * one;
}

int tvmattn_jvp_bwd(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                    const void* tk, const void* tv, const void* o, const void* to, const float* lse,
                    const float* stats, const void* gO, const void* gTO, void* dq, void* dk, void* dv, void* dtq,
                    void* dtk, void* dtv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if (!gO && !gTO) return TVMATTN_INVALID_ARG;
  // one upstream gradient only: 1 = gO (the tangent inputs and outputs take no part), 2 = gTO
  const int mode = !gTO ? 1 : !gO ? 2 : 0;
  const bool m1 = mode == 1;
  const void* const in[] = {q, k, v, unless(m1, tq), unless(m1, tk), unless(m1, tv), o, unless(m1, to), lse,
                            unless(m1, (const void*)stats), unless(mode == 2, gO), unless(m1, gTO)};
  void* const out[] = {dq, dk, dv, unless(m1, dtq), unless(m1, dtk), unless(m1, dtv), workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  const size_t need = tvmattn_jvp_bwd_workspace_bytes(desc);
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::BwdArgs a{q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv,
                 static_cast<float*>(workspace),
                 reinterpret_cast<float*>(static_cast<char*>(workspace) + need / 3),
                 reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * (need / 3)), mode};
  if (m1) {  // not read, not written: whatever was passed
    a.tq = a.tk = a.tv = a.to = nullptr;
    a.stats = nullptr;
    a.dtq = a.dtk = a.dtv = nullptr;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const bool mf = g_path == 0 && tvm::mfma_supported(s, desc->dtype);
  hipError_t e = hipSuccess;
  mark(0, st);
  if (!mf) e = tvm::launch_bwd_pre(s, desc->dtype, a, st);  // the matrix-core query-side kernel does Step 1 itself
  if (e != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  mark(1, st);
  e = mf ? tvm::launch_bwd_row_mfma(s, a, st) : tvm::launch_bwd_row_generic(s, desc->dtype, a, st);
  if (e != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  mark(2, st);
  e = mf ? tvm::launch_bwd_col_mfma(s, a, st) : tvm::launch_bwd_col_generic(s, desc->dtype, a, st);
  mark(3, st);
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}

// ---- RMSNorm with gain as QK-norm, with tangent
namespace {
int norm_wgs(long long rows) {
  const long long w = (rows + tvm::kNormRowsPerWg - 1) / tvm::kNormRowsPerWg;
  return (int)(w < tvm::kNormMaxWg ? w : tvm::kNormMaxWg);
}
void norm_sides(const tvm::Shape& s, tvm::NormArgs* a, float eps) {
  a->B = s.B;
  a->H = s.H;
  a->D = s.D;
  a->eps = eps;
  a->side[0].n = s.M;
  a->side[0].sb = s.qsb;
  a->side[0].sh = s.qsh;
  a->side[0].sn = s.qsn;
  a->side[1].n = s.N;
  a->side[1].sb = s.sb;
  a->side[1].sh = s.sh;
  a->side[1].sn = s.sn;
  for (int i = 0; i < 2; ++i) a->side[i].nwg = norm_wgs((long long)s.B * s.H * a->side[i].n);
}
size_t norm_part_bytes(const tvm::NormArgs& a, int side) {  // padded to a 256-byte multiple
  return ((size_t)a.side[side].nwg * a.D * sizeof(float) + 255) & ~(size_t)255;
}
}  // namespace

int tvmattn_qknorm_jvp_fwd(const tvmattn_desc* desc, const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps, void* qn, void* tqn, void* kn,
                           void* tkn, void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if (!(eps >= 0.f) || isinf(eps)) return TVMATTN_INVALID_ARG;
  const void* const in[] = {q, tq, k, tk, gain_q, gain_k};
  void* const out[] = {qn, tqn, kn, tkn};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  tvm::NormArgs a{};
  norm_sides(s, &a, eps);
  a.side[0].x = q;
  a.side[0].tx = tq;
  a.side[0].g = gain_q;
  a.side[0].y = qn;
  a.side[0].ty = tqn;
  a.side[1].x = k;
  a.side[1].tx = tk;
  a.side[1].g = gain_k;
  a.side[1].y = kn;
  a.side[1].ty = tkn;
  const hipError_t e = tvm::launch_qknorm_fwd(a, desc->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}

size_t tvmattn_qknorm_jvp_bwd_workspace_bytes(const tvmattn_desc* desc) {
  tvm::Shape s;
  if (resolve(desc, &s)) return 0;
  tvm::NormArgs a{};
  norm_sides(s, &a, 0.f);
  return norm_part_bytes(a, 0) + norm_part_bytes(a, 1);  // one partial gain-gradient row per workgroup and side
}

int tvmattn_qknorm_jvp_bwd(const tvmattn_desc* desc, const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps, const void* gqn, const void* gtqn,
                           const void* gkn, const void* gtkn, void* dq, void* dtq, void* dk, void* dtk,
                           float* dgain_q, float* dgain_k, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if (!(eps >= 0.f) || isinf(eps)) return TVMATTN_INVALID_ARG;
  const void* const in[] = {q, tq, k, tk, gain_q, gain_k, gqn, gtqn, gkn, gtkn};
  void* const out[] = {dq, dtq, dk, dtk, dgain_q, dgain_k, workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  if (workspace_bytes < tvmattn_qknorm_jvp_bwd_workspace_bytes(desc)) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::NormArgs a{};
  norm_sides(s, &a, eps);
  a.side[0].x = q;
  a.side[0].tx = tq;
  a.side[0].g = gain_q;
  a.side[0].gy = gqn;
  a.side[0].gty = gtqn;
  a.side[0].y = dq;
  a.side[0].ty = dtq;
  a.side[0].gg = dgain_q;
  a.side[0].part = static_cast<float*>(workspace);
  a.side[1].x = k;
  a.side[1].tx = tk;
  a.side[1].g = gain_k;
  a.side[1].gy = gkn;
  a.side[1].gty = gtkn;
  a.side[1].y = dk;
  a.side[1].ty = dtk;
  a.side[1].gg = dgain_k;
  a.side[1].part = reinterpret_cast<float*>(static_cast<char*>(workspace) + norm_part_bytes(a, 0));
  const hipError_t e = tvm::launch_qknorm_bwd(a, desc->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}

// ---- attention backward with the QK-norm's backward in the kernels' epilogues
namespace {
size_t pad256(size_t n) { return (n + 255) & ~(size_t)255; }
size_t fused_part_bytes(const tvm::Shape& s, bool query_side) {  // one float32 row of D per workgroup (128 rows of a head)
  const size_t blocks = (size_t)(((query_side ? s.M : s.N) + 127) / 128) * s.B * s.H;
  return pad256(blocks * s.D * sizeof(float));
}
bool fused_supported(const tvm::Shape& s, int dtype) {
  return g_path == 0 && tvm::mfma_supported(s, dtype) && s.D <= 96;
}
}  // namespace

size_t tvmattn_jvp_bwd_qknorm_workspace_bytes(const tvmattn_desc* desc) {
  tvm::Shape s;
  if (resolve(desc, &s) || !fused_supported(s, desc->dtype)) return 0;
  return tvmattn_jvp_bwd_workspace_bytes(desc) + fused_part_bytes(s, true) + fused_part_bytes(s, false);
}

int tvmattn_jvp_bwd_qknorm(const tvmattn_desc* desc, const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps, const void* qn, const void* tqn,
                           const void* kn, const void* tkn, const void* v, const void* tv, const void* o, const void* to,
                           const float* lse, const float* stats, const void* gO, const void* gTO, void* dq, void* dk,
                           void* dv, void* dtq, void* dtk, void* dtv, float* dgain_q, float* dgain_k, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if (!(eps >= 0.f) || isinf(eps)) return TVMATTN_INVALID_ARG;
  const void* const in[] = {q, tq, k, tk, gain_q, gain_k, qn, tqn, kn, tkn, v, tv, o, to, lse, stats, gO, gTO};
  void* const out[] = {dq, dk, dv, dtq, dtk, dtv, dgain_q, dgain_k, workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  if (!fused_supported(s, desc->dtype)) return TVMATTN_UNSUPPORTED;
  if (workspace_bytes < tvmattn_jvp_bwd_qknorm_workspace_bytes(desc)) return TVMATTN_WORKSPACE_TOO_SMALL;
  const size_t need0 = tvmattn_jvp_bwd_workspace_bytes(desc);
  char* const ws = static_cast<char*>(workspace);
  tvm::BwdArgs a{qn, kn, v, tqn, tkn, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv,
                 reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws + need0 / 3),
                 reinterpret_cast<float*>(ws + 2 * (need0 / 3)), 0};
  a.nq = q;
  a.ntq = tq;
  a.nk = k;
  a.ntk = tk;
  a.ngq = gain_q;
  a.ngk = gain_k;
  a.neps = eps;
  a.npart_q = reinterpret_cast<float*>(ws + need0);
  a.npart_k = reinterpret_cast<float*>(ws + need0 + fused_part_bytes(s, true));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (tvm::launch_bwd_row_pipe_qknorm(s, a, st) != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  if (tvm::launch_bwd_col_pipe_qknorm(s, a, st) != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  const int rows_q = ((s.M + 127) / 128) * s.B * s.H, rows_k = ((s.N + 127) / 128) * s.B * s.H;
  const hipError_t e = tvm::launch_gain_grad_sum(a.npart_q, rows_q, dgain_q, a.npart_k, rows_k, dgain_k, s.D, st);
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}

// ---- normalised adaptive-layer-norm modulation with tangent
namespace {
int adaln_check(int B, int T, int C, int dtype, float eps) {
  if (B < 1 || T < 1 || C < 1) return TVMATTN_INVALID_ARG;
  if (dtype != TVMATTN_F32 && dtype != TVMATTN_BF16) return TVMATTN_UNSUPPORTED;
  if (!(eps >= 0.f) || isinf(eps)) return TVMATTN_INVALID_ARG;
  if (!tvm::adaln_supported(C, dtype) || (long long)B * T >= (1ll << 31) || B > 65535) return TVMATTN_UNSUPPORTED;
  return TVMATTN_OK;
}
// The forward needs no workspace any more; the query keeps a non-zero answer for valid shapes (0 = unsupported).
constexpr size_t kAdalnFwdWorkspace = 256;
size_t adaln_part_bytes(int B, int T, int C) {
  return pad256((size_t)B * tvm::adaln_wgs(B, T, true, false) * 4 * C * sizeof(float));
}
}  // namespace

size_t tvmattn_adaln_jvp_fwd_workspace_bytes(int B, int T, int C, int dtype) {
  return adaln_check(B, T, C, dtype, 0.f) ? 0 : kAdalnFwdWorkspace;
}

int tvmattn_adaln_jvp_fwd(int B, int T, int C, int dtype, const void* x, const void* tx, const float* a, const float* ta,
                          const float* b, const float* tb, float eps, void* y, void* ty, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  int rc = adaln_check(B, T, C, dtype, eps);
  if (rc) return rc;
  const void* const in[] = {x, tx, a, ta, b, tb};
  void* const out[] = {y, ty, workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  if (workspace_bytes < kAdalnFwdWorkspace) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::AdalnArgs g{};
  g.x = x;
  g.tx = tx;
  g.a = a;
  g.ta = ta;
  g.b = b;
  g.tb = tb;
  g.y = y;
  g.ty = ty;
  g.B = B;
  g.T = T;
  g.C = C;
  g.nwg = tvm::adaln_wgs(B, T, false, false);
  g.eps = eps;
  return tvm::launch_adaln_fwd(g, dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TVMATTN_OK
                                                                                           : TVMATTN_LAUNCH_FAILED;
}

size_t tvmattn_adaln_jvp_bwd_workspace_bytes(int B, int T, int C, int dtype) {
  if (adaln_check(B, T, C, dtype, 0.f)) return 0;
  return adaln_part_bytes(B, T, C);
}

int tvmattn_adaln_jvp_bwd_residual(int B, int T, int C, int dtype, const void* x, const void* tx, const float* a, const float* ta,
                          const float* b, const float* tb, float eps, const void* gy, const void* gty, const void* gres, const void* gtres, void* gx,
                          void* gtx, float* ga, float* gta, float* gb, float* gtb, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  int rc = adaln_check(B, T, C, dtype, eps);
  if (rc) return rc;
  if ((gres == nullptr) != (gtres == nullptr)) return TVMATTN_INVALID_ARG;
  const void* const in[] = {x, tx, a, ta, b, tb, gy, gty, unless(!gres, gres), unless(!gtres, gtres)};
  void* const out[] = {gx, gtx, ga, gta, gb, gtb, workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  if (workspace_bytes < tvmattn_adaln_jvp_bwd_workspace_bytes(B, T, C, dtype)) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::AdalnArgs g{};
  g.x = x;
  g.tx = tx;
  g.gy = gy;
  g.gty = gty;
  g.gres = gres;
  g.gtres = gtres;
  g.a = a;
  g.ta = ta;
  g.b = b;
  g.tb = tb;
  g.y = gx;
  g.ty = gtx;
  g.ga = ga;
  g.gta = gta;
  g.gb = gb;
  g.gtb = gtb;
  g.part = static_cast<float*>(workspace);
  g.B = B;
  g.T = T;
  g.C = C;
  g.nwg = tvm::adaln_wgs(B, T, true, false);
  g.eps = eps;
  return tvm::launch_adaln_bwd(g, dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TVMATTN_OK
                                                                                           : TVMATTN_LAUNCH_FAILED;
}

int tvmattn_adaln_jvp_bwd(int B, int T, int C, int dtype, const void* x, const void* tx, const float* a, const float* ta,
                          const float* b, const float* tb, float eps, const void* gy, const void* gty, void* gx,
                          void* gtx, float* ga, float* gta, float* gb, float* gtb, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  return tvmattn_adaln_jvp_bwd_residual(B, T, C, dtype, x, tx, a, ta, b, tb, eps, gy, gty, nullptr, nullptr, gx, gtx, ga,
                                        gta, gb, gtb, workspace, workspace_bytes, hip_stream);
}

// ---- normalised gate of a residual branch with tangent
size_t tvmattn_gate_jvp_bwd_workspace_bytes(int B, int T, int C, int dtype) {
  if (adaln_check(B, T, C, dtype, 0.f)) return 0;
  return pad256((size_t)B * tvm::adaln_wgs(B, T, true, true) * 2 * C * sizeof(float));
}

int tvmattn_gate_jvp_fwd(int B, int T, int C, int dtype, const void* x, const void* tx, const void* h, const void* th,
                         const float* c, const float* tc, float eps, void* z, void* tz, void* hip_stream) {
  int rc = adaln_check(B, T, C, dtype, eps);
  if (rc) return rc;
  // the stream may be updated in place (z = x and tz = tx, each exactly): a thread reads its 16 bytes of x and tx
  // before it writes the same 16 bytes of z and tz, and nobody else touches them
  const void* const in[] = {z == x ? skip : x, tz == tx ? skip : tx, h, th, c, tc};
  void* const out[] = {z, tz};
  if (!x || !tx || !aligned16(x) || !aligned16(tx)) return TVMATTN_INVALID_ARG;
  rc = check_ptrs(in, out);
  if (rc) return rc;
  tvm::GateArgs g{};
  g.x = x;
  g.tx = tx;
  g.h = h;
  g.th = th;
  g.c = c;
  g.tc = tc;
  g.z = z;
  g.tz = tz;
  g.B = B;
  g.T = T;
  g.C = C;
  g.nwg = tvm::adaln_wgs(B, T, false, true);
  g.eps = eps;
  return tvm::launch_gate_fwd(g, dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TVMATTN_OK
                                                                                          : TVMATTN_LAUNCH_FAILED;
}

int tvmattn_gate_jvp_bwd(int B, int T, int C, int dtype, const void* h, const void* th, const float* c, const float* tc,
                         float eps, const void* gz, const void* gtz, void* gh, void* gth, float* gc, float* gtc,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = adaln_check(B, T, C, dtype, eps);
  if (rc) return rc;
  const void* const in[] = {h, th, c, tc, gz, gtz};
  void* const out[] = {gh, gth, gc, gtc, workspace};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  if (workspace_bytes < tvmattn_gate_jvp_bwd_workspace_bytes(B, T, C, dtype)) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::GateArgs g{};
  g.h = h;
  g.th = th;
  g.gz = gz;
  g.gtz = gtz;
  g.c = c;
  g.tc = tc;
  g.z = gh;
  g.tz = gth;
  g.gc = gc;
  g.gtc = gtc;
  g.part = static_cast<float*>(workspace);
  g.B = B;
  g.T = T;
  g.C = C;
  g.nwg = tvm::adaln_wgs(B, T, true, true);
  g.eps = eps;
  return tvm::launch_gate_bwd(g, dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TVMATTN_OK
                                                                                          : TVMATTN_LAUNCH_FAILED;
}

// ---- the MLP's activation with tangent
namespace {
int gelu_check(long long n, int dtype) {
  if (n < 1) return TVMATTN_INVALID_ARG;
  if (dtype != TVMATTN_F32 && dtype != TVMATTN_BF16) return TVMATTN_UNSUPPORTED;
  if (n % (dtype == TVMATTN_BF16 ? 8 : 4) != 0 || n > (1ll << 40)) return TVMATTN_UNSUPPORTED;
  return TVMATTN_OK;
}
}  // namespace

int tvmattn_gelu_jvp_fwd(long long n, int dtype, const void* u, const void* tu, void* a, void* ta, void* hip_stream) {
  int rc = gelu_check(n, dtype);
  if (rc) return rc;
  const void* const in[] = {u, tu};
  void* const out[] = {a, ta};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  return tvm::launch_gelu_fwd(n, dtype, u, tu, a, ta, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

int tvmattn_gelu_jvp_bwd(long long n, int dtype, const void* u, const void* tu, const void* ga, const void* gta,
                         void* gu, void* gtu, void* hip_stream) {
  int rc = gelu_check(n, dtype);
  if (rc) return rc;
  const void* const in[] = {u, tu, ga, gta};
  void* const out[] = {gu, gtu};
  rc = check_ptrs(in, out);
  if (rc) return rc;
  return tvm::launch_gelu_bwd(n, dtype, u, tu, ga, gta, gu, gtu, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

}  // extern "C"
