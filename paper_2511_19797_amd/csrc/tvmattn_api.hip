// C-ABI entry points: argument validation and dispatch.  No allocation, no synchronisation.
#include "../../include/tvmattn.h"

#include <math.h>

#include <mutex>

#include "tvm_common.h"

namespace {

inline void mark(void* const* events, int i, hipStream_t st) {
  if (events && events[i]) (void)hipEventRecord(static_cast<hipEvent_t>(events[i]), st);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One side's strides: all zero selects `dflt_*`; otherwise row pitch >= D and 16-byte multiples.  The whole tensor
// must fit the 2^47-byte address space (which also keeps every later product of sizes and strides inside 64 bits).
bool side_strides(long long esz, int B, int H, int rows, int D, long long& sb, long long& sh, long long& sn,
                  long long dflt_b, long long dflt_h, long long dflt_n) {
  if (sb == 0 && sh == 0 && sn == 0) {
    sb = dflt_b;
    sh = dflt_h;
    sn = dflt_n;
  }
  constexpr long long kMax = 1ll << 46;  // elements
  if (sn < D || sh < 1 || sb < 1 || sn > kMax || sh > kMax || sb > kMax) return false;
  long long eb, eh, en, ext;
  if (__builtin_mul_overflow((long long)(B - 1), sb, &eb) || __builtin_mul_overflow((long long)(H - 1), sh, &eh) ||
      __builtin_mul_overflow((long long)(rows - 1), sn, &en) || __builtin_add_overflow(eb, eh, &ext) ||
      __builtin_add_overflow(ext, en, &ext) || __builtin_add_overflow(ext, (long long)D, &ext) || ext > kMax)
    return false;
  return (sn * esz) % 16 == 0 && (sh * esz) % 16 == 0 && (sb * esz) % 16 == 0;
}

// Validates the descriptor and resolves sizes, strides and scale.
int resolve(const tvmattn_desc* d, tvm::Shape* s) {
  if (!d) return TVMATTN_INVALID_ARG;
  if (d->B < 1 || d->H < 1 || d->N < 1 || d->D < 1 || d->M < 0 || (d->flags & ~TVMATTN_FLAG_PLAIN_ALU) != 0)
    return TVMATTN_INVALID_ARG;
  if (d->dtype != TVMATTN_F32 && d->dtype != TVMATTN_BF16) return TVMATTN_UNSUPPORTED;
  if (d->D > 256) return TVMATTN_UNSUPPORTED;
  if (!(d->scale >= 0.f) || isinf(d->scale)) return TVMATTN_INVALID_ARG;
  const long long esz = d->dtype == TVMATTN_F32 ? 4 : 2;
  const int M = d->M ? d->M : d->N;
  if ((long long)d->B * d->H >= (1ll << 31) || (long long)d->B * d->H * d->N >= (1ll << 31) ||
      (long long)d->B * d->H * M >= (1ll << 31))
    return TVMATTN_UNSUPPORTED;
  long long sb = d->stride_b, sh = d->stride_h, sn = d->stride_n;
  if (!side_strides(esz, d->B, d->H, d->N, d->D, sb, sh, sn, (long long)d->N * d->D * d->H, (long long)d->N * d->D, d->D))
    return TVMATTN_INVALID_ARG;
  long long qsb = d->qstride_b, qsh = d->qstride_h, qsn = d->qstride_n;
  const bool same = M == d->N;  // self-attention: the query side defaults to the key side's layout
  if (!side_strides(esz, d->B, d->H, M, d->D, qsb, qsh, qsn, same ? sb : (long long)M * d->D * d->H,
                    same ? sh : (long long)M * d->D, same ? sn : d->D))
    return TVMATTN_INVALID_ARG;
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

// A buffer as the overlap check sees it: `dims` levels of (count, byte stride) around an innermost run of
// `inner` bytes.  dims = 0 is a plain range.
struct Buf {
  const void* p;
  int dims;
  long long n[3], s[3];
  long long inner;
  long long extent() const {
    long long e = inner;
    for (int i = 0; i < dims; ++i) e += (n[i] - 1) * s[i];
    return e;
  }
  bool same_layout(const Buf& o) const {
    if (dims != o.dims || inner != o.inner) return false;
    for (int i = 0; i < dims; ++i)
      if (n[i] != o.n[i] || s[i] != o.s[i]) return false;
    return true;
  }
};
const void* const skip = reinterpret_cast<const void*>(uintptr_t(1));  // an entry the call's mode does not use
inline Buf plain(const void* p, long long bytes) { return Buf{p, 0, {0, 0, 0}, {0, 0, 0}, bytes}; }
// One side's [B,H,rows,D] tensor with that side's strides, levels sorted by descending stride.
Buf side_buf(const void* p, const tvm::Shape& s, bool query_side, long long esz) {
  Buf b{p, 3, {s.B, s.H, query_side ? s.M : s.N},
        {(query_side ? s.qsb : s.sb) * esz, (query_side ? s.qsh : s.sh) * esz, (query_side ? s.qsn : s.sn) * esz},
        (long long)s.D * esz};
  for (int i = 0; i < 3; ++i)
    for (int j = i + 1; j < 3; ++j)
      if (b.s[j] > b.s[i]) {
        const long long tn = b.n[i], ts = b.s[i];
        b.n[i] = b.n[j];
        b.s[i] = b.s[j];
        b.n[j] = tn;
        b.s[j] = ts;
      }
  return b;
}
// Do two buffers of ONE layout, `delta` bytes apart, share a byte?  They do iff delta = sum_k d_k s_k + e with
// |d_k| < n_k and |e| < inner.  Where every stride is at least the extent of the levels inside it (any dense or
// sliced tensor), what the inner levels can contribute is smaller than the stride, so only the two multiples of
// s_k around delta can start a solution: a walk of depth `dims` with two branches per level.
bool lattice_hit(const Buf& b, int level, long long delta) {
  if (level == b.dims) return delta > -b.inner && delta < b.inner;
  const long long st = b.s[level];
  long long d0 = delta / st;
  if (delta < 0 && d0 * st != delta) --d0;  // floor
  for (long long d = d0; d <= d0 + 1; ++d)
    if (d > -b.n[level] && d < b.n[level] && lattice_hit(b, level + 1, delta - d * st)) return true;
  return false;
}
bool nested(const Buf& b) {
  long long inside = b.inner;
  for (int i = b.dims - 1; i >= 0; --i) {
    if (b.s[i] < inside) return false;
    inside = (b.n[i] - 1) * b.s[i] + inside;
  }
  return true;
}
bool overlap(const Buf& a, const Buf& b) {
  const long long pa = (long long)reinterpret_cast<uintptr_t>(a.p), pb = (long long)reinterpret_cast<uintptr_t>(b.p);
  if (pa + a.extent() <= pb || pb + b.extent() <= pa) return false;  // disjoint address ranges
  if (a.same_layout(b) && nested(a)) return lattice_hit(a, 0, pb - pa);
  return true;
}
// Every listed pointer must be non-null and 16-byte aligned, and no output may overlap an input or another
// output.  Entries that the call's mode does not use are passed with p == skip (a null there is fine, and the
// buffer takes no part in the overlap check).  `inout`: pairs (output index, input index) that may be the very
// same buffer (an update in place).
template <size_t NI, size_t NO>
int check_bufs(const Buf (&in)[NI], const Buf (&out)[NO], int same_o = -1, int same_i = -1, int same_o2 = -1,
               int same_i2 = -1) {
  for (size_t i = 0; i < NI; ++i)
    if (in[i].p != skip && (!in[i].p || !aligned16(in[i].p))) return TVMATTN_INVALID_ARG;
  for (size_t o = 0; o < NO; ++o) {
    if (out[o].p == skip) continue;
    if (!out[o].p || !aligned16(out[o].p)) return TVMATTN_INVALID_ARG;
    for (size_t i = 0; i < NI; ++i) {
      if (in[i].p == skip) continue;
      const bool allowed = ((int)o == same_o && (int)i == same_i) || ((int)o == same_o2 && (int)i == same_i2);
      if (allowed && out[o].p == in[i].p) continue;
      if (overlap(out[o], in[i])) return TVMATTN_INVALID_ARG;
    }
    for (size_t p = 0; p < o; ++p)
      if (out[p].p != skip && overlap(out[o], out[p])) return TVMATTN_INVALID_ARG;
  }
  return TVMATTN_OK;
}
inline Buf unless(bool unused, Buf b) {
  if (unused) b.p = skip;
  return b;
}
inline long long esz_of(int dtype) { return dtype == TVMATTN_F32 ? 4 : 2; }
inline bool plain_alu(const tvmattn_desc* d) { return (d->flags & TVMATTN_FLAG_PLAIN_ALU) != 0; }

}  // namespace

extern "C" {

int tvmattn_version(void) { return 610; }  // 0.6.1: tvmattn_jvp_fwd_qknorm; 0.6.0: per-call flags instead of process-wide switches, tvmattn_jvp_bwd_timed, tvmattn_jvp_bwd_static, linear layers; 0.5.0: AdaLN modulation, residual gate, MLP activation; 0.4.0: QK-norm entry points; 0.3.0: M != N (the descriptor grew); 0.2.0: one-sided backward, forward that saves nothing

const char* tvmattn_strerror(int status) {
  switch (status) {
    case TVMATTN_OK: return "ok";
    case TVMATTN_INVALID_ARG: return "invalid argument (null/misaligned pointer, bad shape, stride or scale, or aliasing)";
    case TVMATTN_UNSUPPORTED: return "unsupported (dtype, head dimension > 256, or too many rows)";
    case TVMATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TVMATTN_LAUNCH_FAILED: return "kernel launch failed";
    case TVMATTN_SCRATCH_TOO_SMALL:
      return "too many query rows (B*H*M) for the static scratch of tvmattn_jvp_bwd_static; use tvmattn_jvp_bwd with a workspace";
    default: return "unknown status";
  }
}

int tvmattn_jvp_fwd(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                    const void* tk, const void* tv, void* o, void* to, float* lse, float* stats, void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if ((lse == nullptr) != (stats == nullptr)) return TVMATTN_INVALID_ARG;  // saved together or not at all
  const bool nosave = lse == nullptr;
  const long long esz = esz_of(desc->dtype), rvb = (long long)s.B * s.H * s.M * 4;
  const Buf in[] = {side_buf(q, s, true, esz),  side_buf(k, s, false, esz),  side_buf(v, s, false, esz),
                    side_buf(tq, s, true, esz), side_buf(tk, s, false, esz), side_buf(tv, s, false, esz)};
  const Buf out[] = {side_buf(o, s, true, esz), side_buf(to, s, true, esz), unless(nosave, plain(lse, rvb)),
                     unless(nosave, plain(stats, rvb))};
  rc = check_bufs(in, out);
  if (rc) return rc;
  tvm::FwdArgs a{q, k, v, tq, tk, tv, o, to, lse, stats};
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (!plain_alu(desc) && tvm::mfma_supported(s, desc->dtype))
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

namespace {
// The backward proper, with the three row vectors (one float per query row each) wherever the caller's entry
// point keeps them.  Pointer checks of everything but the row vectors included.
int bwd_impl(const tvmattn_desc* desc, const tvm::Shape& s, const void* q, const void* k, const void* v, const void* tq,
             const void* tk, const void* tv, const void* o, const void* to, const float* lse, const float* stats,
             const void* gO, const void* gTO, void* dq, void* dk, void* dv, void* dtq, void* dtk, void* dtv, float* row0,
             float* row1, float* row2, bool rows_fit, void* const* events, void* hip_stream) {
  if (!gO && !gTO) return TVMATTN_INVALID_ARG;
  // one upstream gradient only: 1 = gO (the tangent inputs and outputs take no part), 2 = gTO
  const int mode = !gTO ? 1 : !gO ? 2 : 0;
  const bool m1 = mode == 1;
  const long long esz = esz_of(desc->dtype), rvb = (long long)s.B * s.H * s.M * 4;
  auto qs = [&](const void* p) { return side_buf(p, s, true, esz); };
  auto ks = [&](const void* p) { return side_buf(p, s, false, esz); };
  const Buf in[] = {qs(q), ks(k), ks(v), unless(m1, qs(tq)), unless(m1, ks(tk)), unless(m1, ks(tv)), qs(o),
                    unless(m1, qs(to)), plain(lse, rvb), unless(m1, plain(stats, rvb)), unless(mode == 2, qs(gO)),
                    unless(m1, qs(gTO))};
  const Buf out[] = {qs(dq), ks(dk), ks(dv), unless(m1, qs(dtq)), unless(m1, ks(dtk)), unless(m1, ks(dtv)),
                     plain(row0, rvb), plain(row1, rvb), plain(row2, rvb)};
  const int rc = check_bufs(in, out);
  if (rc) return rc;
  if (!rows_fit) return TVMATTN_WORKSPACE_TOO_SMALL;
  tvm::BwdArgs a{q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv, row0, row1, row2, mode};
  if (m1) {  // not read, not written: whatever was passed
    a.tq = a.tk = a.tv = a.to = nullptr;
    a.stats = nullptr;
    a.dtq = a.dtk = a.dtv = nullptr;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const bool mf = !plain_alu(desc) && tvm::mfma_supported(s, desc->dtype);
  hipError_t e = hipSuccess;
  mark(events, 0, st);
  if (!mf) e = tvm::launch_bwd_pre(s, desc->dtype, a, st);  // the matrix-core query-side kernel does Step 1 itself
  if (e != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  mark(events, 1, st);
  e = mf ? tvm::launch_bwd_row_mfma(s, a, st) : tvm::launch_bwd_row_generic(s, desc->dtype, a, st);
  if (e != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  mark(events, 2, st);
  e = mf ? tvm::launch_bwd_col_mfma(s, a, st) : tvm::launch_bwd_col_generic(s, desc->dtype, a, st);
  mark(events, 3, st);
  return e == hipSuccess ? TVMATTN_OK : TVMATTN_LAUNCH_FAILED;
}
inline size_t row_vector_bytes(const tvm::Shape& s) {  // one float32 per query row, padded to a 256-byte multiple
  return ((size_t)s.B * s.H * s.M * sizeof(float) + 255) & ~(size_t)255;
}
}  // namespace

int tvmattn_jvp_bwd_timed(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                          const void* tk, const void* tv, const void* o, const void* to, const float* lse,
                          const float* stats, const void* gO, const void* gTO, void* dq, void* dk, void* dv, void* dtq,
                          void* dtk, void* dtv, void* workspace, size_t workspace_bytes, void* const* events,
                          void* hip_stream) {
  tvm::Shape s;
  const int rc = resolve(desc, &s);
  if (rc) return rc;
  const size_t one = row_vector_bytes(s);
  char* const ws = static_cast<char*>(workspace);  // (a null workspace fails the pointer checks in bwd_impl)
  return bwd_impl(desc, s, q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv,
                  reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws ? ws + one : nullptr),
                  reinterpret_cast<float*>(ws ? ws + 2 * one : nullptr), workspace_bytes >= 3 * one, events, hip_stream);
}

int tvmattn_jvp_bwd(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                    const void* tk, const void* tv, const void* o, const void* to, const float* lse,
                    const float* stats, const void* gO, const void* gTO, void* dq, void* dk, void* dv, void* dtq,
                    void* dtk, void* dtv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return tvmattn_jvp_bwd_timed(desc, q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv,
                               workspace, workspace_bytes, nullptr, hip_stream);
}

// ---- the same backward for callers that cannot allocate: the row vectors live in a static device array
namespace {
constexpr long long kStaticMaxRows = TVMATTN_STATIC_MAX_ROWS;  // query rows B*H*M served by the static scratch
// Three row vectors of kStaticMaxRows floats each (12 MiB per GPU the library runs on, held until the process ends).
static __device__ __align__(256) float scratch[3 * kStaticMaxRows];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];         // device address of `scratch` on each GPU (its name is no device address)
std::once_flag g_scratch_once[kMaxDevices];
hipError_t g_scratch_err[kMaxDevices];
}  // namespace

int tvmattn_jvp_bwd_static(const tvmattn_desc* desc, const void* q, const void* k, const void* v, const void* tq,
                           const void* tk, const void* tv, const void* o, const void* to, const float* lse,
                           const float* stats, const void* gO, const void* gTO, void* dq, void* dk, void* dv, void* dtq,
                           void* dtk, void* dtv, void* hip_stream) {
  tvm::Shape s;
  const int rc = resolve(desc, &s);
  if (rc) return rc;
  if ((long long)s.B * s.H * s.M > kStaticMaxRows) return TVMATTN_SCRATCH_TOO_SMALL;  // before any HIP call
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TVMATTN_LAUNCH_FAILED;
  // once per device, with that device current: each GPU holds its own copy of the array at its own address
  std::call_once(g_scratch_once[dev], [dev] {
    void* p = nullptr;
    g_scratch_err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    g_scratch_ptr[dev] = g_scratch_err[dev] == hipSuccess ? static_cast<float*>(p) : nullptr;
  });
  float* const base = g_scratch_ptr[dev];
  if (!base) return TVMATTN_LAUNCH_FAILED;
  // nothing has to start at zero: the query-side kernel writes every row's three entries before the key-side
  // kernel, behind it on the same stream, reads them
  return bwd_impl(desc, s, q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, dq, dk, dv, dtq, dtk, dtv, base,
                  base + kStaticMaxRows, base + 2 * kStaticMaxRows, true, nullptr, hip_stream);
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
  const long long esz = esz_of(desc->dtype), gb = (long long)s.D * 4;
  auto qs = [&](const void* p) { return side_buf(p, s, true, esz); };
  auto ks = [&](const void* p) { return side_buf(p, s, false, esz); };
  const Buf in[] = {qs(q), qs(tq), ks(k), ks(tk), plain(gain_q, gb), plain(gain_k, gb)};
  const Buf out[] = {qs(qn), qs(tqn), ks(kn), ks(tkn)};
  rc = check_bufs(in, out);
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

int tvmattn_jvp_fwd_qknorm(const tvmattn_desc* desc, const void* q, const void* tq, const void* k, const void* tk,
                           const float* gain_q, const float* gain_k, float eps, const void* v, const void* tv, void* qn,
                           void* tqn, void* kn, void* tkn, void* o, void* to, float* lse, float* stats,
                           void* hip_stream) {
  tvm::Shape s;
  int rc = resolve(desc, &s);
  if (rc) return rc;
  if (!(eps >= 0.f) || isinf(eps)) return TVMATTN_INVALID_ARG;
  if ((lse == nullptr) != (stats == nullptr)) return TVMATTN_INVALID_ARG;  // saved together or not at all
  if (plain_alu(desc) || !tvm::mfma_supported(s, desc->dtype)) return TVMATTN_UNSUPPORTED;
  const bool nosave = lse == nullptr;
  const long long esz = esz_of(desc->dtype), gb = (long long)s.D * 4, rvb = (long long)s.B * s.H * s.M * 4;
  auto qs = [&](const void* p) { return side_buf(p, s, true, esz); };
  auto ks = [&](const void* p) { return side_buf(p, s, false, esz); };
  const Buf in[] = {qs(q), qs(tq), ks(k), ks(tk), plain(gain_q, gb), plain(gain_k, gb), ks(v), ks(tv)};
  const Buf out[] = {qs(qn), qs(tqn), ks(kn), ks(tkn), qs(o), qs(to), unless(nosave, plain(lse, rvb)),
                     unless(nosave, plain(stats, rvb))};
  rc = check_bufs(in, out);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the key side through the normalisation kernel (no workgroups for the query side) ...
  tvm::NormArgs n{};
  norm_sides(s, &n, eps);
  n.side[0].nwg = 0;
  n.side[1].x = k;
  n.side[1].tx = tk;
  n.side[1].g = gain_k;
  n.side[1].y = kn;
  n.side[1].ty = tkn;
  hipError_t e = tvm::launch_qknorm_fwd(n, desc->dtype, st);
  if (e != hipSuccess) return TVMATTN_LAUNCH_FAILED;
  // ... the query side inside the attention forward, which leaves the normalised rows behind for the backward
  tvm::FwdArgs a{q, kn, v, tq, tkn, tv, o, to, lse, stats};
  a.ngq = gain_q;
  a.neps = eps;
  a.qn = qn;
  a.tqn = tqn;
  e = tvm::launch_fwd_mfma_qnorm(s, a, st);
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
  const long long esz = esz_of(desc->dtype), gb = (long long)s.D * 4;
  const size_t need = tvmattn_qknorm_jvp_bwd_workspace_bytes(desc);
  auto qs = [&](const void* p) { return side_buf(p, s, true, esz); };
  auto ks = [&](const void* p) { return side_buf(p, s, false, esz); };
  const Buf in[] = {qs(q), qs(tq), ks(k), ks(tk), plain(gain_q, gb), plain(gain_k, gb), qs(gqn), qs(gtqn), ks(gkn), ks(gtkn)};
  const Buf out[] = {qs(dq), qs(dtq), ks(dk), ks(dtk), plain(dgain_q, gb), plain(dgain_k, gb), plain(workspace, (long long)need)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
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
bool fused_supported(const tvmattn_desc* d, const tvm::Shape& s) {
  return !plain_alu(d) && tvm::mfma_supported(s, d->dtype) && s.D <= 96;
}
}  // namespace

size_t tvmattn_jvp_bwd_qknorm_workspace_bytes(const tvmattn_desc* desc) {
  tvm::Shape s;
  if (resolve(desc, &s) || !fused_supported(desc, s)) return 0;
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
  if (!fused_supported(desc, s)) return TVMATTN_UNSUPPORTED;
  const long long esz = esz_of(desc->dtype), gb = (long long)s.D * 4, rvb = (long long)s.B * s.H * s.M * 4;
  const size_t need = tvmattn_jvp_bwd_qknorm_workspace_bytes(desc);
  auto qs = [&](const void* p) { return side_buf(p, s, true, esz); };
  auto ks = [&](const void* p) { return side_buf(p, s, false, esz); };
  const Buf in[] = {qs(q),  qs(tq), ks(k), ks(tk), plain(gain_q, gb), plain(gain_k, gb), qs(qn),  qs(tqn),          ks(kn),
                    ks(tkn), ks(v),  ks(tv), qs(o), qs(to),            plain(lse, rvb),   plain(stats, rvb), qs(gO), qs(gTO)};
  const Buf out[] = {qs(dq), ks(dk), ks(dv), qs(dtq), ks(dtk), ks(dtv), plain(dgain_q, gb), plain(dgain_k, gb),
                     plain(workspace, (long long)need)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
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
inline long long tok_bytes(int B, int T, int C, int dtype) { return (long long)B * T * C * esz_of(dtype); }
inline long long mod_bytes(int B, int C) { return (long long)B * C * 4; }
size_t adaln_part_bytes(int B, int T, int C) {  // per-workgroup sums over tokens, and one row per element for their sums
  return pad256((size_t)B * (tvm::adaln_wgs(B, T, true, false) + 1) * 4 * C * sizeof(float));
}
}  // namespace

int tvmattn_adaln_jvp_fwd(int B, int T, int C, int dtype, const void* x, const void* tx, const float* a, const float* ta,
                          const float* b, const float* tb, float eps, void* y, void* ty, void* hip_stream) {
  int rc = adaln_check(B, T, C, dtype, eps);
  if (rc) return rc;
  const long long tb_ = tok_bytes(B, T, C, dtype), mb = mod_bytes(B, C);
  const Buf in[] = {plain(x, tb_), plain(tx, tb_), plain(a, mb), plain(ta, mb), plain(b, mb), plain(tb, mb)};
  const Buf out[] = {plain(y, tb_), plain(ty, tb_)};
  rc = check_bufs(in, out);
  if (rc) return rc;
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
  const long long tb_ = tok_bytes(B, T, C, dtype), mb = mod_bytes(B, C);
  const size_t need = tvmattn_adaln_jvp_bwd_workspace_bytes(B, T, C, dtype);
  const Buf in[] = {plain(x, tb_),  plain(tx, tb_), plain(a, mb),   plain(ta, mb),
                    plain(b, mb),   plain(tb, mb),  plain(gy, tb_), plain(gty, tb_),
                    unless(!gres, plain(gres, tb_)), unless(!gtres, plain(gtres, tb_))};
  const Buf out[] = {plain(gx, tb_), plain(gtx, tb_), plain(ga, mb), plain(gta, mb), plain(gb, mb), plain(gtb, mb),
                     plain(workspace, (long long)need)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
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
  const long long tb_ = tok_bytes(B, T, C, dtype), mb = mod_bytes(B, C);
  const Buf in[] = {plain(x, tb_), plain(tx, tb_), plain(h, tb_), plain(th, tb_), plain(c, mb), plain(tc, mb)};
  const Buf out[] = {plain(z, tb_), plain(tz, tb_)};
  rc = check_bufs(in, out, 0, 0, 1, 1);  // z may be x itself, tz may be tx itself
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
  const long long tb_ = tok_bytes(B, T, C, dtype), mb = mod_bytes(B, C);
  const size_t need = tvmattn_gate_jvp_bwd_workspace_bytes(B, T, C, dtype);
  const Buf in[] = {plain(h, tb_), plain(th, tb_), plain(c, mb), plain(tc, mb), plain(gz, tb_), plain(gtz, tb_)};
  const Buf out[] = {plain(gh, tb_), plain(gth, tb_), plain(gc, mb), plain(gtc, mb), plain(workspace, (long long)need)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
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
  const long long nb = n * esz_of(dtype);
  const Buf in[] = {plain(u, nb), plain(tu, nb)};
  const Buf out[] = {plain(a, nb), plain(ta, nb)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  return tvm::launch_gelu_fwd(n, dtype, u, tu, a, ta, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

int tvmattn_gelu_jvp_bwd(long long n, int dtype, const void* u, const void* tu, const void* ga, const void* gta,
                         void* gu, void* gtu, void* hip_stream) {
  int rc = gelu_check(n, dtype);
  if (rc) return rc;
  const long long nb = n * esz_of(dtype);
  const Buf in[] = {plain(u, nb), plain(tu, nb), plain(ga, nb), plain(gta, nb)};
  const Buf out[] = {plain(gu, nb), plain(gtu, nb)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  return tvm::launch_gelu_bwd(n, dtype, u, tu, ga, gta, gu, gtu, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

// ---- linear layer on a token and its tangent
namespace {
int linear_check(int R, int K, int F, int dtype, long long& ldx, long long& ldy) {
  if (R < 1 || K < 1 || F < 1 || ldx < 0 || ldy < 0) return TVMATTN_INVALID_ARG;
  if (dtype != TVMATTN_F32 && dtype != TVMATTN_BF16) return TVMATTN_UNSUPPORTED;
  if (ldx == 0) ldx = K;
  if (ldy == 0) ldy = F;
  if (ldx < K || ldy < F) return TVMATTN_INVALID_ARG;
  return tvm::linear_supported(R, K, F, ldx, ldy, dtype) ? TVMATTN_OK : TVMATTN_UNSUPPORTED;
}
// R rows of `cols` elements at a pitch of `ld` elements
Buf rows_buf(const void* p, int R, int cols, long long ld, long long esz) {
  return Buf{p, 1, {R, 0, 0}, {ld * esz, 0, 0}, cols * esz};
}
}  // namespace

size_t tvmattn_linear_jvp_bwd_workspace_bytes(int R, int K, int F, int dtype) {
  long long ldx = 0, ldy = 0;
  return linear_check(R, K, F, dtype, ldx, ldy) ? 0 : tvm::linear_bwd_workspace_bytes(R, K, F);
}

int tvmattn_linear_jvp_fwd(int R, int K, int F, int dtype, const void* x, const void* tx, long long ldx, const void* w,
                           const void* bias, void* y, void* ty, long long ldy, void* hip_stream) {
  int rc = linear_check(R, K, F, dtype, ldx, ldy);
  if (rc) return rc;
  const long long e = esz_of(dtype), wb = (long long)F * K * e;
  const Buf in[] = {rows_buf(x, R, K, ldx, e), rows_buf(tx, R, K, ldx, e), plain(w, wb), unless(!bias, plain(bias, F * e))};
  const Buf out[] = {rows_buf(y, R, F, ldy, e), rows_buf(ty, R, F, ldy, e)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  return tvm::launch_linear_fwd(R, K, F, ldx, ldy, x, tx, w, bias, y, ty, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

int tvmattn_linear_jvp_bwd(int R, int K, int F, int dtype, const void* x, const void* tx, long long ldx, const void* w,
                           const void* gy, const void* gty, long long ldy, void* gx, void* gtx, void* gw, void* gbias,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = linear_check(R, K, F, dtype, ldx, ldy);
  if (rc) return rc;
  const long long e = esz_of(dtype), wb = (long long)F * K * e;
  const size_t need = tvm::linear_bwd_workspace_bytes(R, K, F);
  const Buf in[] = {rows_buf(x, R, K, ldx, e), rows_buf(tx, R, K, ldx, e), plain(w, wb), rows_buf(gy, R, F, ldy, e),
                    rows_buf(gty, R, F, ldy, e)};
  const Buf out[] = {rows_buf(gx, R, K, ldx, e), rows_buf(gtx, R, K, ldx, e), plain(gw, wb), unless(!gbias, plain(gbias, F * e)),
                     plain(workspace, (long long)need)};
  rc = check_bufs(in, out);
  if (rc) return rc;
  if (workspace_bytes < need) return TVMATTN_WORKSPACE_TOO_SMALL;
  return tvm::launch_linear_bwd(R, K, F, ldx, ldy, x, tx, w, gy, gty, gx, gtx, gw, gbias, workspace,
                                static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? TVMATTN_OK
             : TVMATTN_LAUNCH_FAILED;
}

}  // extern "C"
