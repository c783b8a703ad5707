// Normalised adaptive-layer-norm modulation (Terminal Velocity Matching, Sec. "Semi-Lipschitz control", the
// equation for AdaLN(x, t); App. "Full Description of Normalization of Modulation"), with its JVP tangent and
// its backward.  With RMSNorm^- the RMSNorm without learnable parameters (mean of squares, eps inside the root):
//     y  = xh o ah + bh,               xh = RMSNorm^-(x) per token, ah, bh = RMSNorm^-(a), RMSNorm^-(b) per batch element
//     ty = txh o ah + xh o tah + tbh   (txh, tah, tbh: the tangents of the three normalisations along tx, ta, tb)
// x, tx, y, ty: [B,T,C]; a, ta, b, tb: [B,C] float32.
// Backward of <gy, y> + <gty, ty>:  g_xh = gy ah + gty tah,  g_txh = gty ah, then RMSNorm^- backward per token (the
// closed form of qknorm.hip with unit gain);  g_ah = sum_t gy xh + gty txh,  g_tah = sum_t gty xh,  g_bh = sum_t gy,
// g_tbh = sum_t gty, then RMSNorm^- backward per batch element for a and b.
// Memory-bound.  A thread owns one 16-byte chunk of columns for the whole kernel: a workgroup is as wide as a row
// (64 to 256 threads), works out its batch element's normalised modulation for its own columns once, into
// registers, and then walks its token rows R at a time (all their loads in flight together, one barrier per R rows
// for the row sums).  The sums over tokens are then per-thread registers: one partial row per workgroup straight
// from registers, no atomics, added in a fixed order by a second, small kernel that also finishes the gradients of
// a and b.
#include "tvm_common.h"

namespace tvm {
namespace {

// A thread's share of a row: 16 bytes, VEC = 4 columns of float32 or 8 of bfloat16.  (Tried: 8 bytes of bfloat16 per
// thread, i.e. half the registers and twice the waves: slower, forward and backward; what counts is the number of
// bytes a compute unit has in flight.)
template <typename T>
struct alignas(16) Chunk {
  static constexpr int VEC = 16 / sizeof(T);
  T v[VEC];
};
template <typename T> using Raw = uint4;
// Nothing is done to the bytes on the way in (arithmetic right behind a load makes the compiler wait for it there
// and then): idle threads read a valid address like the others and drop their share of the sums instead.
// (Non-temporal loads, which gain 5 % in the activation kernels, lose here: forward +10 %, gate backward +40 %.)
template <typename T>
__device__ __forceinline__ Raw<T> load_raw(const T* p) {
  return *reinterpret_cast<const Raw<T>*>(p);
}
template <typename T>
__device__ __forceinline__ void widen(float (&out)[Chunk<T>::VEC], const Raw<T>& raw) {
  const Chunk<T> c = __builtin_bit_cast(Chunk<T>, raw);
#pragma unroll
  for (int e = 0; e < Chunk<T>::VEC; ++e) out[e] = (float)c.v[e];
}
// The bytes as a value the compiler knows nothing about: what was widened from them before is not kept in
// registers across this point but widened again (half the registers for bfloat16).
__device__ __forceinline__ void forget(uint4& raw) { asm volatile("" : "+v"(raw.x), "+v"(raw.y), "+v"(raw.z), "+v"(raw.w)); }
template <typename T>
__device__ __forceinline__ void store_row(T* p, const float (&in)[Chunk<T>::VEC]) {
  Chunk<T> c;
#pragma unroll
  for (int e = 0; e < Chunk<T>::VEC; ++e) c.v[e] = (T)in[e];
  *reinterpret_cast<Raw<T>*>(p) = __builtin_bit_cast(Raw<T>, c);
}
// VEC consecutive floats at a 16-byte aligned address (zeros for idle lanes), and back.
template <int VEC>
__device__ __forceinline__ void load_f32(float (&out)[VEC], const float* p, bool live) {
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
    const float4 v = reinterpret_cast<const float4*>(p)[q];
    out[4 * q] = live ? v.x : 0.f;
    out[4 * q + 1] = live ? v.y : 0.f;
    out[4 * q + 2] = live ? v.z : 0.f;
    out[4 * q + 3] = live ? v.w : 0.f;
  }
}
template <int VEC>
__device__ __forceinline__ void store_f32(float* p, const float (&in)[VEC]) {
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q)
    reinterpret_cast<float4*>(p)[q] = make_float4(in[4 * q], in[4 * q + 1], in[4 * q + 2], in[4 * q + 3]);
}

// Sum over the wave with data-parallel-primitive moves only (no LDS traffic): a butterfly inside each row of 16
// lanes, then row 0 into row 1 and row 2 into row 3, rows 0-1 into rows 2-3; lane 63 holds the whole and is read
// into a scalar, so every lane gets the same bits.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_from(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROWS, 0xf, false));
}
__device__ __forceinline__ float wave_sum_dpp(float x) {
  x += dpp_from<0xB1, 0xf>(x);   // quad_perm [1,0,3,2]
  x += dpp_from<0x4E, 0xf>(x);   // quad_perm [2,3,0,1]
  x += dpp_from<0x141, 0xf>(x);  // row_half_mirror
  x += dpp_from<0x140, 0xf>(x);  // row_mirror
  x += dpp_from<0x142, 0xa>(x);  // lane 15 of the row before, into rows 1 and 3 (the others add 0)
  x += dpp_from<0x143, 0xc>(x);  // lane 31, into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// K sums over the workgroup's NW waves, the same bits in every thread: waves by lane exchange, then the waves in
// order through `red` (NW x K floats).  One barrier: consecutive calls must alternate between two such buffers.
template <int NW, int K>
__device__ __forceinline__ void wg_sums(float (&s)[K], float* red, int wave, int lane) {
#pragma unroll
  for (int k = 0; k < K; ++k) s[k] = wave_sum_dpp(s[k]);
  if constexpr (NW > 1) {
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < K; ++k) red[wave * K + k] = s[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float t = red[k];
#pragma unroll
      for (int w = 1; w < NW; ++w) t += red[w * K + k];
      s[k] = t;
    }
  }
}

// RMSNorm^- with tangent of the C entries at v, tv (float32), the thread's own VEC columns of it (at c0) into out, tout.
template <int NW, int VEC>
__device__ __forceinline__ void norm_own_chunk(const float* v, const float* tv, int c0, bool live, int C, float eps,
                                               float (&out)[VEC], float (&tout)[VEC], float* red, int wave, int lane) {
  float x[VEC], t[VEC];
  load_f32<VEC>(x, v + c0, live);
  load_f32<VEC>(t, tv + c0, live);
  float s[2] = {0.f, 0.f};
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    s[0] = fmaf(x[e], x[e], s[0]);
    s[1] = fmaf(x[e], t[e], s[1]);
  }
  wg_sums<NW, 2>(s, red, wave, lane);
  const float r = 1.0f / sqrtf(s[0] / (float)C + eps), r3m = r * r * r * (s[1] / (float)C);
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    out[e] = x[e] * r;
    tout[e] = t[e] * r - x[e] * r3m;
  }
}

// NW waves to a row (64 NW x VEC >= C; C is a multiple of VEC), R token rows per pass.
template <typename T, int NW, int R>
__global__ __launch_bounds__(64 * NW) void adaln_fwd_kernel(AdalnArgs a) {
  constexpr int VEC = Chunk<T>::VEC, K = 2 * R;
  __shared__ float red[2 * NW * K];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool live = tid * VEC < a.C;
  const int c0 = live ? tid * VEC : 0;
  float ah[VEC], tah[VEC], bh[VEC], tbh[VEC];
  const long long mo = (long long)b * a.C;
  norm_own_chunk<NW, VEC>(a.a + mo, a.ta + mo, c0, live, a.C, a.eps, ah, tah, red, wave, lane);
  norm_own_chunk<NW, VEC>(a.b + mo, a.tb + mo, c0, live, a.C, a.eps, bh, tbh, red + NW * K, wave, lane);
  const float invc = 1.0f / (float)a.C;
  const T* xb = static_cast<const T*>(a.x) + (long long)b * a.T * a.C + c0;
  const T* tb_ = static_cast<const T*>(a.tx) + (long long)b * a.T * a.C + c0;
  T* yb = static_cast<T*>(a.y) + (long long)b * a.T * a.C + c0;
  T* tyb = static_cast<T*>(a.ty) + (long long)b * a.T * a.C + c0;
  int par = 0;
  for (int t0 = blockIdx.x * R; t0 < a.T; t0 += gridDim.x * R, par ^= 1) {
    Raw<T> rx[R], rt[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {  // rows beyond the last one are read as the last one and not stored
      const long long off = (long long)(t0 + j < a.T ? t0 + j : a.T - 1) * a.C;
      rx[j] = load_raw<T>(xb + off);
      rt[j] = load_raw<T>(tb_ + off);
    }
    float s[K];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      float x[VEC], tx[VEC];
      widen<T>(x, rx[j]);
      widen<T>(tx, rt[j]);
      float sxx = 0.f, sxt = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        sxx = fmaf(x[e], x[e], sxx);
        sxt = fmaf(x[e], tx[e], sxt);
      }
      s[2 * j] = live ? sxx : 0.f;
      s[2 * j + 1] = live ? sxt : 0.f;
    }
    wg_sums<NW, K>(s, red + par * NW * K, wave, lane);
#pragma unroll
    for (int j = 0; j < R; ++j) {
      if (!live || t0 + j >= a.T) continue;
      const float r = 1.0f / sqrtf(s[2 * j] * invc + a.eps), r3m = r * r * r * (s[2 * j + 1] * invc);
      float x[VEC], tx[VEC], y[VEC], ty[VEC];
      forget(rx[j]);
      forget(rt[j]);
      widen<T>(x, rx[j]);
      widen<T>(tx, rt[j]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float xh = x[e] * r, txh = tx[e] * r - x[e] * r3m;
        y[e] = fmaf(xh, ah[e], bh[e]);
        ty[e] = fmaf(txh, ah[e], fmaf(xh, tah[e], tbh[e]));
      }
      const long long off = (long long)(t0 + j) * a.C;
      store_row<T>(yb + off, y);
      store_row<T>(tyb + off, ty);
    }
  }
}

// RES: the gradients that reach x and tx by another way (a residual connection around the modulated branch) are
// added to gx and gtx on the way out.
template <typename T, int NW, int R, bool RES>
__global__ __launch_bounds__(64 * NW) void adaln_bwd_kernel(AdalnArgs a) {
  constexpr int VEC = Chunk<T>::VEC, K = 5 * R;
  __shared__ float red[2 * NW * K];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool live = tid * VEC < a.C;
  const int c0 = live ? tid * VEC : 0;
  float ah[VEC], tah[VEC];
  const long long mo = (long long)b * a.C;
  norm_own_chunk<NW, VEC>(a.a + mo, a.ta + mo, c0, live, a.C, a.eps, ah, tah, red + NW * K, wave, lane);
  const float invc = 1.0f / (float)a.C;
  const long long bo = (long long)b * a.T * a.C + c0;
  const T* xb = static_cast<const T*>(a.x) + bo;
  const T* tb_ = static_cast<const T*>(a.tx) + bo;
  const T* gyb = static_cast<const T*>(a.gy) + bo;
  const T* gtb_ = static_cast<const T*>(a.gty) + bo;
  T* gxb = static_cast<T*>(a.y) + bo;
  T* gtxb = static_cast<T*>(a.ty) + bo;
  const T* grb = RES ? static_cast<const T*>(a.gres) + bo : nullptr;
  const T* gtrb = RES ? static_cast<const T*>(a.gtres) + bo : nullptr;
  float pa[VEC], pta[VEC], pb[VEC], ptb[VEC];  // this thread's columns summed over the workgroup's tokens
#pragma unroll
  for (int e = 0; e < VEC; ++e) pa[e] = pta[e] = pb[e] = ptb[e] = 0.f;
  struct Rows {
    Raw<T> x[R], tx[R], gy[R], gty[R];  // as loaded; widened where used
    Raw<T> gr[RES ? R : 1], gtr[RES ? R : 1];
  };
  // rows beyond the last one are read as the last one and take no further part
  auto load = [&](Rows& q, int t0) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const long long off = (long long)(t0 + j < a.T ? t0 + j : a.T - 1) * a.C;
      q.x[j] = load_raw<T>(xb + off);
      q.tx[j] = load_raw<T>(tb_ + off);
      q.gy[j] = load_raw<T>(gyb + off);
      q.gty[j] = load_raw<T>(gtb_ + off);
      if constexpr (RES) {
        q.gr[j] = load_raw<T>(grb + off);
        q.gtr[j] = load_raw<T>(gtrb + off);
      }
    }
  };
  auto pass = [&](Rows& q, int t0, int par) {
    // u = gy ah + gty tah and w = gty ah flow back into the normalised token and its tangent
    float s[K];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      float x[VEC], tx[VEC], gy[VEC], gty[VEC];
      widen<T>(x, q.x[j]);
      widen<T>(tx, q.tx[j]);
      widen<T>(gy, q.gy[j]);
      widen<T>(gty, q.gty[j]);
      float sxx = 0.f, sxt = 0.f, sA = 0.f, sB = 0.f, sC = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = fmaf(gy[e], ah[e], gty[e] * tah[e]), w = gty[e] * ah[e];
        sxx = fmaf(x[e], x[e], sxx);
        sxt = fmaf(x[e], tx[e], sxt);
        sA = fmaf(u, x[e], sA);
        sB = fmaf(w, x[e], sB);
        sC = fmaf(w, tx[e], sC);
      }
      s[5 * j] = live ? sxx : 0.f;
      s[5 * j + 1] = live ? sxt : 0.f;
      s[5 * j + 2] = live ? sA : 0.f;
      s[5 * j + 3] = live ? sB : 0.f;
      s[5 * j + 4] = live ? sC : 0.f;
      __builtin_amdgcn_sched_barrier(0);  // one row at a time: interleaved rows cost more registers than they gain
    }
    wg_sums<NW, K>(s, red + par * NW * K, wave, lane);
#pragma unroll
    for (int j = 0; j < R; ++j) {
      // a row beyond the last one is a copy of the last one: it is worked on like the others, weighs nothing in
      // the sums over tokens and is not stored (no branch around the arithmetic: it would split the sums' registers)
      const float rowf = t0 + j < a.T ? 1.f : 0.f;
      const float sB = s[5 * j + 3];
      const float r = 1.0f / sqrtf(s[5 * j] * invc + a.eps);
      const float r3 = r * r * r, mm = s[5 * j + 1] * invc;
      const float r3m = r3 * mm, kB = r3 * sB * invc;
      const float kx = (3.0f * r3 * r * r * mm * sB - r3 * (s[5 * j + 2] + s[5 * j + 4])) * invc;
      const float rz = r * rowf, r3mz = r3m * rowf;
      float gx[VEC], gtx[VEC], x[VEC], tx[VEC], gy[VEC], gty[VEC];
      forget(q.x[j]);
      forget(q.tx[j]);
      forget(q.gy[j]);
      forget(q.gty[j]);
      widen<T>(x, q.x[j]);
      widen<T>(tx, q.tx[j]);
      widen<T>(gy, q.gy[j]);
      widen<T>(gty, q.gty[j]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = fmaf(gy[e], ah[e], gty[e] * tah[e]), w = gty[e] * ah[e];
        const float xh = x[e] * rz, txh = tx[e] * rz - x[e] * r3mz;
        gtx[e] = r * w - kB * x[e];
        gx[e] = r * u - r3m * w - kB * tx[e] + kx * x[e];
        pa[e] += fmaf(gy[e], xh, gty[e] * txh);
        pta[e] = fmaf(gty[e], xh, pta[e]);
        pb[e] = fmaf(gy[e], rowf, pb[e]);
        ptb[e] = fmaf(gty[e], rowf, ptb[e]);
      }
      if constexpr (RES) {
        float r0[VEC], r1[VEC];
        widen<T>(r0, q.gr[j]);
        widen<T>(r1, q.gtr[j]);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          gx[e] += r0[e];
          gtx[e] += r1[e];
        }
      }
      if (live && t0 + j < a.T) {
        const long long off = (long long)(t0 + j) * a.C;
        store_row<T>(gxb + off, gx);
        store_row<T>(gtxb + off, gtx);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  int par = 0;
  for (int t0 = blockIdx.x * R; t0 < a.T; t0 += gridDim.x * R, par ^= 1) {
    Rows q;
    load(q, t0);
    pass(q, t0, par);
  }
  if (live) {
    float* part = a.part + ((long long)b * gridDim.x + blockIdx.x) * 4 * a.C + c0;
    store_f32<VEC>(part, pa);
    store_f32<VEC>(part + a.C, pta);
    store_f32<VEC>(part + 2 * a.C, pb);
    store_f32<VEC>(part + 3 * a.C, ptb);
  }
}

// The end of a backward for one normalised [C] vector v with tangent tv (a, b or the gate c of a batch element): the
// workgroups' partial rows (u = gradient of the normalised vector, w = of its tangent, at part and part + C, `stride`
// floats from one workgroup's to the next's) added in a fixed order, then RMSNorm^- backward.  1024 threads: first a
// thread sums a quarter of the partial rows for up to two 16-byte chunks of columns (all its loads in flight
// together, v and tv requested before them), the quarters meet in LDS, then a thread owns one chunk of columns.
constexpr int kModNT = 1024, kModWaves = kModNT / 64, kModQ = 4, kModCols = kModNT / kModQ, kModChunks = 2;
__device__ __forceinline__ void mod_bwd_body(const float* part, long long stride, int nwg, int C, float eps, const float* v,
                                             const float* tv, float* gv, float* gtv, float* qsum /* [kModQ][2][C] */,
                                             float* red /* [kModWaves][5] */) {
  const int tid = threadIdx.x;
  const bool live = tid * 4 < C;
  const int c0 = live ? tid * 4 : 0;
  float x[4], t[4];
  load_f32<4>(x, v + c0, live);
  load_f32<4>(t, tv + c0, live);
  {
    const int q = tid / kModCols, ct = tid % kModCols;
    const int g0 = (nwg * q) / kModQ, g1 = (nwg * (q + 1)) / kModQ;
    bool on[kModChunks];
    int cc[kModChunks];
    float4 su[kModChunks], sw[kModChunks];
#pragma unroll
    for (int j = 0; j < kModChunks; ++j) {
      on[j] = (ct + kModCols * j) * 4 < C;
      cc[j] = on[j] ? (ct + kModCols * j) * 4 : 0;
      su[j] = sw[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll 8
    for (int g = g0; g < g1; ++g) {
#pragma unroll
      for (int j = 0; j < kModChunks; ++j) {
        const float4 pu = *reinterpret_cast<const float4*>(part + g * stride + cc[j]);
        const float4 pw = *reinterpret_cast<const float4*>(part + g * stride + C + cc[j]);
        su[j].x += pu.x; su[j].y += pu.y; su[j].z += pu.z; su[j].w += pu.w;
        sw[j].x += pw.x; sw[j].y += pw.y; sw[j].z += pw.z; sw[j].w += pw.w;
      }
    }
#pragma unroll
    for (int j = 0; j < kModChunks; ++j) {
      if (!on[j]) continue;
      *reinterpret_cast<float4*>(qsum + (q * 2) * C + cc[j]) = su[j];
      *reinterpret_cast<float4*>(qsum + (q * 2 + 1) * C + cc[j]) = sw[j];
    }
  }
  __syncthreads();
  float u[4], w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float au = qsum[c0 + e], aw = qsum[C + c0 + e];
#pragma unroll
    for (int q = 1; q < kModQ; ++q) {
      au += qsum[(q * 2) * C + c0 + e];
      aw += qsum[(q * 2 + 1) * C + c0 + e];
    }
    u[e] = live ? au : 0.f;
    w[e] = live ? aw : 0.f;
  }
  float s[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s[0] = fmaf(x[e], x[e], s[0]);
    s[1] = fmaf(x[e], t[e], s[1]);
    s[2] = fmaf(u[e], x[e], s[2]);
    s[3] = fmaf(w[e], x[e], s[3]);
    s[4] = fmaf(w[e], t[e], s[4]);
  }
  wg_sums<kModWaves, 5>(s, red, tid >> 6, tid & 63);
  const float invc = 1.0f / (float)C;
  const float r = 1.0f / sqrtf(s[0] * invc + eps);
  const float r3 = r * r * r, mm = s[1] * invc;
  const float r3m = r3 * mm, kB = r3 * s[3] * invc;
  const float kx = (3.0f * r3 * r * r * mm * s[3] - r3 * (s[2] + s[4])) * invc;
  if (live) {
    float g[4], gt[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      gt[e] = r * w[e] - kB * x[e];
      g[e] = r * u[e] - r3m * w[e] - kB * t[e] + kx * x[e];
    }
    store_f32<4>(gv + c0, g);
    store_f32<4>(gtv + c0, gt);
  }
}

// With many partial rows per batch element the two (or one) workgroups per element of the kernels below would spend
// their time fetching them (64 rows: 15 us, a CU's worth of bandwidth each): this kernel adds the nwg rows of W floats
// of batch element blockIdx.y first, 64 chunks of 16 bytes per workgroup (wave q takes quarter q of the rows, the
// quarters meet in LDS in a fixed order), and leaves one row per element for them.
__global__ __launch_bounds__(256) void part_rows_sum_kernel(const float* __restrict__ part, int nwg, int W,
                                                            float* __restrict__ out) {
  __shared__ float4 red[4][64];
  const int q = threadIdx.x >> 6, ct = threadIdx.x & 63, b = blockIdx.y;
  const int c = (blockIdx.x * 64 + ct) * 4;
  const bool on = c < W;
  const float* p = part + (long long)b * nwg * W + (on ? c : 0);
  const int g0 = (nwg * q) / 4, g1 = (nwg * (q + 1)) / 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 16
  for (int g = g0; g < g1; ++g) {
    const float4 v = *reinterpret_cast<const float4*>(p + (long long)g * W);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  red[q][ct] = s;
  __syncthreads();
  if (q == 0 && on) {
    const float4 r0 = red[0][ct], r1 = red[1][ct], r2 = red[2][ct], r3 = red[3][ct];
    const float4 t = make_float4((r0.x + r1.x) + (r2.x + r3.x), (r0.y + r1.y) + (r2.y + r3.y),
                                 (r0.z + r1.z) + (r2.z + r3.z), (r0.w + r1.w) + (r2.w + r3.w));
    *reinterpret_cast<float4*>(out + (long long)b * W + c) = t;
  }
}
constexpr int kPartRowsDirect = 16;  // up to this many partial rows the end kernels fetch them themselves

// Workgroup (which, b): which = 0: g_ah, g_tah and the gradients of a, ta; which = 1: g_bh, g_tbh and those of b, tb.
__global__ __launch_bounds__(kModNT) void adaln_mod_bwd_kernel(AdalnArgs a) {
  extern __shared__ float qsum[];
  __shared__ float red[kModWaves * 5];
  const int which = blockIdx.x, b = blockIdx.y;
  const long long o = (long long)b * a.C;
  mod_bwd_body(a.part + (long long)b * a.nwg * 4 * a.C + which * 2 * a.C, (long long)4 * a.C, a.nwg, a.C, a.eps,
               (which ? a.b : a.a) + o, (which ? a.tb : a.ta) + o, (which ? a.gb : a.ga) + o,
               (which ? a.gtb : a.gta) + o, qsum, red);
}

// ---- Normalised gate of a residual branch (App. "Full Description of Normalization of Modulation", the layer
// equations): z = x + ch o h, tz = tx + tch o h + ch o th with ch, tch = RMSNorm^-(c) and its tangent per batch
// element.  Backward of <gz, z> + <gtz, tz>: gh = ch gz + tch gtz, gth = ch gtz (the gradients of x and tx are gz
// and gtz themselves and are not written), g_ch = sum_t gz h + gtz th, g_tch = sum_t gtz h, then RMSNorm^- backward
// for c.  No row sums: pure streaming, the same thread-per-chunk layout, R rows per pass, no barrier in the loop.
template <typename T, int NW, int R>
__global__ __launch_bounds__(64 * NW) void gate_fwd_kernel(GateArgs a) {
  constexpr int VEC = Chunk<T>::VEC;
  __shared__ float red[NW * 2];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool live = tid * VEC < a.C;
  const int c0 = live ? tid * VEC : 0;
  float ch[VEC], tch[VEC];
  const long long mo = (long long)b * a.C;
  norm_own_chunk<NW, VEC>(a.c + mo, a.tc + mo, c0, live, a.C, a.eps, ch, tch, red, wave, lane);
  if (!live) return;  // no barrier from here on
  const long long bo = (long long)b * a.T * a.C + c0;
  const T* xb = static_cast<const T*>(a.x) + bo;
  const T* txb = static_cast<const T*>(a.tx) + bo;
  const T* hb = static_cast<const T*>(a.h) + bo;
  const T* thb = static_cast<const T*>(a.th) + bo;
  T* zb = static_cast<T*>(a.z) + bo;
  T* tzb = static_cast<T*>(a.tz) + bo;
  for (int t0 = blockIdx.x * R; t0 < a.T; t0 += gridDim.x * R) {
    Raw<T> rx[R], rtx[R], rh[R], rth[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {  // rows beyond the last one are read as the last one and not stored
      const long long off = (long long)(t0 + j < a.T ? t0 + j : a.T - 1) * a.C;
      rx[j] = load_raw<T>(xb + off);
      rtx[j] = load_raw<T>(txb + off);
      rh[j] = load_raw<T>(hb + off);
      rth[j] = load_raw<T>(thb + off);
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      if (t0 + j >= a.T) continue;
      float x[VEC], tx[VEC], h[VEC], th[VEC], z[VEC], tz[VEC];
      widen<T>(x, rx[j]);
      widen<T>(tx, rtx[j]);
      widen<T>(h, rh[j]);
      widen<T>(th, rth[j]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        z[e] = fmaf(ch[e], h[e], x[e]);
        tz[e] = fmaf(tch[e], h[e], fmaf(ch[e], th[e], tx[e]));
      }
      const long long off = (long long)(t0 + j) * a.C;
      store_row<T>(zb + off, z);
      store_row<T>(tzb + off, tz);
    }
  }
}

template <typename T, int NW, int R>
__global__ __launch_bounds__(64 * NW) void gate_bwd_kernel(GateArgs a) {
  constexpr int VEC = Chunk<T>::VEC;
  __shared__ float red[NW * 2];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool live = tid * VEC < a.C;
  const int c0 = live ? tid * VEC : 0;
  float ch[VEC], tch[VEC];
  const long long mo = (long long)b * a.C;
  norm_own_chunk<NW, VEC>(a.c + mo, a.tc + mo, c0, live, a.C, a.eps, ch, tch, red, wave, lane);
  if (!live) return;  // no barrier from here on
  const long long bo = (long long)b * a.T * a.C + c0;
  const T* hb = static_cast<const T*>(a.h) + bo;
  const T* thb = static_cast<const T*>(a.th) + bo;
  const T* gzb = static_cast<const T*>(a.gz) + bo;
  const T* gtzb = static_cast<const T*>(a.gtz) + bo;
  T* ghb = static_cast<T*>(a.z) + bo;
  T* gthb = static_cast<T*>(a.tz) + bo;
  float pc[VEC], ptc[VEC];  // this thread's columns summed over the workgroup's tokens
#pragma unroll
  for (int e = 0; e < VEC; ++e) pc[e] = ptc[e] = 0.f;
  for (int t0 = blockIdx.x * R; t0 < a.T; t0 += gridDim.x * R) {
    Raw<T> rh[R], rth[R], rgz[R], rgtz[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const long long off = (long long)(t0 + j < a.T ? t0 + j : a.T - 1) * a.C;
      rh[j] = load_raw<T>(hb + off);
      rth[j] = load_raw<T>(thb + off);
      rgz[j] = load_raw<T>(gzb + off);
      rgtz[j] = load_raw<T>(gtzb + off);
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const float rowf = t0 + j < a.T ? 1.f : 0.f;  // a copy of the last row weighs nothing and is not stored
      float h[VEC], th[VEC], gz[VEC], gtz[VEC], gh[VEC], gth[VEC];
      widen<T>(h, rh[j]);
      widen<T>(th, rth[j]);
      widen<T>(gz, rgz[j]);
      widen<T>(gtz, rgtz[j]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        gh[e] = fmaf(ch[e], gz[e], tch[e] * gtz[e]);
        gth[e] = ch[e] * gtz[e];
        const float hv = h[e] * rowf;
        pc[e] += fmaf(gz[e], hv, gtz[e] * th[e] * rowf);
        ptc[e] = fmaf(gtz[e], hv, ptc[e]);
      }
      if (t0 + j < a.T) {
        const long long off = (long long)(t0 + j) * a.C;
        store_row<T>(ghb + off, gh);
        store_row<T>(gthb + off, gth);
      }
    }
  }
  float* part = a.part + ((long long)b * gridDim.x + blockIdx.x) * 2 * a.C + c0;
  store_f32<VEC>(part, pc);
  store_f32<VEC>(part + a.C, ptc);
}

// Workgroup b: g_ch, g_tch and the gradients of c, tc.
__global__ __launch_bounds__(kModNT) void gate_mod_bwd_kernel(GateArgs a) {
  extern __shared__ float qsum[];
  __shared__ float red[kModWaves * 5];
  const int b = blockIdx.x;
  const long long o = (long long)b * a.C;
  mod_bwd_body(a.part + (long long)b * a.nwg * 2 * a.C, (long long)2 * a.C, a.nwg, a.C, a.eps, a.c + o, a.tc + o,
               a.gc + o, a.gtc + o, qsum, red);
}

template <typename T>
int waves_per_row(int C) { return (C / Chunk<T>::VEC + 63) / 64; }

// Rows per pass and the number of workgroups aimed at, measured at 16 x 1024 tokens x 1152 (us per call with the
// tail kernel): AdaLN backward 2 rows on 1024 workgroups 57-58 (4 on 512: 63, 2 on 512: 63, 1 on 1024: 58, 2 on
// 2048: 73, 8 on 512: 88); gate backward 2 on 256: 41 (4 on 512: 45, 4 on 256: 44, 2 on 384: 42.5, 1 on 256: 46, 4 on
// 128: 54): fewer workgroups leave fewer partial rows to the tail kernel, shorter passes stall less at the
// barrier.  Forward 4 on 1024 (2 or 8 rows, 768 or 2048 workgroups: the same or worse).
#ifndef ADALN_RF
#define ADALN_RF 4
#define ADALN_TF 1024
#define ADALN_RB 2
#define ADALN_TB 1024
#define GATE_RB 2
#define GATE_TB 256
#endif
constexpr int kRowsFwd = ADALN_RF, kRowsBwd = ADALN_RB, kRowsGateBwd = GATE_RB;

}  // namespace

#define TVM_ADALN_BY_SIZE(KERNEL, T, ...)                                                            \
  switch (waves_per_row<T>(a.C)) {                                                                   \
    case 1: hipLaunchKernelGGL((KERNEL<T, 1, __VA_ARGS__>), grid, dim3(64), 0, st, a); break;        \
    case 2: hipLaunchKernelGGL((KERNEL<T, 2, __VA_ARGS__>), grid, dim3(128), 0, st, a); break;       \
    case 3: hipLaunchKernelGGL((KERNEL<T, 3, __VA_ARGS__>), grid, dim3(192), 0, st, a); break;       \
    case 4: hipLaunchKernelGGL((KERNEL<T, 4, __VA_ARGS__>), grid, dim3(256), 0, st, a); break;       \
    default: return hipErrorNotSupported;                                                            \
  }

// Workgroups per batch element: R token rows per pass, at most about `total` workgroups in all, and every one the
// same number of passes where T allows.
int adaln_wgs(int B, int T, bool backward, bool gate) {
  const int R = !backward ? kRowsFwd : gate ? kRowsGateBwd : kRowsBwd;
  const int total = !backward ? ADALN_TF : gate ? GATE_TB : ADALN_TB;
  const int groups = (T + R - 1) / R, cap = total / B > 1 ? total / B : 1;
  const int passes = (groups + cap - 1) / cap;
  return (groups + passes - 1) / passes;
}

bool adaln_supported(int C, int dtype) {
  const int vec = dtype == 1 ? 8 : 4;
  return C % vec == 0 && C / vec <= 256;  // a thread per 16-byte chunk, at most 256 threads
}

hipError_t launch_gate_fwd(const GateArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.nwg, a.B);
  if (dtype == 1) {
    TVM_ADALN_BY_SIZE(gate_fwd_kernel, bf16, kRowsFwd)
  } else {
    TVM_ADALN_BY_SIZE(gate_fwd_kernel, float, kRowsFwd)
  }
  return hipGetLastError();
}

hipError_t launch_gate_bwd(const GateArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.nwg, a.B);
  if (dtype == 1) {
    TVM_ADALN_BY_SIZE(gate_bwd_kernel, bf16, kRowsGateBwd)
  } else {
    TVM_ADALN_BY_SIZE(gate_bwd_kernel, float, kRowsGateBwd)
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gate_mod_bwd_kernel, dim3(a.B), dim3(kModNT), (size_t)kModQ * 2 * a.C * sizeof(float), st, a);
  return hipGetLastError();
}

hipError_t launch_adaln_fwd(const AdalnArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.nwg, a.B);
  if (dtype == 1) {
    TVM_ADALN_BY_SIZE(adaln_fwd_kernel, bf16, kRowsFwd)
  } else {
    TVM_ADALN_BY_SIZE(adaln_fwd_kernel, float, kRowsFwd)
  }
  return hipGetLastError();
}

hipError_t launch_adaln_bwd(const AdalnArgs& a, int dtype, hipStream_t st) {
  const dim3 grid(a.nwg, a.B);
  if (dtype == 1) {
    if (a.gres) {
      TVM_ADALN_BY_SIZE(adaln_bwd_kernel, bf16, kRowsBwd, true)
    } else {
      TVM_ADALN_BY_SIZE(adaln_bwd_kernel, bf16, kRowsBwd, false)
    }
  } else {
    if (a.gres) {
      TVM_ADALN_BY_SIZE(adaln_bwd_kernel, float, kRowsBwd, true)
    } else {
      TVM_ADALN_BY_SIZE(adaln_bwd_kernel, float, kRowsBwd, false)
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  AdalnArgs m = a;
  if (a.nwg > kPartRowsDirect) {  // the partial rows of an element are added first, into [B][4][C] behind all of them
    const int W = 4 * a.C;
    float* sum = a.part + (long long)a.B * a.nwg * W;
    hipLaunchKernelGGL(part_rows_sum_kernel, dim3((W / 4 + 63) / 64, a.B), dim3(256), 0, st, a.part, a.nwg, W, sum);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    m.part = sum;
    m.nwg = 1;
  }
  hipLaunchKernelGGL(adaln_mod_bwd_kernel, dim3(2, a.B), dim3(kModNT), (size_t)kModQ * 2 * a.C * sizeof(float), st, m);
  return hipGetLastError();
}

}  // namespace tvm
