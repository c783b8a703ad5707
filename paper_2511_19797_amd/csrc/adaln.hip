// Normalised adaptive-layer-norm modulation (Terminal Velocity Matching, Sec. "Semi-Lipschitz control", the
// equation for AdaLN(x, t); App. "Full Description of Normalization of Modulation"), with its JVP tangent and
// its backward.  With RMSNorm^- the RMSNorm without learnable parameters (mean of squares, eps inside the root):
//     y  = xh o ah + bh,               xh = RMSNorm^-(x) per token, ah, bh = RMSNorm^-(a), RMSNorm^-(b) per batch element
//     ty = txh o ah + xh o tah + tbh   (txh, tah, tbh: the tangents of the three normalisations along tx, ta, tb)
// x, tx, y, ty: [B,T,C]; a, ta, b, tb: [B,C] float32.
// Backward of <gy, y> + <gty, ty>:  g_xh = gy ah + gty tah,  g_txh = gty ah, then RMSNorm^- backward per token (the
// closed form of qknorm.hip with unit gain);  g_ah = sum_t gy xh + gty txh,  g_tah = sum_t gty xh,  g_bh = sum_t gy,
// g_tbh = sum_t gty, then RMSNorm^- backward per batch element for a and b.
// Memory-bound: a wave per token row, 16 bytes per lane and tensor; the normalised modulation vectors are worked
// out once per batch element by a small kernel and sit in LDS while a workgroup walks its tokens.  The sums over
// tokens use no atomics: column sums per thread, per workgroup through LDS, one partial row per workgroup, added
// in a fixed order by a small kernel, and a last one finishes the gradients of a and b.
#include "tvm_common.h"

namespace tvm {
namespace {

constexpr int kNT = 256;
constexpr int kWaves = kNT / 64;

template <typename T>
struct alignas(16) Chunk16 {
  static constexpr int VEC = 16 / sizeof(T);
  T v[VEC];
};
template <typename T>
__device__ __forceinline__ void load16(float (&out)[Chunk16<T>::VEC], const T* p, bool live) {
  uint4 raw = *reinterpret_cast<const uint4*>(p);  // callers pass a valid address also for idle lanes
  raw.x = live ? raw.x : 0u;
  raw.y = live ? raw.y : 0u;
  raw.z = live ? raw.z : 0u;
  raw.w = live ? raw.w : 0u;
  const Chunk16<T> c = __builtin_bit_cast(Chunk16<T>, raw);
#pragma unroll
  for (int e = 0; e < Chunk16<T>::VEC; ++e) out[e] = (float)c.v[e];
}
// The same in two steps, for kernels that keep the 16 bytes as loaded and widen them where they are used (half the
// registers for bfloat16).
template <typename T>
__device__ __forceinline__ uint4 load16_raw(const T* p, bool live) {
  uint4 raw = *reinterpret_cast<const uint4*>(p);
  raw.x = live ? raw.x : 0u;
  raw.y = live ? raw.y : 0u;
  raw.z = live ? raw.z : 0u;
  raw.w = live ? raw.w : 0u;
  return raw;
}
template <typename T>
__device__ __forceinline__ void widen16(float (&out)[Chunk16<T>::VEC], const uint4& raw) {
  const Chunk16<T> c = __builtin_bit_cast(Chunk16<T>, raw);
#pragma unroll
  for (int e = 0; e < Chunk16<T>::VEC; ++e) out[e] = (float)c.v[e];
}
template <typename T>
__device__ __forceinline__ void store16(T* p, const float (&in)[Chunk16<T>::VEC]) {
  Chunk16<T> c;
#pragma unroll
  for (int e = 0; e < Chunk16<T>::VEC; ++e) c.v[e] = (T)in[e];
  *reinterpret_cast<uint4*>(p) = __builtin_bit_cast(uint4, c);
}

// VEC consecutive floats from LDS at a 16-byte aligned address, as 16-byte reads.
template <int VEC>
__device__ __forceinline__ void lds_vec(float (&out)[VEC], const float* p) {
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
    const float4 v = reinterpret_cast<const float4*>(p)[q];
    out[4 * q] = v.x;
    out[4 * q + 1] = v.y;
    out[4 * q + 2] = v.z;
    out[4 * q + 3] = v.w;
  }
}

// Sum over the workgroup, the same bits in every thread: waves by lane exchange, then the four waves in order.
__device__ __forceinline__ float block_sum(float v, float* red4, int tid) {
  v = wave_sum(v);
  __syncthreads();  // red4 may still be read from the previous call
  if ((tid & 63) == 0) red4[tid >> 6] = v;
  __syncthreads();
  return ((red4[0] + red4[1]) + red4[2]) + red4[3];
}

// RMSNorm^- with tangent of the C entries at v, tv (float32) into out, tout (float32): one workgroup.
__device__ __forceinline__ void norm_row_block(const float* v, const float* tv, float* out, float* tout, int C, float eps,
                                               float* red4, int tid) {
  float sxx = 0.f, sxt = 0.f;
  for (int c = tid; c < C; c += kNT) {
    sxx = fmaf(v[c], v[c], sxx);
    sxt = fmaf(v[c], tv[c], sxt);
  }
  sxx = block_sum(sxx, red4, tid);
  sxt = block_sum(sxt, red4, tid);
  const float r = 1.0f / sqrtf(sxx / (float)C + eps), r3m = r * r * r * (sxt / (float)C);
  for (int c = tid; c < C; c += kNT) {
    out[c] = v[c] * r;
    tout[c] = tv[c] * r - v[c] * r3m;
  }
}

// mod[b][0..3][C] = ah, tah, bh, tbh of batch element b.
__global__ __launch_bounds__(kNT) void adaln_mod_kernel(AdalnArgs a) {
  __shared__ float red4[kWaves];
  const int b = blockIdx.x, tid = threadIdx.x;
  const long long o = (long long)b * a.C;
  float* m = a.mod + (long long)b * 4 * a.C;
  norm_row_block(a.a + o, a.ta + o, m, m + a.C, a.C, a.eps, red4, tid);
  norm_row_block(a.b + o, a.tb + o, m + 2 * a.C, m + 3 * a.C, a.C, a.eps, red4, tid);
}

// MAXC: 16-byte chunks per lane (64 lanes x MAXC x VEC >= C; C is a multiple of VEC).
template <typename T, int MAXC>
__global__ __launch_bounds__(kNT) void adaln_fwd_kernel(AdalnArgs a) {
  constexpr int VEC = Chunk16<T>::VEC;
  extern __shared__ float lds[];  // ah, tah, bh, tbh: 4 x C floats
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* m = a.mod + (long long)b * 4 * a.C;
  for (int c = tid; c < 4 * a.C; c += kNT) lds[c] = m[c];
  __syncthreads();
  const float invc = 1.0f / (float)a.C;
  for (int t = blockIdx.x * kWaves + wave; t < a.T; t += gridDim.x * kWaves) {
    const long long off = ((long long)b * a.T + t) * a.C;
    const T* xp = static_cast<const T*>(a.x) + off;
    const T* tp = static_cast<const T*>(a.tx) + off;
    float x[MAXC][VEC], tx[MAXC][VEC];
    float sxx = 0.f, sxt = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c0 = (lane + 64 * i) * VEC;
      const bool live = c0 < a.C;
      load16<T>(x[i], xp + (live ? c0 : 0), live);
      load16<T>(tx[i], tp + (live ? c0 : 0), live);
    }
#pragma unroll
    for (int i = 0; i < MAXC; ++i)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        sxx = fmaf(x[i][e], x[i][e], sxx);
        sxt = fmaf(x[i][e], tx[i][e], sxt);
      }
    sxx = wave_sum(sxx);
    sxt = wave_sum(sxt);
    const float r = 1.0f / sqrtf(sxx * invc + a.eps), r3m = r * r * r * (sxt * invc);
    T* yp = static_cast<T*>(a.y) + off;
    T* typ = static_cast<T*>(a.ty) + off;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c0 = (lane + 64 * i) * VEC;
      if (c0 >= a.C) continue;
      float y[VEC], ty[VEC], ah[VEC], tah[VEC], bh[VEC], tbh[VEC];
      lds_vec<VEC>(ah, lds + c0);
      lds_vec<VEC>(tah, lds + a.C + c0);
      lds_vec<VEC>(bh, lds + 2 * a.C + c0);
      lds_vec<VEC>(tbh, lds + 3 * a.C + c0);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float xh = x[i][e] * r, txh = tx[i][e] * r - x[i][e] * r3m;
        y[e] = fmaf(xh, ah[e], bh[e]);
        ty[e] = fmaf(txh, ah[e], fmaf(xh, tah[e], tbh[e]));
      }
      store16<T>(yp + c0, y);
      store16<T>(typ + c0, ty);
    }
  }
}

template <typename T, int MAXC>
__global__ __launch_bounds__(kNT) void adaln_bwd_kernel(AdalnArgs a) {
  constexpr int VEC = Chunk16<T>::VEC;
  extern __shared__ float lds[];  // ah, tah (2 x C floats), then the workgroup's column sums (4 x C floats)
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* m = a.mod + (long long)b * 4 * a.C;
  for (int c = tid; c < 2 * a.C; c += kNT) lds[c] = m[c];
  __syncthreads();
  const float invc = 1.0f / (float)a.C;
  float pa[MAXC][VEC], pta[MAXC][VEC], pb[MAXC][VEC], ptb[MAXC][VEC];  // column sums over this wave's tokens
#pragma unroll
  for (int i = 0; i < MAXC; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) pa[i][e] = pta[i][e] = pb[i][e] = ptb[i][e] = 0.f;
  for (int t = blockIdx.x * kWaves + wave; t < a.T; t += gridDim.x * kWaves) {
    const long long off = ((long long)b * a.T + t) * a.C;
    const T* xp = static_cast<const T*>(a.x) + off;
    const T* tp = static_cast<const T*>(a.tx) + off;
    const T* gyp = static_cast<const T*>(a.gy) + off;
    const T* gtp = static_cast<const T*>(a.gty) + off;
    uint4 rx[MAXC], rtx[MAXC], rgy[MAXC], rgt[MAXC];  // as loaded; widened where used
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c0 = (lane + 64 * i) * VEC;
      const bool live = c0 < a.C;
      const int cl = live ? c0 : 0;
      rx[i] = load16_raw<T>(xp + cl, live);
      rtx[i] = load16_raw<T>(tp + cl, live);
      rgy[i] = load16_raw<T>(gyp + cl, live);
      rgt[i] = load16_raw<T>(gtp + cl, live);
    }
    // u = gy ah + gty tah and w = gty ah flow back into the normalised token and its tangent
    float sxx = 0.f, sxt = 0.f, sA = 0.f, sB = 0.f, sC = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c0 = (lane + 64 * i) * VEC;
      const int cl = c0 < a.C ? c0 : 0;
      float x[VEC], tx[VEC], gy[VEC], gty[VEC], ah[VEC], tah[VEC];
      widen16<T>(x, rx[i]);
      widen16<T>(tx, rtx[i]);
      widen16<T>(gy, rgy[i]);
      widen16<T>(gty, rgt[i]);
      lds_vec<VEC>(ah, lds + cl);
      lds_vec<VEC>(tah, lds + a.C + cl);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = fmaf(gy[e], ah[e], gty[e] * tah[e]), w = gty[e] * ah[e];
        sxx = fmaf(x[e], x[e], sxx);
        sxt = fmaf(x[e], tx[e], sxt);
        sA = fmaf(u, x[e], sA);
        sB = fmaf(w, x[e], sB);
        sC = fmaf(w, tx[e], sC);
      }
    }
    sxx = wave_sum(sxx);
    sxt = wave_sum(sxt);
    sA = wave_sum(sA);
    sB = wave_sum(sB);
    sC = wave_sum(sC);
    const float r = 1.0f / sqrtf(sxx * invc + a.eps);
    const float r3 = r * r * r, mm = sxt * invc;
    const float r3m = r3 * mm, kB = r3 * sB * invc;
    const float kx = (3.0f * r3 * r * r * mm * sB - r3 * (sA + sC)) * invc;
    T* gxp = static_cast<T*>(a.y) + off;
    T* gtxp = static_cast<T*>(a.ty) + off;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c0 = (lane + 64 * i) * VEC;
      if (c0 >= a.C) continue;
      float gx[VEC], gtx[VEC], x[VEC], tx[VEC], gy[VEC], gty[VEC], ah[VEC], tah[VEC];
      widen16<T>(x, rx[i]);
      widen16<T>(tx, rtx[i]);
      widen16<T>(gy, rgy[i]);
      widen16<T>(gty, rgt[i]);
      lds_vec<VEC>(ah, lds + c0);
      lds_vec<VEC>(tah, lds + a.C + c0);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float u = fmaf(gy[e], ah[e], gty[e] * tah[e]), w = gty[e] * ah[e];
        const float xh = x[e] * r, txh = tx[e] * r - x[e] * r3m;
        gtx[e] = r * w - kB * x[e];
        gx[e] = r * u - r3m * w - kB * tx[e] + kx * x[e];
        pa[i][e] += fmaf(gy[e], xh, gty[e] * txh);
        pta[i][e] = fmaf(gty[e], xh, pta[i][e]);
        pb[i][e] += gy[e];
        ptb[i][e] += gty[e];
      }
      store16<T>(gxp + c0, gx);
      store16<T>(gtxp + c0, gtx);
    }
  }
  // column sums of this workgroup: its four waves add theirs one after the other, in order
  float* sums = lds + 2 * a.C;
  for (int k = 0; k < kWaves; ++k) {
    if (wave == k) {
#pragma unroll
      for (int i = 0; i < MAXC; ++i) {
        const int c0 = (lane + 64 * i) * VEC;
        if (c0 >= a.C) continue;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float* s = sums + c0 + e;
          s[0] = (k ? s[0] : 0.f) + pa[i][e];
          s[a.C] = (k ? s[a.C] : 0.f) + pta[i][e];
          s[2 * a.C] = (k ? s[2 * a.C] : 0.f) + pb[i][e];
          s[3 * a.C] = (k ? s[3 * a.C] : 0.f) + ptb[i][e];
        }
      }
    }
    __syncthreads();
  }
  float* part = a.part + ((long long)b * gridDim.x + blockIdx.x) * 4 * a.C;
  for (int c = tid; c < 4 * a.C; c += kNT) part[c] = sums[c];
}

// gsum[b][0..3][C] (in place of mod, which nobody reads any more) = the partial rows of batch element b added in
// order: a thread per column, four loads in flight.
__global__ __launch_bounds__(kNT) void adaln_sum_kernel(AdalnArgs a) {
  const int b = blockIdx.y, c = blockIdx.x * kNT + threadIdx.x;
  if (c >= 4 * a.C) return;
  const float* part = a.part + (long long)b * a.nwg * 4 * a.C + c;
  const long long stride = (long long)4 * a.C;
  float s = 0.f;
  int w = 0;
  for (; w + 3 < a.nwg; w += 4) {
    const float v0 = part[w * stride], v1 = part[(w + 1) * stride], v2 = part[(w + 2) * stride], v3 = part[(w + 3) * stride];
    s = (((s + v0) + v1) + v2) + v3;
  }
  for (; w < a.nwg; ++w) s += part[w * stride];
  a.mod[(long long)b * 4 * a.C + c] = s;
}

// Per batch element: RMSNorm^- backward for a (from the sums g_ah, g_tah) and for b (from g_bh, g_tbh).
__global__ __launch_bounds__(kNT) void adaln_mod_bwd_kernel(AdalnArgs a) {
  __shared__ float red4[kWaves];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* gsum = a.mod + (long long)b * 4 * a.C;
  const long long o = (long long)b * a.C;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const float* v = (which ? a.b : a.a) + o;
    const float* tv = (which ? a.tb : a.ta) + o;
    const float* u = gsum + (which ? 2 : 0) * a.C;   // gradient of the normalised vector
    const float* w = u + a.C;                         // ... of its tangent
    float* gv = (which ? a.gb : a.ga) + o;
    float* gtv = (which ? a.gtb : a.gta) + o;
    float sxx = 0.f, sxt = 0.f, sA = 0.f, sB = 0.f, sC = 0.f;
    for (int c = tid; c < a.C; c += kNT) {
      sxx = fmaf(v[c], v[c], sxx);
      sxt = fmaf(v[c], tv[c], sxt);
      sA = fmaf(u[c], v[c], sA);
      sB = fmaf(w[c], v[c], sB);
      sC = fmaf(w[c], tv[c], sC);
    }
    sxx = block_sum(sxx, red4, tid);
    sxt = block_sum(sxt, red4, tid);
    sA = block_sum(sA, red4, tid);
    sB = block_sum(sB, red4, tid);
    sC = block_sum(sC, red4, tid);
    const float invc = 1.0f / (float)a.C;
    const float r = 1.0f / sqrtf(sxx * invc + a.eps);
    const float r3 = r * r * r, mm = sxt * invc;
    const float r3m = r3 * mm, kB = r3 * sB * invc;
    const float kx = (3.0f * r3 * r * r * mm * sB - r3 * (sA + sC)) * invc;
    for (int c = tid; c < a.C; c += kNT) {
      gtv[c] = r * w[c] - kB * v[c];
      gv[c] = r * u[c] - r3m * w[c] - kB * tv[c] + kx * v[c];
    }
  }
}

template <typename T>
int chunks_per_lane(int C) { return (C / Chunk16<T>::VEC + 63) / 64; }

}  // namespace

#define TVM_ADALN_BY_SIZE(KERNEL, T, SHMEM)                                                    \
  switch (chunks_per_lane<T>(a.C)) {                                                           \
    case 1: hipLaunchKernelGGL((KERNEL<T, 1>), grid, dim3(kNT), SHMEM, st, a); break;          \
    case 2: hipLaunchKernelGGL((KERNEL<T, 2>), grid, dim3(kNT), SHMEM, st, a); break;          \
    case 3: hipLaunchKernelGGL((KERNEL<T, 3>), grid, dim3(kNT), SHMEM, st, a); break;          \
    case 4: hipLaunchKernelGGL((KERNEL<T, 4>), grid, dim3(kNT), SHMEM, st, a); break;          \
    default: return hipErrorNotSupported;                                                      \
  }

bool adaln_supported(int C, int dtype) {
  const int vec = dtype == 1 ? 8 : 4;
  return C % vec == 0 && C / vec <= 256;  // at most four 16-byte chunks per lane
}

hipError_t launch_adaln_fwd(const AdalnArgs& a, int dtype, hipStream_t st) {
  hipLaunchKernelGGL(adaln_mod_kernel, dim3(a.B), dim3(kNT), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(a.nwg, a.B);
  const size_t shmem = (size_t)4 * a.C * sizeof(float);
  if (dtype == 1) {
    TVM_ADALN_BY_SIZE(adaln_fwd_kernel, bf16, shmem)
  } else {
    TVM_ADALN_BY_SIZE(adaln_fwd_kernel, float, shmem)
  }
  return hipGetLastError();
}

hipError_t launch_adaln_bwd(const AdalnArgs& a, int dtype, hipStream_t st) {
  hipLaunchKernelGGL(adaln_mod_kernel, dim3(a.B), dim3(kNT), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(a.nwg, a.B);
  const size_t shmem = (size_t)6 * a.C * sizeof(float);
  if (dtype == 1) {
    TVM_ADALN_BY_SIZE(adaln_bwd_kernel, bf16, shmem)
  } else {
    TVM_ADALN_BY_SIZE(adaln_bwd_kernel, float, shmem)
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(adaln_sum_kernel, dim3((4 * a.C + kNT - 1) / kNT, a.B), dim3(kNT), 0, st, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(adaln_mod_bwd_kernel, dim3(a.B), dim3(kNT), 0, st, a);
  return hipGetLastError();
}

}  // namespace tvm
