// The activation between the MLP's two linear layers, with its JVP tangent and its backward (the MLP branch of the
// block in Terminal Velocity Matching, App. "Full Description of Normalization of Modulation"; the network's JVP,
// Sec. 4, runs through it).  The paper does not name the activation; DiT's is taken, the GELU in its tanh form:
//     gelu(u) = u/2 (1 + t),   t = tanh(w),   w = k (u + c u^3),   k = sqrt(2/pi),  c = 0.044715
//     a = gelu(u),   ta = gelu'(u) tu
//     gelu'  = (1 + t)/2 + u/2 (1 - t^2) w'                      w'  = k (1 + 3 c u^2)
//     gelu'' = (1 - t^2) w' + u/2 (1 - t^2) (w'' - 2 t w'^2)      w'' = 6 k c u
// Backward of <ga, a> + <gta, ta>:  gu = ga gelu' + gta tu gelu'',  gtu = gta gelu'.
// Pointwise: 16 bytes per thread and tensor, float32 arithmetic, tanh(w) = 1 - 2 / (exp(2w) + 1) (exact limits for
// large |w|: exp overflows to inf or underflows to 0).  About as much unpacked float32 arithmetic as memory time.
#include "tvm_common.h"

namespace tvm {
namespace {

#ifndef GELU_UNROLL
#define GELU_UNROLL 1     // chunks per thread in flight (1 with a thread per chunk measured best: 108 / 168 us
#define GELU_MAXGRID 65535  // forward / backward at 16 x 1024 x 4608 against 114 / 177 us with 4 and 8192 workgroups)
#endif
constexpr int kNT = 256, kUnroll = GELU_UNROLL;
constexpr float kK = 0.7978845608028654f, kC = 0.044715f, kTwoLog2e = 2.8853900817779268f;

template <typename T>
struct alignas(16) Chunk {
  static constexpr int VEC = 16 / sizeof(T);
  T v[VEC];
};
template <typename T>
__device__ __forceinline__ void widen(float (&out)[Chunk<T>::VEC], const uint4& raw) {
  const Chunk<T> c = __builtin_bit_cast(Chunk<T>, raw);
#pragma unroll
  for (int e = 0; e < Chunk<T>::VEC; ++e) out[e] = (float)c.v[e];
}
template <typename T>
__device__ __forceinline__ uint4 narrow(const float (&in)[Chunk<T>::VEC]) {
  Chunk<T> c;
#pragma unroll
  for (int e = 0; e < Chunk<T>::VEC; ++e) c.v[e] = (T)in[e];
  return __builtin_bit_cast(uint4, c);
}

// Loads of data that is touched once are non-temporal (bit 0 of GELU_NT; measured 5.5 % faster, forward and
// backward); non-temporal stores (bit 1) change nothing.
#ifndef GELU_NT
#define GELU_NT 1
#endif
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_once(const uint4* p) {
#if GELU_NT & 1
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
#else
  return *p;
#endif
}
__device__ __forceinline__ void st_once(uint4* p, uint4 v) {
#if GELU_NT & 2
  __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
#else
  *p = v;
#endif
}

struct Gelu {
  float half_1pt, g1, g2;  // (1 + t)/2, gelu', gelu''
};
// With e = exp(2w) and r = 1/(e + 1):  t = 1 - 2r,  (1 + t)/2 = 1 - r =: h,  1 - t^2 = 4 r h.  For large |w| the
// exponential overflows to inf (r = 0, h = 1) or underflows to 0 (r = 1, h = 0): the limits come out exact.
template <bool SECOND>
__device__ __forceinline__ Gelu gelu_parts(float u) {
  const float u2 = u * u;
  const float e = __builtin_amdgcn_exp2f(u * fmaf(kTwoLog2e * kK * kC, u2, kTwoLog2e * kK));  // exp(2w)
  const float r = __builtin_amdgcn_rcpf(e + 1.0f);
  const float h = 1.0f - r;
  const float q = u * r * h;                               // u (1 - t^2) / 4
  const float wp = fmaf(3.0f * kK * kC, u2, kK);           // w'
  Gelu g;
  g.half_1pt = h;
  g.g1 = fmaf(2.0f * q, wp, h);
  // gelu'' = (1 - t^2) w' + u/2 (1 - t^2) (w'' - 2 t w'^2),  t = 1 - 2r
  g.g2 = SECOND ? fmaf(2.0f * q, fmaf(wp * wp, fmaf(4.0f, r, -2.0f), 6.0f * kK * kC * u), 4.0f * r * h * wp) : 0.f;
  return g;
}

// chunks: number of 16-byte chunks per tensor
template <typename T>
__global__ __launch_bounds__(kNT) void gelu_fwd_kernel(const uint4* __restrict__ u, const uint4* __restrict__ tu,
                                                        uint4* __restrict__ a, uint4* __restrict__ ta, long long chunks) {
  constexpr int VEC = Chunk<T>::VEC;
  const long long stride = (long long)gridDim.x * kNT;
  for (long long i0 = (long long)blockIdx.x * kNT + threadIdx.x; i0 < chunks; i0 += stride * kUnroll) {
    uint4 ru[kUnroll], rt[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {  // chunks past the end are read as the last one and not stored
      const long long i = i0 + k * stride < chunks ? i0 + k * stride : chunks - 1;
      ru[k] = ld_once(u + i);
      rt[k] = ld_once(tu + i);
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const long long i = i0 + k * stride;
      if (i >= chunks) break;
      float x[VEC], tx[VEC], y[VEC], ty[VEC];
      widen<T>(x, ru[k]);
      widen<T>(tx, rt[k]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const Gelu g = gelu_parts<false>(x[e]);
        y[e] = x[e] * g.half_1pt;
        ty[e] = g.g1 * tx[e];
      }
      st_once(a + i, narrow<T>(y));
      st_once(ta + i, narrow<T>(ty));
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kNT) void gelu_bwd_kernel(const uint4* __restrict__ u, const uint4* __restrict__ tu,
                                                        const uint4* __restrict__ ga, const uint4* __restrict__ gta,
                                                        uint4* __restrict__ gu, uint4* __restrict__ gtu, long long chunks) {
  constexpr int VEC = Chunk<T>::VEC;
  const long long stride = (long long)gridDim.x * kNT;
  for (long long i0 = (long long)blockIdx.x * kNT + threadIdx.x; i0 < chunks; i0 += stride * kUnroll) {
    uint4 ru[kUnroll], rt[kUnroll], rg[kUnroll], rgt[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const long long i = i0 + k * stride < chunks ? i0 + k * stride : chunks - 1;
      ru[k] = ld_once(u + i);
      rt[k] = ld_once(tu + i);
      rg[k] = ld_once(ga + i);
      rgt[k] = ld_once(gta + i);
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const long long i = i0 + k * stride;
      if (i >= chunks) break;
      float x[VEC], tx[VEC], g[VEC], gt[VEC], ox[VEC], otx[VEC];
      widen<T>(x, ru[k]);
      widen<T>(tx, rt[k]);
      widen<T>(g, rg[k]);
      widen<T>(gt, rgt[k]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const Gelu p = gelu_parts<true>(x[e]);
        ox[e] = fmaf(g[e], p.g1, gt[e] * tx[e] * p.g2);
        otx[e] = gt[e] * p.g1;
      }
      st_once(gu + i, narrow<T>(ox));
      st_once(gtu + i, narrow<T>(otx));
    }
  }
}

int grid_for(long long chunks) {
  const long long want = (chunks + (long long)kNT * kUnroll - 1) / ((long long)kNT * kUnroll);
  return (int)(want < 1 ? 1 : want > GELU_MAXGRID ? GELU_MAXGRID : want);
}

}  // namespace

hipError_t launch_gelu_fwd(long long n, int dtype, const void* u, const void* tu, void* a, void* ta, hipStream_t st) {
  const long long chunks = n / (dtype == 1 ? 8 : 4);
  const dim3 grid(grid_for(chunks));
  if (dtype == 1)
    hipLaunchKernelGGL(gelu_fwd_kernel<bf16>, grid, dim3(kNT), 0, st, (const uint4*)u, (const uint4*)tu, (uint4*)a,
                       (uint4*)ta, chunks);
  else
    hipLaunchKernelGGL(gelu_fwd_kernel<float>, grid, dim3(kNT), 0, st, (const uint4*)u, (const uint4*)tu, (uint4*)a,
                       (uint4*)ta, chunks);
  return hipGetLastError();
}

hipError_t launch_gelu_bwd(long long n, int dtype, const void* u, const void* tu, const void* ga, const void* gta,
                           void* gu, void* gtu, hipStream_t st) {
  const long long chunks = n / (dtype == 1 ? 8 : 4);
  const dim3 grid(grid_for(chunks));
  if (dtype == 1)
    hipLaunchKernelGGL(gelu_bwd_kernel<bf16>, grid, dim3(kNT), 0, st, (const uint4*)u, (const uint4*)tu,
                       (const uint4*)ga, (const uint4*)gta, (uint4*)gu, (uint4*)gtu, chunks);
  else
    hipLaunchKernelGGL(gelu_bwd_kernel<float>, grid, dim3(kNT), 0, st, (const uint4*)u, (const uint4*)tu,
                       (const uint4*)ga, (const uint4*)gta, (uint4*)gu, (uint4*)gtu, chunks);
  return hipGetLastError();
}

}  // namespace tvm
