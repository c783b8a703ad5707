// Microbenchmarks of the two ceilings the attention kernels are priced against, measured on the card itself:
// the rate of the one matrix-core instruction they use (v_mfma_f32_32x32x16_bf16) and the HBM rate of a plain
// copy and of a plain read.  Built into a library of its own (libtvmpeaks.so, used by bench.py only): nothing
// of it is part of the product library.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kAcc = 4;     // independent accumulators per wave
constexpr int kUnroll = 4;  // products per accumulator and loop iteration

// Every wave issues iters * kAcc * kUnroll products back to back; operands never change, results are summed into
// one float per thread so that nothing is optimised away.
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* __restrict__ out, int iters, float seed) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(seed + (float)(threadIdx.x & 7) * 0.001f);
    b[e] = (__bf16)(seed * 0.5f);
  }
  f32x16 acc[kAcc];
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int n = 0; n < kAcc; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same stream of products on operands that look like data: every accumulator has fragments of its own, filled
// with pseudo-random values in [-1, 1) that differ from lane to lane, and the two operands change places from one
// product of an accumulator to the next.  The rate in products per cycle is the same; what differs is the power the
// matrix cores draw with operand bits that toggle, and with it the clock the card holds.
// live_rows < 32: the first operand's rows from live_rows on are zero in every second product of an accumulator (the
// products where it is the A operand), as the rows of a padded head dim are in the output products of the attention
// kernels (8 of 32 live in the last block of d = 72).
__global__ __launch_bounds__(256) void mfma_rate_random_kernel(float* __restrict__ out, int iters, unsigned seed,
                                                               int live_rows) {
  bf16x8 a[kAcc], b[kAcc];
  unsigned h = seed ^ (blockIdx.x * 2654435761u) ^ (threadIdx.x * 40503u);
  const bool live = (int)(threadIdx.x & 31) < live_rows;  // (a lane holds row lane % 32 of the A operand)
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      a[n][e] = live ? (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.0f) - 1.0f) : (__bf16)0.f;
      h = h * 1664525u + 1013904223u;
      b[n][e] = (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.0f) - 1.0f);
    }
  f32x16 acc[kAcc];
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int n = 0; n < kAcc; ++n)
        acc[n] = (u & 1) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[n], a[(n + 1) % kAcc], acc[n], 0, 0, 0)
                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n], b[n], acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 16 bytes per thread and step, consecutive threads on consecutive chunks, four steps in flight.
__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    dst[i] = v0;
    dst[i + stride] = v1;
    dst[i + 2 * stride] = v2;
    dst[i + 3 * stride] = v3;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ out) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  unsigned x = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    x ^= v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = src[i];
    x ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (x == 0x9E3779B9u) out[0] = x;  // (practically never: the read must not be optimised away)
}

// What a backward kernel that forms dQ, dtQ in its key-side pass would have to do: every wave adds float32 partial
// tiles into the query-side gradients of its head, which other workgroups of the head add to as well.  Each
// workgroup (four waves) owns 1/wgs_per_head of a head's keys and walks the head's `rows` queries in blocks of
// 32; per block every wave adds 2 x 32 x cols floats, 256 contiguous bytes per wave instruction (the friendliest
// pattern a kernel could stage through LDS), to the head's [2][rows][cols] region, which the XCD's L2 holds.
__global__ __launch_bounds__(256) void atomic_tile_kernel(float* __restrict__ base, int wgs_per_head, int rows, int cols,
                                                          int reps, int waves) {
  if ((int)(threadIdx.x >> 6) >= waves) return;  // (waves < 4: as if the workgroup had summed its waves' tiles first)
  const int head = blockIdx.x / wgs_per_head;
  const int lane = threadIdx.x & 63;
  float* region = base + (size_t)head * 2 * rows * cols;
  const float v = 1.0f + (float)(threadIdx.x & 3);
  for (int rep = 0; rep < reps; ++rep)
    for (int qb = 0; qb < rows / 32; ++qb) {
      float* tile = region + (size_t)qb * 32 * cols;
      for (int t = 0; t < 2; ++t)
        for (int e = lane; e < 32 * cols; e += 64) atomicAdd(tile + (size_t)t * rows * cols + e, v);
    }
}

}  // namespace

extern "C" {

// Launches the matrix-core rate kernel on `blocks` workgroups of four waves.  `out`: device memory for
// blocks * 256 floats.  Returns the number of floating-point operations the launch performs (0 on a bad argument
// or a failed launch): blocks * 4 waves * iters * 16 products * 32 * 32 * 16 * 2.
double tvmpeaks_mfma_bf16(int blocks, int iters, void* out, void* hip_stream) {
  if (blocks < 1 || iters < 1 || !out) return 0.0;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<float*>(out), iters, 1.0f);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)blocks * 4.0 * iters * (kAcc * kUnroll) * (32.0 * 32.0 * 16.0 * 2.0);
}

// The same launch with operands that differ from product to product (see mfma_rate_random_kernel).
double tvmpeaks_mfma_bf16_random(int blocks, int iters, void* out, void* hip_stream) {
  if (blocks < 1 || iters < 1 || !out) return 0.0;
  hipLaunchKernelGGL(mfma_rate_random_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<float*>(out), iters, 12345u, 32);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)blocks * 4.0 * iters * (kAcc * kUnroll) * (32.0 * 32.0 * 16.0 * 2.0);
}
// ... and with only `live_rows` (1..32) of the 32 rows of one operand non-zero: what padded products cost.  Returns the
// operations issued (zeros included), as above.
double tvmpeaks_mfma_bf16_random_padded(int blocks, int iters, int live_rows, void* out, void* hip_stream) {
  if (blocks < 1 || iters < 1 || live_rows < 1 || live_rows > 32 || !out) return 0.0;
  hipLaunchKernelGGL(mfma_rate_random_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<float*>(out), iters, 12345u, live_rows);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)blocks * 4.0 * iters * (kAcc * kUnroll) * (32.0 * 32.0 * 16.0 * 2.0);
}

// Copies `bytes` (a multiple of 16; both pointers 16-byte aligned, device memory).  Returns 0 on success.
int tvmpeaks_copy(void* dst, const void* src, size_t bytes, int blocks, void* hip_stream) {
  if (!dst || !src || bytes % 16 != 0 || blocks < 1 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) return -1;
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Reads `bytes` once.  `out`: device memory for one unsigned.  Returns 0 on success.
int tvmpeaks_read(const void* src, size_t bytes, void* out, int blocks, void* hip_stream) {
  if (!src || !out || bytes % 16 != 0 || blocks < 1 || (uintptr_t)src % 16 != 0) return -1;
  hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const u32x4*>(src), bytes / 16, static_cast<unsigned*>(out));
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Launches the atomic-add pattern above on heads * wgs_per_head workgroups.  `base`: device memory for
// heads * 2 * rows * cols floats (rows a multiple of 32).  Returns the number of bytes added atomically (0 on a bad
// argument or a failed launch): heads * wgs_per_head * waves * reps * rows * cols * 2 tensors * 4 (waves: 1..4 of a
// workgroup's waves take part).
double tvmpeaks_atomic_add(void* base, int heads, int wgs_per_head, int rows, int cols, int reps, int waves,
                           void* hip_stream) {
  if (!base || heads < 1 || wgs_per_head < 1 || rows < 32 || rows % 32 != 0 || cols < 1 || reps < 1 || waves < 1 || waves > 4)
    return 0.0;
  hipLaunchKernelGGL(atomic_tile_kernel, dim3(heads * wgs_per_head), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<float*>(base), wgs_per_head, rows, cols, reps, waves);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)heads * wgs_per_head * waves * reps * rows * cols * 2.0 * 4.0;
}

}  // extern "C"
