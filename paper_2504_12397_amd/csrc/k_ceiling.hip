// Measured ceilings of the machine the library runs on, for pricing the kernels next to the
// published peaks: a register-only bf16 MFMA loop and a streaming read of a buffer far larger
// than the last-level cache.
#include "mfma_kernels.h"

namespace alora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// every wave issues `iters` x 8 independent 32x32x16 MFMAs (8 accumulators, no memory traffic)
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(int iters, float *sink) {
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  const u32x4 ua = u32x4{0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 a = __builtin_bit_cast(bf16x8, ua), b = a;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0];
  if (s == 12345.678f) sink[0] = s;      // keeps the loop alive
}

// The same loop fed with operands that differ per lane, per register and per instruction
// (pseudo-random bf16 values in [1, 2) and their negatives): the clock the chip sustains depends on
// how much the operand bits toggle, so this is the ceiling a kernel working on real data can reach.
__global__ __launch_bounds__(256) void mfma_ceiling_random_kernel(int iters, float *sink) {
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  u32x4 fa[8], fb[8];
  uint32_t h = (threadIdx.x + 1u) * 2654435761u ^ (blockIdx.x * 40503u);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      h = h * 1664525u + 1013904223u;
      // two bf16 per word: random sign and mantissa, exponent of 1.0
      w[j] = ((h >> 8) & 0x807f807fu) | 0x3f803f80u;
    }
    fa[i] = u32x4{w[0], w[1], w[2], w[3]};
    fb[i] = u32x4{w[4], w[5], w[6], w[7]};
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                       __builtin_bit_cast(bf16x8, fb[(i + it) & 7]), acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0];
  if (s == 12345.678f) sink[0] = s;
}

__global__ __launch_bounds__(256) void read_ceiling_kernel(const u32x4 *__restrict__ src, int64_t n, uint32_t *sink) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * 256;
  uint32_t x = 0;
  for (; i + 7 * stride < n; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) x ^= v[u].x ^ v[u].w;
  }
  if (x == 0x12345678u) sink[0] = x;
}

// kind 0: bf16 MFMA TFLOP/s, constant operands; kind 1: HBM read GB/s; kind 2: bf16 MFMA TFLOP/s on
// random operands.  Returns a negative value on a HIP error.
double measure_ceiling(int kind, int n_cu, hipStream_t s) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.0;
  double out = -1.0;
  float ms = 0.f;
  if (kind == 0 || kind == 2) {
    float *sink = nullptr;
    if (hipMalloc((void **)&sink, 256) != hipSuccess) return -1.0;
    const int iters = 4096, grid = n_cu * 8;
    auto kern = kind == 0 ? mfma_ceiling_kernel : mfma_ceiling_random_kernel;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, s, 64, sink);
    (void)hipEventRecord(e0, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, s, iters, sink);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f)
      out = (double)grid * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12;
    (void)hipFree(sink);
  } else {
    const int64_t bytes = (int64_t)4 << 30;
    u32x4 *buf = nullptr;
    uint32_t *sink = nullptr;
    if (hipMalloc((void **)&buf, bytes) != hipSuccess) return -1.0;
    if (hipMalloc((void **)&sink, 256) != hipSuccess) { (void)hipFree(buf); return -1.0; }
    (void)hipMemsetAsync(buf, 1, bytes, s);
    const int64_t n = bytes / 16;
    hipLaunchKernelGGL(read_ceiling_kernel, dim3(n_cu * 8), dim3(256), 0, s, buf, n, sink);
    (void)hipEventRecord(e0, s);
    for (int r = 0; r < 4; ++r)
      hipLaunchKernelGGL(read_ceiling_kernel, dim3(n_cu * 8), dim3(256), 0, s, buf, n, sink);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f)
      out = 4.0 * (double)bytes / (ms * 1e-3) / 1e9;
    (void)hipFree(buf);
    (void)hipFree(sink);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return out;
}

}  // namespace alora
