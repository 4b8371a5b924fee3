// Output head for the first token (Section 3 measures the time to it): logits of a few rows against
// the whole vocabulary, and the greedy choice.  The projection itself runs through the bf16 MFMA
// GEMM where the shape allows; what is here is the any-shape fp32-FMA projection and the argmax.
#include "common.h"

namespace alora {

// logits[b, v] = <xh[b], W[v]>: one wave per vocabulary row, every row of xh against it
template <typename T>
__global__ __launch_bounds__(256) void lm_logits_plain_kernel(const T *__restrict__ xh, const T *__restrict__ W, int B,
                                                              int V, int d, float *__restrict__ logits) {
  const int lane = threadIdx.x & 63;
  const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (v >= V) return;
  const T *w = W + (int64_t)v * d;
  for (int b0 = 0; b0 < B; b0 += 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = lane; c < d; c += 64) {
      const float wv = to_f32<T>(w[c]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (b0 + i < B) acc[i] += wv * to_f32<T>(xh[(int64_t)(b0 + i) * d + c]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float t = wave_sum(acc[i]);
      if (lane == 0 && b0 + i < B) logits[(int64_t)(b0 + i) * V + v] = t;
    }
  }
}

// (value, index) with the larger value, the lower index among equals; NaN never wins
__device__ __forceinline__ void take_better(float &bv, int &bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

constexpr int ARGMAX_SLAB = 8192;

__global__ __launch_bounds__(256) void argmax_partial_kernel(const float *__restrict__ logits, int V, int n_slabs,
                                                             float *__restrict__ pv, int *__restrict__ pi) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int b = blockIdx.y, slab = blockIdx.x;
  const int lo = slab * ARGMAX_SLAB, hi = min(V, lo + ARGMAX_SLAB);
  const float *row = logits + (int64_t)b * V;
  float bv = -INFINITY;
  int bi = lo;                                     // an all-NaN or all -inf slab answers its first index
  for (int c = lo + threadIdx.x; c < hi; c += 256) take_better(bv, bi, row[c], c);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) take_better(bv, bi, __shfl_xor(bv, o, 64), __shfl_xor(bi, o, 64));
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) take_better(bv, bi, sv[w], si[w]);
    pv[b * n_slabs + slab] = bv;
    pi[b * n_slabs + slab] = bi;
  }
}

__global__ __launch_bounds__(64) void argmax_final_kernel(const float *__restrict__ pv, const int *__restrict__ pi,
                                                          int n_slabs, int32_t *__restrict__ token) {
  const int b = blockIdx.x;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int s = threadIdx.x; s < n_slabs; s += 64) take_better(bv, bi, pv[b * n_slabs + s], pi[b * n_slabs + s]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) take_better(bv, bi, __shfl_xor(bv, o, 64), __shfl_xor(bi, o, 64));
  if (threadIdx.x == 0) token[b] = bi == 0x7fffffff ? 0 : bi;
}

template <typename T>
void launch_lm_logits_plain(const T *xh, const T *W, int B, int V, int d, float *logits, hipStream_t s) {
  if (B == 0 || V == 0) return;
  hipLaunchKernelGGL(lm_logits_plain_kernel<T>, dim3((V + 3) / 4), dim3(256), 0, s, xh, W, B, V, d, logits);
}
template void launch_lm_logits_plain<float>(const float *, const float *, int, int, int, float *, hipStream_t);
template void launch_lm_logits_plain<bf16>(const bf16 *, const bf16 *, int, int, int, float *, hipStream_t);

int argmax_slabs(int V) { return (V + ARGMAX_SLAB - 1) / ARGMAX_SLAB; }

void launch_argmax(const float *logits, int B, int V, float *pv, int *pi, int32_t *token, hipStream_t s) {
  if (B == 0) return;
  const int n_slabs = argmax_slabs(V);
  hipLaunchKernelGGL(argmax_partial_kernel, dim3(n_slabs, B), dim3(256), 0, s, logits, V, n_slabs, pv, pi);
  hipLaunchKernelGGL(argmax_final_kernel, dim3(B), dim3(64), 0, s, pv, pi, n_slabs, token);
}

}  // namespace alora
