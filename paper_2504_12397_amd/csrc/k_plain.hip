// Plain kernels: every step of the path in straightforward fp32-FMA HIP, for any dtype and
// any shape.  They are the fp32 path (small single-block configuration) and the fallback
// for shapes the MFMA kernels do not cover.
#include "common.h"

namespace alora {

// ---------------------------------------------------------------------------------------
// rotary table: table[pos * half + c] = (cos, sin)(pos * theta^(-2c/h)), evaluated in
// double so that positions in the tens of thousands keep full fp32 accuracy.
// ---------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2 *table, int n_pos, int half, double log2_theta) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)n_pos * half) return;
  int pos = (int)(i / half), c = (int)(i % half);
  double inv = exp2(-(double)c / (double)half * log2_theta);   // theta^(-2c/h), h = 2*half
  double ang = (double)pos * inv;
  double sn, cs;
  sincos(ang, &sn, &cs);
  table[i] = make_float2((float)cs, (float)sn);
}

// The same entries for the positions of given rows only: table[row * half + c] for position pos[row] (callers
// that may not allocate a table of all positions keep one line per row).  Same arithmetic, same bits.
__global__ void rope_rows_kernel(float2 *table, const int32_t *__restrict__ pos, int n_rows, int half, double log2_theta) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)n_rows * half) return;
  int row = (int)(i / half), c = (int)(i % half);
  double inv = exp2(-(double)c / (double)half * log2_theta);
  double ang = (double)pos[row] * inv;
  double sn, cs;
  sincos(ang, &sn, &cs);
  table[i] = make_float2((float)cs, (float)sn);
}

void launch_rope_rows(float2 *table, const int32_t *pos, int n_rows, int half_dim, float theta, hipStream_t s) {
  int64_t n = (int64_t)n_rows * half_dim;
  if (n == 0) return;
  hipLaunchKernelGGL(rope_rows_kernel, dim3((int)((n + 255) / 256)), dim3(256), 0, s, table, pos, n_rows, half_dim,
                     log2((double)theta));
}

void launch_rope_table(float2 *table, int n_pos, int half_dim, float theta, hipStream_t s) {
  int64_t n = (int64_t)n_pos * half_dim;
  if (n == 0) return;
  int grid = (int)((n + 255) / 256);
  hipLaunchKernelGGL(rope_table_kernel, dim3(grid), dim3(256), 0, s, table, n_pos, half_dim,
                     log2((double)theta));
}

// ---------------------------------------------------------------------------------------
// row preparation: per-row metadata, RMSNorm, and the low-rank down projection
// t = s_a * A_a x_hat for adapted rows (Eq.6's Delta applied right to left).
// One workgroup per packed row.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void prep_rows_kernel(const T *__restrict__ x, const T *__restrict__ gain,
                                                        float eps, int d, const SeqMeta *__restrict__ seqs,
                                                        int n_seqs, int pos_shift, const T *__restrict__ A, int rank,
                                                        int write_meta, T *__restrict__ xh,
                                                        float *__restrict__ tlow, bf16 *__restrict__ tlow16,
                                                        RowMeta rm) {
  extern __shared__ float xs[];
  __shared__ float red[4];
  __shared__ int s_adapter;
  __shared__ float s_scale;
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) {
    int adapter = -1;
    float scale = 0.f;
    if (seqs != nullptr) {
      int lo = 0, hi = n_seqs - 1;   // last sequence whose first row is <= row
      while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (seqs[mid].row_start <= row) lo = mid; else hi = mid - 1;
      }
      SeqMeta sm = seqs[lo];
      int pos = sm.P + pos_shift + (row - sm.row_start);
      if (sm.adapter >= 0 && pos >= sm.k) { adapter = sm.adapter; scale = sm.scale; }
      if (write_meta) {
        rm.seq[row] = lo;
        rm.pos[row] = pos;
        rm.adapter[row] = adapter;
        rm.slot[row] = sm.pool_off + pos;
      }
    }
    s_adapter = adapter;
    s_scale = scale;
  }
  const T *xr = x + (int64_t)row * d;
  float ssq = 0.f;
  for (int c = tid; c < d; c += 256) {
    float v = to_f32<T>(xr[c]);
    xs[c] = v;
    ssq += v * v;
  }
  ssq = wave_sum(ssq);
  if (lane == 0) red[wave] = ssq;
  __syncthreads();
  float rinv = 1.f;
  if (gain != nullptr) rinv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
  for (int c = tid; c < d; c += 256) {
    float v = xs[c];
    if (gain != nullptr) v = v * to_f32<T>(gain[c]) * rinv;
    T stored = from_f32<T>(v);
    xh[(int64_t)row * d + c] = stored;
    xs[c] = to_f32<T>(stored);      // the projections consume the stored (rounded) value
  }
  __syncthreads();
  const int a = s_adapter;
  if (a < 0 || rank == 0) return;
  const float scale = s_scale;
  for (int j = wave; j < 3 * rank; j += 4) {
    const T *ar = A + ((int64_t)a * 3 * rank + j) * d;
    float acc = 0.f;
    for (int c = lane; c < d; c += 64) acc += to_f32<T>(ar[c]) * xs[c];
    acc = wave_sum(acc);
    if (lane == 0) {
      const float t = scale * acc;
      if (tlow16) {
        // bf16 pair (hi, lo) with hi + lo = t to ~2^-17: the MFMA path feeds both as extra k-steps,
        // so the low-rank term keeps fp32-level accuracy.  Layout [row][p][hi|lo][rank].
        const int p = j / rank, jj = j % rank;
        const bf16 hi = (bf16)t;
        bf16 *dst = tlow16 + (((int64_t)row * 3 + p) * 2) * rank + jj;
        dst[0] = hi;
        dst[rank] = (bf16)(t - (float)hi);
      } else {
        tlow[(int64_t)row * 3 * rank + j] = t;
      }
    }
  }
}

template <typename T>
void launch_prep_rows(const T *x, const T *gain, float eps, int T_rows, int d, const SeqMeta *seqs,
                      int n_seqs, int pos_shift, const T *A, int rank, bool write_meta, T *xh, float *tlow,
                      bf16 *tlow16, RowMeta rm, hipStream_t s) {
  if (T_rows == 0) return;
  hipLaunchKernelGGL((prep_rows_kernel<T>), dim3(T_rows), dim3(256), (size_t)d * sizeof(float), s, x, gain,
                     eps, d, seqs, n_seqs, pos_shift, A, rank, write_meta ? 1 : 0, xh, tlow, tlow16, rm);
}
template void launch_prep_rows<float>(const float *, const float *, float, int, int, const SeqMeta *, int, int,
                                      const float *, int, bool, float *, float *, bf16 *, RowMeta, hipStream_t);
template void launch_prep_rows<bf16>(const bf16 *, const bf16 *, float, int, int, const SeqMeta *, int, int,
                                     const bf16 *, int, bool, bf16 *, float *, bf16 *, RowMeta, hipStream_t);

// ---------------------------------------------------------------------------------------
// plain tiled GEMM  C[M,N] = A[M,K] B[N,K]^T, 64x64 tile, 16-deep, 4x4 outputs per thread
// ---------------------------------------------------------------------------------------
struct LoraEpi {
  const float *tlow;
  const void *Bq, *Bk, *Bv;
  const int32_t *row_adapter;
  int rank, n_q, n_kv;
};

template <typename T, int MODE>
__global__ __launch_bounds__(256) void gemm_plain_kernel(const T *__restrict__ A, const T *__restrict__ B,
                                                         const T *__restrict__ R, void *__restrict__ Cv,
                                                         int M, int N, int K, LoraEpi epi) {
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int kk = k0 + lk + i;
      int ar = m0 + lr, br = n0 + lr;
      As[lk + i][lr] = (ar < M && kk < K) ? to_f32<T>(A[(int64_t)ar * K + kk]) : 0.f;
      Bs[lk + i][lr] = (br < N && kk < K) ? to_f32<T>(B[(int64_t)br * K + kk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = m0 + ty * 4 + i;
    if (row >= M) continue;
    int a = -1;
    if (MODE == EPI_F32_LORA) a = epi.row_adapter[row];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int col = n0 + tx * 4 + j;
      if (col >= N) continue;
      float v = acc[i][j];
      if (MODE == EPI_F32_LORA) {
        if (a >= 0) {     // adapted row: add s * B (A x); other rows get nothing added
          const int r = epi.rank;
          const T *bp;
          int p;
          if (col < epi.n_q) { p = 0; bp = (const T *)epi.Bq + ((int64_t)a * epi.n_q + col) * r; }
          else if (col < epi.n_q + epi.n_kv) { p = 1; bp = (const T *)epi.Bk + ((int64_t)a * epi.n_kv + (col - epi.n_q)) * r; }
          else { p = 2; bp = (const T *)epi.Bv + ((int64_t)a * epi.n_kv + (col - epi.n_q - epi.n_kv)) * r; }
          const float *t = epi.tlow + (int64_t)row * 3 * r + p * r;
          float lo = 0.f;
          for (int jj = 0; jj < r; ++jj) lo += t[jj] * to_f32<T>(bp[jj]);
          v += lo;
        }
        ((float *)Cv)[(int64_t)row * N + col] = v;
      } else if (MODE == EPI_STORE_F32) {
        ((float *)Cv)[(int64_t)row * N + col] = v;
      } else {
        if (MODE == EPI_STORE_RESIDUAL) v += to_f32<T>(R[(int64_t)row * N + col]);
        ((T *)Cv)[(int64_t)row * N + col] = from_f32<T>(v);
      }
    }
  }
}

template <typename T>
void launch_qkv_gemm_plain(const T *xh, const T *W, const float *tlow, const T *Bq, const T *Bk,
                           const T *Bv, const LayerDims &L, RowMeta rm, int T_rows, float *Y,
                           hipStream_t s) {
  if (T_rows == 0) return;
  LoraEpi epi{tlow, Bq, Bk, Bv, rm.adapter, L.rank, L.n_q, L.n_kv};
  dim3 grid((L.n_qkv + 63) / 64, (T_rows + 63) / 64);
  hipLaunchKernelGGL((gemm_plain_kernel<T, EPI_F32_LORA>), grid, dim3(256), 0, s, xh, W, (const T *)nullptr,
                     (void *)Y, T_rows, L.n_qkv, L.d, epi);
}
template void launch_qkv_gemm_plain<float>(const float *, const float *, const float *, const float *,
                                           const float *, const float *, const LayerDims &, RowMeta, int,
                                           float *, hipStream_t);
template void launch_qkv_gemm_plain<bf16>(const bf16 *, const bf16 *, const float *, const bf16 *,
                                          const bf16 *, const bf16 *, const LayerDims &, RowMeta, int,
                                          float *, hipStream_t);

template <typename T>
void launch_gemm_plain(const T *A, const T *B, const T *R, T *C, int M, int N, int K, hipStream_t s) {
  if (M == 0 || N == 0) return;
  LoraEpi epi{};
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (R)
    hipLaunchKernelGGL((gemm_plain_kernel<T, EPI_STORE_RESIDUAL>), grid, dim3(256), 0, s, A, B, R, (void *)C,
                       M, N, K, epi);
  else
    hipLaunchKernelGGL((gemm_plain_kernel<T, EPI_STORE>), grid, dim3(256), 0, s, A, B, R, (void *)C, M, N, K,
                       epi);
}
template <typename T>
void launch_gemm_plain_f32(const T *A, const T *B, float *C, int M, int N, int K, hipStream_t s) {
  if (M == 0 || N == 0) return;
  LoraEpi epi{};
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  hipLaunchKernelGGL((gemm_plain_kernel<T, EPI_STORE_F32>), grid, dim3(256), 0, s, A, B, (const T *)nullptr, (void *)C, M,
                     N, K, epi);
}
template void launch_gemm_plain_f32<float>(const float *, const float *, float *, int, int, int, hipStream_t);
template void launch_gemm_plain_f32<bf16>(const bf16 *, const bf16 *, float *, int, int, int, hipStream_t);
template void launch_gemm_plain<float>(const float *, const float *, const float *, float *, int, int, int,
                                       hipStream_t);
template void launch_gemm_plain<bf16>(const bf16 *, const bf16 *, const bf16 *, bf16 *, int, int, int,
                                      hipStream_t);

// ---------------------------------------------------------------------------------------
// rotary embedding + cache append (Eq.3: K_{1:t} = [K_{1:t-1}; K_t]).
// ---------------------------------------------------------------------------------------
// One wave per (row, head slot), four slots per workgroup: slots 0..Hq-1 are query heads, then the
// key heads, then the value heads.  Every lane handles whole rotation pairs, all loads are
// independent.
template <typename T, bool MULTI>      // MULTI: Y arrives as several partial sums
__global__ __launch_bounds__(256) void rope_append_kernel(const float *__restrict__ Y, int n_parts,
                                                         int64_t part_stride, LayerDims L, RowMeta rm,
                                                         const float2 *__restrict__ table, int table_by_row,
                                                         float q_scale, int q_half, T *__restrict__ Q,
                                                         T *__restrict__ cacheK,
                                                         T *__restrict__ cacheV) {
  const int row = blockIdx.x, slot_id = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int h = L.head_dim, h2 = h >> 1;
  if (slot_id >= L.n_q_heads + 2 * L.n_kv_heads) return;
  const float *y = Y + (int64_t)row * L.n_qkv;
  // Y may arrive as n_parts partial sums over the reduction axis: add them in a fixed order
  // (the first eight are requested together: a loop over the run-time count costs a memory round trip per part)
  auto ysum = [&](const float *p) {
    if constexpr (!MULTI) return p[0];
    float t[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      if (s < n_parts) t[s] = p[(int64_t)s * part_stride];
    float v = t[0];
#pragma unroll
    for (int s = 1; s < 8; ++s)
      if (s < n_parts) v += t[s];
    for (int s = 8; s < n_parts; ++s) v += p[(int64_t)s * part_stride];
    return v;
  };
  if (slot_id < L.n_q_heads + L.n_kv_heads) {
    const bool is_q = slot_id < L.n_q_heads;
    const int head = is_q ? slot_id : slot_id - L.n_q_heads;
    const int base = (is_q ? 0 : L.n_q) + head * h;
    const float2 *tab = table + (int64_t)(table_by_row ? row : rm.pos[row]) * h2;
    T *dst = is_q ? Q + (int64_t)row * L.n_q + head * h : cacheK + rm.slot[row] * L.n_kv + head * h;
    // q_scale: the attention kernel that follows may want its queries premultiplied (softmax scale and
    // log2 e, so that its scores come out of the MFMA ready for exp2); keys are never scaled
    const float qs = is_q ? q_scale : 1.0f;
    for (int c = lane; c < h2; c += 64) {
      const float u = ysum(y + base + c), w = ysum(y + base + c + h2);
      const float2 cs = tab[c];
      const float lo = (u * cs.x - w * cs.y) * qs, hi = (w * cs.x + u * cs.y) * qs;
      if (is_q && q_half == 1) {
        // the MFMA attention kernels want their queries as fp16
        _Float16 *dq = reinterpret_cast<_Float16 *>(Q) + (int64_t)row * L.n_q + head * h;
        dq[c] = (_Float16)lo;
        dq[c + h2] = (_Float16)hi;
      } else if (is_q && q_half == 2) {
        // the plain attention kernel keeps them in fp32
        float *dq = reinterpret_cast<float *>(Q) + (int64_t)row * L.n_q + head * h;
        dq[c] = lo;
        dq[c + h2] = hi;
      } else {
        dst[c] = from_f32<T>(lo);
        dst[c + h2] = from_f32<T>(hi);
      }
    }
  } else {
    const int head = slot_id - L.n_q_heads - L.n_kv_heads;
    const float *yv = y + L.n_q + L.n_kv + head * h;
    T *dst = cacheV + rm.slot[row] * L.n_kv + head * h;
    for (int c = lane; c < h; c += 64) dst[c] = from_f32<T>(ysum(yv + c));
  }
}

template <typename T>
void launch_rope_append(const float *Y, int n_parts, const LayerDims &L, RowMeta rm, int T_rows,
                        const float2 *rope_table, bool table_by_row, float q_scale, int q_half, void *Q, T *cacheK,
                        T *cacheV, hipStream_t s) {
  if (T_rows == 0) return;
  dim3 grid(T_rows, (L.n_q_heads + 2 * L.n_kv_heads + 3) / 4);
  if (n_parts > 1)
    hipLaunchKernelGGL((rope_append_kernel<T, true>), grid, dim3(256), 0, s, Y, n_parts, (int64_t)T_rows * L.n_qkv, L, rm,
                       rope_table, table_by_row ? 1 : 0, q_scale, q_half, (T *)Q, cacheK, cacheV);
  else
    hipLaunchKernelGGL((rope_append_kernel<T, false>), grid, dim3(256), 0, s, Y, n_parts, (int64_t)T_rows * L.n_qkv, L, rm,
                       rope_table, table_by_row ? 1 : 0, q_scale, q_half, (T *)Q, cacheK, cacheV);
}
template void launch_rope_append<float>(const float *, int, const LayerDims &, RowMeta, int, const float2 *, bool, float, int,
                                        void *, float *, float *, hipStream_t);
template void launch_rope_append<bf16>(const float *, int, const LayerDims &, RowMeta, int, const float2 *, bool, float, int,
                                       void *, bf16 *, bf16 *, hipStream_t);

// ---------------------------------------------------------------------------------------
// plain split-KV attention (Eq.1 / Eq.4, causal, GQA).  One wave per (row, kv head, chunk of
// up to 8 query heads, key split).  Scores: one key per lane; values: lanes across head_dim.
// Partial layout: part[(((row*Hq + hq) * n_splits) + split) * (h + 2)] = acc[h], m, l.
// ---------------------------------------------------------------------------------------
#define ATT_GMAX 8
#define ATT_DMAX 4     // head_dim <= 256

template <typename T>
__global__ __launch_bounds__(64) void attn_partial_kernel(const float *__restrict__ Q, const T *__restrict__ cacheK,
                                                          const T *__restrict__ cacheV,
                                                          const SeqMeta *__restrict__ seqs, RowMeta rm,
                                                          LayerDims L, int n_splits, float *__restrict__ part) {
  extern __shared__ float smem[];       // qs[GMAX][h] then ps[GMAX][64]
  const int lane = threadIdx.x;
  const int h = L.head_dim;
  const int G = L.n_q_heads / L.n_kv_heads;
  const int row = blockIdx.x / L.n_kv_heads, g = blockIdx.x % L.n_kv_heads;
  const int split = blockIdx.y;
  const int g0 = blockIdx.z * ATT_GMAX;
  const int ng = min(ATT_GMAX, G - g0);
  float *qs = smem, *ps = smem + ATT_GMAX * h;
  const int n_keys = rm.pos[row] + 1;
  int chunk = (n_keys + n_splits - 1) / n_splits;
  chunk = (chunk + 63) & ~63;
  const int begin = split * chunk, end = min(n_keys, begin + chunk);
  const SeqMeta sm = seqs[rm.seq[row]];
  const float sm_scale = 1.0f / sqrtf((float)h);
  for (int i = lane; i < ng * h; i += 64) {
    int gi = i / h, c = i % h;
    qs[gi * h + c] = Q[(int64_t)row * L.n_q + (g * G + g0 + gi) * h + c] * sm_scale;
  }
  __syncthreads();
  float m[ATT_GMAX], l[ATT_GMAX], acc[ATT_GMAX][ATT_DMAX];
#pragma unroll
  for (int gi = 0; gi < ATT_GMAX; ++gi) {
    m[gi] = -INFINITY; l[gi] = 0.f;
#pragma unroll
    for (int dd = 0; dd < ATT_DMAX; ++dd) acc[gi][dd] = 0.f;
  }
  for (int t0 = begin; t0 < end; t0 += 64) {
    const int key = t0 + lane;
    const bool valid = key < end;
    float sc[ATT_GMAX];
#pragma unroll
    for (int gi = 0; gi < ATT_GMAX; ++gi) sc[gi] = 0.f;
    if (valid) {
      const T *kr = cacheK + seq_pool_row(sm, key) * L.n_kv + g * h;
      for (int c = 0; c < h; ++c) {
        float kv = to_f32<T>(kr[c]);
#pragma unroll
        for (int gi = 0; gi < ATT_GMAX; ++gi)
          if (gi < ng) sc[gi] += qs[gi * h + c] * kv;
      }
    }
    __syncthreads();      // previous tile's ps fully consumed
#pragma unroll
    for (int gi = 0; gi < ATT_GMAX; ++gi) {
      if (gi < ng) {
        float s = valid ? sc[gi] : -INFINITY;
        float mn = fmaxf(m[gi], wave_max(s));
        float p = valid ? __expf(s - mn) : 0.f;
        float corr = __expf(m[gi] - mn);
        l[gi] = l[gi] * corr + wave_sum(p);
        m[gi] = mn;
#pragma unroll
        for (int dd = 0; dd < ATT_DMAX; ++dd) acc[gi][dd] *= corr;
        ps[gi * 64 + lane] = p;
      }
    }
    __syncthreads();
    const int nk = min(64, end - t0);
    for (int j = 0; j < nk; ++j) {
      const T *vr = cacheV + seq_pool_row(sm, t0 + j) * L.n_kv + g * h;
#pragma unroll
      for (int dd = 0; dd < ATT_DMAX; ++dd) {
        int c = lane + 64 * dd;
        if (c < h) {
          float vv = to_f32<T>(vr[c]);
#pragma unroll
          for (int gi = 0; gi < ATT_GMAX; ++gi)
            if (gi < ng) acc[gi][dd] += ps[gi * 64 + j] * vv;
        }
      }
    }
  }
#pragma unroll
  for (int gi = 0; gi < ATT_GMAX; ++gi) {
    if (gi < ng) {
      float *o = part + (((int64_t)row * L.n_q_heads + (g * G + g0 + gi)) * n_splits + split) * (h + 2);
#pragma unroll
      for (int dd = 0; dd < ATT_DMAX; ++dd) {
        int c = lane + 64 * dd;
        if (c < h) o[c] = acc[gi][dd];
      }
      if (lane == 0) { o[h] = m[gi]; o[h + 1] = l[gi]; }
    }
  }
}

// One wave per (row, query head), four per workgroup.  The per-split maxima are fetched by the
// first lanes in parallel, and the accumulators are read MU splits at a time (added in ascending order whatever
// MU is: a short batch over a long cache has few (row, head) pairs and a hundred records each, and every group
// of records is a memory round trip).
template <typename T, int MU>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part, LayerDims L, int n_splits,
                                                         int64_t n_rh, T *__restrict__ out) {
  const int lane = threadIdx.x & 63, h = L.head_dim;
  const int64_t rh = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);       // row * Hq + hq
  if (rh >= n_rh) return;
  const float *p = part + rh * n_splits * (h + 2);
  float M = -INFINITY;
  for (int s0 = 0; s0 < n_splits; s0 += 64) {
    const int s = s0 + lane;
    M = fmaxf(M, s < n_splits ? p[s * (h + 2) + h] : -INFINITY);
  }
  M = wave_max(M);
  float denom = 0.f;
  float acc[ATT_DMAX] = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < n_splits; s0 += MU) {
    float ms[MU], ls[MU], v[MU][ATT_DMAX];
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      const int s = min(s0 + u, n_splits - 1);
      const float *ps = p + s * (h + 2);
      ms[u] = ps[h];
      ls[u] = ps[h + 1];
#pragma unroll
      for (int dd = 0; dd < ATT_DMAX; ++dd) {
        const int c = lane + 64 * dd;
        v[u][dd] = c < h ? ps[c] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      const float w = (s0 + u >= n_splits || ms[u] == -INFINITY) ? 0.f : __expf(ms[u] - M);
      denom += w * ls[u];
#pragma unroll
      for (int dd = 0; dd < ATT_DMAX; ++dd) acc[dd] += w * v[u][dd];
    }
  }
  const float inv = 1.0f / denom;
#pragma unroll
  for (int dd = 0; dd < ATT_DMAX; ++dd) {
    int c = lane + 64 * dd;
    if (c < h) out[rh * h + c] = from_f32<T>(acc[dd] * inv);
  }
}

// The same merge for few (row, head) pairs with many records each (a handful of sequences decoding over long
// caches): one workgroup per pair, its four waves take the records w, w + 4, w + 8, ... (eight in flight each, two
// columns per lane and load), and their sums are added in wave order.  head_dim <= 128.
template <typename T>
__global__ __launch_bounds__(256) void attn_merge_wide_kernel(const float *__restrict__ part, LayerDims L, int n_splits,
                                                              T *__restrict__ out) {
  __shared__ float s_acc[4][130];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = L.head_dim;
  const int64_t rh = blockIdx.x;
  const float *p = part + rh * n_splits * (h + 2);
  float M = -INFINITY;
  for (int s0 = 0; s0 < n_splits; s0 += 64) {
    const int s = s0 + lane;
    M = fmaxf(M, s < n_splits ? p[s * (h + 2) + h] : -INFINITY);
  }
  M = wave_max(M);
  float denom = 0.f;
  float2 acc = make_float2(0.f, 0.f);
  const bool col_ok = 2 * lane < h;
  constexpr int MU = 8;
  for (int s0 = wave; s0 < n_splits; s0 += 4 * MU) {
    float ms[MU], ls[MU];
    float2 v[MU];
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      const int s = min(s0 + 4 * u, n_splits - 1);
      const float *ps = p + s * (h + 2);
      ms[u] = ps[h];
      ls[u] = ps[h + 1];
      v[u] = col_ok ? *reinterpret_cast<const float2 *>(ps + 2 * lane) : make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      const float w = (s0 + 4 * u >= n_splits || ms[u] == -INFINITY) ? 0.f : __expf(ms[u] - M);
      denom += w * ls[u];
      acc.x += w * v[u].x;
      acc.y += w * v[u].y;
    }
  }
  if (col_ok) { s_acc[wave][2 * lane] = acc.x; s_acc[wave][2 * lane + 1] = acc.y; }
  if (lane == 0) s_acc[wave][128] = denom;
  __syncthreads();
  if (wave == 0 && col_ok) {
    const float d = ((s_acc[0][128] + s_acc[1][128]) + s_acc[2][128]) + s_acc[3][128];
    const float inv = 1.0f / d;
    const float x = ((s_acc[0][2 * lane] + s_acc[1][2 * lane]) + s_acc[2][2 * lane]) + s_acc[3][2 * lane];
    const float y = ((s_acc[0][2 * lane + 1] + s_acc[1][2 * lane + 1]) + s_acc[2][2 * lane + 1]) + s_acc[3][2 * lane + 1];
    out[rh * h + 2 * lane] = from_f32<T>(x * inv);
    out[rh * h + 2 * lane + 1] = from_f32<T>(y * inv);
  }
}

size_t attn_plain_partial_floats(const LayerDims &L, int T_rows, int n_splits) {
  return (size_t)T_rows * L.n_q_heads * n_splits * (L.head_dim + 2);
}

template <typename T>
void launch_attn_plain(const float *Q, const T *cacheK, const T *cacheV, const SeqMeta *seqs, RowMeta rm,
                       const LayerDims &L, int T_rows, int n_splits, float *partials, hipStream_t s) {
  if (T_rows == 0) return;
  const int G = L.n_q_heads / L.n_kv_heads;
  dim3 grid(T_rows * L.n_kv_heads, n_splits, (G + ATT_GMAX - 1) / ATT_GMAX);
  size_t smem = (size_t)(ATT_GMAX * L.head_dim + ATT_GMAX * 64) * sizeof(float);
  hipLaunchKernelGGL((attn_partial_kernel<T>), grid, dim3(64), smem, s, Q, cacheK, cacheV, seqs, rm, L, n_splits,
                     partials);
}
template void launch_attn_plain<float>(const float *, const float *, const float *, const SeqMeta *, RowMeta,
                                       const LayerDims &, int, int, float *, hipStream_t);
template void launch_attn_plain<bf16>(const float *, const bf16 *, const bf16 *, const SeqMeta *, RowMeta,
                                      const LayerDims &, int, int, float *, hipStream_t);

template <typename T>
void launch_attn_merge(const float *partials, const LayerDims &L, int T_rows, int n_splits, T *out, hipStream_t s) {
  if (T_rows == 0) return;
  const int64_t n_rh = (int64_t)T_rows * L.n_q_heads;
  if (n_splits >= 16 && n_rh <= 512 && L.head_dim <= 128 && L.head_dim % 2 == 0)
    hipLaunchKernelGGL((attn_merge_wide_kernel<T>), dim3((unsigned)n_rh), dim3(256), 0, s, partials, L, n_splits, out);
  else if (n_splits > 16)
    hipLaunchKernelGGL((attn_merge_kernel<T, 32>), dim3((unsigned)((n_rh + 3) / 4)), dim3(256), 0, s, partials, L, n_splits,
                       n_rh, out);
  else
    hipLaunchKernelGGL((attn_merge_kernel<T, 8>), dim3((unsigned)((n_rh + 3) / 4)), dim3(256), 0, s, partials, L, n_splits,
                       n_rh, out);
}
template void launch_attn_merge<float>(const float *, const LayerDims &, int, int, float *, hipStream_t);
template void launch_attn_merge<bf16>(const float *, const LayerDims &, int, int, bf16 *, hipStream_t);

// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void silu_mul_kernel(const T *__restrict__ gate, const T *__restrict__ up, T *__restrict__ out,
                                int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float gv = to_f32<T>(gate[i]);
    float uv = to_f32<T>(up[i]);
    out[i] = from_f32<T>(gv / (1.0f + __expf(-gv)) * uv);
  }
}

template <typename T>
void launch_silu_mul(const T *gate, const T *up, T *out, int64_t n, hipStream_t s) {
  if (n == 0) return;
  int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL((silu_mul_kernel<T>), dim3(grid), dim3(256), 0, s, gate, up, out, n);
}
template <typename T>
__global__ void silu_mul_f32_kernel(const float *__restrict__ gate, const float *__restrict__ up, T *__restrict__ out,
                                    int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const float gv = gate[i];
    out[i] = from_f32<T>(gv / (1.0f + __expf(-gv)) * up[i]);
  }
}
template <typename T>
void launch_silu_mul_f32(const float *gate, const float *up, T *out, int64_t n, hipStream_t s) {
  if (n == 0) return;
  int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL((silu_mul_f32_kernel<T>), dim3(grid), dim3(256), 0, s, gate, up, out, n);
}
template void launch_silu_mul_f32<float>(const float *, const float *, float *, int64_t, hipStream_t);
template void launch_silu_mul_f32<bf16>(const float *, const float *, bf16 *, int64_t, hipStream_t);

template <typename T>
__global__ void residual_store_kernel(const float *__restrict__ C, const T *__restrict__ R, T *__restrict__ out,
                                      int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = from_f32<T>(C[i] + (R != nullptr ? to_f32<T>(R[i]) : 0.f));
}
template <typename T>
void launch_residual_store(const float *C, const T *R, T *out, int64_t n, hipStream_t s) {
  if (n == 0) return;
  int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL((residual_store_kernel<T>), dim3(grid), dim3(256), 0, s, C, R, out, n);
}
template void launch_residual_store<float>(const float *, const float *, float *, int64_t, hipStream_t);
template void launch_residual_store<bf16>(const float *, const bf16 *, bf16 *, int64_t, hipStream_t);
template void launch_silu_mul<float>(const float *, const float *, float *, int64_t, hipStream_t);
template void launch_silu_mul<bf16>(const bf16 *, const bf16 *, bf16 *, int64_t, hipStream_t);

// Gated low-rank term of Eq.6 added to an already computed linear, any shape and dtype:
// C[row, :] += s_a * B_a (A_{a,part} x[row]) for adapted rows (a = row_adapter[row] >= 0).  One workgroup per row.
template <typename T, typename TC>
__global__ __launch_bounds__(256) void lowrank_add_plain_kernel(const T *__restrict__ x, int K, const T *__restrict__ A,
                                                                int parts, int part, const T *__restrict__ B, int N,
                                                                int rank, const int32_t *__restrict__ row_adapter,
                                                                const float *__restrict__ scale, TC *__restrict__ C) {
  __shared__ float t[256];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int a = row_adapter[row];
  if (a < 0) return;
  const T *xr = x + (int64_t)row * K;
  const float sc = scale[a];
  for (int j = wave; j < rank; j += 4) {
    const T *ar = A + (((int64_t)a * parts + part) * rank + j) * K;
    float acc = 0.f;
    for (int c = lane; c < K; c += 64) acc += to_f32<T>(ar[c]) * to_f32<T>(xr[c]);
    acc = wave_sum(acc);
    if (lane == 0) t[j] = acc * sc;
  }
  __syncthreads();
  for (int col = tid; col < N; col += 256) {
    const T *br = B + ((int64_t)a * N + col) * rank;
    float acc = 0.f;
    for (int j = 0; j < rank; ++j) acc += to_f32<T>(br[j]) * t[j];
    const int64_t o = (int64_t)row * N + col;
    C[o] = from_f32<TC>(to_f32<TC>(C[o]) + acc);
  }
}

template <typename T, typename TC>
void launch_lowrank_add_plain(const T *x, int K, const T *A, int parts, int part, const T *B, int N, int rank,
                              const int32_t *row_adapter, const float *scale, TC *C, int M, hipStream_t s) {
  if (M == 0) return;
  hipLaunchKernelGGL((lowrank_add_plain_kernel<T, TC>), dim3(M), dim3(256), 0, s, x, K, A, parts, part, B, N, rank,
                     row_adapter, scale, C);
}
template void launch_lowrank_add_plain<float, float>(const float *, int, const float *, int, int, const float *, int, int,
                                                     const int32_t *, const float *, float *, int, hipStream_t);
template void launch_lowrank_add_plain<bf16, bf16>(const bf16 *, int, const bf16 *, int, int, const bf16 *, int, int,
                                                   const int32_t *, const float *, bf16 *, int, hipStream_t);
template void launch_lowrank_add_plain<bf16, float>(const bf16 *, int, const bf16 *, int, int, const bf16 *, int, int,
                                                    const int32_t *, const float *, float *, int, hipStream_t);

}  // namespace alora
