// Shared declarations of the libalora kernels (device side and their host launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace alora {

typedef __bf16 bf16;

// Per-sequence metadata staged to the device once per call.
struct SeqMeta {
  int32_t row_start;   // first packed row of the sequence's new tokens
  int32_t n_new;       // S_b
  int32_t P;           // rows already valid in the cache
  int32_t k;           // invocation index (first adapted absolute position)
  int32_t adapter;     // adapter id or -1
  float scale;         // s_a of that adapter (0 if none)
  int64_t pool_off;    // pool row of position 0 if the own rows started there: position j >= prefix_len
                       // sits at pool_off + j (= seq_offset - prefix_len + j)
  int64_t prefix_off;  // pool row of position 0 of the shared prefix (positions < prefix_len)
  int32_t prefix_len;  // 0: no shared prefix
  int32_t pad_;
};

// pool row of cached position j of a sequence
__device__ __forceinline__ int64_t seq_pool_row(const SeqMeta &sm, int j) {
  return (j < sm.prefix_len ? sm.prefix_off : sm.pool_off) + j;
}

// Per-row metadata written by the row-preparation kernel and read by everything after it.
struct RowMeta {
  int32_t *seq;        // [T] sequence index
  int32_t *pos;        // [T] absolute position p(i)
  int32_t *adapter;    // [T] adapter id if the row is adapted (a >= 0 and p >= k), else -1
  int64_t *slot;       // [T] pool row where this token's key/value go
  unsigned long long *present16;   // [ceil(T / 16)] bit a set: a row of this group of 16 is adapted by adapter a
                                   // (written by the MFMA row preparation; nullptr when nobody writes it)
};

struct LayerDims {
  int d, n_q_heads, n_kv_heads, head_dim, rank, n_adapters;
  int n_q, n_kv, n_qkv;
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- launchers: plain kernels (any dtype, any shape) ------------------------------------
enum GemmEpilogue { EPI_F32_LORA = 0, EPI_STORE = 1, EPI_STORE_RESIDUAL = 2, EPI_STORE_F32 = 3 };

void launch_rope_table(float2 *table, int n_pos, int half_dim, float theta, hipStream_t s);
// one table line per row (entry row * half_dim + c belongs to position pos[row])
void launch_rope_rows(float2 *table, const int32_t *pos, int n_rows, int half_dim, float theta, hipStream_t s);

template <typename T>
void launch_prep_rows(const T *x, const T *gain, float eps, int T_rows, int d, const SeqMeta *seqs,
                      int n_seqs, int pos_shift, const T *A, int rank, bool write_meta, T *xh, float *tlow,
                      bf16 *tlow16, RowMeta rm, hipStream_t s);

// Y[T, n_qkv] (fp32) = xh W^T + gated low-rank term (Eq.6)
template <typename T>
void launch_qkv_gemm_plain(const T *xh, const T *W, const float *tlow, const T *Bq, const T *Bk,
                           const T *Bv, const LayerDims &L, RowMeta rm, int T_rows, float *Y,
                           hipStream_t s);

// C[M,N] (T) = A[M,K] B[N,K]^T (+ R[M,N])
template <typename T>
void launch_gemm_plain(const T *A, const T *B, const T *R, T *C, int M, int N, int K, hipStream_t s);
// The same product left in fp32 (no rounding to the storage type), for the callers that still add to it:
// low-rank term, residual, SwiGLU -- so that a stored activation is rounded once, as in the fused MFMA epilogues.
template <typename T>
void launch_gemm_plain_f32(const T *A, const T *B, float *C, int M, int N, int K, hipStream_t s);
// out = T(C + R) (R may be nullptr), and out = T(silu(gate) * up), from fp32 inputs
template <typename T>
void launch_residual_store(const float *C, const T *R, T *out, int64_t n, hipStream_t s);
template <typename T>
void launch_silu_mul_f32(const float *gate, const float *up, T *out, int64_t n, hipStream_t s);

// q_mode: how the rotated queries are stored -- 0: as T, 1: as fp16 (operand type of the MFMA attention kernels),
// 2: as fp32 (the plain attention kernel)
template <typename T>
void launch_rope_append(const float *Y, int n_parts, const LayerDims &L, RowMeta rm, int T_rows,
                        const float2 *rope_table, bool table_by_row, float q_scale, int q_mode, void *Q, T *cacheK,
                        T *cacheV, hipStream_t s);

// C[M, N] += gated low-rank term (Eq.6) of one linear: s_a B_a (A_{a,part} x) for rows with row_adapter >= 0
// (TC: the type C is held in -- the storage type, or float for a sum that has not been rounded yet)
template <typename T, typename TC>
void launch_lowrank_add_plain(const T *x, int K, const T *A, int parts, int part, const T *B, int N, int rank,
                              const int32_t *row_adapter, const float *scale, TC *C, int M, hipStream_t s);

// output head: fp32 logits[B, V] = xh[B, d] W[V, d]^T (any shape), and the greedy token of every row
template <typename T>
void launch_lm_logits_plain(const T *xh, const T *W, int B, int V, int d, float *logits, hipStream_t s);
int argmax_slabs(int V);
void launch_argmax(const float *logits, int B, int V, float *pv, int *pi, int32_t *token, hipStream_t s);

// split-KV attention with plain fp32 arithmetic: partial pass + merge
template <typename T>
void launch_attn_plain(const float *Q, const T *cacheK, const T *cacheV, const SeqMeta *seqs, RowMeta rm,
                       const LayerDims &L, int T_rows, int n_splits, float *partials, hipStream_t s);
// merge of the per-split partials (log-sum-exp weights); partial layout per (row, q head, split):
// head_dim accumulators, running max, running sum
template <typename T>
void launch_attn_merge(const float *partials, const LayerDims &L, int T_rows, int n_splits, T *out, hipStream_t s);

template <typename T>
void launch_silu_mul(const T *gate, const T *up, T *out, int64_t n, hipStream_t s);

size_t attn_plain_partial_floats(const LayerDims &L, int T_rows, int n_splits);

}  // namespace alora
