// Launchers of the MFMA (bf16, gfx950) kernels.
#pragma once
#include "common.h"

namespace alora {

enum GemmEpi { GEMM_EPI_PARTIAL = 0, GEMM_EPI_BF16 = 1, GEMM_EPI_SWIGLU = 2, GEMM_EPI_ROPE = 3 };

// C[M,N] = A[M,K] B[N,K]^T, bf16 operands, fp32 accumulation.
struct GemmArgs {
  const bf16 *A; int lda;      // [M, K]
  const bf16 *B; int ldb;      // [N, K]
  const bf16 *B2;              // SwiGLU only: the "up" weights; B holds the "gate" weights, N = 2 * I
  int M, N, K;
  int tile_hint;               // 0 = automatic; 1 = 128x128 (4 waves), 2 = 256x128, 3 = 256x256, 4 = 128x64,
                               // 5 / 6 = 128x128 with 8 waves of 32x64 / 64x32
  int k_splits;                // PARTIAL only: workgroups per output tile along the reduction axis, 1 or k_segments
  int k_segments;              // equal segments the reduction axis is cut in, each summed from zero and the sums added
                               // in ascending order (by the consumer of the partials when k_splits == k_segments, by
                               // the kernel itself when k_splits == 1); K / k_segments must be a multiple of 64
  int lora_split;              // PARTIAL only, 1: the low-rank term gets workgroups of its own that write partial
                               // number k_splits (Cpart then holds k_splits + 1 partials), instead of riding on split 0
  float *Cpart;                // PARTIAL: [k_splits, M, N] fp32 partial sums
  bf16 *C; int ldc;            // BF16 / SWIGLU output
  const bf16 *R;               // BF16: optional residual [M, ldc]
  // gated low-rank term (Eq.6); tlow == nullptr switches it off
  const bf16 *tlow;            // [M, lr_parts, 2, rank]: s_a * A_{a,p} x for adapted rows as bf16 (hi, lo) pairs
  int rank;
  int lr_parts;                // 3: parts are the column ranges q | k | v (widths n_q, n_kv, n_kv; up-matrices Bq,
                               // Bk, Bv); 1: every column is part 0 (n_q = N, Bq); SwiGLU, 2: gate (Bq) and up
                               // (Bk) columns, n_q = I
  const bf16 *Bq, *Bk, *Bv;
  int n_q, n_kv;
  const int32_t *row_adapter;  // [M]: adapter id of adapted rows, -1 otherwise
  const unsigned long long *present16;   // [ceil(M / 16)] adapters among each 16 rows as a bit mask, or nullptr (the
                               // workgroup then finds the adapters of its rows itself: one more memory round trip)
  // ROPE epilogue (the QKV projection with an unsplit reduction and head_dim = 128 = the column tile): q and k
  // heads are rotated (Eq.3's K_t before it is appended) and every head goes where the rotary kernel would have
  // put it -- Q [M, n_q], the cache rows rope_slot[row] of K and V -- without the fp32 round trip through memory
  const int32_t *rope_pos;     // [M] absolute positions
  const int64_t *rope_slot;    // [M] pool rows
  const float2 *rope_table;    // [positions, 64] (cos, sin)
  float q_scale;               // multiplies the rotated queries
  int q_half;                  // 1: Qout receives fp16 (the MFMA prefill attention kernel's operand type) instead of bf16
  bf16 *Qout, *cacheK, *cacheV;
};
bool gemm_mfma_rope_supported(const GemmArgs &g, int head_dim);

// Row preparation: metadata, RMSNorm, t = s_a * A_a x_hat as bf16 (hi, lo) pairs.
struct PrepArgs {
  const bf16 *x;            // [T, d]
  const bf16 *gain;         // [d] or nullptr
  float eps;
  int T, d;
  const SeqMeta *seqs;      // nullptr: no metadata / adapters (plain RMSNorm)
  int n_seqs;
  SeqMeta one;              // a copy of seqs[0] when n_seqs == 1: the kernel then needs no memory round trip
                            // to know its rows' positions and adapter, and fetches A together with x
  int pos_shift;            // added to every position (step index of a multi-step decode)
  const bf16 *A;            // [n_adapters, 3, rank, d] or nullptr
  int rank;
  int n_adapters;           // adapters stored in A (a short batch gives every adapter workgroups of its own)
  int write_meta;
  bf16 *xh;                 // [T, d]
  bf16 *tlow16;             // [T, 3, 2, rank]
  RowMeta rm;
};
bool prep_rows_mfma_supported(int d, int rank);
void launch_prep_rows_mfma(const PrepArgs &a, hipStream_t s);
// metadata and RMSNorm only (A, rank, tlow16 unused), for many rows of a call without adapters: x_hat and
// metadata bit-identical to launch_prep_rows_mfma's
bool norm_rows_mfma_supported(int d);
void launch_norm_rows_mfma(const PrepArgs &a, hipStream_t s);

// One workgroup of the prefill attention kernel: up to 256/G consecutive packed rows (tokens) against the key
// positions [kbeg, kend) of one kv head, counted from pool row key_row0.  Own rows of one sequence: key_row0 is
// its first own row, pos0 the position of the first token counted from there, and the causal mask applies.
// Rows of several consecutive sequences over the shared prefix they all name (Section 2, "Cache reuse patterns",
// several adapters on one context): key_row0 is the prefix, pos0 lies beyond every key, the prefix tile is
// fetched once for all of them.
struct AttnItem {
  int64_t key_row0;         // pool row that holds key position 0 of this item
  int32_t kbeg, kend;       // key positions of this item
  int32_t n_addr;           // key positions that may be addressed from key_row0 (loads beyond kend are clamped to it)
  int32_t row0, ntok;       // packed rows row0 .. row0 + ntok - 1; ntok <= 0: padding item
  int32_t pos0;             // position of row0's token (token i sits at pos0 + i)
  int32_t g;                // kv head
  int32_t part;             // which of the n_parts partial records of a (row, head) this item writes
  int32_t pad_[2];
};
// Prefill attention (Eq.1 with the causal mask) over the pool cache.
struct AttnArgs {
  const _Float16 *Q;        // [T, n_q] rotated queries of the new rows, as fp16
  const bf16 *K, *V;        // pool [tokens, n_kv]
  const AttnItem *work;     // one item per workgroup
  int n_q, n_kv, n_q_heads, n_kv_heads;
  int n_parts;              // partial records per (row, head); 1: the kernel writes the final output
  float sm_scale;           // 1 / sqrt(head_dim)
  int q_prescaled;          // Q already carries sm_scale * log2(e): scores leave the MFMA in the exp2 domain
  float lazy;               // the running maximum moves only when a block exceeds it by more than this (log2 units)
  float *partials;          // [T, n_q_heads, n_parts, head_dim + 2] (acc, max, sum), used when out == nullptr
  int compact;              // partial records in the compact form (ATTN_REC16 bytes each) that launch_attn_merge16 reads
  bf16 *out;                // [T, n_q] final output, only with n_parts == 1
};
constexpr int ATTN_REC16 = 272;      // 128 fp16 + (reference, row sum, scale) as fp32 + 4 bytes of padding
bool attn_prefill_mfma_supported(const LayerDims &L);
void launch_attn_merge16(const float *partials, const LayerDims &L, int T_rows, int n_splits, bf16 *out, hipStream_t s);
int attn_prefill_mfma_tokens_per_tile(const LayerDims &L, int waves);      // waves per workgroup: 8 or 4
// with a.q_prescaled the kernels run their folded-softmax form (attn_prefill_mfma_q_scale tells the rotation
// kernel what to multiply the queries by)
void launch_attn_prefill_mfma(const AttnArgs &a, int n_work, int G, int waves, bool prefix, hipStream_t s);
float attn_prefill_mfma_q_scale(const LayerDims &L, bool fold);

// Decode attention (Eq.4): one query row per sequence over its whole cache.
// One workgroup of the decode kernel: the query heads of up to 16 / G rows, for up to eight kv heads (one wave
// each), against one range of keys.  shared = 0: the row's own cached positions [prefix_len, pos];
// shared = 1: the prefix [0, prefix_len) that all the item's rows name (one physical copy), so
// its keys and values are read once for all of them.
struct DecItem {
  int32_t n_rows;           // rows whose heads fill the MFMA columns (column = row index * G + head)
  int32_t g;                // first kv head of the workgroup (its waves take g, g + 1, ...)
  int32_t split, n_splits;  // this item's share of its key range
  int32_t part;             // which of the n_parts partial records of (row, head) it writes
  int32_t shared;
  int32_t pad_[2];
  int32_t rows[16];
};
struct DecodeArgs {
  const _Float16 *Q;        // [rows, n_q] rotated queries as fp16
  const bf16 *K, *V;        // pool [tokens, n_kv]
  const SeqMeta *seqs;
  RowMeta rm;               // seq and pos of every row
  const DecItem *items;     // one per workgroup
  int n_q, n_kv, n_q_heads, n_kv_heads;
  int n_parts;              // partial records per (row, head)
  int heads_per_wg;         // kv heads a workgroup covers (one wave each) and ...
  int ranges_per_wg;        // ... sub-ranges its key split is cut in; heads_per_wg * ranges_per_wg <= 8 waves
  int cols_max;             // largest n_rows * G over the items (MFMA columns in use; sizes the merge buffer)
  float sm_scale;
  float *partials;          // [rows, n_q_heads, n_parts, head_dim + 2]
};
bool attn_decode_mfma_supported(const LayerDims &L);
void launch_attn_decode_mfma(const DecodeArgs &a, int n_items, hipStream_t s);
void decode_mfma_shape(int n_kv_heads, int *heads_per_wg, int *ranges_per_wg);

bool gemm_mfma_supported(int M, int N, int K);
int gemm_mfma_pick_splits(int M, int N, int K, int n_cu);
int gemm_mfma_fixed_segments(int N, int K, int n_cu);      // reduction segments of a linear: from the weight shape alone
bool gemm_mfma_split_segments(int M, int N, int n_cu);     // one workgroup per segment (few row tiles) or one for all
void launch_gemm_mfma(GemmArgs g, int epi, hipStream_t s);
// tlow[row, p, {hi, lo}, j] = s_a * sum over splits of Y[split, row, (a * parts + p) * rank + j] for adapted rows
// (a = row_adapter[row] >= 0): picks each row's adapter out of a projection on all adapters' down-matrices
void launch_tlow_select(const float *Y, int splits, int M, int n_adapters, int parts, int rank,
                        const int32_t *row_adapter, const float *scale, bf16 *tlow, hipStream_t s);
// C[mn] = bf16(sum_s part[s][mn] + R[mn]); mn must be a multiple of 4
void launch_splitk_reduce(const float *part, int splits, int64_t mn, const bf16 *R, bf16 *C, hipStream_t s);
// the same for whole rows plus the RMSNorm of the summed row: C = bf16(h), Cn = bf16(RMSNorm(h; gain))
bool splitk_reduce_norm_supported(int N);
void launch_splitk_reduce_norm(const float *part, int splits, int M, int N, const bf16 *R, const bf16 *gain, float eps,
                               bf16 *C, bf16 *Cn, hipStream_t s);

}  // namespace alora
