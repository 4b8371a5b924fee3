// Launchers of the MFMA (bf16, gfx950) kernels.
#pragma once
#include "common.h"

namespace alora {

enum GemmEpi { GEMM_EPI_PARTIAL = 0, GEMM_EPI_BF16 = 1, GEMM_EPI_SWIGLU = 2 };

// C[M,N] = A[M,K] B[N,K]^T, bf16 operands, fp32 accumulation.
struct GemmArgs {
  const bf16 *A; int lda;      // [M, K]
  const bf16 *B; int ldb;      // [N, K]
  const bf16 *B2;              // SwiGLU only: the "up" weights; B holds the "gate" weights, N = 2 * I
  int M, N, K;
  int k_splits;                // PARTIAL only: grid.z; K / k_splits must be a multiple of 64
  float *Cpart;                // PARTIAL: [k_splits, M, N] fp32 partial sums
  bf16 *C; int ldc;            // BF16 / SWIGLU output
  const bf16 *R;               // BF16: optional residual [M, ldc]
  // gated low-rank term (Eq.6); tlow == nullptr switches it off
  const bf16 *tlow;            // [M, 3, 2, rank]: s_a * A_{a,p} x for adapted rows as bf16 (hi, lo) pairs
  int rank;
  const bf16 *Bq, *Bk, *Bv;
  int n_q, n_kv;
  const int32_t *row_adapter;  // [M]: adapter id of adapted rows, -1 otherwise
};

// Prefill attention (Eq.1 with the causal mask) over the pool cache.
struct AttnArgs {
  const bf16 *Q;            // [T, n_q] rotated queries of the new rows
  const bf16 *K, *V;        // pool [tokens, n_kv]
  const SeqMeta *seqs;
  const int2 *qtiles;       // per q-tile: (sequence, first new-token index of the tile)
  int n_q, n_kv, n_q_heads, n_kv_heads;
  int n_splits;             // key splits (grid.z)
  float sm_scale;           // 1 / sqrt(head_dim)
  float *partials;          // [T, n_q_heads, n_splits, head_dim + 2] (acc, max, sum), used when out == nullptr
  bf16 *out;                // [T, n_q] final output, only with n_splits == 1
};
bool attn_prefill_mfma_supported(const LayerDims &L);
int attn_prefill_mfma_tokens_per_tile(const LayerDims &L);
void launch_attn_prefill_mfma(const AttnArgs &a, int n_qtiles, int G, hipStream_t s);

bool gemm_mfma_supported(int M, int N, int K);
int gemm_mfma_pick_splits(int M, int N, int K, int n_cu);
void launch_gemm_mfma(GemmArgs g, int epi, hipStream_t s);

}  // namespace alora
