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
  const bf16 *tlow;            // [M, 3, rank]: s_a * A_{a,p} x for adapted rows
  int rank;
  const bf16 *Bq, *Bk, *Bv;
  int n_q, n_kv;
  const int32_t *row_adapter;  // [M]: adapter id of adapted rows, -1 otherwise
};

bool gemm_mfma_supported(int M, int N, int K);
int gemm_mfma_pick_splits(int M, int N, int K, int n_cu);
void launch_gemm_mfma(GemmArgs g, int epi, hipStream_t s);

}  // namespace alora
