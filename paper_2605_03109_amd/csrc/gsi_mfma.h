// Host interface of the matrix-core GEMM used by the image build and the prefill-sized batched path.
#pragma once
#include "gsi_internal.h"

namespace gsi {

enum { EPI_STORE_BF16 = 0, EPI_STORE_F32 = 1, EPI_RESIDUAL = 2, EPI_SCATTER_ADD = 3 };

// D = A B^T, A[M,K] (bf16, or fp32 split into two bf16 terms), B[N,K] bf16, both row-major.
struct GemmArgs {
  const void* A;
  int64_t lda;
  int a_f32;
  const void* B;
  int64_t ldb;
  void* D;                    // bf16 or fp32 [.., ldd]
  int64_t ldd;
  int M, N, K;                // K a multiple of 32
  const int32_t* row_idx;     // optional: row i of A is A[row_idx[i]], and (scatter-add) row i of D is D[row_idx[i]]
  const int32_t* n_rows_dev;  // optional: device count of valid rows (<= M)
  // residual epilogue: D = X - A B^T and per-row partial sums of squares
  const void* X;
  int xdtype;
  int64_t ldx;
  float* part_n;              // [tiles of N][part_tokens][2]
  int part_tokens;
};

hipError_t mfma_gemm_nt(const GemmArgs& g, int epi, hipStream_t s);
hipError_t mfma_transpose_bf16(const void* U, void* Ut, int rows, int cols, hipStream_t s);
int mfma_res_tiles(int64_t d);  // column tiles of the residual GEMM = partial norms per token

}  // namespace gsi
