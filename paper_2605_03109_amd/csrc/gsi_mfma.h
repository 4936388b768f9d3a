// Host interface of the matrix-core GEMM used by the image build and the prefill-sized batched path.
#pragma once
#include "gsi_internal.h"

namespace gsi {

enum { EPI_STORE_BF16 = 0, EPI_STORE_F32 = 1, EPI_RESIDUAL = 2, EPI_SCATTER_ADD = 3, EPI_SCATTER_STORE = 4, EPI_MULTI = 5 };

// One right-hand factor of a product with several (EPI_MULTI): the same A against B_0, B_1, ... side by side in
// one launch, each with its own output and epilogue (EPI_RESIDUAL or EPI_STORE_F32).
struct GemmSeg {
  const void* B;
  int64_t ldb;
  void* D;
  int64_t ldd;
  int N;
  int tile_begin;  // first column tile of this factor in the launch (filled by mfma_gemm_nt)
  int epi;
};
constexpr int kMaxGemmSegs = 4;

// D = A B^T, A[M,K] (bf16, or fp32 split into two bf16 terms), B[N,K] bf16, both row-major.
struct GemmArgs {
  const void* A;
  int64_t lda;
  int a_f32;                  // A is 0: bf16; 1: fp32, fed as bf16 head + tail (two passes); 2: fp32, rounded once to bf16
  const void* B;
  int64_t ldb;
  void* D;                    // bf16 or fp32 [.., ldd]
  int64_t ldd;
  int M, N, K;                // K a multiple of 64; M * N below 2^31
  const int32_t* row_idx;     // optional: row i of A is A[row_idx[i]], and (scatter-add) row i of D is D[row_idx[i]]
  const int32_t* n_rows_dev;  // optional: device count of valid rows (<= M)
  // residual epilogue: D = X - A B^T and per-row partial sums of squares
  const void* X;
  int xdtype;
  int64_t ldx;
  float* part_n;              // [tiles of N][part_tokens][2]
  int part_tokens;
  // split contraction: workspace [splits][M][N] of partial sums, or null (then no split); `splits` is set
  // by mfma_gemm_nt from mfma_splits()
  float* part;
  int splits;
  // EPI_MULTI: the right-hand factors (B, ldb, D, ldd, N above are then unused)
  GemmSeg seg[kMaxGemmSegs];
  int nseg;
};

// how many ways mfma_gemm_nt splits the contraction of an M x N x K problem, and the workspace that takes
int mfma_splits(int64_t M, int64_t N, int64_t K, int epi);
size_t mfma_part_bytes(int64_t M, int64_t N, int64_t K, int epi);

hipError_t mfma_gemm_nt(const GemmArgs& g, int epi, hipStream_t s);
hipError_t mfma_transpose_bf16(const void* U, void* Ut, int rows, int cols, hipStream_t s);
int mfma_res_tiles(int64_t d);  // column tiles of the residual GEMM = partial norms per token

}  // namespace gsi
