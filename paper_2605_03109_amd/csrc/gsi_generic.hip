// Generic kernels of libgsi: correct for every shape and alignment (scalar element access, fp32
// accumulation in a fixed order).  They serve odd/tiny shapes; aligned shapes take the vectorised
// kernels in the other translation units.
#include "gsi_device.h"
#include "gsi_internal.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;

// c[t][j] = sum_i U[i][j] x[t][i]          (Algorithm 1, line 1)
template <class T>
__global__ __launch_bounds__(kBlock) void gen_proj_c(const typename T::storage* __restrict__ U,
                                                     const void* __restrict__ X, int xdtype, int64_t d, int64_t k,
                                                     int64_t B, float* __restrict__ C) {
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= k) return;
  for (int64_t t = blockIdx.y; t < B; t += gridDim.y) {
    float acc = 0.f;
    for (int64_t i = 0; i < d; ++i) acc = fmaf(T::load(U, i * k + j), load_act(X, xdtype, t * d + i), acc);
    C[t * k + j] = acc;
  }
}

// r[t][i] = x[t][i] - sum_j U[i][j] c[t][j]   (Algorithm 1, line 2): one wave per row i
template <class T>
__global__ __launch_bounds__(kBlock) void gen_residual(const typename T::storage* __restrict__ U,
                                                       const void* __restrict__ X, int xdtype, int64_t d,
                                                       int64_t k, int64_t B, const float* __restrict__ C,
                                                       float* __restrict__ R) {
  const int lane = threadIdx.x % kWave;
  const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (i >= d) return;
  for (int64_t t = blockIdx.y; t < B; t += gridDim.y) {
    float acc = 0.f;
    for (int64_t j = lane; j < k; j += kWave) acc = fmaf(T::load(U, i * k + j), C[t * k + j], acc);
    acc = group_sum<kWave>(acc);
    if (lane == 0) R[t * d + i] = load_act(X, xdtype, t * d + i) - acc;
  }
}

// rnorm[t] = |r_t|, xnorm[t] = |x_t|        (Algorithm 1, line 3): one workgroup per token
__global__ __launch_bounds__(kBlock) void gen_norms(const void* __restrict__ X, int xdtype,
                                                    const float* __restrict__ R, int64_t d, int64_t B,
                                                    float* __restrict__ rnorm, float* __restrict__ xnorm) {
  __shared__ float sr[kBlock / kWave], sx[kBlock / kWave];
  for (int64_t t = blockIdx.x; t < B; t += gridDim.x) {
    float ar = 0.f, ax = 0.f;
    for (int64_t i = threadIdx.x; i < d; i += kBlock) {
      const float r = R[t * d + i], x = load_act(X, xdtype, t * d + i);
      ar = fmaf(r, r, ar);
      ax = fmaf(x, x, ax);
    }
    ar = group_sum<kWave>(ar);
    ax = group_sum<kWave>(ax);
    if (threadIdx.x % kWave == 0) {
      sr[threadIdx.x / kWave] = ar;
      sx[threadIdx.x / kWave] = ax;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      float tr = 0.f, tx = 0.f;
      for (int w = 0; w < kBlock / kWave; ++w) {
        tr += sr[w];
        tx += sx[w];
      }
      rnorm[t] = sqrtf(tr);
      xnorm[t] = sqrtf(tx);
    }
    __syncthreads();
  }
}

// Y[t][row] = M[row,:] . C[t,:]  for all t, then  Y[f][row] += W[row,:] . R[f,:]  for fired f.
// One wave per row; the same lane writes and later updates an output, so no atomics are needed.
template <class T>
__global__ __launch_bounds__(kBlock) void gen_gated_linear(const typename T::storage* __restrict__ W,
                                                           const typename T::storage* __restrict__ M,
                                                           const float* __restrict__ C,
                                                           const float* __restrict__ R,
                                                           const int32_t* __restrict__ fired_idx,
                                                           const int32_t* __restrict__ n_fired, int64_t m,
                                                           int64_t d, int64_t k, int64_t B, float* __restrict__ Y,
                                                           const void* __restrict__ X, int xdtype) {
  // X non-null: a fired token gets y = W x (Algorithm 1, line 7) instead of M c + W r
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (row >= m) return;
  for (int64_t t = 0; t < B; ++t) {
    float acc = 0.f;
    for (int64_t j = lane; j < k; j += kWave) acc = fmaf(T::load(M, row * k + j), C[t * k + j], acc);
    acc = group_sum<kWave>(acc);
    if (lane == 0) Y[t * m + row] = acc;
  }
  int nf = n_fired[0];
  if (nf > B) nf = (int)B;
  for (int f = 0; f < nf; ++f) {
    const int64_t t = fired_idx[f];
    if (t < 0 || t >= B) continue;
    float acc = 0.f;
    for (int64_t i = lane; i < d; i += kWave)
      acc = fmaf(T::load(W, row * d + i), X ? load_act(X, xdtype, t * d + i) : R[t * d + i], acc);
    acc = group_sum<kWave>(acc);
    if (lane == 0) Y[t * m + row] = X ? acc : Y[t * m + row] + acc;
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void gen_dense_linear(const typename T::storage* __restrict__ W,
                                                           const void* __restrict__ X, int xdtype, int64_t m,
                                                           int64_t d, int64_t B, float* __restrict__ Y) {
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (row >= m) return;
  for (int64_t t = 0; t < B; ++t) {
    float acc = 0.f;
    for (int64_t i = lane; i < d; i += kWave) acc = fmaf(T::load(W, row * d + i), load_act(X, xdtype, t * d + i), acc);
    acc = group_sum<kWave>(acc);
    if (lane == 0) Y[t * m + row] = acc;
  }
}

// M[row][j] = sum_i W[row][i] U[i][j]       (Eq. (exact): the cached image)
template <class T>
__global__ __launch_bounds__(kBlock) void gen_build_image(const typename T::storage* __restrict__ W,
                                                          const typename T::storage* __restrict__ U,
                                                          typename T::storage* __restrict__ M, int64_t m,
                                                          int64_t d, int64_t k) {
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= k) return;
  for (int64_t row = blockIdx.y; row < m; row += gridDim.y) {
    float acc = 0.f;
    for (int64_t i = 0; i < d; ++i) acc = fmaf(T::load(W, row * d + i), T::load(U, i * k + j), acc);
    T::store(M, row * k + j, acc);
  }
}

inline unsigned grid_y(int64_t n) { return (unsigned)(n < 65535 ? (n < 1 ? 1 : n) : 65535); }

}  // namespace

hipError_t generic_build_image(const void* W, const void* U, void* M, int64_t m, int64_t d, int64_t k, int wdtype,
                               hipStream_t s) {
  dim3 grid((unsigned)ceil_div(k, kBlock), grid_y(m));
  if (wdtype == GSI_BF16)
    gen_build_image<BF16><<<grid, kBlock, 0, s>>>((const uint16_t*)W, (const uint16_t*)U, (uint16_t*)M, m, d, k);
  else
    gen_build_image<F32><<<grid, kBlock, 0, s>>>((const float*)W, (const float*)U, (float*)M, m, d, k);
  return hipGetLastError();
}

hipError_t generic_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype,
                           float* C, float* R, float* rnorm, float* xnorm, hipStream_t s) {
  dim3 g1((unsigned)ceil_div(k, kBlock), grid_y(B));
  dim3 g2((unsigned)ceil_div(d, kBlock / kWave), grid_y(B));
  if (udtype == GSI_BF16) {
    gen_proj_c<BF16><<<g1, kBlock, 0, s>>>((const uint16_t*)U, X, xdtype, d, k, B, C);
    gen_residual<BF16><<<g2, kBlock, 0, s>>>((const uint16_t*)U, X, xdtype, d, k, B, C, R);
  } else {
    gen_proj_c<F32><<<g1, kBlock, 0, s>>>((const float*)U, X, xdtype, d, k, B, C);
    gen_residual<F32><<<g2, kBlock, 0, s>>>((const float*)U, X, xdtype, d, k, B, C, R);
  }
  gen_norms<<<grid_y(B), kBlock, 0, s>>>(X, xdtype, R, d, B, rnorm, xnorm);
  return hipGetLastError();
}

hipError_t generic_gated_linear(const void* W, const void* M, const float* C, const float* R,
                                const int32_t* fired_idx, const int32_t* n_fired, int64_t m, int64_t d, int64_t k,
                                int64_t B, int wdtype, float* Y, hipStream_t s, const void* X, int xdtype) {
  const unsigned grid = (unsigned)ceil_div(m, kBlock / kWave);
  if (wdtype == GSI_BF16)
    gen_gated_linear<BF16><<<grid, kBlock, 0, s>>>((const uint16_t*)W, (const uint16_t*)M, C, R, fired_idx,
                                                   n_fired, m, d, k, B, Y, X, xdtype);
  else
    gen_gated_linear<F32><<<grid, kBlock, 0, s>>>((const float*)W, (const float*)M, C, R, fired_idx, n_fired, m,
                                                  d, k, B, Y, X, xdtype);
  return hipGetLastError();
}

hipError_t generic_dense_linear(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int wdtype,
                                int xdtype, float* Y, hipStream_t s) {
  const unsigned grid = (unsigned)ceil_div(m, kBlock / kWave);
  if (wdtype == GSI_BF16)
    gen_dense_linear<BF16><<<grid, kBlock, 0, s>>>((const uint16_t*)W, X, xdtype, m, d, B, Y);
  else
    gen_dense_linear<F32><<<grid, kBlock, 0, s>>>((const float*)W, X, xdtype, m, d, B, Y);
  return hipGetLastError();
}

// E = U^T U - I in fp64 (one-time companion of a basis for the single-pass gate): a 16 x 16 tile of E per
// workgroup, 64 rows of the two column strips of U staged in LDS per step, one fp64 accumulator per thread.
template <class T>
__global__ __launch_bounds__(kBlock) void gen_gram(const typename T::storage* __restrict__ U, int64_t d, int64_t k,
                                                   float* __restrict__ E) {
  __shared__ float a[64][17], b[64][17];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int64_t i0 = (int64_t)blockIdx.y * 16, j0 = (int64_t)blockIdx.x * 16;
  double acc = 0.0;
  for (int64_t r0 = 0; r0 < d; r0 += 64) {
    for (int e = threadIdx.x; e < 64 * 16; e += kBlock) {
      const int rr = e / 16, cc = e % 16;
      const int64_t r = r0 + rr;
      a[rr][cc] = (r < d && i0 + cc < k) ? T::load(U, r * k + i0 + cc) : 0.f;
      b[rr][cc] = (r < d && j0 + cc < k) ? T::load(U, r * k + j0 + cc) : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int rr = 0; rr < 64; ++rr) acc = fma((double)a[rr][ty], (double)b[rr][tx], acc);
    __syncthreads();
  }
  const int64_t i = i0 + ty, j = j0 + tx;
  if (i < k && j < k) E[i * k + j] = (float)(acc - (i == j ? 1.0 : 0.0));
}

hipError_t generic_build_gram(const void* U, int64_t d, int64_t k, int udtype, float* E, hipStream_t s) {
  const dim3 grid((unsigned)ceil_div(k, 16), (unsigned)ceil_div(k, 16));
  if (udtype == GSI_BF16) gen_gram<BF16><<<grid, kBlock, 0, s>>>((const uint16_t*)U, d, k, E);
  else gen_gram<F32><<<grid, kBlock, 0, s>>>((const float*)U, d, k, E);
  return hipGetLastError();
}

}  // namespace gsi
