// Online basis maintenance of libgsi: one DGKS rank-1 extension of a basis of fixed capacity, with the matching
// append to the cached images (Section 5.3 "The cascade initialization", Section 5.4 "Time-dimension tracking",
// Section 7 "Online basis adaptation").
//
// The basis lives in U[d, K] whose columns from k on are zero (a zero column changes neither c, r nor y, so every
// other kernel of the library runs on it unchanged at rank K).  Given the residual r = x - U U^T x of a token and
// its norms (what the projection of the layer already produced), the step is
//     candidate   iff  |x| > 0, |r| / |x| >= tau, k < K
//     s = U^T r,  r2 = r - U s                    (the re-orthogonalisation pass of classical Gram-Schmidt)
//     u = r2 / |r2| rounded to the basis' storage type  ->  column k of U
//     M[:, k] = W u   for every map that reads this basis, from the STORED u, so that M = W U keeps holding
//     E[:, k] = E[k, :] = U^T u - e_k             (when the caller keeps E = U^T U - I for the single-pass gate)
//     k <- k + 1
// Everything is decided on the device (k is a device counter): every kernel below starts by reading the verdict of
// the one before and leaves at once when there is nothing to do, so a token that does not extend the basis costs a
// handful of empty launches and no pass over U or W.  All sums have a fixed order.
#include <hip/hip_runtime.h>

#include "gsi_device.h"
#include "gsi_extend.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kCols = 64;  // columns of U per workgroup in the projection

__global__ void ext_decide(const float* __restrict__ rnorm, const float* __restrict__ xnorm, float tau,
                           const int32_t* __restrict__ k_cur, int K, ExtState* __restrict__ st) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int k = k_cur[0];
  st->kc = k;
  st->cand = (k >= 0 && k < K && gate_fires(rnorm[0], xnorm[0], tau)) ? 1 : 0;
  st->ext = 0;
  st->inv = 0.f;
}

// part[slab][j] = sum over the slab's rows of U[i, j] v[i]   (grid: column blocks x slabs)
template <class T>
__global__ __launch_bounds__(kBlock) void ext_proj(const typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                   const float* __restrict__ v, const int* __restrict__ go,
                                                   float* __restrict__ part, int rows_per_slab) {
  if (!go[0]) return;
  __shared__ float sh[kBlock / kCols][kCols];
  const int col = blockIdx.x * kCols + threadIdx.x % kCols, rl = threadIdx.x / kCols;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
  const int64_t r1 = r0 + rows_per_slab < d ? r0 + rows_per_slab : d;
  float acc = 0.f;
  if (col < K)
    for (int64_t i = r0 + rl; i < r1; i += kBlock / kCols) acc = fmaf(T::load(U, i * K + col), v[i], acc);
  sh[rl][threadIdx.x % kCols] = acc;
  __syncthreads();
  if (rl == 0 && col < K) {
    float s = 0.f;
    for (int q = 0; q < kBlock / kCols; ++q) s += sh[q][threadIdx.x];
    part[(int64_t)blockIdx.y * K + col] = s;
  }
}

__global__ __launch_bounds__(kBlock) void ext_sum(const float* __restrict__ part, int slabs, int64_t K,
                                                  const int* __restrict__ go, float* __restrict__ s) {
  if (!go[0]) return;
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= K) return;
  float t = 0.f;
  for (int q = 0; q < slabs; ++q) t += part[(int64_t)q * K + j];
  s[j] = t;
}

// r2[i] = v[i] - sum_j U[i, j] s[j], a wave per row; pn[workgroup] = the workgroup's share of |r2|^2
template <class T>
__global__ __launch_bounds__(kBlock) void ext_resid(const typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                    const float* __restrict__ v, const float* __restrict__ s,
                                                    const int* __restrict__ go, float* __restrict__ r2,
                                                    float* __restrict__ pn, int rows_per_wg) {
  if (!go[0]) return;
  __shared__ float shn[kWaves];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg;
  const int64_t r1 = r0 + rows_per_wg < d ? r0 + rows_per_wg : d;
  float nn = 0.f;
  for (int64_t i = r0 + wave; i < r1; i += kWaves) {
    float acc = 0.f;
    for (int64_t j = lane; j < K; j += kWave) acc = fmaf(T::load(U, i * K + j), s[j], acc);
    acc = group_sum<kWave>(acc);
    const float r = v[i] - acc;
    if (lane == 0) r2[i] = r;
    nn = fmaf(r, r, nn);  // (every lane holds the same value)
  }
  if (lane == 0) shn[wave] = nn;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < kWaves; ++w) t += shn[w];
    pn[blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(kBlock) void ext_finalize(const float* __restrict__ pn, int n, ExtState* __restrict__ st,
                                                       int32_t* __restrict__ k_cur, int32_t* __restrict__ extended) {
  __shared__ float sh[kBlock];
  float t = 0.f;
  if (st->cand)
    for (int q = threadIdx.x; q < n; q += kBlock) t += pn[q];
  sh[threadIdx.x] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int q = 0; q < kBlock; ++q) tot += sh[q];
    const float n2 = sqrtf(tot);
    const int ext = (st->cand && n2 > 0.f) ? 1 : 0;
    st->ext = ext;
    st->inv = ext ? 1.f / n2 : 0.f;
    if (ext) k_cur[0] = st->kc + 1;
    if (extended) extended[0] = ext;
  }
}

// column kc of U <- r2 / |r2| rounded to storage; ust = the stored values widened
template <class T>
__global__ __launch_bounds__(kBlock) void ext_column(typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                     const float* __restrict__ r2, const ExtState* __restrict__ st,
                                                     float* __restrict__ ust) {
  if (!st->ext) return;
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= d) return;
  const int64_t at = i * K + st->kc;
  T::store(U, at, r2[i] * st->inv);
  ust[i] = T::load(U, at);
}

// M[row, kc] = sum_i W[row, i] ust[i], a wave per row (16-byte loads when the row allows them)
template <class T>
__global__ __launch_bounds__(kBlock) void ext_image(const typename T::storage* __restrict__ W,
                                                    typename T::storage* __restrict__ M, int64_t m, int64_t d, int64_t K,
                                                    const float* __restrict__ ust, const ExtState* __restrict__ st,
                                                    int vec_ok) {
  if (!st->ext) return;
  constexpr int V = T::kVec;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t row = (int64_t)blockIdx.x * kWaves + wave;
  if (row >= m) return;  // (whole waves leave together)
  const typename T::storage* w = W + row * d;
  float acc = 0.f;
  if (vec_ok) {
    for (int64_t c = lane; c < d / V; c += kWave) {
      float f[V];
      T::load_vec(w + c * V, f);
#pragma unroll
      for (int e = 0; e < V; ++e) acc = fmaf(f[e], ust[c * V + e], acc);
    }
  } else {
    for (int64_t i = lane; i < d; i += kWave) acc = fmaf(T::load(w, i), ust[i], acc);
  }
  acc = group_sum<kWave>(acc);
  if (lane == 0) T::store(M, row * K + st->kc, acc);
}

// E[j, kc] = E[kc, j] = s[j] - (j == kc), s = U^T u over the extended basis
__global__ __launch_bounds__(kBlock) void ext_gram(float* __restrict__ E, int64_t K, const float* __restrict__ s,
                                                   const ExtState* __restrict__ st) {
  if (!st->ext) return;
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= K) return;
  const int kc = st->kc;
  const float v = s[j] - (j == kc ? 1.f : 0.f);
  E[j * K + kc] = v;
  E[(int64_t)kc * K + j] = v;
}

struct Geom {
  int slabs, rows_per_slab, wgs, rows_per_wg;
};
Geom geom(int64_t d) {
  Geom g;
  g.slabs = (int)(d < 64 * 32 ? ceil_div(d, 64) : 32);
  g.rows_per_slab = (int)ceil_div(d, g.slabs);
  g.slabs = (int)ceil_div(d, g.rows_per_slab);
  g.rows_per_wg = 32;
  g.wgs = (int)ceil_div(d, g.rows_per_wg);
  return g;
}

}  // namespace

size_t extend_ws_bytes(int64_t d, int64_t K) {
  const Geom g = geom(d);
  return align_up(sizeof(ExtState), 256) + align_up((size_t)g.slabs * K * 4, 256) + align_up((size_t)K * 4, 256) +
         2 * align_up((size_t)d * 4, 256) + align_up((size_t)g.wgs * 4, 256);
}

template <class T>
static hipError_t extend_launch(void* U, int64_t d, int64_t K, int32_t* k_cur, const float* R, const float* rnorm,
                                const float* xnorm, float tau, const ExtMap* maps, int n_maps, float* gram,
                                int32_t* extended, void* ws, hipStream_t s) {
  using S = typename T::storage;
  const Geom g = geom(d);
  char* p = static_cast<char*>(ws);
  ExtState* st = reinterpret_cast<ExtState*>(p);
  p += align_up(sizeof(ExtState), 256);
  float* part = reinterpret_cast<float*>(p);
  p += align_up((size_t)g.slabs * K * 4, 256);
  float* sv = reinterpret_cast<float*>(p);
  p += align_up((size_t)K * 4, 256);
  float* r2 = reinterpret_cast<float*>(p);
  p += align_up((size_t)d * 4, 256);
  float* ust = reinterpret_cast<float*>(p);
  p += align_up((size_t)d * 4, 256);
  float* pn = reinterpret_cast<float*>(p);
  const dim3 pgrid((unsigned)ceil_div(K, kCols), (unsigned)g.slabs);
  const unsigned kgrid = (unsigned)ceil_div(K, kBlock);

  ext_decide<<<1, 1, 0, s>>>(rnorm, xnorm, tau, k_cur, (int)K, st);
  ext_proj<T><<<pgrid, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, R, &st->cand, part, g.rows_per_slab);
  ext_sum<<<kgrid, kBlock, 0, s>>>(part, g.slabs, K, &st->cand, sv);
  ext_resid<T><<<g.wgs, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, R, sv, &st->cand, r2, pn, g.rows_per_wg);
  ext_finalize<<<1, kBlock, 0, s>>>(pn, g.wgs, st, k_cur, extended);
  ext_column<T><<<(unsigned)ceil_div(d, kBlock), kBlock, 0, s>>>(static_cast<S*>(U), d, K, r2, st, ust);
  for (int j = 0; j < n_maps; ++j) {
    const int vec_ok = d % T::kVec == 0 && reinterpret_cast<uintptr_t>(maps[j].W) % 16 == 0;
    ext_image<T><<<(unsigned)ceil_div(maps[j].m, kWaves), kBlock, 0, s>>>(static_cast<const S*>(maps[j].W),
                                                                        static_cast<S*>(maps[j].M), maps[j].m, d, K, ust,
                                                                        st, vec_ok);
  }
  if (gram) {
    ext_proj<T><<<pgrid, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, ust, &st->ext, part, g.rows_per_slab);
    ext_sum<<<kgrid, kBlock, 0, s>>>(part, g.slabs, K, &st->ext, sv);
    ext_gram<<<kgrid, kBlock, 0, s>>>(gram, K, sv, st);
  }
  return hipGetLastError();
}

hipError_t extend_basis(void* U, int64_t d, int64_t K, int udtype, int32_t* k_cur, const float* R, const float* rnorm,
                        const float* xnorm, float tau, const ExtMap* maps, int n_maps, float* gram, int32_t* extended,
                        void* ws, hipStream_t s) {
  return udtype == GSI_BF16
             ? extend_launch<BF16>(U, d, K, k_cur, R, rnorm, xnorm, tau, maps, n_maps, gram, extended, ws, s)
             : extend_launch<F32>(U, d, K, k_cur, R, rnorm, xnorm, tau, maps, n_maps, gram, extended, ws, s);
}

}  // namespace gsi
