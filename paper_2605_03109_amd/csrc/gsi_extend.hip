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
// Everything is decided on the device (k is a device counter): every kernel below starts by reading (or, the
// first one, forming) the verdict and leaves at once when there is nothing to do, so a token that does not extend
// the basis costs a handful of empty launches and no pass over U or W.  All sums have a fixed order.
//
// Launches: s partials (+ the candidate verdict) | s | r2 and shares of |r2|^2 | final verdict + the stored column
// | image columns of all maps | U^T u partials | E's row and column.  An extension moves U three times and every
// W once; operands whose rows are 16-byte aligned are read with 16-byte loads, several in flight per lane.
#include <hip/hip_runtime.h>

#include "gsi_device.h"
#include "gsi_extend.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kCols = 64;       // columns of U per workgroup in the projections
constexpr int kRowsPerWg = 32;  // rows of U per workgroup in the residual
constexpr int kMaxExtMaps = 8;  // maps per image launch

struct ExtImg {
  const void* W;
  void* M;
  int m;
  int blk_begin;
};
struct ExtImgs {
  ExtImg t[kMaxExtMaps];
  int n;
};

// part[slab][j] = sum over the slab's rows of U[i, j] v[i]   (grid: column blocks x slabs).
// first: this is the projection s = U^T r of the step: every workgroup forms the candidate verdict from the token's
// norms and the column counter (the first one records it); else the projection U^T u for E, run iff the basis grew.
template <class T>
__global__ __launch_bounds__(kBlock) void ext_proj(const typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                   const float* __restrict__ v, float* __restrict__ part,
                                                   int rows_per_slab, int vec, int first, ExtState* __restrict__ st,
                                                   const float* __restrict__ rnorm, const float* __restrict__ xnorm,
                                                   float tau, const int32_t* __restrict__ k_cur) {
  if (first) {
    const int k = k_cur[0];
    const bool cand = k >= 0 && k < K && gate_fires(rnorm[0], xnorm[0], tau);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
      st->kc = k;
      st->cand = cand ? 1 : 0;
      st->ext = 0;
      st->inv = 0.f;
    }
    if (!cand) return;
  } else if (!st->ext) {
    return;
  }
  constexpr int V = T::kVec;
  constexpr int TPR = kCols / V;        // threads per row segment of 64 columns
  constexpr int RG = kBlock / TPR;      // rows in flight per pass of the workgroup
  __shared__ float sh[RG][kCols + 1];
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
  const int64_t r1 = r0 + rows_per_slab < d ? r0 + rows_per_slab : d;
  if (vec) {
    const int rg = threadIdx.x / TPR, cv = threadIdx.x % TPR;
    const int64_t col0 = (int64_t)blockIdx.x * kCols + cv * V;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    if (col0 < K) {  // K is a multiple of V here: whole vectors
      for (int64_t i = r0 + rg; i < r1; i += 4 * RG) {
        float f[4][V], w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {  // four rows requested before the first is used; rows past the slab repeat
          const int64_t ii = i + q * RG;  // the last one with weight zero
          const int64_t ic = ii < r1 ? ii : r1 - 1;
          T::load_vec(U + ic * K + col0, f[q]);
          w[q] = ii < r1 ? v[ic] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[e] = fmaf(f[q][e], w[q], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) sh[rg][cv * V + e] = acc[e];
    __syncthreads();
    const int64_t col = (int64_t)blockIdx.x * kCols + threadIdx.x;
    if (threadIdx.x < kCols && col < K) {
      float s = 0.f;
      for (int q = 0; q < RG; ++q) s += sh[q][threadIdx.x];
      part[(int64_t)blockIdx.y * K + col] = s;
    }
  } else {
    constexpr int RL = kBlock / kCols;
    const int64_t col = (int64_t)blockIdx.x * kCols + threadIdx.x % kCols;
    const int rl = threadIdx.x / kCols;
    float acc = 0.f;
    if (col < K)
      for (int64_t i = r0 + rl; i < r1; i += RL) acc = fmaf(T::load(U, i * K + col), v[i], acc);
    sh[rl][threadIdx.x % kCols] = acc;
    __syncthreads();
    if (rl == 0 && col < K) {
      float s = 0.f;
      for (int q = 0; q < RL; ++q) s += sh[q][threadIdx.x];
      part[(int64_t)blockIdx.y * K + col] = s;
    }
  }
}

// sum over the slabs, in slab order, of part[slab][j]; eight requests in flight
__device__ __forceinline__ float slab_sum(const float* __restrict__ part, int slabs, int64_t K, int64_t j) {
  float t = 0.f;
  for (int q0 = 0; q0 < slabs; q0 += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)min(q0 + u, slabs - 1) * K + j];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (q0 + u < slabs) t += v[u];
  }
  return t;
}

constexpr int kSumBlock = 64;  // a wave per workgroup: K / 64 workgroups instead of K / 256
__global__ __launch_bounds__(kSumBlock) void ext_sum(const float* __restrict__ part, int slabs, int64_t K,
                                                     const int* __restrict__ go, float* __restrict__ s) {
  if (!go[0]) return;
  const int64_t j = (int64_t)blockIdx.x * kSumBlock + threadIdx.x;
  if (j >= K) return;
  s[j] = slab_sum(part, slabs, K, j);
}

// r2[i] = v[i] - sum_j U[i, j] s[j], a wave per row (two rows at a time); pn[workgroup] = the workgroup's share
// of |r2|^2
template <class T>
__global__ __launch_bounds__(kBlock) void ext_resid(const typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                    const float* __restrict__ v, const float* __restrict__ s,
                                                    const int* __restrict__ go, float* __restrict__ r2,
                                                    float* __restrict__ pn, int vec) {
  if (!go[0]) return;
  constexpr int V = T::kVec;
  __shared__ float shn[kWaves];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t r0 = (int64_t)blockIdx.x * kRowsPerWg;
  const int64_t r1 = r0 + kRowsPerWg < d ? r0 + kRowsPerWg : d;
  float nn = 0.f;
  if (vec) {
    const int64_t chunks = K / V;
    for (int64_t i = r0 + wave; i < r1; i += 2 * kWaves) {
      const int64_t i2 = i + kWaves < r1 ? i + kWaves : i;  // the second row of the pair, or the first again
      float a0 = 0.f, a1 = 0.f;
      for (int64_t c = lane; c < chunks; c += kWave) {
        float f0[V], f1[V], sv[V];
        T::load_vec(U + i * K + c * V, f0);
        T::load_vec(U + i2 * K + c * V, f1);
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
          const float4 x = *reinterpret_cast<const float4*>(s + c * V + 4 * q);
          sv[4 * q] = x.x; sv[4 * q + 1] = x.y; sv[4 * q + 2] = x.z; sv[4 * q + 3] = x.w;
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
          a0 = fmaf(f0[e], sv[e], a0);
          a1 = fmaf(f1[e], sv[e], a1);
        }
      }
      a0 = group_sum<kWave>(a0);
      a1 = group_sum<kWave>(a1);
      const float ra = v[i] - a0;
      if (lane == 0) r2[i] = ra;
      nn = fmaf(ra, ra, nn);  // (every lane holds the same value)
      if (i2 != i) {
        const float rb = v[i2] - a1;
        if (lane == 0) r2[i2] = rb;
        nn = fmaf(rb, rb, nn);
      }
    }
  } else {
    for (int64_t i = r0 + wave; i < r1; i += kWaves) {
      float acc = 0.f;
      for (int64_t j = lane; j < K; j += kWave) acc = fmaf(T::load(U, i * K + j), s[j], acc);
      acc = group_sum<kWave>(acc);
      const float r = v[i] - acc;
      if (lane == 0) r2[i] = r;
      nn = fmaf(r, r, nn);
    }
  }
  if (lane == 0) shn[wave] = nn;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < kWaves; ++w) t += shn[w];
    pn[blockIdx.x] = t;
  }
}

// The final verdict (every workgroup adds the n shares of |r2|^2 in the same fixed order; the first one records the
// verdict, the column counter and the caller's flag), then column kc of U <- r2 / |r2| rounded to storage;
// ust = the stored values widened.
template <class T>
__global__ __launch_bounds__(kBlock) void ext_column(typename T::storage* __restrict__ U, int64_t d, int64_t K,
                                                     const float* __restrict__ r2, const float* __restrict__ pn, int n,
                                                     ExtState* __restrict__ st, int32_t* __restrict__ k_cur,
                                                     int32_t* __restrict__ extended, float* __restrict__ ust) {
  __shared__ float sh[kBlock];
  __shared__ float s_inv;
  const int cand = st->cand, kc = st->kc;
  float t = 0.f;
  if (cand)
    for (int q = threadIdx.x; q < n; q += kBlock) t += pn[q];
  sh[threadIdx.x] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int q = 0; q < kBlock; ++q) tot += sh[q];
    const float n2 = sqrtf(tot);
    const int ext = (cand && n2 > 0.f) ? 1 : 0;
    s_inv = ext ? 1.f / n2 : 0.f;
    if (blockIdx.x == 0) {
      st->ext = ext;
      st->inv = s_inv;
      if (ext) k_cur[0] = kc + 1;
      if (extended) extended[0] = ext;
    }
  }
  __syncthreads();
  const float inv = s_inv;
  if (inv == 0.f) return;  // uniform
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= d) return;
  const int64_t at = i * K + kc;
  T::store(U, at, r2[i] * inv);
  ust[i] = T::load(U, at);
}

// M[row, kc] = sum_i W[row, i] ust[i] for every map of the launch.  A workgroup takes kImgRows rows of one map, a
// wave one row at a time (16-byte loads, eight in flight per lane, when the rows allow them); u is staged in LDS
// once per workgroup when it fits (lds = 1), else read through the caches.
constexpr int kImgRows = 16;
template <class T>
__global__ __launch_bounds__(kBlock) void ext_image(const ExtImgs im, int64_t d, int64_t K,
                                                    const float* __restrict__ ust, const ExtState* __restrict__ st,
                                                    int vec, int lds) {
  extern __shared__ __align__(16) float us[];
  if (!st->ext) return;
  constexpr int V = T::kVec;
  constexpr int NL = 8;
  using S = typename T::storage;
  int ti = 0;
#pragma unroll
  for (int q = 1; q < kMaxExtMaps; ++q)
    if (q < im.n && (int)blockIdx.x >= im.t[q].blk_begin) ti = q;
  const ExtImg& p = im.t[ti];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const float* uv = ust;
  if (lds) {  // (d is a multiple of 4 on this path)
    for (int64_t i = 4 * (int64_t)threadIdx.x; i < d; i += 4 * kBlock)
      *reinterpret_cast<float4*>(us + i) = *reinterpret_cast<const float4*>(ust + i);
    __syncthreads();
    uv = us;
  }
  const int64_t row_begin = (int64_t)(blockIdx.x - p.blk_begin) * kImgRows;
  const int kc = st->kc;
  for (int r = wave; r < kImgRows; r += kWaves) {
    const int64_t row = row_begin + r;
    if (row >= p.m) break;  // (whole waves leave together)
    const S* w = static_cast<const S*>(p.W) + row * d;
    float acc = 0.f;
    if (vec) {
      const int64_t chunks = d / V;
      for (int64_t c0 = 0; c0 < chunks; c0 += (int64_t)kWave * NL) {
        uint4 raw[NL];
#pragma unroll
        for (int q = 0; q < NL; ++q) {  // chunks past the row repeat its last one and are not used
          int64_t c = c0 + lane + (int64_t)q * kWave;
          c = c < chunks ? c : chunks - 1;
          raw[q] = load_stream16(w + c * V);
        }
#pragma unroll
        for (int q = 0; q < NL; ++q) {
          const int64_t c = c0 + lane + (int64_t)q * kWave;
          if (c < chunks) {
            float f[V];
            T::widen(raw[q], f);
#pragma unroll
            for (int e4 = 0; e4 < V / 4; ++e4) {
              const float4 x = *reinterpret_cast<const float4*>(uv + c * V + 4 * e4);
              acc = fmaf(f[4 * e4], x.x, acc);
              acc = fmaf(f[4 * e4 + 1], x.y, acc);
              acc = fmaf(f[4 * e4 + 2], x.z, acc);
              acc = fmaf(f[4 * e4 + 3], x.w, acc);
            }
          }
        }
      }
    } else {
      for (int64_t i = lane; i < d; i += kWave) acc = fmaf(T::load(w, i), uv[i], acc);
    }
    acc = group_sum<kWave>(acc);
    if (lane == 0) T::store(static_cast<S*>(p.M), row * K + kc, acc);
  }
}

// E[j, kc] = E[kc, j] = (U^T u)[j] - (j == kc), the projection over the extended basis added over its slabs
__global__ __launch_bounds__(kSumBlock) void ext_gram(float* __restrict__ E, int64_t K, const float* __restrict__ part,
                                                      int slabs, const ExtState* __restrict__ st) {
  if (!st->ext) return;
  const int64_t j = (int64_t)blockIdx.x * kSumBlock + threadIdx.x;
  if (j >= K) return;
  const float t = slab_sum(part, slabs, K, j);
  const int kc = st->kc;
  const float v = t - (j == kc ? 1.f : 0.f);
  E[j * K + kc] = v;
  E[(int64_t)kc * K + j] = v;
}

struct Geom {
  int slabs, rows_per_slab, wgs;
};
Geom geom(int64_t d) {
  Geom g;
  g.slabs = (int)(d < 64 * 32 ? ceil_div(d, 64) : 32);
  g.rows_per_slab = (int)ceil_div(d, g.slabs);
  g.slabs = (int)ceil_div(d, g.rows_per_slab);
  g.wgs = (int)ceil_div(d, kRowsPerWg);
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
  const unsigned kgrid = (unsigned)ceil_div(K, kSumBlock);
  // 16-byte loads along the rows of U: whole vectors per row, rows that start on 16 bytes
  const int uvec = K % T::kVec == 0 && reinterpret_cast<uintptr_t>(U) % 16 == 0;

  ext_proj<T><<<pgrid, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, R, part, g.rows_per_slab, uvec, 1, st, rnorm, xnorm,
                                       tau, k_cur);
  ext_sum<<<kgrid, kSumBlock, 0, s>>>(part, g.slabs, K, &st->cand, sv);
  ext_resid<T><<<g.wgs, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, R, sv, &st->cand, r2, pn, uvec);
  ext_column<T><<<(unsigned)ceil_div(d, kBlock), kBlock, 0, s>>>(static_cast<S*>(U), d, K, r2, pn, g.wgs, st, k_cur,
                                                               extended, ust);
  for (int j0 = 0; j0 < n_maps; j0 += kMaxExtMaps) {
    ExtImgs im;
    im.n = n_maps - j0 < kMaxExtMaps ? n_maps - j0 : kMaxExtMaps;
    int total = 0, vec = d % T::kVec == 0;
    for (int q = 0; q < kMaxExtMaps; ++q) {
      const ExtMap& mp = maps[j0 + (q < im.n ? q : 0)];
      im.t[q] = ExtImg{mp.W, mp.M, (int)mp.m, total};
      if (q < im.n) {
        total += (int)ceil_div(mp.m, kImgRows);
        if (reinterpret_cast<uintptr_t>(mp.W) % 16) vec = 0;
      }
    }
    // u in LDS when it fits beside nothing else (160 KB per compute unit; two workgroups of 64 KB still share one)
    const int lds = d % 4 == 0 && d * 4 <= 65536;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&ext_image<T>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    if (attr != hipSuccess) return attr;
    ext_image<T><<<total, kBlock, lds ? (size_t)d * 4 : 0, s>>>(im, d, K, ust, st, vec, lds);
  }
  if (gram) {
    ext_proj<T><<<pgrid, kBlock, 0, s>>>(static_cast<const S*>(U), d, K, ust, part, g.rows_per_slab, uvec, 0, st, rnorm,
                                         xnorm, tau, k_cur);
    ext_gram<<<kgrid, kSumBlock, 0, s>>>(gram, K, part, g.slabs, st);
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
