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
//
// Every launch covers ALL bases of a call (one grid dimension is the basis, or the map): a token's pass over the
// bases of a whole model is these seven launches, not seven per basis, and what it costs when no basis grows is
// seven nearly empty launches.  The records of a call with several bases sit in a table in the workspace (copied
// there by the call); a call with one basis carries its record in the kernel arguments.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "gsi_decode.h"
#include "gsi_device.h"
#include "gsi_extend.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kCols = 64;       // columns of U per workgroup in the projections
constexpr int kRowsPerWg = 32;  // rows of U per workgroup in the residual
constexpr int kImgRows = kWaves;  // rows of W per workgroup and turn in the image launch: one per wave
constexpr int kFewMaps = 8;     // maps whose records fit the kernel arguments
constexpr int kSumBlock = 64;   // a wave per workgroup in the slab sums

struct ExtArg {  // the bases of a launch: a device table, or (tab == null) the one record
  const ExtIn* tab;
  ExtIn one;
};
struct ExtMapArg {  // the maps of an image launch: a device table, or up to kFewMaps records
  const ExtMapRec* tab;
  ExtMapRec few[kFewMaps];
};

struct ExtWs {
  ExtState* st;
  float *part, *sv, *r2, *ust, *pn;
};
__host__ __device__ __forceinline__ size_t a256(size_t b) { return (b + 255) / 256 * 256; }
__host__ __device__ __forceinline__ ExtWs ext_ws(const ExtIn& in) {
  ExtWs w;
  char* p = in.ws;
  w.st = reinterpret_cast<ExtState*>(p);
  p += a256(sizeof(ExtState));
  w.part = reinterpret_cast<float*>(p);
  p += a256((size_t)in.slabs * in.K * 4);
  w.sv = reinterpret_cast<float*>(p);
  p += a256((size_t)in.K * 4);
  w.r2 = reinterpret_cast<float*>(p);
  p += a256((size_t)in.d * 4);
  w.ust = reinterpret_cast<float*>(p);
  p += a256((size_t)in.d * 4);
  w.pn = reinterpret_cast<float*>(p);
  return w;
}

// part[slab][j] = sum over the slab's rows of U[i, j] v[i]   (grid: column blocks x slabs x bases).
// first: this is the projection s = U^T r of the step: every workgroup forms the candidate verdict from the token's
// norms and the column counter (the first one of a basis records it); else the projection U^T u for E, run iff the
// basis grew and the caller keeps E.
template <class T>
__global__ __launch_bounds__(kBlock) void ext_proj(const ExtArg a, float tau, int first) {
  using S = typename T::storage;
  const ExtIn in = a.tab ? a.tab[blockIdx.z] : a.one;
  const ExtWs w = ext_ws(in);
  const int64_t d = in.d, K = in.K;
  if ((int64_t)blockIdx.x * kCols >= K || (int)blockIdx.y >= in.slabs) return;  // (the grid is sized for the largest basis)
  const float* v;
  if (first) {
    const int k = in.k_cur[0];
    const bool cand = k >= 0 && k < K && gate_fires(in.rnorm[0], in.xnorm[0], tau);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
      w.st->kc = k;
      w.st->cand = cand ? 1 : 0;
      w.st->ext = 0;
      w.st->inv = 0.f;
    }
    if (!cand) return;
    v = in.R;
  } else {
    if (!in.gram || !w.st->ext) return;
    v = w.ust;
  }
  const S* U = static_cast<const S*>(in.U);
  float* part = w.part;
  constexpr int V = T::kVec;
  constexpr int TPR = kCols / V;        // threads per row segment of 64 columns
  constexpr int RG = kBlock / TPR;      // rows in flight per pass of the workgroup
  __shared__ float sh[RG][kCols + 1];
  // (a call with many bases launches fewer workgroups per basis than it has slabs: the workgroup takes several)
  for (int slab = blockIdx.y; slab < in.slabs; slab += gridDim.y) {
  const int64_t r0 = (int64_t)slab * in.rows_per_slab;
  const int64_t r1 = r0 + in.rows_per_slab < d ? r0 + in.rows_per_slab : d;
  if (in.uvec) {
    const int rg = threadIdx.x / TPR, cv = threadIdx.x % TPR;
    const int64_t col0 = (int64_t)blockIdx.x * kCols + cv * V;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    if (col0 < K) {  // K is a multiple of V here: whole vectors
      for (int64_t i = r0 + rg; i < r1; i += 4 * RG) {
        float f[4][V], wt[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {  // four rows requested before the first is used; rows past the slab repeat
          const int64_t ii = i + q * RG;  // the last one with weight zero
          const int64_t ic = ii < r1 ? ii : r1 - 1;
          T::load_vec(U + ic * K + col0, f[q]);
          wt[q] = ii < r1 ? v[ic] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[e] = fmaf(f[q][e], wt[q], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) sh[rg][cv * V + e] = acc[e];
    __syncthreads();
    const int64_t col = (int64_t)blockIdx.x * kCols + threadIdx.x;
    if (threadIdx.x < kCols && col < K) {
      float s = 0.f;
      for (int q = 0; q < RG; ++q) s += sh[q][threadIdx.x];
      part[(int64_t)slab * K + col] = s;
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
      part[(int64_t)slab * K + col] = s;
    }
  }
  __syncthreads();  // the sums have been read before the next slab's are written
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

__global__ __launch_bounds__(kSumBlock) void ext_sum(const ExtArg a) {
  const ExtIn in = a.tab ? a.tab[blockIdx.y] : a.one;
  const ExtWs w = ext_ws(in);
  if (!w.st->cand) return;
  const int64_t j = (int64_t)blockIdx.x * kSumBlock + threadIdx.x;
  if (j >= in.K) return;
  w.sv[j] = slab_sum(w.part, in.slabs, in.K, j);
}

// r2[i] = r[i] - sum_j U[i, j] s[j], a wave per row (two rows at a time); pn[workgroup] = the workgroup's share
// of |r2|^2
template <class T>
__global__ __launch_bounds__(kBlock) void ext_resid(const ExtArg a) {
  using S = typename T::storage;
  const ExtIn in = a.tab ? a.tab[blockIdx.y] : a.one;
  const ExtWs w = ext_ws(in);
  if ((int)blockIdx.x >= in.wgs || !w.st->cand) return;
  const int64_t d = in.d, K = in.K;
  const S* U = static_cast<const S*>(in.U);
  const float* v = in.R;
  const float* s = w.sv;
  float* r2 = w.r2;
  constexpr int V = T::kVec;
  __shared__ float shn[kWaves];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  for (int blk = blockIdx.x; blk < in.wgs; blk += gridDim.x) {
  const int64_t r0 = (int64_t)blk * kRowsPerWg;
  const int64_t r1 = r0 + kRowsPerWg < d ? r0 + kRowsPerWg : d;
  float nn = 0.f;
  if (in.uvec) {
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
    for (int q = 0; q < kWaves; ++q) t += shn[q];
    w.pn[blk] = t;
  }
  __syncthreads();
  }
}

// The final verdict (every workgroup of a basis adds the shares of |r2|^2 in the same fixed order; the first one
// records the verdict, the column counter and the caller's flag), then column kc of U <- r2 / |r2| rounded to
// storage; ust = the stored values widened.
template <class T>
__global__ __launch_bounds__(kBlock) void ext_column(const ExtArg a) {
  using S = typename T::storage;
  const ExtIn in = a.tab ? a.tab[blockIdx.y] : a.one;
  const ExtWs w = ext_ws(in);
  const int64_t d = in.d, K = in.K;
  if ((int64_t)blockIdx.x * kBlock >= d) return;  // (block 0 of a basis always stays)
  __shared__ float sh[kBlock];
  __shared__ float s_inv;
  const int cand = w.st->cand, kc = w.st->kc;
  float t = 0.f;
  if (cand)
    for (int q = threadIdx.x; q < in.wgs; q += kBlock) t += w.pn[q];
  sh[threadIdx.x] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int q = 0; q < kBlock; ++q) tot += sh[q];
    const float n2 = sqrtf(tot);
    const int ext = (cand && n2 > 0.f) ? 1 : 0;
    s_inv = ext ? 1.f / n2 : 0.f;
    if (blockIdx.x == 0) {
      w.st->ext = ext;
      w.st->inv = s_inv;
      if (ext) in.k_cur[0] = kc + 1;
      if (in.extended) in.extended[0] = ext;
    }
  }
  __syncthreads();
  const float inv = s_inv;
  if (inv == 0.f) return;  // uniform
  S* U = static_cast<S*>(in.U);
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < d; i += (int64_t)gridDim.x * kBlock) {
    const int64_t at = i * K + kc;
    T::store(U, at, w.r2[i] * inv);
    w.ust[i] = T::load(U, at);
  }
}

// M[row, kc] = sum_i W[row, i] ust[i] (grid: row blocks x maps).  A workgroup takes kImgRows rows of one map, a
// wave one row at a time (16-byte loads, eight in flight per lane, when the rows allow them).
template <class T>
__global__ __launch_bounds__(kBlock) void ext_image(const ExtArg a, const ExtMapArg ma) {
  using S = typename T::storage;
  const ExtMapRec p = ma.tab ? ma.tab[blockIdx.y] : ma.few[blockIdx.y];
  if ((int64_t)blockIdx.x * kImgRows >= p.m) return;
  const ExtIn in = a.tab ? a.tab[p.in] : a.one;
  const ExtWs w = ext_ws(in);
  if (!w.st->ext) return;
  constexpr int V = T::kVec;
  constexpr int NL = 8;
  const int64_t d = in.d, K = in.K;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const float* uv = w.ust;
  const int kc = w.st->kc;
  for (int64_t row_begin = (int64_t)blockIdx.x * kImgRows; row_begin < p.m; row_begin += (int64_t)gridDim.x * kImgRows)
  for (int r = wave; r < kImgRows; r += kWaves) {
    const int64_t row = row_begin + r;
    if (row >= p.m) break;  // (whole waves leave together)
    const S* wr = static_cast<const S*>(p.W) + row * d;
    float acc = 0.f;
    if (p.vec) {
      const int64_t chunks = d / V;
      for (int64_t c0 = 0; c0 < chunks; c0 += (int64_t)kWave * NL) {
        uint4 raw[NL];
#pragma unroll
        for (int q = 0; q < NL; ++q) {  // chunks past the row repeat its last one and are not used
          int64_t c = c0 + lane + (int64_t)q * kWave;
          c = c < chunks ? c : chunks - 1;
          raw[q] = load_stream16(wr + c * V);
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
      for (int64_t i = lane; i < d; i += kWave) acc = fmaf(T::load(wr, i), uv[i], acc);
    }
    acc = group_sum<kWave>(acc);
    if (lane == 0) T::store(static_cast<S*>(p.M), row * K + kc, acc);
  }
}

// E[j, kc] = E[kc, j] = (U^T u)[j] - (j == kc), the projection over the extended basis added over its slabs
__global__ __launch_bounds__(kSumBlock) void ext_gram(const ExtArg a) {
  const ExtIn in = a.tab ? a.tab[blockIdx.y] : a.one;
  const ExtWs w = ext_ws(in);
  if (!in.gram || !w.st->ext) return;
  const int64_t K = in.K;
  const int64_t j = (int64_t)blockIdx.x * kSumBlock + threadIdx.x;
  if (j >= K) return;
  const float t = slab_sum(w.part, in.slabs, K, j);
  const int kc = w.st->kc;
  const float v = t - (j == kc ? 1.f : 0.f);
  in.gram[j * K + kc] = v;
  in.gram[(int64_t)kc * K + j] = v;
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

template <class T>
hipError_t launch_all(const ExtIn* in, int n, const ExtMapRec* maps, int n_maps, float tau, void* table, hipStream_t s) {
  ExtArg a;
  std::memset(&a, 0, sizeof(a));
  const ExtMapRec* mtab = nullptr;
  if (n == 1) {
    a.one = in[0];
  } else {  // the records go to the table in the workspace: bases first, then maps
    const size_t ib = align_up((size_t)n * sizeof(ExtIn), 256), mb = align_up((size_t)n_maps * sizeof(ExtMapRec), 256);
    std::vector<char> host(ib + mb, 0);
    std::memcpy(host.data(), in, (size_t)n * sizeof(ExtIn));
    if (n_maps) std::memcpy(host.data() + ib, maps, (size_t)n_maps * sizeof(ExtMapRec));
    if (hipError_t e = upload_launch(host.data(), host.size(), table, s); e != hipSuccess) return e;
    a.tab = static_cast<const ExtIn*>(table);
    mtab = reinterpret_cast<const ExtMapRec*>(static_cast<const char*>(table) + ib);
  }
  int64_t K_max = 0, d_max = 0, m_max = 0;
  int slabs_max = 0, wgs_max = 0, any_gram = 0;
  for (int i = 0; i < n; ++i) {
    K_max = std::max<int64_t>(K_max, in[i].K);
    d_max = std::max<int64_t>(d_max, in[i].d);
    slabs_max = std::max(slabs_max, in[i].slabs);
    wgs_max = std::max(wgs_max, in[i].wgs);
    any_gram |= in[i].gram != nullptr;
  }
  for (int j = 0; j < n_maps; ++j) m_max = std::max<int64_t>(m_max, maps[j].m);
  // A launch is about kGridCap workgroups at most: every workgroup of a basis that does not grow reads its record and
  // leaves, which is what a token costs nearly always, so a call with many bases gives each fewer workgroups (they
  // take several slabs, row blocks ... in turn; what a workgroup computes per slab or row does not change).
  constexpr int64_t kGridCap = 2048;
  const int64_t pc = ceil_div(K_max, kCols);
  const dim3 pgrid((unsigned)pc, (unsigned)std::min<int64_t>(slabs_max, std::max<int64_t>(1, kGridCap / (pc * n))), (unsigned)n);
  const dim3 kgrid((unsigned)ceil_div(K_max, kSumBlock), (unsigned)n);
  const int64_t per_basis = std::max<int64_t>(8, kGridCap / n);
  ext_proj<T><<<pgrid, kBlock, 0, s>>>(a, tau, 1);
  ext_sum<<<kgrid, kSumBlock, 0, s>>>(a);
  ext_resid<T><<<dim3((unsigned)std::min<int64_t>(wgs_max, per_basis), (unsigned)n), kBlock, 0, s>>>(a);
  ext_column<T><<<dim3((unsigned)std::min<int64_t>(ceil_div(d_max, kBlock), per_basis), (unsigned)n), kBlock, 0, s>>>(a);
  if (n_maps > 0) {
    ExtMapArg ma;
    std::memset(&ma, 0, sizeof(ma));
    if (mtab) {
      ma.tab = mtab;
      const int64_t per_map = std::max<int64_t>(8, 2 * kGridCap / n_maps);
      ext_image<T><<<dim3((unsigned)std::min<int64_t>(ceil_div(m_max, kImgRows), per_map), (unsigned)n_maps), kBlock, 0, s>>>(a, ma);
    } else {
      for (int j0 = 0; j0 < n_maps; j0 += kFewMaps) {
        const int nm = std::min(kFewMaps, n_maps - j0);
        int64_t mm = 0;
        for (int q = 0; q < nm; ++q) {
          ma.few[q] = maps[j0 + q];
          mm = std::max<int64_t>(mm, maps[j0 + q].m);
        }
        ext_image<T><<<dim3((unsigned)ceil_div(mm, kImgRows), (unsigned)nm), kBlock, 0, s>>>(a, ma);
      }
    }
  }
  if (any_gram) {
    ext_proj<T><<<pgrid, kBlock, 0, s>>>(a, tau, 0);
    ext_gram<<<kgrid, kSumBlock, 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace

size_t extend_ws_bytes(int64_t d, int64_t K) {
  const Geom g = geom(d);
  return align_up(sizeof(ExtState), 256) + align_up((size_t)g.slabs * K * 4, 256) + align_up((size_t)K * 4, 256) +
         2 * align_up((size_t)d * 4, 256) + align_up((size_t)g.wgs * 4, 256);
}

size_t extend_table_bytes(int n, int n_maps) {
  return n > 1 ? align_up((size_t)n * sizeof(ExtIn), 256) + align_up((size_t)n_maps * sizeof(ExtMapRec), 256) : 0;
}

void extend_fill(ExtIn& in, int udtype) {
  const Geom g = geom(in.d);
  in.slabs = g.slabs;
  in.rows_per_slab = g.rows_per_slab;
  in.wgs = g.wgs;
  // 16-byte loads along the rows of U: whole vectors per row, rows that start on 16 bytes
  const int V = udtype == GSI_BF16 ? 8 : 4;
  in.uvec = in.K % V == 0 && reinterpret_cast<uintptr_t>(in.U) % 16 == 0;
}

void extend_fill_map(ExtMapRec& mp, int64_t d, int udtype) {
  const int V = udtype == GSI_BF16 ? 8 : 4;
  mp.vec = d % V == 0 && reinterpret_cast<uintptr_t>(mp.W) % 16 == 0;
}

hipError_t extend_many(const ExtIn* in, int n, const ExtMapRec* maps, int n_maps, int udtype, float tau, void* table,
                       hipStream_t s) {
  if (n <= 0) return hipSuccess;
  return udtype == GSI_BF16 ? launch_all<BF16>(in, n, maps, n_maps, tau, table, s)
                            : launch_all<F32>(in, n, maps, n_maps, tau, table, s);
}

}  // namespace gsi
