// Linear-map kernels of libgsi for small token counts (decode): Algorithm 1 lines 4-7 in the
// y = M c (+ W r when the gate fires) form of Eq. (exact), and the dense baseline y = W x.
//
// stream_rows (one token): a persistent grid of a few workgroups per CU.  Every wave first learns
//   the gate of every input group (either from the published count, or by reducing the residual
//   kernel's partial norms itself -- identical arithmetic in every wave, so the decision is uniform
//   across the grid without any communication).  The projection coefficients of all groups are
//   staged in LDS once.  Rows of maps whose input did not fire are "short" (k elements of the image M,
//   several rows per 1-KB wave load); rows of fired maps are "long" (d elements of W plus the row of
//   M), one row per wave with four 16-byte loads in flight per lane and the activation vector in LDS.
//   Rows are dealt round-robin over all waves of the grid, so concurrently running waves stream
//   neighbouring rows.  Every output element is written exactly once, by one wave.
//   A map whose input did not fire never issues a load from W.
//
// gated_rows / dense_rows (several tokens): one workgroup per tile of 16 output rows; token tiles of
//   four for the image term, one fired token at a time (from the device-side list) for the W term.
#include <cstdlib>

#include "gsi_decode.h"
#include "gsi_device.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

__device__ __forceinline__ int find_task(const int* begin, int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < kMaxTasks; ++i)
    if (i < n && b >= begin[i]) t = i;
  return t;
}

// V consecutive floats from a 16-byte aligned LDS address, as 128-bit reads
template <int V>
__device__ __forceinline__ void lds_vec(const float* p, float (&f)[V]) {
#pragma unroll
  for (int q = 0; q < V / 4; ++q) {
    const float4 x = reinterpret_cast<const float4*>(p)[q];
    f[4 * q + 0] = x.x; f[4 * q + 1] = x.y; f[4 * q + 2] = x.z; f[4 * q + 3] = x.w;
  }
}

template <int V>
__device__ __forceinline__ float dotv(const float (&a)[V], const float (&b)[V], float acc) {
#pragma unroll
  for (int e = 0; e < V; ++e) acc = fmaf(a[e], b[e], acc);
  return acc;
}

// ------------------------------------------------------------------------------------------------
// single token
// ------------------------------------------------------------------------------------------------
template <class T, int UNR>
__global__ __launch_bounds__(kBlock) void stream_rows(const LinBatch lb) {
  constexpr int V = T::kVec;
  extern __shared__ __align__(16) float smem[];  // [coefficients of every group][one activation vector]
  using S = typename T::storage;

  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int gw = blockIdx.x * kWaves + wave;  // this wave's index in the grid
  const int GW = gridDim.x * kWaves;

  // ---- gate of every group, identical in every wave --------------------------------------------
  unsigned fired_mask = 0;
  int sumk = 0;
  auto coff = [&](int gi) {  // offset of group gi's coefficients in LDS
    int o = 0;
    for (int i = 0; i < gi; ++i) o += lb.g[i].k;
    return o;
  };
  for (int gi = 0; gi < kMaxTasks; ++gi) {
    if (gi < lb.ng) {
      const LinGroup& g = lb.g[gi];
      bool f;
      if (lb.dense) {
        f = true;
      } else if (lb.inline_gate) {
        float sr, sx;
        wave_norm_sums(g.part_n, g.b_slabs, 1, 0, sr, sx);
        const float rn = sqrtf(sr), xn = sqrtf(sx);
        f = gate_fires(rn, xn, lb.eps);
        if (blockIdx.x == 0 && threadIdx.x == 0) {  // publish, as the stand-alone norm + gate kernels would
          g.rnorm[0] = rn;
          g.xnorm[0] = xn;
          g.mask[0] = f ? 1 : 0;
          if (f) g.fired_idx_out[0] = 0;
          g.n_fired_out[0] = f ? 1 : 0;
        }
      } else {
        f = g.n_fired[0] > 0;
      }
      if (f) fired_mask |= 1u << gi;
      if (!lb.dense) sumk += g.k;
    }
  }
  float* xs = smem + sumk;

  // ---- image rows of the maps that did not fire --------------------------------------------------
  if (!lb.dense) {
    for (int gi = 0; gi < lb.ng; ++gi) {
      const LinGroup& g = lb.g[gi];
      const int co = coff(gi);
      for (int idx = threadIdx.x; idx < g.k; idx += kBlock) smem[co + idx] = g.C[idx];
    }
    __syncthreads();
  }
  int off = 0;  // running item offset, so the round-robin deal continues across tasks
  if (!lb.dense) {
    for (int ti = 0; ti < lb.n; ++ti) {
      const LinTask& t = lb.t[ti];
      if ((fired_mask >> t.group) & 1u) continue;
      const int k = lb.g[t.group].k, m = t.m;
      const float* cv = smem + coff(t.group);
      const S* M = reinterpret_cast<const S*>(t.M);
      const int chunks = k / V;
      int lpr = kWave;
      while (lpr / 2 >= chunks && lpr > 1) lpr >>= 1;  // lanes per row: smallest power of two >= chunks
      const int rpw = kWave / lpr, sub = lane / lpr, l = lane % lpr;
      const int ri = 4 * rpw;  // rows per item: four loads per lane
      const int items = (m + ri - 1) / ri;
      int it = (gw - off % GW + GW) % GW;
      for (; it < items; it += GW) {
        const int rb = it * ri + sub;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c = l; c < chunks; c += lpr) {
          float w[4][V], cvv[V];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int row = rb + u * rpw;
            if (row < m) {
              T::load_vec(M + (int64_t)row * k + c * V, w[u]);
            } else {
#pragma unroll
              for (int e = 0; e < V; ++e) w[u][e] = 0.f;
            }
          }
          lds_vec<V>(cv + c * V, cvv);
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[u] = dotv<V>(w[u], cvv, acc[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float s = group_sum_rt(acc[u], lpr);
          const int row = rb + u * rpw;
          if (l == 0 && row < m) t.Y[row] = s;
        }
      }
      off += items;
    }
  }

  // ---- rows of fired maps (or every map in the dense baseline), one input group at a time ---------
  for (int gi = 0; gi < lb.ng; ++gi) {
    if (!((fired_mask >> gi) & 1u)) continue;  // uniform across the grid
    const LinGroup& g = lb.g[gi];
    const int d = g.d, k = g.k;
    __syncthreads();
    if (lb.dense) {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) xs[idx] = load_act(g.X, g.xdtype, idx);
    } else {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) xs[idx] = g.R[idx];
    }
    __syncthreads();
    const int chunks = d / V;
    const int kchunks = lb.dense ? 0 : k / V;
    const float* cv = smem + coff(gi);
    for (int ti = 0; ti < lb.n; ++ti) {
      const LinTask& t = lb.t[ti];
      if (t.group != gi) continue;
      const S* W = reinterpret_cast<const S*>(t.W);
      const S* M = reinterpret_cast<const S*>(t.M);
      const int m = t.m;
      int row = (gw - off % GW + GW) % GW;
      for (; row < m; row += GW) {
        const S* wr = W + (int64_t)row * d;
        float acc = 0.f;
        // the row of the image goes in flight together with the first loads of W
        for (int c = lane; c < kchunks; c += kWave) {
          float mv[V], cvv[V];
          T::load_vec(M + (int64_t)row * k + c * V, mv);
          lds_vec<V>(cv + c * V, cvv);
          acc = dotv<V>(mv, cvv, acc);
        }
        int c = lane;
        for (; c + (UNR - 1) * kWave < chunks; c += UNR * kWave) {
          float w[UNR][V];
#pragma unroll
          for (int u = 0; u < UNR; ++u) T::load_vec(wr + (int64_t)(c + u * kWave) * V, w[u]);
#pragma unroll
          for (int u = 0; u < UNR; ++u) {
            float xv[V];
            lds_vec<V>(xs + (c + u * kWave) * V, xv);
            acc = dotv<V>(w[u], xv, acc);
          }
        }
        for (; c < chunks; c += kWave) {
          float w[V], xv[V];
          T::load_vec(wr + (int64_t)c * V, w);
          lds_vec<V>(xs + c * V, xv);
          acc = dotv<V>(w, xv, acc);
        }
        acc = group_sum<kWave>(acc);
        if (lane == 0) t.Y[row] = acc;
      }
      off += m;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// several tokens
// ------------------------------------------------------------------------------------------------
// Row dot products: the calling wave computes A[row, 0:len] . v_t for its rows and up to TB vectors
// v_t held in LDS as fp32.  Results go to out[(row - row_base) * TB + t] in LDS.
template <class T, int TB>
__device__ __forceinline__ void rows_dot(const typename T::storage* __restrict__ A, int64_t ld, int len,
                                         int row_begin, int row_end, int row_base, const float* __restrict__ v,
                                         int vstride, int nt, float* __restrict__ out) {
  constexpr int V = T::kVec;
  constexpr int UNR = 4;
  const int lane = threadIdx.x % kWave;
  const int chunks = len / V;
  int lpr = kWave;
  while (lpr / 2 >= chunks && lpr > 1) lpr >>= 1;
  const int rpw = kWave / lpr;
  const int sub = lane / lpr, l = lane % lpr;
  for (int rb = row_begin; rb < row_end; rb += rpw) {
    const int row = rb + sub;
    const bool live = row < row_end;
    float acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = 0.f;
    if (live) {
      const typename T::storage* a = A + (int64_t)row * ld;
      int c = l;
      for (; c + (UNR - 1) * lpr < chunks; c += UNR * lpr) {
        float w[UNR][V];
#pragma unroll
        for (int u = 0; u < UNR; ++u) T::load_vec(a + (int64_t)(c + u * lpr) * V, w[u]);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
          for (int t = 0; t < TB; ++t) {
            if (t < nt) {
              float vv[V];
              lds_vec<V>(v + t * vstride + (c + u * lpr) * V, vv);
              acc[t] = dotv<V>(w[u], vv, acc[t]);
            }
          }
        }
      }
      for (; c < chunks; c += lpr) {
        float w[V];
        T::load_vec(a + (int64_t)c * V, w);
#pragma unroll
        for (int t = 0; t < TB; ++t) {
          if (t < nt) {
            float vv[V];
            lds_vec<V>(v + t * vstride + c * V, vv);
            acc[t] = dotv<V>(w, vv, acc[t]);
          }
        }
      }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
      const float s = group_sum_rt(acc[t], lpr);
      if (live && l == 0 && t < nt) out[(row - row_base) * TB + t] = s;
    }
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void gated_rows(const LinBatch lb) {
  extern __shared__ __align__(16) float vec[];  // max(kTokTile * k, d) floats
  __shared__ float ya[kRowsPerBlock * kTokTile];
  __shared__ float yb[kRowsPerBlock];
  using S = typename T::storage;

  const int ti = find_task(lb.blk_begin, lb.n, blockIdx.x);
  const LinTask& p = lb.t[ti];
  const LinGroup& g = lb.g[p.group];
  const int B = lb.B;
  const int m = p.m, d = g.d, k = g.k;
  const int row0 = (blockIdx.x - lb.blk_begin[ti]) * kRowsPerBlock;
  const int rows = min(kRowsPerBlock, m - row0);
  const int wave = threadIdx.x / kWave;
  constexpr int RW = kRowsPerBlock / kWaves;
  const int wr0 = row0 + wave * RW;
  const int wr1 = min(wr0 + RW, row0 + rows);
  const S* W = reinterpret_cast<const S*>(p.W);
  const S* M = reinterpret_cast<const S*>(p.M);
  int nf = g.n_fired[0];
  nf = nf < 0 ? 0 : (nf > B ? B : nf);

  for (int t0 = 0; t0 < B; t0 += kTokTile) {
    const int nt = min(kTokTile, B - t0);
    __syncthreads();
    for (int idx = threadIdx.x; idx < nt * k; idx += kBlock) vec[idx] = g.C[(int64_t)t0 * k + idx];
    __syncthreads();
    rows_dot<T, kTokTile>(M, k, k, wr0, wr1, row0, vec, k, nt, ya);
    __syncthreads();
    for (int idx = threadIdx.x; idx < nt * rows; idx += kBlock) {
      const int tt = idx / rows, rr = idx % rows;
      p.Y[(int64_t)(t0 + tt) * m + row0 + rr] = ya[rr * kTokTile + tt];
    }
  }
  for (int f = 0; f < nf; ++f) {
    const int t = g.fired_idx[f];
    if (t < 0 || t >= B) continue;  // uniform across the workgroup
    __syncthreads();
    for (int idx = threadIdx.x; idx < d; idx += kBlock) vec[idx] = g.R[(int64_t)t * d + idx];
    __syncthreads();
    rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
    __syncthreads();
    if (threadIdx.x < rows) p.Y[(int64_t)t * m + row0 + threadIdx.x] += yb[threadIdx.x];
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void dense_rows(const LinBatch lb) {
  extern __shared__ __align__(16) float vec[];
  __shared__ float yb[kRowsPerBlock];
  using S = typename T::storage;
  const int ti = find_task(lb.blk_begin, lb.n, blockIdx.x);
  const LinTask& p = lb.t[ti];
  const LinGroup& g = lb.g[p.group];
  const int B = lb.B;
  const int m = p.m, d = g.d;
  const int row0 = (blockIdx.x - lb.blk_begin[ti]) * kRowsPerBlock;
  const int rows = min(kRowsPerBlock, m - row0);
  const int wave = threadIdx.x / kWave;
  constexpr int RW = kRowsPerBlock / kWaves;
  const int wr0 = row0 + wave * RW;
  const int wr1 = min(wr0 + RW, row0 + rows);
  const S* W = reinterpret_cast<const S*>(p.W);
  for (int t = 0; t < B; ++t) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < d; idx += kBlock) vec[idx] = load_act(g.X, g.xdtype, (int64_t)t * d + idx);
    __syncthreads();
    rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
    __syncthreads();
    if (threadIdx.x < rows) p.Y[(int64_t)t * m + row0 + threadIdx.x] = yb[threadIdx.x];
  }
}

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  if (!v || !*v) return dflt;
  const int x = std::atoi(v);
  return x > 0 ? x : dflt;
}

int num_cus() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) return 256;
    return cu;
  }();
  return n;
}

size_t stream_smem(const LinBatch& lb) {
  size_t sumk = 0, maxd = 0;
  for (int i = 0; i < lb.ng; ++i) {
    if (!lb.dense) sumk += (size_t)lb.g[i].k;
    if ((size_t)lb.g[i].d > maxd) maxd = (size_t)lb.g[i].d;
  }
  return (sumk + maxd) * sizeof(float);
}

size_t tile_smem(const LinBatch& lb) {
  size_t fl = 0;
  for (int i = 0; i < lb.ng; ++i) {
    size_t need = (size_t)lb.g[i].d;
    if (!lb.dense && (size_t)kTokTile * lb.g[i].k > need) need = (size_t)kTokTile * lb.g[i].k;
    if (need > fl) fl = need;
  }
  return fl * sizeof(float);
}

}  // namespace

bool decode_linear_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M) {
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  if (d % V || (k > 0 && k % V)) return false;
  if (d > kMaxLinD || kTokTile * k > kMaxLinD || k > kMaxSumK) return false;
  if (reinterpret_cast<uintptr_t>(W) % 16) return false;
  if (M && reinterpret_cast<uintptr_t>(M) % 16) return false;
  return m < (1ll << 30);
}

bool decode_linear_fits(const LinBatch& lb) {
  if (lb.B == 1) {
    size_t sumk = 0;
    for (int i = 0; i < lb.ng; ++i) sumk += (size_t)lb.g[i].k;
    return sumk <= (size_t)kMaxSumK && stream_smem(lb) <= (size_t)(kMaxLinD + kMaxSumK) * sizeof(float);
  }
  return tile_smem(lb) <= (size_t)kMaxLinD * sizeof(float);
}

hipError_t decode_linear_launch(LinBatch& lb, int wdtype, hipStream_t s) {
  if (lb.n == 0 || lb.B == 0) return hipSuccess;
  if (lb.B == 1) {
    // persistent grid: a few workgroups per CU, never more waves than rows
    static const int per_cu = env_int("GSI_LIN_WGS_PER_CU", 2);
    static const int unr8 = env_int("GSI_LIN_UNROLL", 4) == 8;
    int64_t rows = 0;
    for (int i = 0; i < lb.n; ++i) rows += lb.t[i].m;
    int64_t grid = (int64_t)per_cu * num_cus();
    if (grid > ceil_div(rows, kWaves)) grid = ceil_div(rows, kWaves);
    if (grid < 1) grid = 1;
    const size_t smem = stream_smem(lb);
    static const hipError_t attr = [] {  // the kernels may use more than the default 64 KB of dynamic LDS
      const int cap = (kMaxLinD + kMaxSumK) * (int)sizeof(float);
      hipError_t e = hipSuccess, r;
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<BF16, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, cap); if (r != hipSuccess) e = r;
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<BF16, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, cap); if (r != hipSuccess) e = r;
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<F32, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, cap); if (r != hipSuccess) e = r;
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<F32, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, cap); if (r != hipSuccess) e = r;
      return e;
    }();
    if (attr != hipSuccess) return attr;
    if (wdtype == GSI_BF16) {
      if (unr8) stream_rows<BF16, 8><<<(unsigned)grid, kBlock, smem, s>>>(lb);
      else stream_rows<BF16, 4><<<(unsigned)grid, kBlock, smem, s>>>(lb);
    } else {
      if (unr8) stream_rows<F32, 8><<<(unsigned)grid, kBlock, smem, s>>>(lb);
      else stream_rows<F32, 4><<<(unsigned)grid, kBlock, smem, s>>>(lb);
    }
    return hipGetLastError();
  }
  int total = 0;
  for (int i = 0; i < lb.n; ++i) {
    lb.blk_begin[i] = total;
    total += (int)ceil_div(lb.t[i].m, kRowsPerBlock);
  }
  const size_t smem = tile_smem(lb);
  if (lb.dense) {
    if (wdtype == GSI_BF16) dense_rows<BF16><<<total, kBlock, smem, s>>>(lb);
    else dense_rows<F32><<<total, kBlock, smem, s>>>(lb);
  } else {
    if (wdtype == GSI_BF16) gated_rows<BF16><<<total, kBlock, smem, s>>>(lb);
    else gated_rows<F32><<<total, kBlock, smem, s>>>(lb);
  }
  return hipGetLastError();
}

}  // namespace gsi
