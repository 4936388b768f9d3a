// Linear-map kernels of libgsi for a few tokens per call (decode batches): Algorithm 1 lines 4-7 in
// the y = M c (+ W r when the gate fires) form of Eq. (exact), and the dense baseline y = W x.
//
// gated_rows / dense_rows: one workgroup per tile of 16 output rows; token tiles of four for the image
//   term, one fired token at a time (from the device-side list) for the W term.  The single-token
//   case is served by the persistent streaming kernel in gsi_stream.hip.
#include <cstdlib>

#include "gsi_decode.h"
#include "gsi_device.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

template <int N>
__device__ __forceinline__ int find_task(const int (&begin)[N], int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < N; ++i)
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
    for (int idx = threadIdx.x; idx < d; idx += kBlock)
      vec[idx] = g.wx ? load_act(g.X, g.xdtype, (int64_t)t * d + idx) : g.R[(int64_t)t * d + idx];
    __syncthreads();
    rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
    __syncthreads();
    if (threadIdx.x < rows) {
      float* y = p.Y + (int64_t)t * m + row0 + threadIdx.x;
      *y = g.wx ? yb[threadIdx.x] : *y + yb[threadIdx.x];  // W x replaces the image term, W r is added to it
    }
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

bool decode_linear_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M, int64_t B) {
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  if (d % V || (k > 0 && k % V)) return false;
  if (d > kMaxStreamD || kTokTile * k > kMaxLinD || k > kMaxSumK) return false;
  // a longer input than the LDS vector: one token streams it a block of columns at a time; a decode batch must be
  // one that the matrix-core kernel takes (it stages slices of the tokens' vectors, never a whole one)
  if (d > kMaxLinD && B != 1 && !tile_rows_shape_ok(m, d, k, B, wdtype)) return false;
  if (k / V > kWave) return false;  // one 16-byte chunk of an image row per lane
  if (reinterpret_cast<uintptr_t>(W) % 16) return false;
  if (M && reinterpret_cast<uintptr_t>(M) % 16) return false;
  return m < (1ll << 30);
}

bool decode_linear_fits(const LinBatch& lb, int wdtype) {
  if (lb.B == 1) return stream_smem_bytes(lb) <= (size_t)kMaxLinD * sizeof(float);
  if (tile_rows_ok(lb, wdtype)) return true;
  return tile_smem(lb) <= (size_t)kMaxLinD * sizeof(float);
}

hipError_t decode_linear_launch(LinBatch& lb, int wdtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (lb.n == 0 || lb.B == 0) return hipSuccess;
  if (lb.B == 1) return stream_rows_launch(lb, wdtype, s, e0, e1);
  if (tile_rows_ok(lb, wdtype)) return tile_rows_launch(lb, s);
  if (tile_smem(lb) > (size_t)kMaxLinD * sizeof(float)) return hipErrorInvalidValue;  // (callers rule this out)
  int total = 0;
  for (int i = 0; i < lb.n; ++i) {
    lb.blk_begin[i] = total;
    total += (int)ceil_div(lb.t[i].m, kRowsPerBlock);
  }
  const size_t smem = tile_smem(lb);
  // one activation vector of up to kMaxLinD floats beside the kernels' static LDS: more than the default 64 KB
  static const hipError_t attr = [] {
    const int bytes = kMaxLinD * (int)sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dense_rows<BF16>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dense_rows<F32>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gated_rows<BF16>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gated_rows<F32>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e;
  }();
  if (attr != hipSuccess) return attr;
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
