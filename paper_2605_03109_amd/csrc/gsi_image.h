// Image rows y = M c for ONE token (Algorithm 1, line 5): device code of one 256-thread workgroup,
// shared by the fused residual + image launch of a layer stack and by the stand-alone image kernel.
//
// A workgroup takes eight items of one map (two per wave); an item is four 16-byte loads per lane, i.e. 4 * rpw rows
// of M where rpw = 64 / (lanes per row).  The rows of M are requested first; the projection
// coefficients are then either summed from the row-slab partials (fixed slab order -- the same
// function the residual kernel uses, hence the same bits) or read from C, staged in LDS, and the rows
// are reduced with DPP row sums.  One lane writes each output element.
#pragma once
#include "gsi_decode.h"
#include "gsi_device.h"

namespace gsi {

constexpr int kImgItemsPerBlock = 8;   // two per wave
constexpr int kImgLoads = 4;           // 16-byte loads per lane and item
constexpr int kImgPerWave = kImgItemsPerBlock / 4;

// c_j = sum over row slabs of the partial projections, slab order fixed
__device__ __forceinline__ float sum_partials(const float* __restrict__ pc, int64_t stride, int a_slabs) {
  float s = 0.f;
  int sl = 0;
  for (; sl + 16 <= a_slabs; sl += 16) {
    float v[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) v[q] = pc[(sl + q) * stride];
#pragma unroll
    for (int q = 0; q < 16; ++q) s += v[q];
  }
  for (; sl + 8 <= a_slabs; sl += 8) {
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = pc[(sl + q) * stride];
#pragma unroll
    for (int q = 0; q < 8; ++q) s += v[q];
  }
  for (; sl < a_slabs; ++sl) s += pc[sl * stride];
  return s;
}

// STREAM: the image is larger than the caches keep from one step to the next (many maps in one launch): its rows
// are loaded non-temporally
template <class T, int ITEMS = kImgItemsPerBlock, bool STREAM = false>
__device__ __forceinline__ void image_block_as(const ImgTask& t, int local_block, float* __restrict__ cs) {
  constexpr int kPerWave = ITEMS / 4;
  constexpr int V = T::kVec;
  using S = typename T::storage;
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int k = t.k, m = t.m;
  const int chunks = k / V;
  const int lsh = chunks <= 1 ? 0 : 32 - __builtin_clz(chunks - 1);
  const int lpr = 1 << lsh, rpw = kWave >> lsh;  // lanes per row (power of two >= chunks), rows per wave load
  const int l = lane & (lpr - 1), sub = lane >> lsh;
  const bool live = l * V < k;
  const int col = live ? l * V : k - V;
  const S* M = reinterpret_cast<const S*>(t.M) + col;
  const int item0 = local_block * ITEMS + wave * kPerWave;
  uint4 raw[kPerWave][kImgLoads];
#pragma unroll
  for (int it = 0; it < kPerWave; ++it)
#pragma unroll
    for (int u = 0; u < kImgLoads; ++u) {
      const int row = ((item0 + it) * kImgLoads + u) * rpw + sub;
      const S* src = M + (int64_t)(row < m ? row : m - 1) * k;
      raw[it][u] = STREAM ? load_stream16(src) : *reinterpret_cast<const uint4*>(src);
    }
  // E4M3 codes: the rows' power-of-two scales, requested with the rows (a load at the point of use would put one
  // more memory round trip at the end of the workgroup)
  float rscale[kPerWave][kImgLoads];
  if constexpr (T::kVec == 16) {
#pragma unroll
    for (int it = 0; it < kPerWave; ++it)
#pragma unroll
      for (int u = 0; u < kImgLoads; ++u) {
        const int row = ((item0 + it) * kImgLoads + u) * rpw + sub;
        rscale[it][u] = t.scale[row < m ? row : m - 1];
      }
  }
  for (int j = threadIdx.x; j < k; j += 256) cs[j] = t.part_c ? sum_partials(t.part_c + j, k, t.a_slabs) : t.C[j];
  __syncthreads();
  float cvv[V];
#pragma unroll
  for (int q = 0; q < V / 4; ++q) {
    const float4 x = reinterpret_cast<const float4*>(cs + col)[q];
    cvv[4 * q + 0] = x.x; cvv[4 * q + 1] = x.y; cvv[4 * q + 2] = x.z; cvv[4 * q + 3] = x.w;
  }
#pragma unroll
  for (int it = 0; it < kPerWave; ++it)
#pragma unroll
    for (int u = 0; u < kImgLoads; ++u) {
      float w[V];
      T::widen(raw[it][u], w);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < V; ++e) s = fmaf(w[e], cvv[e], s);
      s = group_sum_rt(live ? s : 0.f, lpr);
      const int row = ((item0 + it) * kImgLoads + u) * rpw + sub;
      if (l == 0 && row < m) {
        if constexpr (T::kVec == 16) s *= rscale[it][u];
        t.Y[row] = s;
      }
    }
}

// T: storage of an image in the weights' dtype; a task with row scales holds E4M3 codes instead (Section 7,
// "Combination with quantization").  The choice is uniform over the workgroup.
template <class T, int ITEMS = kImgItemsPerBlock, bool STREAM = false>
__device__ __forceinline__ void image_block(const ImgTask& t, int local_block, float* __restrict__ cs) {
  if (t.scale) image_block_as<FP8, ITEMS, STREAM>(t, local_block, cs);
  else image_block_as<T, ITEMS, STREAM>(t, local_block, cs);
}

// workgroups a map needs in an image launch
inline int image_blocks(int64_t m, int64_t k, int wdtype, bool fp8 = false, int items = kImgItemsPerBlock) {
  const int V = fp8 ? 16 : wdtype == GSI_BF16 ? 8 : 4;
  int lpr = 1;
  while (lpr < k / V) lpr <<= 1;
  const int64_t rows_per_item = (int64_t)kImgLoads * (kWave / lpr);
  return (int)ceil_div(ceil_div(m, rows_per_item), items);
}

}  // namespace gsi
