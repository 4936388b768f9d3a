// Single-token linear-map kernel of libgsi: Algorithm 1 lines 4-7 in the y = M c (+ W r when the
// gate fires) form of Eq. (exact), and the dense baseline y = W x, for one decode token.
//
// A persistent grid of two 512-thread workgroups per CU (sixteen waves per CU).  Structure of one launch:
//   1. gate of every input group, evaluated redundantly by every wave from the residual kernel's
//      partial norms (identical arithmetic => identical decision everywhere, no communication), or
//      read from the published count;
//   2. the projection coefficients of all groups are staged in LDS;
//   3. "short" phase: rows of the image M of maps whose input did NOT fire.  Items of four 16-byte
//      loads per lane (several rows per 1-KB wave load when k is small), dealt round-robin over the
//      waves of the grid;
//   4. "long" phase, once per fired group: the residual vector is staged in LDS, then rows of W (and
//      the matching row of M) are streamed, one row per wave, in units of eight 16-byte loads per lane.
// In 3 and 4 the next unit's loads are issued before the current unit is consumed (two register
// buffers, all loads unconditional with clamped addresses) so that a wave always has loads in flight.
// Every output element is written exactly once, by one lane.  A map whose input did not fire never
// issues a load from W.
#include <hip/hip_ext.h>

#include <cstdlib>

#include "gsi_decode.h"
#include "gsi_device.h"

// Phase markers: empty in the library; a profiling build may define GSI_MARK(i) to record a timestamp.
#ifndef GSI_MARK
#define GSI_MARK(i)
#endif

namespace gsi {
namespace {

constexpr int kBlock = 512;  // eight waves share one staged activation vector
constexpr int kWaves = kBlock / kWave;
constexpr int kSU = 4;  // loads per lane in a short item
constexpr int kLU = 8;  // loads per lane in a long unit

template <class T>
struct Raw {  // 16 bytes as loaded; widened to fp32 when consumed
  uint4 v;
  __device__ __forceinline__ void load(const typename T::storage* p) { v = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void widen(float (&f)[T::kVec]) const;
};
template <>
__device__ __forceinline__ void Raw<BF16>::widen(float (&f)[8]) const {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}
template <>
__device__ __forceinline__ void Raw<F32>::widen(float (&f)[4]) const {
  f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}

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

template <class T, bool DENSE, bool TAIL>
__global__ __launch_bounds__(kBlock) void stream_rows(const LinBatch lb) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  extern __shared__ __align__(16) float smem[];  // [coefficients of every group][one activation vector]

  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform by construction
  const int gw = blockIdx.x * kWaves + wave;  // this wave's index in the grid
  const int GW = gridDim.x * kWaves;
  const int ng = lb.ng, n = lb.n;
  GSI_MARK(0);

  // ---- 0. the first two image-row items of this wave go in flight before anything else ------------
  // (they do not depend on the gate; an item of a map that turns out to have fired is dropped)
  struct Item {
    const S* base;  // this lane's chunk in row 0 of the task's image
    float* y;
    int row0, rpw, lpr, m, k, coff, group, live;
  };
  auto coff = [&](int gi) {
    int o = 0;
    for (int i = 0; i < gi; ++i) o += lb.g[i].k;
    return o;
  };
  const int total_items = DENSE ? 0 : lb.short_begin[n];
  auto locate = [&](int v) {
    Item it;
    it.live = v < total_items;
    v = it.live ? v : total_items - 1;
    // every task's fields are read at fixed argument offsets (independent scalar loads), then selected
    const LinTask* tp = &lb.t[0];
    int base = 0;
    const void* Mp = tp->M;
    it.y = tp->Y;
    it.m = tp->m;
    it.group = tp->group;
    it.k = tp->k;
    int co = tp->coff;
#pragma unroll
    for (int i = 1; i < kMaxTasks; ++i) {
      const bool ge = i < n && v >= lb.short_begin[i];
      const LinTask& t = lb.t[i];
      base = ge ? lb.short_begin[i] : base;
      Mp = ge ? t.M : Mp;
      it.y = ge ? t.Y : it.y;
      it.m = ge ? t.m : it.m;
      it.group = ge ? t.group : it.group;
      it.k = ge ? t.k : it.k;
      co = ge ? t.coff : co;
    }
    const int chunks = it.k / V;
    const int lsh = chunks <= 1 ? 0 : 32 - __builtin_clz(chunks - 1);
    it.lpr = 1 << lsh;  // lanes per row: smallest power of two >= chunks
    it.rpw = kWave >> lsh;
    it.row0 = (v - base) * kSU * it.rpw + (lane >> lsh);
    const int l = lane & (it.lpr - 1);
    const int col = l * V < it.k ? l * V : it.k - V;
    it.live = it.live && (l * V < it.k);
    it.base = reinterpret_cast<const S*>(Mp) + col;
    it.coff = co + col;
    return it;
  };
  auto issue = [&](const Item& it, Raw<T> (&buf)[kSU]) {
#pragma unroll
    for (int u = 0; u < kSU; ++u) {
      const int row = it.row0 + u * it.rpw;
      buf[u].load(it.base + (int64_t)(row < it.m ? row : it.m - 1) * it.k);
    }
  };
  auto consume = [&](const Item& it, const Raw<T> (&buf)[kSU], unsigned fired) {
    float cvv[V];
    lds_vec<V>(smem + it.coff, cvv);
    const bool live = it.live && !((fired >> it.group) & 1u);
    const bool head = (lane & (it.lpr - 1)) == 0;
#pragma unroll
    for (int u = 0; u < kSU; ++u) {
      float w[V];
      buf[u].widen(w);
      float s = live ? dotv<V>(w, cvv, 0.f) : 0.f;
      s = group_sum_rt(s, it.lpr);
      const int row = it.row0 + u * it.rpw;
      if (live && head && row < it.m) it.y[row] = s;
    }
  };
  Raw<T> bufA[kSU], bufB[kSU];
  Item itA, itB;
  const bool haveB = gw + GW < total_items;  // wave-uniform
  if constexpr (!DENSE) {
    if (total_items > 0) {
      itA = locate(gw);
      issue(itA, bufA);
      if (haveB) {
        itB = locate(gw + GW);
        issue(itB, bufB);
      }
    }
  }

  GSI_MARK(1);
  // ---- 1. gates: one wave per group in every workgroup (identical arithmetic in every workgroup, hence
  //         the same decision across the grid without communication) -----------------------------------
  __shared__ unsigned s_fired_g[kMaxTasks];
  if constexpr (!DENSE) {
    for (int gi = wave; gi < ng; gi += kWaves) {  // wave gi evaluates the gate of group gi
      const LinGroup& g = lb.g[gi];
      bool f;
      if (lb.inline_gate) {
        const float2* pn = reinterpret_cast<const float2*>(g.part_n);
        const int ns = g.b_slabs;
        float2 v[kMaxResSlabs / kWave];
#pragma unroll
        for (int q = 0; q < kMaxResSlabs / kWave; ++q) {  // clamped: the loads are unconditional
          const int sl = lane + q * kWave;
          v[q] = pn[sl < ns ? sl : ns - 1];
        }
        float ar = 0.f, ax = 0.f;
#pragma unroll
        for (int q = 0; q < kMaxResSlabs / kWave; ++q) {
          const bool ok = lane + q * kWave < ns;
          ar += ok ? v[q].x : 0.f;
          ax += ok ? v[q].y : 0.f;
        }
        const float rn = sqrtf(group_sum<kWave>(ar)), xn = sqrtf(group_sum<kWave>(ax));
        f = gate_fires(rn, xn, lb.eps);
        if (blockIdx.x == 0 && lane == 0) {  // publish what the norm and gate kernels would write
          g.rnorm[0] = rn;
          g.xnorm[0] = xn;
          g.mask[0] = f ? 1 : 0;
          if (f) g.fired_idx_out[0] = 0;
          g.n_fired_out[0] = f ? 1 : 0;
        }
      } else {
        f = g.n_fired[0] > 0;
      }
      if (lane == 0) s_fired_g[gi] = f ? 1u : 0u;
    }
  }

  GSI_MARK(2);
  // ---- 2. coefficients of every group into LDS: the last waves of the workgroup stage them while the
  //         first ones evaluate the gates (group gi is staged by wave kWaves - 1 - gi) -----------------
  int sumk = 0;
  if constexpr (!DENSE) {
    for (int gi = 0; gi < ng; ++gi) sumk += lb.g[gi].k;
    for (int gi = kWaves - 1 - wave; gi < ng; gi += kWaves) {
      const LinGroup& g = lb.g[gi];
      const int k = g.k;  // <= 512: at most two float4 per lane
      float* dst = smem + coff(gi);
      const int i0 = lane * 4, i1 = lane * 4 + kWave * 4;
      const float4 a = *reinterpret_cast<const float4*>(g.C + (i0 < k ? i0 : k - 4));
      const float4 b2 = *reinterpret_cast<const float4*>(g.C + (i1 < k ? i1 : k - 4));
      if (i0 < k) *reinterpret_cast<float4*>(dst + i0) = a;
      if (i1 < k) *reinterpret_cast<float4*>(dst + i1) = b2;
    }
  }
  GSI_MARK(3);
  __syncthreads();
  GSI_MARK(4);
  unsigned fired_mask = 0;
  if constexpr (DENSE) {
    fired_mask = (1u << ng) - 1u;
  } else {
    for (int gi = 0; gi < ng; ++gi) fired_mask |= s_fired_g[gi] << gi;
    fired_mask = __builtin_amdgcn_readfirstlane(fired_mask);
  }
  float* xs = smem + sumk;

  // ---- 3. short phase: image rows of maps whose input did not fire --------------------------------------
  if constexpr (!DENSE) {
    if (total_items > 0) {
      consume(itA, bufA, fired_mask);
      if (haveB) consume(itB, bufB, fired_mask);
      for (int v = gw + 2 * GW; v < total_items; v += 2 * GW) {  // only when the grid is small for the maps
        itA = locate(v);
        itB = locate(v + GW);
        issue(itA, bufA);
        issue(itB, bufB);
        consume(itA, bufA, fired_mask);
        consume(itB, bufB, fired_mask);
      }
    }
  }

  GSI_MARK(5);
  // ---- 4. long phase: rows of W of fired maps (every map in the dense baseline) ------------------------
  for (int gi = 0; gi < ng; ++gi) {
    if (!((fired_mask >> gi) & 1u)) continue;  // uniform across the grid
    const LinGroup& g = lb.g[gi];
    const int d = g.d;
    const int k = DENSE ? V : g.k;
    const int chunks = d / V;
    const int nseg = (chunks + kWave * kLU - 1) / (kWave * kLU);  // units per row

    // stage the activation vector (readers of the previous group's vector are past the barrier)
    __syncthreads();
    if (DENSE && g.xdtype != GSI_F32) {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) xs[idx] = load_act(g.X, g.xdtype, idx);
    } else {
      const float4* src = reinterpret_cast<const float4*>(DENSE ? reinterpret_cast<const float*>(g.X) : g.R);
      float4* dst = reinterpret_cast<float4*>(xs);
      const int n4 = d / 4;
      int i = threadIdx.x;
      for (; i + 3 * kBlock < n4; i += 4 * kBlock) {  // four independent loads per thread and trip
        const float4 a = src[i], b = src[i + kBlock], c = src[i + 2 * kBlock], e = src[i + 3 * kBlock];
        dst[i] = a;
        dst[i + kBlock] = b;
        dst[i + 2 * kBlock] = c;
        dst[i + 3 * kBlock] = e;
      }
      for (; i < n4; i += kBlock) dst[i] = src[i];
    }
    __syncthreads();

    // this lane's chunk of the group's coefficients (zero beyond k)
    float cvv[V];
    const int mcol = lane * V < k ? lane * V : k - V;
    if constexpr (!DENSE) {
      lds_vec<V>(smem + coff(gi) + mcol, cvv);
      if (lane * V >= k) {
#pragma unroll
        for (int e = 0; e < V; ++e) cvv[e] = 0.f;
      }
    }

    int first = gw;  // rows of the group's maps are dealt round-robin, map after map
    for (int ti = 0; ti < n; ++ti) {
      const LinTask& t = lb.t[ti];
      if (t.group != gi) continue;  // uniform
      const int m = t.m;
      const S* W = reinterpret_cast<const S*>(t.W);
      const S* M = reinterpret_cast<const S*>(t.M);
      for (int row = first; row < m; row += GW) {
        const S* wr = W + (int64_t)row * d + (int64_t)lane * V;
        float acc = 0.f;
        Raw<T> mb;
        if constexpr (!DENSE) mb.load(M + (int64_t)row * k + mcol);
        for (int sg = 0; sg < nseg; ++sg) {
          Raw<T> buf[kLU];
          const int cb = sg * kWave * kLU + lane;
#pragma unroll
          for (int q = 0; q < kLU; ++q) {
            int c = cb + q * kWave;
            if (TAIL) c = c < chunks ? c : chunks - 1;
            buf[q].load(W + (int64_t)row * d + (int64_t)c * V);
          }
          if (!DENSE && sg == 0) {
            float mv[V];
            mb.widen(mv);
            acc = dotv<V>(mv, cvv, acc);
          }
#pragma unroll
          for (int q = 0; q < kLU; ++q) {
            const int c = cb + q * kWave;
            float w[V], xv[V];
            buf[q].widen(w);
            if (TAIL) {
              lds_vec<V>(xs + (c < chunks ? c : chunks - 1) * V, xv);
              const float part = dotv<V>(w, xv, 0.f);
              acc += c < chunks ? part : 0.f;
            } else {
              lds_vec<V>(xs + c * V, xv);
              acc = dotv<V>(w, xv, acc);
            }
          }
        }
        (void)wr;
        acc = group_sum<kWave>(acc);
        if (lane == 0) t.Y[row] = acc;
      }
      // continue the deal: the next map starts with the wave after the one that took this map's last row
      first = (first - m % GW + GW) % GW;
    }
  }
  GSI_MARK(6);
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

template <class T, bool DENSE, bool TAIL>
hipError_t launch_one(const LinBatch& lb, unsigned grid, size_t smem, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  static const hipError_t attr =  // the kernel may use more than the default 64 KB of dynamic LDS
      hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<T, DENSE, TAIL>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (kMaxLinD + kMaxSumK) * (int)sizeof(float));
  if (attr != hipSuccess) return attr;
  if (e0 && e1) {  // the events take the dispatch's own start and stop timestamps
    hipExtLaunchKernelGGL((stream_rows<T, DENSE, TAIL>), dim3(grid), dim3(kBlock), smem, s, e0, e1, 0, lb);
  } else {
    stream_rows<T, DENSE, TAIL><<<grid, kBlock, smem, s>>>(lb);
  }
  return hipGetLastError();
}

template <class T>
hipError_t launch_dtype(const LinBatch& lb, bool tail, unsigned grid, size_t smem, hipStream_t s, hipEvent_t e0,
                        hipEvent_t e1) {
  if (lb.dense)
    return tail ? launch_one<T, true, true>(lb, grid, smem, s, e0, e1) : launch_one<T, true, false>(lb, grid, smem, s, e0, e1);
  return tail ? launch_one<T, false, true>(lb, grid, smem, s, e0, e1) : launch_one<T, false, false>(lb, grid, smem, s, e0, e1);
}

}  // namespace

size_t stream_smem_bytes(const LinBatch& lb) {
  size_t sumk = 0, maxd = 0;
  for (int i = 0; i < lb.ng; ++i) {
    if (!lb.dense) sumk += (size_t)lb.g[i].k;
    if ((size_t)lb.g[i].d > maxd) maxd = (size_t)lb.g[i].d;
  }
  return (sumk + maxd) * sizeof(float);
}

hipError_t stream_rows_launch(LinBatch& lb, int wdtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  // persistent grid: a few workgroups per CU, never more waves than rows
  static const int per_cu = env_int("GSI_LIN_WGS_PER_CU", 2);
  int64_t rows = 0;
  bool tail = false;
  int items = 0;
  for (int i = 0; i < lb.n; ++i) {
    rows += lb.t[i].m;
    const LinGroup& g = lb.g[lb.t[i].group];
    lb.t[i].k = g.k;
    lb.t[i].coff = 0;
    for (int gi = 0; gi < lb.t[i].group; ++gi) lb.t[i].coff += lb.g[gi].k;
    if ((g.d / V) % (kWave * kLU)) tail = true;
    lb.short_begin[i] = items;
    if (!lb.dense) {
      const int chunks = g.k / V;
      int lpr = 1;
      while (lpr < chunks) lpr <<= 1;
      items += (int)ceil_div(lb.t[i].m, (int64_t)kSU * (kWave / lpr));
    }
  }
  for (int i = lb.n; i <= kMaxTasks; ++i) lb.short_begin[i] = items;
  int64_t grid = (int64_t)per_cu * num_cus();
  if (grid > ceil_div(rows, kWaves)) grid = ceil_div(rows, kWaves);
  if (grid < 1) grid = 1;
  const size_t smem = stream_smem_bytes(lb);
  return wdtype == GSI_BF16 ? launch_dtype<BF16>(lb, tail, (unsigned)grid, smem, s, e0, e1)
                            : launch_dtype<F32>(lb, tail, (unsigned)grid, smem, s, e0, e1);
}

}  // namespace gsi
