// Rows of one weight matrix streamed against a vector staged in LDS: the slow-path product W r (or W x) of
// Eq. (exact) / Algorithm 1 line 7 for ONE token.  Device code shared by the stand-alone weight-streaming
// kernel and by the fused single-token kernel, so that both give the same bits for a row.
//
// The waves of the grid are dealt rows round-robin (wave `first`, first + GW, ...).  A row is consumed in
// units of kLU 16-byte loads per lane; fp32 FMA against the staged vector, a DPP wave reduction, and one
// lane updates the output element (exactly one lane of the grid touches each element).
#pragma once
#include "gsi_device.h"

namespace gsi {

constexpr int kLU = 8;  // 16-byte loads per lane in a unit

template <class T>
struct Raw {  // 16 bytes as loaded; widened to fp32 when consumed
  uint4 v;
  // NT: a launch that streams far more than the caches hold loads its weights non-temporally (6.7 TB/s against
  // 6.0 TB/s on 1.6 GB); a launch whose weights may still be in the 256 MB memory-side cache from the step before
  // loads them normally (non-temporal loads would forfeit those hits)
  template <bool NT>
  __device__ __forceinline__ void load(const typename T::storage* p) {
    if constexpr (NT) v = load_stream16(p);
    else v = *reinterpret_cast<const uint4*>(p);
  }
  __device__ __forceinline__ void widen(float (&f)[T::kVec]) const { T::widen(v, f); }
};

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

// How the old value of an output element is read when the product is added to it: a plain load, or a load
// that is coherent across the chip (the element was written earlier in the same launch by another workgroup).
template <bool COHERENT>
__device__ __forceinline__ float load_old(const float* p) {
  if constexpr (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

// Rows first, first + GW, ... (< m) of a matrix by the calling wave: d columns of every row, rows ld elements apart
// (ld = d for a whole matrix W[m, d]; a block of columns of a longer row otherwise); xs = the staged vector
// (d floats, LDS).
// whole: the product replaces y (dense baseline, W x form of the slow path); else it is added to y.
// TAIL: d / kVec is not a multiple of 64 * kLU (loads clamped, surplus products dropped).
template <class T, bool TAIL, bool COHERENT, bool NT = false>
__device__ __forceinline__ void stream_map_rows(const typename T::storage* __restrict__ W, float* __restrict__ Y,
                                                int m, int d, int64_t ld, const float* __restrict__ xs, bool whole,
                                                int first, int GW, int lane) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  const int chunks = d / V;
  const int nseg = (chunks + kWave * kLU - 1) / (kWave * kLU);  // units per row
  if constexpr (!TAIL) {
    // Software-pipelined: units of kLU loads per lane, two register buffers; the loads of the next
    // unit are issued before the current one is consumed.  The loop body is straight-line code
    // with unconditional loads and no stores (results are parked in lane (row index mod 64) of a
    // register and written once per 64 rows), so a wave always has a unit in flight.
    const int nrows = first < m ? (m - first + GW - 1) / GW : 0;
    const int64_t seg_step = (int64_t)kWave * kLU * V;                       // elements to the next unit of a row
    const int64_t row_step = (int64_t)GW * ld - (int64_t)(nseg - 1) * seg_step;  // last unit of a row -> next row
    for (int j0 = 0; j0 < nrows; j0 += kWave) {
      const int cnt = min(kWave, nrows - j0);
      const int nu = cnt * nseg;
      const S* p0 = W + (int64_t)(first + (int64_t)j0 * GW) * ld + (int64_t)lane * V;
      float res = 0.f, acc = 0.f;
      Raw<T> A[kLU], Bb[kLU];
      auto issue = [&](Raw<T> (&buf)[kLU], const S* ptr) {
        __builtin_amdgcn_sched_barrier(0);  // keep the loads here: ahead of the arithmetic that follows
#pragma unroll
        for (int q = 0; q < kLU; ++q) buf[q].template load<NT>(ptr + (int64_t)q * kWave * V);
        __builtin_amdgcn_sched_barrier(0);
      };
      auto consume = [&](const Raw<T> (&buf)[kLU], int jj, int sg) {
        const float* xp = xs + (sg * kWave * kLU + lane) * V;
#pragma unroll
        for (int q = 0; q < kLU; ++q) {
          float w[V], xv[V];
          buf[q].widen(w);
          lds_vec<V>(xp + q * kWave * V, xv);
          acc = dotv<V>(w, xv, acc);
        }
        const bool last = sg == nseg - 1;
        const float sum = group_sum<kWave>(acc);
        res = (last && lane == jj) ? sum : res;
        acc = last ? 0.f : acc;
      };
      // unit u: row index jj = u / nseg, segment sg = u % nseg; pointers advance incrementally
      const S* pa = p0;
      int jja = 0, sga = 0;
      issue(A, pa);
      int u = 0;
      while (u + 2 < nu) {
        const S* pb = pa + (sga == nseg - 1 ? row_step : seg_step);
        const int jjb = sga == nseg - 1 ? jja + 1 : jja, sgb = sga == nseg - 1 ? 0 : sga + 1;
        issue(Bb, pb);
        consume(A, jja, sga);
        pa = pb + (sgb == nseg - 1 ? row_step : seg_step);
        jja = sgb == nseg - 1 ? jjb + 1 : jjb;
        sga = sgb == nseg - 1 ? 0 : sgb + 1;
        issue(A, pa);
        consume(Bb, jjb, sgb);
        u += 2;
      }
      if (u + 1 < nu) {
        const S* pb = pa + (sga == nseg - 1 ? row_step : seg_step);
        const int jjb = sga == nseg - 1 ? jja + 1 : jja, sgb = sga == nseg - 1 ? 0 : sga + 1;
        issue(Bb, pb);
        consume(A, jja, sga);
        consume(Bb, jjb, sgb);
      } else {
        consume(A, jja, sga);
      }
      if (lane < cnt) {  // lane j holds the sum of this wave's row j0 + j
        float* yp = Y + first + (int64_t)(j0 + lane) * GW;
        float old = 0.f;
        if (!whole) old = load_old<COHERENT>(yp);  // image term written earlier (uniform branch)
        *yp = old + res;
      }
    }
  } else {
    for (int row = first; row < m; row += GW) {
      float acc = 0.f;
      float yold = 0.f;
      if (!whole) yold = load_old<COHERENT>(Y + row);  // the image term written earlier
      for (int sg = 0; sg < nseg; ++sg) {
        Raw<T> buf[kLU];
        const int cb = sg * kWave * kLU + lane;
#pragma unroll
        for (int q = 0; q < kLU; ++q) {
          int c = cb + q * kWave;
          c = c < chunks ? c : chunks - 1;
          buf[q].template load<NT>(W + (int64_t)row * ld + (int64_t)c * V);
        }
#pragma unroll
        for (int q = 0; q < kLU; ++q) {
          const int c = cb + q * kWave;
          float w[V], xv[V];
          buf[q].widen(w);
          lds_vec<V>(xs + (c < chunks ? c : chunks - 1) * V, xv);
          const float part = dotv<V>(w, xv, 0.f);
          acc += c < chunks ? part : 0.f;
        }
      }
      acc = group_sum<kWave>(acc);
      if (lane == 0) Y[row] = yold + acc;
    }
  }
}

}  // namespace gsi
