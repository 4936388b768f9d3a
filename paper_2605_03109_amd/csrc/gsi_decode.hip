// Decode-time kernels of libgsi (small token counts): bandwidth-bound, 128-bit coalesced loads of
// the stored operands, fp32 accumulation, fixed reduction orders (bit-reproducible run to run).
//
// Three kernel families, each launched over a small table of tasks passed by value, so that the
// projections of several inputs and the linear maps of several weights share one launch:
//
//   proj_partial   : per row-slab of U, partial c = U_slab^T x_slab              (Alg. 1 line 1)
//   proj_residual  : c = sum of partials;  r = x - U c on the slab;  partial |r|^2, |x|^2
//                                                                                 (Alg. 1 lines 2-3)
//   proj_norms     : |r|, |x| from the slab partials (optionally fused with the gate + compaction)
//   gated_rows     : y[rows] = M[rows,:] c  (+ W[rows,:] r for fired tokens)      (Alg. 1 lines 5-7,
//                    in the M c + W r form of Eq. (exact));  also the dense baseline y = W x
//
// Data layout in the workspace of one projection: part_c[nslab][B][k] then part_n[nslab][B][2].
#include "gsi_decode.h"
#include "gsi_device.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

__device__ __forceinline__ int find_task(const int* blk_begin, int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < kMaxTasks; ++i)
    if (i < n && b >= blk_begin[i]) t = i;
  return t;
}

// ------------------------------------------------------------------------------------------------
// proj_partial: one workgroup per (input, row slab).  Thread (ro, cc) owns column chunk cc (kVec
// columns) of rows ro, ro + RPS, ... of the slab and accumulates kVec partial sums per token; the
// RPS row groups are then combined through LDS in a fixed order.
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kBlock) void proj_partial(const ProjBatch pb) {
  constexpr int V = T::kVec;
  __shared__ float xs[kTokTile][kMaxSlabRows];
  __shared__ float red[kBlock * kTokTile * V];  // [ro][tt][cc*V + e] flattened as tid-major

  const int ti = find_task(pb.blk_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  const int slab = blockIdx.x - pb.blk_begin[ti];
  const int d = p.d, k = p.k, B = pb.B;
  const int cpr = k / V;            // column chunks per row (power of two, <= 64)
  const int rps = kBlock / cpr;     // rows per step
  const int cc = threadIdx.x % cpr;
  const int ro = threadIdx.x / cpr;
  const int row0 = slab * p.slab_rows;
  const int rows = min(p.slab_rows, d - row0);
  const typename T::storage* U = reinterpret_cast<const typename T::storage*>(p.U);

  for (int t0 = 0; t0 < B; t0 += kTokTile) {
    const int nt = min(kTokTile, B - t0);
    for (int idx = threadIdx.x; idx < nt * rows; idx += kBlock) {
      const int tt = idx / rows, i = idx % rows;
      xs[tt][i] = load_act(p.X, p.xdtype, (int64_t)(t0 + tt) * d + row0 + i);
    }
    __syncthreads();
    float acc[kTokTile][V];
#pragma unroll
    for (int tt = 0; tt < kTokTile; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) acc[tt][e] = 0.f;
#pragma unroll 4
    for (int i = ro; i < rows; i += rps) {
      float u[V];
      T::load_vec(U + (int64_t)(row0 + i) * k + cc * V, u);
#pragma unroll
      for (int tt = 0; tt < kTokTile; ++tt) {
        if (tt < nt) {
          const float xv = xs[tt][i];
#pragma unroll
          for (int e = 0; e < V; ++e) acc[tt][e] = fmaf(u[e], xv, acc[tt][e]);
        }
      }
    }
    // red[(ro * kTokTile + tt) * k + cc*V + e]
#pragma unroll
    for (int tt = 0; tt < kTokTile; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) red[(ro * kTokTile + tt) * k + cc * V + e] = acc[tt][e];
    __syncthreads();
    for (int idx = threadIdx.x; idx < nt * k; idx += kBlock) {
      const int tt = idx / k, j = idx % k;
      float s = 0.f;
      for (int g = 0; g < rps; ++g) s += red[(g * kTokTile + tt) * k + j];
      p.part_c[((int64_t)slab * B + t0 + tt) * k + j] = s;
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// proj_residual: same decomposition.  Every workgroup first rebuilds the full c of the token tile
// from the slab partials (fixed slab order), then forms r on its rows and the slab's share of the
// two squared norms.
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kBlock) void proj_residual(const ProjBatch pb) {
  constexpr int V = T::kVec;
  __shared__ float cs[kTokTile][kMaxK];
  __shared__ float nr[kWaves][kTokTile], nx[kWaves][kTokTile];

  const int ti = find_task(pb.blk_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  const int slab = blockIdx.x - pb.blk_begin[ti];
  const int d = p.d, k = p.k, B = pb.B;
  const int cpr = k / V;
  const int rps = kBlock / cpr;
  const int cc = threadIdx.x % cpr;
  const int ro = threadIdx.x / cpr;
  const int row0 = slab * p.slab_rows;
  const int rows = min(p.slab_rows, d - row0);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const typename T::storage* U = reinterpret_cast<const typename T::storage*>(p.U);

  for (int t0 = 0; t0 < B; t0 += kTokTile) {
    const int nt = min(kTokTile, B - t0);
    for (int idx = threadIdx.x; idx < nt * k; idx += kBlock) {
      const int tt = idx / k, j = idx % k;
      float s = 0.f;
      for (int sl = 0; sl < p.nslab; ++sl) s += p.part_c[((int64_t)sl * B + t0 + tt) * k + j];
      cs[tt][j] = s;
      if (slab == 0) p.C[(int64_t)(t0 + tt) * k + j] = s;
    }
    __syncthreads();
    float c[kTokTile][V];
#pragma unroll
    for (int tt = 0; tt < kTokTile; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) c[tt][e] = cs[tt][cc * V + e];
    float ar[kTokTile], ax[kTokTile];
#pragma unroll
    for (int tt = 0; tt < kTokTile; ++tt) ar[tt] = ax[tt] = 0.f;
    // every lane of a row group walks the same rows, so the cross-lane sums below are convergent
    const int steps = (rows + rps - 1) / rps;
    for (int st = 0; st < steps; ++st) {
      const int i = st * rps + ro;
      const bool live = i < rows;
      float u[V];
      if (live) {
        T::load_vec(U + (int64_t)(row0 + i) * k + cc * V, u);
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) u[e] = 0.f;
      }
#pragma unroll
      for (int tt = 0; tt < kTokTile; ++tt) {
        if (tt < nt) {
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < V; ++e) s = fmaf(u[e], c[tt][e], s);
          s = group_sum_rt(s, cpr);
          if (live && cc == 0) {
            const int64_t off = (int64_t)(t0 + tt) * d + row0 + i;
            const float x = load_act(p.X, p.xdtype, off);
            const float r = x - s;
            p.R[off] = r;
            ar[tt] = fmaf(r, r, ar[tt]);
            ax[tt] = fmaf(x, x, ax[tt]);
          }
        }
      }
    }
#pragma unroll
    for (int tt = 0; tt < kTokTile; ++tt) {
      const float sr = group_sum<kWave>(ar[tt]);
      const float sx = group_sum<kWave>(ax[tt]);
      if (lane == 0) {
        nr[wave][tt] = sr;
        nx[wave][tt] = sx;
      }
    }
    __syncthreads();
    if (threadIdx.x < nt) {
      float sr = 0.f, sx = 0.f;
      for (int w = 0; w < kWaves; ++w) {
        sr += nr[w][threadIdx.x];
        sx += nx[w][threadIdx.x];
      }
      float* pn = p.part_n + ((int64_t)slab * B + t0 + threadIdx.x) * 2;
      pn[0] = sr;
      pn[1] = sx;
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// proj_norms: |r_t|, |x_t| from the slab partials; one workgroup per input.  With do_gate != 0 the
// same workgroup also evaluates the gate and compacts the fired tokens (ascending order), exactly
// as the stand-alone gate kernel does.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void proj_norms(const ProjBatch pb, int do_gate, float eps) {
  __shared__ int wave_count[kWaves];
  const ProjTask& p = pb.t[blockIdx.x];
  const int B = pb.B;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  int base = 0;
  for (int t0 = 0; t0 < B; t0 += kBlock) {
    const int t = t0 + threadIdx.x;
    bool fired = false;
    if (t < B) {
      float sr = 0.f, sx = 0.f;
      for (int sl = 0; sl < p.nslab; ++sl) {
        const float* pn = p.part_n + ((int64_t)sl * B + t) * 2;
        sr += pn[0];
        sx += pn[1];
      }
      const float rn = sqrtf(sr), xn = sqrtf(sx);
      p.rnorm[t] = rn;
      p.xnorm[t] = xn;
      if (do_gate) {
        fired = (xn > 0.f) && (rn / xn >= eps);
        p.mask[t] = fired ? 1 : 0;
      }
    }
    if (do_gate) {
      const unsigned long long ballot = __ballot(fired);
      const int rank_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
      if (lane == 0) wave_count[wave] = __popcll(ballot);
      __syncthreads();
      int before = 0, total = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const int c = wave_count[w];
        if (w < wave) before += c;
        total += c;
      }
      if (fired) p.fired_idx[base + before + rank_in_wave] = t;
      base += total;
      __syncthreads();
    }
  }
  if (do_gate && threadIdx.x == 0) p.n_fired[0] = base;
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

// ------------------------------------------------------------------------------------------------
// Row dot products: the calling wave computes  A[row, 0:len] . v_t  for its rows and up to TB
// vectors v_t held in LDS as fp32.  A row of `chunks` = len / kVec 16-byte chunks is read by
// LPR = min(64, pow2ceil(chunks)) lanes, so short rows (the image M) pack several rows per wave
// load and long rows (W) use the whole wave with eight independent loads in flight per lane.
// Results go to out[(row - row_base) * TB + t] in LDS.
// ------------------------------------------------------------------------------------------------
template <class T, int TB>
__device__ __forceinline__ void rows_dot(const typename T::storage* __restrict__ A, int64_t ld, int len,
                                         int row_begin, int row_end, int row_base, const float* __restrict__ v,
                                         int vstride, int nt, float* __restrict__ out) {
  constexpr int V = T::kVec;
  constexpr int UNR = 8;
  const int lane = threadIdx.x % kWave;
  const int chunks = len / V;
  int lpr = kWave;
  while (lpr / 2 >= chunks && lpr > 1) lpr >>= 1;  // smallest power of two >= chunks, capped at 64
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
#pragma unroll
              for (int e = 0; e < V; ++e) acc[t] = fmaf(w[u][e], vv[e], acc[t]);
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
#pragma unroll
            for (int e = 0; e < V; ++e) acc[t] = fmaf(w[e], vv[e], acc[t]);
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

// ------------------------------------------------------------------------------------------------
// gated_rows: one workgroup per (map, tile of kRowsPerBlock output rows).
//   phase A: Y[t, rows] = M[rows,:] c_t for every token t (tiles of kTokTile tokens, c in LDS)
//   phase B: for each fired token f (device-side list): Y[f, rows] += W[rows,:] r_f  (r_f in LDS)
// With one token the two phases are summed in LDS and Y is written once.  When n_fired == 0 the
// workgroup never issues a load from W.
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kBlock) void gated_rows(const LinBatch lb) {
  extern __shared__ __align__(16) float vec[];  // max(kTokTile * k, d) floats
  __shared__ float ya[kRowsPerBlock * kTokTile];
  __shared__ float yb[kRowsPerBlock];

  const int ti = find_task(lb.blk_begin, lb.n, blockIdx.x);
  const LinTask& p = lb.t[ti];
  const int B = lb.B;
  const int m = p.m, d = p.d, k = p.k;
  const int row0 = (blockIdx.x - lb.blk_begin[ti]) * kRowsPerBlock;
  const int rows = min(kRowsPerBlock, m - row0);
  const int wave = threadIdx.x / kWave;
  constexpr int RW = kRowsPerBlock / kWaves;
  const int wr0 = row0 + wave * RW;
  const int wr1 = min(wr0 + RW, row0 + rows);
  const typename T::storage* W = reinterpret_cast<const typename T::storage*>(p.W);
  const typename T::storage* M = reinterpret_cast<const typename T::storage*>(p.M);
  int nf = p.n_fired[0];
  nf = nf < 0 ? 0 : (nf > B ? B : nf);

  for (int t0 = 0; t0 < B; t0 += kTokTile) {
    const int nt = min(kTokTile, B - t0);
    for (int idx = threadIdx.x; idx < nt * k; idx += kBlock) vec[idx] = p.C[(int64_t)t0 * k + idx];
    __syncthreads();
    rows_dot<T, kTokTile>(M, k, k, wr0, wr1, row0, vec, k, nt, ya);
    __syncthreads();
    if (B > 1) {
      for (int idx = threadIdx.x; idx < nt * rows; idx += kBlock) {
        const int tt = idx / rows, rr = idx % rows;
        p.Y[(int64_t)(t0 + tt) * m + row0 + rr] = ya[rr * kTokTile + tt];
      }
    }
  }
  if (B == 1) {
    if (nf > 0) {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) vec[idx] = p.R[idx];
      __syncthreads();
      rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
      __syncthreads();
    }
    if (threadIdx.x < rows) {
      float y = ya[threadIdx.x * kTokTile];
      if (nf > 0) y += yb[threadIdx.x];
      p.Y[row0 + threadIdx.x] = y;
    }
    return;
  }
  for (int f = 0; f < nf; ++f) {
    const int t = p.fired_idx[f];
    if (t < 0 || t >= B) continue;  // uniform across the workgroup
    __syncthreads();
    for (int idx = threadIdx.x; idx < d; idx += kBlock) vec[idx] = p.R[(int64_t)t * d + idx];
    __syncthreads();
    rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
    __syncthreads();
    if (threadIdx.x < rows) p.Y[(int64_t)t * m + row0 + threadIdx.x] += yb[threadIdx.x];
  }
}

// dense baseline: Y[t, rows] = W[rows,:] x_t for every token (same row kernel as phase B above)
template <class T>
__global__ __launch_bounds__(kBlock) void dense_rows(const LinBatch lb) {
  extern __shared__ __align__(16) float vec[];
  __shared__ float yb[kRowsPerBlock];
  const int ti = find_task(lb.blk_begin, lb.n, blockIdx.x);
  const LinTask& p = lb.t[ti];
  const int B = lb.B;
  const int m = p.m, d = p.d;
  const int row0 = (blockIdx.x - lb.blk_begin[ti]) * kRowsPerBlock;
  const int rows = min(kRowsPerBlock, m - row0);
  const int wave = threadIdx.x / kWave;
  constexpr int RW = kRowsPerBlock / kWaves;
  const int wr0 = row0 + wave * RW;
  const int wr1 = min(wr0 + RW, row0 + rows);
  const typename T::storage* W = reinterpret_cast<const typename T::storage*>(p.W);
  for (int t = 0; t < B; ++t) {
    if (t > 0) __syncthreads();
    for (int idx = threadIdx.x; idx < d; idx += kBlock) vec[idx] = load_act(p.X, p.xdtype, (int64_t)t * d + idx);
    __syncthreads();
    rows_dot<T, 1>(W, d, d, wr0, wr1, row0, vec, d, 1, yb);
    __syncthreads();
    if (threadIdx.x < rows) p.Y[(int64_t)t * m + row0 + threadIdx.x] = yb[threadIdx.x];
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
bool decode_project_ok(int64_t d, int64_t k, int udtype, const void* U) {
  const int V = udtype == GSI_BF16 ? 8 : 4;
  if (k % V) return false;
  const int64_t cpr = k / V;
  if (cpr > kWave || (cpr & (cpr - 1))) return false;  // chunks per row: power of two, one wave at most
  if (k > kMaxK || d > (1 << 24)) return false;
  return (reinterpret_cast<uintptr_t>(U) % 16) == 0;
}

int decode_slab_rows(int64_t d, int64_t k, int udtype) {
  const int V = udtype == GSI_BF16 ? 8 : 4;
  const int rps = kBlock / (int)(k / V);
  int64_t rows = ceil_div(d, kTargetSlabs);
  rows = ceil_div(rows, rps) * rps;
  if (rows > kMaxSlabRows) rows = kMaxSlabRows / rps * rps;
  if (rows < rps) rows = rps;
  return (int)rows;
}

size_t decode_project_ws(int64_t d, int64_t k, int64_t B, int udtype) {
  const int64_t nslab = ceil_div(d, decode_slab_rows(d, k, udtype));
  return align_up((size_t)nslab * B * k * 4, 256) + align_up((size_t)nslab * B * 2 * 4, 256);
}

void decode_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws) {
  t.d = (int)d;
  t.k = (int)k;
  t.slab_rows = decode_slab_rows(d, k, t.udtype);
  t.nslab = (int)ceil_div(d, t.slab_rows);
  t.part_c = reinterpret_cast<float*>(ws);
  t.part_n = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + align_up((size_t)t.nslab * B * k * 4, 256));
}

hipError_t decode_project_launch(ProjBatch& pb, int udtype, bool with_gate, float eps, hipStream_t s) {
  int total = 0;
  for (int i = 0; i < pb.n; ++i) {
    pb.blk_begin[i] = total;
    total += pb.t[i].nslab;
  }
  if (total == 0 || pb.B == 0) return hipSuccess;
  if (udtype == GSI_BF16) {
    proj_partial<BF16><<<total, kBlock, 0, s>>>(pb);
    proj_residual<BF16><<<total, kBlock, 0, s>>>(pb);
  } else {
    proj_partial<F32><<<total, kBlock, 0, s>>>(pb);
    proj_residual<F32><<<total, kBlock, 0, s>>>(pb);
  }
  proj_norms<<<pb.n, kBlock, 0, s>>>(pb, with_gate ? 1 : 0, eps);
  return hipGetLastError();
}

bool decode_linear_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M) {
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  if (d % V || (k > 0 && k % V)) return false;
  if (d > kMaxLinD || kTokTile * k > kMaxLinD) return false;
  if (reinterpret_cast<uintptr_t>(W) % 16) return false;
  if (M && reinterpret_cast<uintptr_t>(M) % 16) return false;
  return m < (1ll << 30);
}

static size_t lin_smem(const LinBatch& lb, bool dense) {
  size_t fl = 0;
  for (int i = 0; i < lb.n; ++i) {
    size_t need = (size_t)lb.t[i].d;
    if (!dense && (size_t)kTokTile * lb.t[i].k > need) need = (size_t)kTokTile * lb.t[i].k;
    if (need > fl) fl = need;
  }
  return fl * sizeof(float);
}

static int lin_grid(LinBatch& lb) {
  int total = 0;
  for (int i = 0; i < lb.n; ++i) {
    lb.blk_begin[i] = total;
    total += (int)ceil_div(lb.t[i].m, kRowsPerBlock);
  }
  return total;
}

hipError_t decode_gated_launch(LinBatch& lb, int wdtype, hipStream_t s) {
  const int total = lin_grid(lb);
  if (total == 0 || lb.B == 0) return hipSuccess;
  const size_t smem = lin_smem(lb, false);
  if (wdtype == GSI_BF16)
    gated_rows<BF16><<<total, kBlock, smem, s>>>(lb);
  else
    gated_rows<F32><<<total, kBlock, smem, s>>>(lb);
  return hipGetLastError();
}

hipError_t decode_dense_launch(LinBatch& lb, int wdtype, hipStream_t s) {
  const int total = lin_grid(lb);
  if (total == 0 || lb.B == 0) return hipSuccess;
  const size_t smem = lin_smem(lb, true);
  if (wdtype == GSI_BF16)
    dense_rows<BF16><<<total, kBlock, smem, s>>>(lb);
  else
    dense_rows<F32><<<total, kBlock, smem, s>>>(lb);
  return hipGetLastError();
}

}  // namespace gsi
