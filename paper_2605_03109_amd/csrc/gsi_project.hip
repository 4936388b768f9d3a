// Projection kernels of libgsi for small token counts (decode): Algorithm 1, lines 1-3.
//
//   proj_partial   one workgroup per (input, 64-column block of U, row slab): partial
//                  c_j = sum over the slab's rows of U[i,j] x[i]; 128-byte row segments per load group,
//                  fp32 accumulation, the row groups of the workgroup combined through LDS in a
//                  fixed order.  kPartSlabs partials per coefficient.
//   proj_residual  one workgroup per (input, row slab): rebuilds c from the partials (fixed slab
//                  order), forms r = x - U c on its rows, writes R and the slab's share of |r|^2, |x|^2.
//                  The slab of U is requested before the partials so both latencies overlap.
//   proj_norms     |r|, |x| from the slab shares; optionally the gate and the ordered compaction.
//
// Workgroups are handed to the chip's 8 XCDs in turn, each with an L2 of its own.  Both launches therefore walk
// their row slabs in an order that puts the workgroups of the same rows of U on the same XCD, so that the
// residual launch finds the basis in the L2 the partial projection filled.
//
// All reductions have a fixed order: results are bit-identical run to run.
#include <hip/hip_ext.h>

#include <algorithm>

#include "gsi_decode.h"
#include "gsi_device.h"
#include "gsi_image.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kResSlabRows = 64;  // rows of U per residual workgroup, lower bound

template <int N>
__device__ __forceinline__ int find_task(const int (&begin)[N], int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < N; ++i)
    if (i < n && b >= begin[i]) t = i;
  return t;
}

template <class T, int TB>
__global__ __launch_bounds__(kBlock) void proj_partial(const ProjBatch pb) {
  constexpr int V = T::kVec;
  __shared__ float red[kBlock * TB * V];  // [row group][token][column of the block]

  const int ti = find_task(pb.a_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  const int local = blockIdx.x - pb.a_begin[ti];
  // column blocks of one row slab are a_slabs workgroups apart: with a_slabs a multiple of 8 they run on the same
  // XCD (workgroups go to the 8 XCDs in turn), whose L2 then holds all columns of the slab for the residual launch
  const int slab = local % p.a_slabs, cb = local / p.a_slabs;
  const int d = p.d, k = p.k, B = pb.B;
  const int cbw = k < kColBlock ? k : kColBlock;  // columns of this block
  const int lps = cbw / V;                        // lanes per row segment (a power of two)
  const int rps = kBlock / lps;                   // rows per step
  const int lsh = __builtin_ctz(lps);
  const int l = threadIdx.x & (lps - 1), ro = threadIdx.x >> lsh;
  const int col0 = cb * kColBlock + l * V;
  const int row0 = slab * p.a_rows;
  const int rows = min(p.a_rows, d - row0);
  const typename T::storage* U = reinterpret_cast<const typename T::storage*>(p.U) + (int64_t)row0 * k + col0;

  for (int t0 = 0; t0 < B; t0 += TB) {
    const int nt = min(TB, B - t0);
    // token rows of X read by this tile (clamped: loads are unconditional, surplus tokens are dropped below)
    int64_t xoff[TB];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) xoff[tt] = (int64_t)min(t0 + tt, B - 1) * d + row0;
    float acc[TB][V];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) acc[tt][e] = 0.f;
    int i = ro;
    // sixteen (then eight, four) row steps at a time: all loads of a batch are issued before the first use
    for (; i + 15 * rps < rows; i += 16 * rps) {
      uint4 raw[16];
      float xv[16][TB];
#pragma unroll
      for (int q = 0; q < 16; ++q) raw[q] = *reinterpret_cast<const uint4*>(U + (int64_t)(i + q * rps) * k);
#pragma unroll
      for (int q = 0; q < 16; ++q)
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) xv[q][tt] = load_act(p.X, p.xdtype, xoff[tt] + i + q * rps);
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        float u[V];
        T::widen(raw[q], u);
#pragma unroll
        for (int tt = 0; tt < TB; ++tt)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[tt][e] = fmaf(u[e], xv[q][tt], acc[tt][e]);
      }
    }
    for (; i + 7 * rps < rows; i += 8 * rps) {
      uint4 raw[8];
      float xv[8][TB];
#pragma unroll
      for (int q = 0; q < 8; ++q) raw[q] = *reinterpret_cast<const uint4*>(U + (int64_t)(i + q * rps) * k);
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) xv[q][tt] = load_act(p.X, p.xdtype, xoff[tt] + i + q * rps);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float u[V];
        T::widen(raw[q], u);
#pragma unroll
        for (int tt = 0; tt < TB; ++tt)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[tt][e] = fmaf(u[e], xv[q][tt], acc[tt][e]);
      }
    }
    for (; i + 3 * rps < rows; i += 4 * rps) {
      uint4 raw[4];
      float xv[4][TB];
#pragma unroll
      for (int q = 0; q < 4; ++q) raw[q] = *reinterpret_cast<const uint4*>(U + (int64_t)(i + q * rps) * k);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) xv[q][tt] = load_act(p.X, p.xdtype, xoff[tt] + i + q * rps);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float u[V];
        T::widen(raw[q], u);
#pragma unroll
        for (int tt = 0; tt < TB; ++tt)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[tt][e] = fmaf(u[e], xv[q][tt], acc[tt][e]);
      }
    }
    for (; i < rows; i += rps) {
      float u[V];
      T::load_vec(U + (int64_t)i * k, u);
#pragma unroll
      for (int tt = 0; tt < TB; ++tt) {
        const float xv = load_act(p.X, p.xdtype, xoff[tt] + i);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[tt][e] = fmaf(u[e], xv, acc[tt][e]);
      }
    }
#pragma unroll
    for (int tt = 0; tt < TB; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) red[(ro * TB + tt) * cbw + l * V + e] = acc[tt][e];
    __syncthreads();
    for (int idx = threadIdx.x; idx < nt * cbw; idx += kBlock) {
      const int tt = idx / cbw, j = idx % cbw;
      const float* rp = red + tt * cbw + j;
      const int gstride = TB * cbw;
      float s = 0.f;
      for (int g = 0; g < rps; g += 8) {  // rps is a multiple of 8: eight LDS reads in flight, fixed order of adds
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = rp[(g + q) * gstride];
#pragma unroll
        for (int q = 0; q < 8; ++q) s += v[q];
      }
      p.part_c[((int64_t)slab * B + t0 + tt) * k + cb * kColBlock + j] = s;
    }
    __syncthreads();
  }
}

template <class T, int TB>
__global__ __launch_bounds__(kBlock) void proj_residual(const ProjBatch pb) {
  constexpr int V = T::kVec;
  constexpr int PF = 4;  // row steps of U held in registers
  __shared__ __align__(16) float cs[TB][kMaxK];
  __shared__ float nr[kWaves][TB], nx[kWaves][TB];

  const int ti = find_task(pb.b_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  int slab = blockIdx.x - pb.b_begin[ti];
  if (p.b_perm) {
    // walk the slabs so that a workgroup lands on the XCD whose L2 the partial projection left these rows of U in:
    // workgroup j = 8 q + x runs on XCD x (relative to the task's first); it takes residual slab u = q % r of
    // partial-projection slab t = 8 (q / r) + x, which ran on XCD x as well
    const int r = p.b_perm, x = slab & 7, q = slab >> 3;
    slab = ((q / r) * 8 + x) * r + q % r;
  }
  const int d = p.d, k = p.k, B = pb.B;
  const int cpr = k / V;         // 16-byte chunks per row (power of two, <= 64)
  const int rps = kBlock / cpr;  // rows per step
  const int cc = threadIdx.x & (cpr - 1), ro = threadIdx.x >> __builtin_ctz(cpr);
  const int row0 = slab * p.b_rows;
  const int rows = min(p.b_rows, d - row0);
  const int steps = (rows + rps - 1) / rps;
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const typename T::storage* U = reinterpret_cast<const typename T::storage*>(p.U) + (int64_t)row0 * k + cc * V;

  // the slab of U goes in flight first (row index clamped: loads are unconditional) ...
  float upf[PF][V];
#pragma unroll
  for (int q = 0; q < PF; ++q) T::load_vec(U + (int64_t)min(q * rps + ro, rows - 1) * k, upf[q]);

  for (int t0 = 0; t0 < B; t0 += TB) {
    const int nt = min(TB, B - t0);
    // ... with the slab's activations ...
    float xpf[PF][TB];
#pragma unroll
    for (int q = 0; q < PF; ++q)
#pragma unroll
      for (int tt = 0; tt < TB; ++tt)
        xpf[q][tt] = load_act(p.X, p.xdtype, (int64_t)min(t0 + tt, B - 1) * d + row0 + min(q * rps + ro, rows - 1));
    // ... then the partials: c_j = sum over slabs, slab order fixed
    for (int idx = threadIdx.x; idx < nt * k; idx += kBlock) {
      const int tt = idx / k, j = idx % k;
      const float s = sum_partials(p.part_c + (int64_t)(t0 + tt) * k + j, (int64_t)B * k, p.a_slabs);
      cs[tt][j] = s;
      if (slab == 0) p.C[(int64_t)(t0 + tt) * k + j] = s;
    }
    __syncthreads();
    float c[TB][V];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt)
#pragma unroll
      for (int e = 0; e < V; ++e) c[tt][e] = cs[tt][cc * V + e];
    float ar[TB], ax[TB];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) ar[tt] = ax[tt] = 0.f;
    // every lane of a row group walks the same steps, so the cross-lane sums are convergent
    auto row_step = [&](const float (&u)[V], const float (&xv)[TB], int st) {
      const int i = st * rps + ro;
      const bool live = i < rows;
#pragma unroll
      for (int tt = 0; tt < TB; ++tt) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) s = fmaf(u[e], c[tt][e], s);
        s = group_sum_rt(s, cpr);
        if (live && cc == 0 && tt < nt) {
          const float x = xv[tt];
          const float r = x - s;
          p.R[(int64_t)(t0 + tt) * d + row0 + i] = r;
          ar[tt] = fmaf(r, r, ar[tt]);
          ax[tt] = fmaf(x, x, ax[tt]);
        }
      }
    };
#pragma unroll
    for (int q = 0; q < PF; ++q)
      if (q < steps) row_step(upf[q], xpf[q], q);
    for (int st0 = PF; st0 < steps; st0 += PF) {  // further steps, PF at a time with all loads issued first
      float u[PF][V], xv[PF][TB];
#pragma unroll
      for (int q = 0; q < PF; ++q) {
        const int i = min((st0 + q) * rps + ro, rows - 1);
        T::load_vec(U + (int64_t)i * k, u[q]);
#pragma unroll
        for (int tt = 0; tt < TB; ++tt)
          xv[q][tt] = load_act(p.X, p.xdtype, (int64_t)min(t0 + tt, B - 1) * d + row0 + i);
      }
#pragma unroll
      for (int q = 0; q < PF; ++q)
        if (st0 + q < steps) row_step(u[q], xv[q], st0 + q);
    }
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) {
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

// |r_t|, |x_t| (and the gate): one workgroup per input; each wave takes tokens w, w + 4, ... of a
// 256-token chunk, then the chunk is compacted exactly as in the stand-alone gate kernel.
__global__ __launch_bounds__(kBlock) void proj_norms(const ProjBatch pb, int do_gate, float eps) {
  __shared__ int wave_count[kWaves];
  __shared__ unsigned char flag[kBlock];
  const ProjTask& p = pb.t[blockIdx.x];
  const int B = pb.B;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  int base = 0;
  for (int t0 = 0; t0 < B; t0 += kBlock) {
    const int tend = min(B, t0 + kBlock);
    for (int t = t0 + wave; t < tend; t += kWaves) {
      float sr, sx;
      wave_norm_sums(p.part_n, p.b_slabs, B, t, sr, sx);
      if (lane == 0) {
        const float rn = sqrtf(sr), xn = sqrtf(sx);
        p.rnorm[t] = rn;
        p.xnorm[t] = xn;
        flag[t - t0] = gate_fires(rn, xn, eps) ? 1 : 0;
      }
    }
    if (do_gate) {
      __syncthreads();
      const int t = t0 + threadIdx.x;
      const bool fired = t < B && flag[threadIdx.x];
      if (t < B) p.mask[t] = fired ? 1 : 0;
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

// |r|, |x| for many tokens: one thread per token adds the slab shares in slab order (neighbouring
// threads read neighbouring tokens of a slab).  The gate, when asked for, follows as its own launch.
__global__ __launch_bounds__(kBlock) void norms_tokens(const ProjBatch pb) {
  const ProjTask& p = pb.t[blockIdx.y];
  const int B = pb.B;
  const int t = blockIdx.x * kBlock + threadIdx.x;
  if (t >= B) return;
  const float2* src = reinterpret_cast<const float2*>(p.part_n) + t;
  float sr = 0.f, sx = 0.f;
  for (int s0 = 0; s0 < p.b_slabs; s0 += 8) {
    float2 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = src[(int64_t)min(s0 + u, p.b_slabs - 1) * B];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < p.b_slabs) { sr += q[u].x; sx += q[u].y; }
  }
  p.rnorm[t] = sqrtf(sr);
  p.xnorm[t] = sqrtf(sx);
}

// stand-alone image launch (one token): y = M c with c read from C
template <class T>
__global__ __launch_bounds__(kBlock) void image_rows(const ImgBatch ib) {
  __shared__ __align__(16) float cs[kMaxSumK];
  const int b = blockIdx.x;
  int ti = 0;
#pragma unroll
  for (int i = 1; i < kMaxLinTasks; ++i)
    if (i < ib.n && b >= ib.t[i].blk_begin) ti = i;
  image_block<T>(ib.t[ti], b - ib.t[ti].blk_begin, cs);
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
  if (k > kMaxK || d > (int64_t)kPartSlabs * kStageMaxRows) return false;  // 32 slabs of 2048 rows at most
  return (reinterpret_cast<uintptr_t>(U) % 16) == 0;
}

namespace {
struct ProjGeom {
  int a_rows, a_slabs, a_cblocks, b_rows, b_slabs;
};
ProjGeom proj_geom(int64_t d, int64_t k, int udtype) {
  const int V = udtype == GSI_BF16 ? 8 : 4;
  ProjGeom g;
  const int cbw = (int)(k < kColBlock ? k : kColBlock);
  const int rps_a = kBlock / (cbw / V);
  g.a_cblocks = (int)ceil_div(k, kColBlock);
  // one batch of eight row steps per workgroup, unless that would need more than kPartSlabs slabs
  int64_t ar = ceil_div(d, kPartSlabs);
  if (ar < 8 * rps_a) ar = 8 * rps_a;
  g.a_rows = (int)(ceil_div(ar, rps_a) * rps_a);
  g.a_slabs = (int)ceil_div(d, g.a_rows);
  const int rps_b = kBlock / (int)(k / V);
  // At least four row steps and at least 64 rows per workgroup (unless that needs too many slabs).  Measured on
  // GPT-J-sized blocks for k = 64 .. 512: with the image rows riding along, slabs of 64 rows keep the residual
  // launch within one residency round (four workgroups per CU); smaller slabs spill into a second round, larger
  // ones leave too few workgroups to cover the load latency.
  int64_t br = ceil_div(d, kMaxResSlabs);
  if (br < 4 * rps_b) br = 4 * rps_b;
  if (br < kResSlabRows) br = kResSlabRows;
  g.b_rows = (int)(ceil_div(br, rps_b) * rps_b);
  g.b_slabs = (int)ceil_div(d, g.b_rows);
  return g;
}
}  // namespace

size_t decode_project_ws(int64_t d, int64_t k, int64_t B, int udtype) {
  const ProjGeom g = proj_geom(d, k, udtype);
  int s_rows = 0, s_slabs = 0;
  if (B == 1) stage_geom(d, k, udtype, s_rows, s_slabs, true);  // the finer of the two geometries
  const size_t part_slabs = (size_t)std::max(g.a_slabs, s_slabs);
  // (a single token's slab shares of the norms, or the kGateDoubles doubles of the single-pass gate)
  // (B == 1: twice, for the low parts of the partials that the single-pass gate keeps)
  size_t need = align_up(part_slabs * B * k * 4 * (B == 1 ? 2 : 1), 256) +
                align_up(std::max((size_t)g.b_slabs * B * 2 * 4, sizeof(double) * kGateDoubles), 256);
  if (tile_project_shape_ok(d, k, B, udtype)) need = std::max(need, tile_project_ws(d, k, B));
  return need;
}

void decode_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws) {
  t.tile = 0;
  if (tile_project_shape_ok(d, k, B, t.udtype) && t.xdtype == GSI_F32 && reinterpret_cast<uintptr_t>(t.X) % 16 == 0 &&
      reinterpret_cast<uintptr_t>(t.C) % 16 == 0 && reinterpret_cast<uintptr_t>(t.R) % 16 == 0) {
    tile_project_fill(t, d, k, B, ws);
    return;
  }
  const ProjGeom g = proj_geom(d, k, t.udtype);
  t.d = (int)d;
  t.k = (int)k;
  t.a_rows = g.a_rows; t.a_slabs = g.a_slabs; t.a_cblocks = g.a_cblocks;
  t.b_rows = g.b_rows; t.b_slabs = g.b_slabs;
  t.s_rows = t.s_slabs = 0;
  int f_rows = 0, f_slabs = 0;
  if (B == 1) {
    stage_geom(d, k, t.udtype, t.s_rows, t.s_slabs);
    stage_geom(d, k, t.udtype, f_rows, f_slabs, true);
  }
  const size_t part_slabs = (size_t)std::max(g.a_slabs, std::max(t.s_slabs, f_slabs));
  t.part_c = reinterpret_cast<float*>(ws);
  t.part_n = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + align_up(part_slabs * B * k * 4 * (B == 1 ? 2 : 1), 256));
}

hipError_t decode_norms_launch(const ProjBatch& pb, bool with_gate, float eps, hipStream_t s) {
  if (pb.n == 0 || pb.B == 0) return hipSuccess;
  if (pb.B > 4 * kBlock) {  // many tokens: a thread per token, then the stand-alone gate kernel per input
    const dim3 grid((unsigned)ceil_div(pb.B, kBlock), (unsigned)pb.n);
    norms_tokens<<<grid, kBlock, 0, s>>>(pb);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    if (with_gate)
      for (int i = 0; i < pb.n; ++i)
        if (hipError_t e = launch_gate(pb.t[i].rnorm, pb.t[i].xnorm, pb.B, eps, pb.t[i].mask, pb.t[i].fired_idx,
                                       pb.t[i].n_fired, s);
            e != hipSuccess)
          return e;
    return hipSuccess;
  }
  proj_norms<<<pb.n, kBlock, 0, s>>>(pb, with_gate ? 1 : 0, eps);
  return hipGetLastError();
}

hipError_t decode_image_launch(ImgBatch& ib, int wdtype, hipStream_t s) {
  int total = 0;
  for (int i = 0; i < ib.n; ++i) {
    ib.t[i].blk_begin = total;
    total += image_blocks(ib.t[i].m, ib.t[i].k, wdtype, ib.t[i].scale != nullptr);
  }
  ib.total = total;
  if (total == 0) return hipSuccess;
  if (wdtype == GSI_BF16) image_rows<BF16><<<total, kBlock, 0, s>>>(ib);
  else image_rows<F32><<<total, kBlock, 0, s>>>(ib);
  return hipGetLastError();
}

hipError_t decode_project_launch(ProjBatch& pb, int udtype, bool with_norms, bool with_gate, float eps,
                                 hipStream_t s, ImgBatch* img) {
  if (pb.n == 0 || pb.B == 0) return hipSuccess;
  if (pb.B == 1) {
    // one token: the staged kernel, first the partial projections, then residuals (+ the image rows that ride along)
    StageArgs a;
    stage_clear(a, eps);
    for (int i = 0; i < pb.n; ++i) stage_add_part(a, pb.t[i]);
    if (hipError_t e = stage_launch(a, udtype, s); e != hipSuccess) return e;
    stage_clear(a, eps);
    for (int i = 0; i < pb.n; ++i) stage_add_res(a, pb.t[i], false);
    if (img)
      for (int j = 0; j < img->n; ++j) {
        const ImgTask& it = img->t[j];
        int res = -1;
        for (int i = 0; i < pb.n; ++i)
          if (pb.t[i].part_c == it.part_c) res = i;
        if (res < 0) return hipErrorInvalidValue;
        stage_add_img(a, res, it.M, it.Y, it.scale, it.m);
      }
    if (hipError_t e = stage_launch(a, udtype, s); e != hipSuccess) return e;
    if (with_norms) proj_norms<<<pb.n, kBlock, 0, s>>>(pb, with_gate ? 1 : 0, eps);
    return hipGetLastError();
  }
  // tasks of a decode batch that take the matrix-core kernels go in a launch set of their own
  {
    ProjBatch tile_pb = pb, rest = pb;
    tile_pb.n = rest.n = 0;
    for (int i = 0; i < pb.n; ++i) {
      if (pb.t[i].tile) tile_pb.t[tile_pb.n++] = pb.t[i];
      else rest.t[rest.n++] = pb.t[i];
    }
    if (tile_pb.n > 0) {
      if (hipError_t e = tile_project_launch(tile_pb, with_norms, with_gate, eps, s); e != hipSuccess) return e;
      if (rest.n == 0) return hipSuccess;
      pb = rest;
    }
  }
  // the tasks are independent: the largest input goes first so that its workgroups start first
  for (int i = 1; i < pb.n; ++i)
    for (int j = i; j > 0 && (int64_t)pb.t[j].d * pb.t[j].k > (int64_t)pb.t[j - 1].d * pb.t[j - 1].k; --j) {
      const ProjTask tmp = pb.t[j];
      pb.t[j] = pb.t[j - 1];
      pb.t[j - 1] = tmp;
    }
  int ta = 0, tb = 0;
  for (int i = 0; i < pb.n; ++i) {
    pb.a_begin[i] = ta;
    pb.b_begin[i] = tb;
    ta += pb.t[i].a_slabs * pb.t[i].a_cblocks;
    tb += pb.t[i].b_slabs;
  }
  if (ta == 0 || pb.B == 0) return hipSuccess;
  pb.b_total = tb;
  for (int i = 0; i < pb.n; ++i) {
    ProjTask& t = pb.t[i];
    t.b_perm = 0;
    if (t.b_rows > 0 && t.a_rows % t.b_rows == 0) {
      const int r = t.a_rows / t.b_rows;
      if (t.a_slabs % 8 == 0 && t.b_slabs % (8 * r) == 0 && pb.a_begin[i] % 8 == pb.b_begin[i] % 8 &&
          (int64_t)t.a_slabs * t.a_rows == t.d && (int64_t)t.b_slabs * t.b_rows == t.d)
        t.b_perm = r;
    }
  }
  if (udtype == GSI_BF16) {
    proj_partial<BF16, kTokTile><<<ta, kBlock, 0, s>>>(pb);
    proj_residual<BF16, kTokTile><<<tb, kBlock, 0, s>>>(pb);
  } else {
    proj_partial<F32, kTokTile><<<ta, kBlock, 0, s>>>(pb);
    proj_residual<F32, kTokTile><<<tb, kBlock, 0, s>>>(pb);
  }
  if (with_norms) proj_norms<<<pb.n, kBlock, 0, s>>>(pb, with_gate ? 1 : 0, eps);
  return hipGetLastError();
}

}  // namespace gsi
