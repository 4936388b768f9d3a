// Single-token projection kernel of libgsi: Algorithm 1, lines 1-5 for ONE token, as stages of one kernel.
//
// A launch holds up to four kinds of 256-thread workgroups, told apart by their index:
//   partial    one per (input, row slab): whole rows of U (contiguous slabs), partial c_j over the slab's rows, the
//              row groups combined through LDS in a fixed order;
//   sum        one per input: c = the partials added in slab order, written to C (calls of one set skip this
//              stage: their residual and image workgroups add the partials themselves, with the same function);
//   residual   one per (input, row slab): r = x - U c on the slab's rows, R, the slab's share of |r|^2, |x|^2;
//   image      rows y = M c of the maps that read the residual inputs (gsi_image.h);
//   gate       one per input: |r|, |x| from the slab shares in a fixed order, Eq. (gate), and what the stand-alone
//              gate kernel would publish (rnorm, xnorm, mask, fired_idx, n_fired), so the weight kernel that
//              follows reads one count per input.
// Sets of inputs are independent of each other, so launch L holds the partial projections of set L, the sums of
// set L - 1, the residuals and image rows of set L - 2 and the gates of set L - 3: the ramp and tail of one stage
// fill with the others and a call of n sets makes n + 3 launches instead of 3 n.  Nothing inside a launch waits
// for anything else in it: every dependency is a launch boundary.
//
//
// Single-pass gate (inputs with a cached E = U^T U - I): |r|^2 = |x|^2 - |c|^2 + c^T E c holds for ANY stored U when
// c = U^T x, so the gate needs no second pass over U.  The partial workgroups also write their slab's share of
// |x|^2; the sum stage becomes kGramBlocks workgroups per input that add the partials, take a block of rows of E
// each and write their share of c^T E c; every residual workgroup then evaluates the gate from those shares
// (identical arithmetic, so the verdict is uniform without communication), workgroup 0 of the input publishes
// it, and r = x - U c is formed only when the gate fires.  The shares of the two large terms and the final
// combination are fp64: their difference is 400 times smaller than either at the threshold 0.05.
//
// All sums have a fixed order: results are bit-identical run to run.
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "gsi_decode.h"
#include "gsi_device.h"
#include "gsi_image.h"

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

// sum over the wave in a fixed (butterfly) order; every lane gets the total
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Eq. (gate) from the single-pass shares of one input: gw = [slabs shares of |x|^2][kGramBlocks shares of
// c^T E c][|c|^2].  Called by whole waves: the lanes load the shares side by side (a few memory latencies in all,
// not one per share), the sums run in a fixed order (lane-strided, then a butterfly over the wave), so every wave
// of every workgroup reaches the same verdict.
__device__ __forceinline__ bool single_pass_gate(const double* __restrict__ gw, int slabs, float eps, float& rn,
                                                 float& xn) {
  const int lane = threadIdx.x % kWave;
  double a = 0.0;
  for (int s = lane; s < slabs; s += kWave) a += gw[s];
  const double v = lane < kGramBlocks + kC2Shares ? gw[slabs + lane] : 0.0;
  const double x2 = wave_sum_f64(a);
  const double q = wave_sum_f64(lane < kGramBlocks ? v : 0.0);
  const double c2 = wave_sum_f64(lane >= kGramBlocks ? v : 0.0);
  const double r2 = x2 - c2 + q;
  rn = (float)sqrt(r2 > 0.0 ? r2 : 0.0);
  xn = (float)sqrt(x2);
  return gate_fires(rn, xn, eps);
}

__device__ __forceinline__ void publish_gate(const StageGate& g, float rn, float xn, bool f) {
  g.rnorm[0] = rn;
  g.xnorm[0] = xn;
  g.mask[0] = f ? 1 : 0;
  if (f) g.fired_idx[0] = 0;
  g.n_fired[0] = f ? 1 : 0;
}

// STREAM: the first two batches of U are loaded non-temporally (a launch over many inputs: nothing is read again soon)
template <class T, bool STREAM = false>
__device__ __forceinline__ void partial_block(const StagePart& p, int local, float* __restrict__ red,
                                              float* __restrict__ xs, double* __restrict__ dsh) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  // A small call splits the columns of U into ncb blocks of w = k / ncb (a workgroup then reads w-wide pieces of its
  // rows), so that a few inputs still give the chip hundreds of workgroups; a large call takes whole rows (ncb = 1).
  const int d = p.d, k = p.k_rows & 0xffff, prow = p.k_rows >> 16;
  const int slabs = p.slabs_x & 0xffff, ncb = max(1, (p.slabs_x >> 20) & 0xff);
  const int slab = local % slabs, col0 = (local / slabs) * (k / ncb);
  const int w = k / ncb;
  const int cpr = w / V;         // lanes per row piece (a power of two, one wave at most)
  const int rps = kBlock / cpr;  // rows per step
  const int lsh = __builtin_ctz(cpr);
  const int cc = threadIdx.x & (cpr - 1), ro = threadIdx.x >> lsh;
  const int row0 = slab * prow;
  const int rows = min(prow, d - row0);
  const S* U = reinterpret_cast<const S*>(p.U) + (int64_t)row0 * k + col0 + cc * V;
  const int xdtype = (p.slabs_x >> 16) & 0xf;

  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  int i = ro;
  // the first two batches of U go in flight (64 KB per workgroup, a whole slab of the fine geometry), then the
  // slab's activations are staged in LDS (one coalesced load)
  uint4 raw[8], raw2[8];
  const bool first = i + 7 * rps < rows, second = i + 15 * rps < rows;
  if (first) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const S* src = U + (int64_t)(i + q * rps) * k;
      raw[q] = STREAM ? load_stream16(src) : *reinterpret_cast<const uint4*>(src);
    }
  }
  if (second) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const S* src = U + (int64_t)(i + (8 + q) * rps) * k;
      raw2[q] = STREAM ? load_stream16(src) : *reinterpret_cast<const uint4*>(src);
    }
  }
  double x2 = 0.0;  // this thread's share of the slab's |x|^2 (single-pass gate)
  for (int r = threadIdx.x; r < rows; r += kBlock) {
    const float xv = load_act(p.X, xdtype, row0 + r);
    xs[r] = xv;
    x2 = fma((double)xv, (double)xv, x2);
  }
  __syncthreads();
  if (first) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float u[V];
      T::widen(raw[q], u);
      const float xv = xs[i + q * rps];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = fmaf(u[e], xv, acc[e]);
    }
    i += 8 * rps;
  }
  if (second) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float u[V];
      T::widen(raw2[q], u);
      const float xv = xs[i + q * rps];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = fmaf(u[e], xv, acc[e]);
    }
    i += 8 * rps;
  }
  // eight (then four) row steps at a time: all loads of a batch are issued before the first use
  for (; i + 7 * rps < rows; i += 8 * rps) {
#pragma unroll
    for (int q = 0; q < 8; ++q) raw[q] = *reinterpret_cast<const uint4*>(U + (int64_t)(i + q * rps) * k);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float u[V];
      T::widen(raw[q], u);
      const float xv = xs[i + q * rps];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = fmaf(u[e], xv, acc[e]);
    }
  }
  for (; i + 3 * rps < rows; i += 4 * rps) {
#pragma unroll
    for (int q = 0; q < 4; ++q) raw[q] = *reinterpret_cast<const uint4*>(U + (int64_t)(i + q * rps) * k);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float u[V];
      T::widen(raw[q], u);
      const float xv = xs[i + q * rps];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = fmaf(u[e], xv, acc[e]);
    }
  }
  for (; i < rows; i += rps) {
    float u[V];
    T::load_vec(U + (int64_t)i * k, u);
    const float xv = xs[i];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = fmaf(u[e], xv, acc[e]);
  }
#pragma unroll
  for (int q = 0; q < V / 4; ++q)
    reinterpret_cast<float4*>(red + ro * w + cc * V)[q] = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
  if (p.x2_off) {
    x2 = wave_sum_f64(x2);
    if (threadIdx.x % kWave == 0) dsh[threadIdx.x / kWave] = x2;
  }
  __syncthreads();
  if (p.x2_off && threadIdx.x == 0 && col0 == 0) {
    double t = 0.0;
    for (int w = 0; w < kWaves; ++w) t += dsh[w];
    reinterpret_cast<double*>(reinterpret_cast<char*>(p.part_c) + p.x2_off)[slab] = t;
  }
  if (p.x2_off) {  // single-pass gate: the row groups are added in fp64 and the partial is kept as high + low part
    for (int j = threadIdx.x; j < w; j += kBlock) {
      double s = 0.0;
      for (int g = 0; g < rps; g += 4) {
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = red[(g + q) * w + j];
#pragma unroll
        for (int q = 0; q < 4; ++q) s += (double)v[q];
      }
      const float hi = (float)s;
      p.part_c[(int64_t)slab * k + col0 + j] = hi;
      p.part_c[(int64_t)(slabs + slab) * k + col0 + j] = (float)(s - (double)hi);
    }
    return;
  }
  for (int j = threadIdx.x; j < w; j += kBlock) {
    float s = 0.f;
    for (int g = 0; g < rps; g += 4) {  // rps is a multiple of 4: four LDS reads in flight, fixed order of adds
      float v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = red[(g + q) * w + j];
#pragma unroll
      for (int q = 0; q < 4; ++q) s += v[q];
    }
    p.part_c[(int64_t)slab * k + col0 + j] = s;
  }
}

// c = the partials of one input added in slab order (one workgroup)
__device__ __forceinline__ void cred_block(const StageCRed& p) {
  const int k = p.k_slabs & 0xffff, slabs = p.k_slabs >> 16;
  for (int j = threadIdx.x; j < k; j += kBlock) p.C[j] = sum_partials(p.part_c + j, k, slabs);
}

// Single-pass gate: block `blk` of kGramBlocks adds the partials of one input (block 0 writes C and |c|^2), then
// takes rows [blk * rpb, (blk + 1) * rpb) of E: share = sum_i c_i (sum_j E_ij c_j).  A wave takes a row at a time,
// a lane the 16-byte pieces lane, lane + 64, ... of it.
// c_j to double precision: high and low parts of the slab partials ([slabs][k] each, low parts behind the high
// parts), slab order fixed
__device__ __forceinline__ double sum_partials_f64(const float* __restrict__ pc, int k, int slabs) {
  double s = 0.0;
  const float* __restrict__ lo = pc + (int64_t)slabs * k;
  int sl = 0;
  for (; sl + 8 <= slabs; sl += 8) {
    float h[8], l[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      h[q] = pc[(int64_t)(sl + q) * k];
      l[q] = lo[(int64_t)(sl + q) * k];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) s += (double)h[q] + (double)l[q];
  }
  for (; sl < slabs; ++sl) s += (double)pc[(int64_t)sl * k] + (double)lo[(int64_t)sl * k];
  return s;
}

// c_ready: C already holds the sums (a launch before this one added the partials)
__device__ __forceinline__ void gram_block(const StageCRed& p, double* __restrict__ gw, bool c_ready, int blk,
                                           float* __restrict__ cs, double* __restrict__ dsh) {
  const int k = p.k_slabs & 0xffff, slabs = p.k_slabs >> 16;
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  double c2 = 0.0;  // block 0, when it adds the partials itself: |c|^2 of the unrounded sums
  if (c_ready) {
    for (int j = threadIdx.x; j < k; j += kBlock) cs[j] = p.C[j];
  } else {
    for (int j = threadIdx.x; j < k; j += kBlock) {
      const double cd = sum_partials_f64(p.part_c + j, k, slabs);
      const float c = (float)cd;
      cs[j] = c;
      if (blk == 0) {
        p.C[j] = c;
        c2 = fma(cd, cd, c2);
      }
    }
  }
  __syncthreads();
  const int rpb = (k + kGramBlocks - 1) / kGramBlocks;
  const int row_end = min(k, (blk + 1) * rpb);
  const int pieces = k / 4;  // k is a multiple of four on this path
  double acc = 0.0;
  for (int i = blk * rpb + wave; i < row_end; i += kWaves) {
    const float4* __restrict__ row = reinterpret_cast<const float4*>(p.E + (int64_t)i * k);
    float s = 0.f;
    for (int q = lane; q < pieces; q += kWave) {
      const float4 e = row[q];
      const float4 c = reinterpret_cast<const float4*>(cs)[q];
      s = fmaf(e.x, c.x, s);
      s = fmaf(e.y, c.y, s);
      s = fmaf(e.z, c.z, s);
      s = fmaf(e.w, c.w, s);
    }
    s = group_sum<kWave>(s);
    acc = fma((double)cs[i], (double)s, acc);
  }
  if (lane == 0) dsh[wave] = acc;
  if (blk == 0 && !c_ready) {  // |c|^2: each thread its coefficients j, j + 256, ...; waves in order
    c2 = wave_sum_f64(c2);
    if (lane == 0) dsh[kWaves + wave] = c2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kWaves; ++w) t += dsh[w];
    gw[slabs + blk] = t;
    if (blk == 0 && !c_ready) {
      double t2 = 0.0;
      for (int w = 0; w < kWaves; ++w) t2 += dsh[kWaves + w];
      gw[slabs + kGramBlocks] = t2;
      for (int q = 1; q < kC2Shares; ++q) gw[slabs + kGramBlocks + q] = 0.0;
    }
  }
}

template <class T>
__device__ __forceinline__ void residual_block(const StageRes& p, const StageGate* gates, float eps, int slab,
                                               float* __restrict__ cs, float* __restrict__ xs, float* nr, float* nx) {
  constexpr int V = T::kVec;
  constexpr int PF = 4;  // row steps of U held in registers
  using S = typename T::storage;
  const int d = p.d, k = p.k_rows & 0xffff, b_rows = p.k_rows >> 16;
  const int xdtype = p.slabs_x >> 24, a_slabs = (p.slabs_x >> 16) & 0xff;
  if (const int r = p.gate >> 8) {
    // Workgroups go to the eight XCDs round-robin.  The launch before this one read the rows of partial-projection
    // slab ps on XCD ps % 8 (the host checked the offsets); r residual slabs cover one such slab, so the residual
    // slabs are walked in an order that puts slab r * ps + h on XCD ps % 8 too: the second read of the basis then
    // comes out of the L2 that holds it.
    const int chunk = slab / (8 * r), within = slab % (8 * r);
    slab = r * (8 * chunk + within % 8) + within / 8;
  }
  if (p.gate & 0xff) {  // single-pass gate: the verdict first; an input that did not fire needs no residual
    const StageGate& g = gates[(p.gate & 0xff) - 1];
    float rn, xn;
    const bool f = single_pass_gate(reinterpret_cast<const double*>(g.part_n), g.b_slabs, eps, rn, xn);
    if (slab == 0 && threadIdx.x == 0) publish_gate(g, rn, xn, f);
    if (!f || g.skip_fired_image) return;  // (the W x form of the slow path reads x, not r)
  }
  const int cpr = k / V;         // 16-byte chunks per row (power of two, <= 64)
  const int rps = kBlock / cpr;  // rows per step
  const int cc = threadIdx.x & (cpr - 1), ro = threadIdx.x >> __builtin_ctz(cpr);
  const int row0 = slab * b_rows;
  const int rows = min(b_rows, d - row0);
  const int steps = (rows + rps - 1) / rps;
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const S* U = reinterpret_cast<const S*>(p.U) + (int64_t)row0 * k + cc * V;

  // the slab of U goes in flight first (row index clamped: loads are unconditional), then the slab's activations
  // (one coalesced load, staged in LDS) and the coefficients
  uint4 upf[PF];
#pragma unroll
  for (int q = 0; q < PF; ++q) upf[q] = *reinterpret_cast<const uint4*>(U + (int64_t)min(q * rps + ro, rows - 1) * k);
  for (int r = threadIdx.x; r < rows; r += kBlock) xs[r] = load_act(p.X, xdtype, row0 + r);
  if (p.part_c) {
    for (int j = threadIdx.x; j < k; j += kBlock) {
      const float s = sum_partials(p.part_c + j, k, a_slabs);
      cs[j] = s;
      if (slab == 0) p.C[j] = s;
    }
  } else {
    for (int j = threadIdx.x; j < k; j += kBlock) cs[j] = p.C[j];
  }
  __syncthreads();
  float c[V];
#pragma unroll
  for (int e = 0; e < V; ++e) c[e] = cs[cc * V + e];
  float ar = 0.f, ax = 0.f;
  // every lane of a row group walks the same steps, so the cross-lane sums are convergent
  auto row_step = [&](const uint4& raw, float x, int st) {
    const int i = st * rps + ro;
    float u[V];
    T::widen(raw, u);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < V; ++e) s = fmaf(u[e], c[e], s);
    s = group_sum_rt(s, cpr);
    if (i < rows && cc == 0) {
      const float r = x - s;
      p.R[row0 + i] = r;
      ar = fmaf(r, r, ar);
      ax = fmaf(x, x, ax);
    }
  };
#pragma unroll
  for (int q = 0; q < PF; ++q)
    if (q < steps) row_step(upf[q], xs[min(q * rps + ro, rows - 1)], q);
  for (int st0 = PF; st0 < steps; st0 += PF) {  // further steps, PF at a time with all loads issued first
    uint4 u[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q)
      u[q] = *reinterpret_cast<const uint4*>(U + (int64_t)min((st0 + q) * rps + ro, rows - 1) * k);
#pragma unroll
    for (int q = 0; q < PF; ++q)
      if (st0 + q < steps) row_step(u[q], xs[min((st0 + q) * rps + ro, rows - 1)], st0 + q);
  }
  if (p.gate & 0xff) return;  // the norms came from the single-pass shares
  const float sr = group_sum<kWave>(ar);
  const float sx = group_sum<kWave>(ax);
  if (lane == 0) {
    nr[wave] = sr;
    nx[wave] = sx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tr = 0.f, tx = 0.f;
    for (int w = 0; w < kWaves; ++w) {
      tr += nr[w];
      tx += nx[w];
    }
    p.part_n[slab * 2 + 0] = tr;
    p.part_n[slab * 2 + 1] = tx;
  }
}

// one wave: the same sums, in the same order, as the stand-alone norm kernel
__device__ __forceinline__ void gate_block(const StageGate& g, float eps) {
  if (threadIdx.x >= kWave) return;
  float tr, tx;
  wave_norm_sums(g.part_n, g.b_slabs, 1, 0, tr, tx);
  if (threadIdx.x == 0) {
    const float rn = sqrtf(tr), xn = sqrtf(tx);
    publish_gate(g, rn, xn, gate_fires(rn, xn, eps));
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void proj_stage(const StageArgs a) {
  __shared__ __align__(16) float lds[kBlock * 8];  // partial: [row group][k]; residual, image: the coefficients
  __shared__ float xs[kStageMaxRows];              // the slab's activations
  __shared__ float nr[kWaves], nx[kWaves];
  __shared__ double dsh[2 * kWaves];
  int b = blockIdx.x;
  // single-pass gate: the residual workgroups (nearly all of which only evaluate the gate and leave) go last
  if (a.gram) b = b + a.b_total < (int)gridDim.x ? b + a.b_total : b + a.b_total - (int)gridDim.x;
  if (b < a.b_total) {
    const int ti = find_task(a.b_begin, a.nb, b);
    residual_block<T>(a.b[ti], a.g, a.eps, b - a.b_begin[ti], lds, xs, nr, nx);
    return;
  }
  b -= a.b_total;
  if (b < a.a_total) {
    const int ti = find_task(a.a_begin, a.na, b);
    partial_block<T>(a.a[ti], b - a.a_begin[ti], lds, xs, dsh);
    return;
  }
  b -= a.a_total;
  if (b < a.i_total) {
    int ti = 0;
#pragma unroll
    for (int i = 1; i < kMaxLinTasks; ++i)
      if (i < a.ni && b >= (a.im[i].blk_res & 0xffffff)) ti = i;
    const StageImg& im = a.im[ti];
    const StageRes& r = a.b[im.blk_res >> 24];
    if ((r.gate & 0xff) && a.g[(r.gate & 0xff) - 1].skip_fired_image) {  // fired: the weight kernel writes y = W x
      const StageGate& g = a.g[(r.gate & 0xff) - 1];
      float rn, xn;
      if (single_pass_gate(reinterpret_cast<const double*>(g.part_n), g.b_slabs, a.eps, rn, xn)) return;
    }
    ImgTask t;
    t.M = im.M; t.Y = im.Y; t.part_c = r.part_c; t.C = r.C; t.scale = im.scale;
    t.m = im.m; t.k = r.k_rows & 0xffff; t.a_slabs = (r.slabs_x >> 16) & 0xff; t.blk_begin = im.blk_res & 0xffffff;
    image_block<T>(t, b - t.blk_begin, lds);
    return;
  }
  b -= a.i_total;
  if (a.gram) {
    if (b < a.ncr * kGramBlocks) {
      const StageCRed& p = a.cr[b / kGramBlocks];
      gram_block(p, reinterpret_cast<double*>(reinterpret_cast<char*>(const_cast<float*>(p.part_c)) + p.gw_off), false,
                 b % kGramBlocks, lds, dsh);
    }
    return;
  }
  if (b < a.ncr) {
    cred_block(a.cr[b]);
    return;
  }
  gate_block(a.g[b - a.ncr], a.eps);
}

// ---- the same stages over a table in device memory (many inputs, single-pass gate) ------------------------------
// first-workgroup table of n tasks staged in LDS, then a binary search: the task that holds workgroup b
__device__ __forceinline__ int find_in_table(const int* __restrict__ begin, int n, int b, int* __restrict__ sh) {
  for (int i = threadIdx.x; i < n; i += kBlock) sh[i] = begin[i];
  __syncthreads();
  int lo = 0, hi = n - 1;  // begin[0] = 0 <= b
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sh[mid] <= b) lo = mid;
    else hi = mid - 1;
  }
  return __builtin_amdgcn_readfirstlane(lo);
}

template <class T, bool NT>
__global__ __launch_bounds__(kBlock) void table_partial(const TabIn* __restrict__ ins, const int* __restrict__ pbegin,
                                                        int n_in) {
  __shared__ __align__(16) float lds[kBlock * 8];
  __shared__ float xs[kStageMaxRows];
  __shared__ double dsh[2 * kWaves];
  __shared__ int tab[kMaxTabIn];
  const int b = blockIdx.x;
  const int i = find_in_table(pbegin, n_in, b, tab);
  const TabIn& in = ins[i];
  StagePart p;
  p.U = in.U; p.X = in.X; p.part_c = in.part_c; p.d = in.d; p.k_rows = in.k_rows;
  p.slabs_x = (in.slabs & 0xffff) | (((in.r_rows_x >> 16) & 0xf) << 16);
  p.x2_off = in.gw_off;
  partial_block<T, NT>(p, b - tab[i], lds, xs, dsh);
}

// c = the partials added in slab order: a workgroup per (input, 64 columns); its four waves take every fourth slab
// (16 loads in flight per lane) and are combined through LDS in wave order
__global__ __launch_bounds__(kBlock) void table_cred(const TabIn* __restrict__ ins, const int* __restrict__ cbegin,
                                                     int n_in) {
  __shared__ double sh[kWaves][kWave];
  __shared__ int tab[kMaxTabIn];
  const int i = find_in_table(cbegin, n_in, blockIdx.x, tab);
  const TabIn& in = ins[i];
  const int k = in.k_rows & 0xffff, slabs = in.slabs & 0xffff;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int cblk = blockIdx.x - tab[i];
  const int j = cblk * kWave + lane;
  double s = 0.0;
  if (j < k) {
    const float* __restrict__ pc = in.part_c + j;
    const float* __restrict__ lo = pc + (int64_t)slabs * k;
    int sl = wave;
    for (; sl + 7 * kWaves < slabs; sl += 8 * kWaves) {
      float h[8], l[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        h[q] = pc[(int64_t)(sl + q * kWaves) * k];
        l[q] = lo[(int64_t)(sl + q * kWaves) * k];
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) s += (double)h[q] + (double)l[q];
    }
    for (; sl < slabs; sl += kWaves) s += (double)pc[(int64_t)sl * k] + (double)lo[(int64_t)sl * k];
  }
  sh[wave][lane] = s;
  __syncthreads();
  if (wave == 0) {  // (whole wave: the sum over its lanes below needs every lane)
    const double cd = (sh[0][lane] + sh[1][lane]) + (sh[2][lane] + sh[3][lane]);
    if (j < k) in.C[j] = (float)cd;
    const double c2 = wave_sum_f64(j < k ? cd * cd : 0.0);  // this block's share of |c|^2, from the unrounded sums
    double* gw = reinterpret_cast<double*>(reinterpret_cast<char*>(in.part_c) + in.gw_off);
    if (lane == 0) {
      gw[slabs + kGramBlocks + cblk] = c2;
      if (cblk == 0)  // shares that no block writes (k / 64 < kC2Shares) are zero
        for (int q = (k + kWave - 1) / kWave; q < kC2Shares; ++q) gw[slabs + kGramBlocks + q] = 0.0;
    }
  }
}

// merged: no launch added the partials before this one; every workgroup adds them itself (fixed order) and the first
// of an input writes C and |c|^2
__global__ __launch_bounds__(kBlock) void table_gram(const TabIn* __restrict__ ins, int merged) {
  __shared__ __align__(16) float lds[kMaxK];
  __shared__ double dsh[2 * kWaves];
  const TabIn& in = ins[blockIdx.x / kGramBlocks];
  StageCRed p;
  p.part_c = merged ? in.part_c : nullptr; p.C = in.C; p.E = in.E;
  p.k_slabs = (in.k_rows & 0xffff) | ((in.slabs & 0xffff) << 16);
  p.gw_off = 0;
  gram_block(p, reinterpret_cast<double*>(reinterpret_cast<char*>(in.part_c) + in.gw_off), !merged, blockIdx.x % kGramBlocks,
             lds, dsh);
}

// the residual workgroups first (they evaluate the gate, publish it, and form r only for an input that fired: few
// and slow, so they start early and run beside the image stream), then the image rows of every map
template <class T, bool NT>
__global__ __launch_bounds__(kBlock) void table_rows(const TabIn* __restrict__ ins, const TabMap* __restrict__ maps,
                                                     const int* __restrict__ ibegin, const int* __restrict__ rbegin,
                                                     int n_in, int n_maps, int r_total, float eps) {
  __shared__ __align__(16) float lds[kBlock * 8];
  __shared__ float xs[kStageMaxRows];
  __shared__ float nr[kWaves], nx[kWaves];
  __shared__ int tab[kMaxTabMaps];
  int b = blockIdx.x;
  if (b >= r_total) {
    b -= r_total;
    const int j = find_in_table(ibegin, n_maps, b, tab);
    const TabMap& mp = maps[j];
    if (mp.gw) {  // W x form of the slow path: a fired input's rows are left to the weight kernel
      float rn, xn;
      if (single_pass_gate(mp.gw, mp.slabs, eps, rn, xn)) return;
    }
    ImgTask t;
    t.M = mp.M; t.Y = mp.Y; t.part_c = nullptr; t.C = mp.C; t.scale = mp.scale;
    t.m = mp.m; t.k = mp.k; t.a_slabs = 0; t.blk_begin = tab[j];
    image_block<T, kTabImgItems, NT>(t, b - t.blk_begin, lds);
    return;
  }
  const int i = find_in_table(rbegin, n_in, b, tab);
  const TabIn& in = ins[i];
  StageGate g;
  g.part_n = reinterpret_cast<const float*>(reinterpret_cast<const char*>(in.part_c) + in.gw_off);
  g.rnorm = in.rnorm; g.xnorm = in.xnorm; g.mask = in.mask; g.fired_idx = in.fired_idx; g.n_fired = in.n_fired;
  g.b_slabs = in.slabs & 0xffff;
  g.skip_fired_image = (in.r_rows_x >> 20) & 1;
  StageRes p;
  p.U = in.U; p.X = in.X; p.part_c = nullptr; p.C = in.C; p.R = in.R; p.part_n = nullptr;
  p.d = in.d; p.k_rows = (in.k_rows & 0xffff) | ((in.r_rows_x & 0xffff) << 16);
  p.slabs_x = (in.slabs >> 16) | ((in.slabs & 0xff) << 16) | (((in.r_rows_x >> 16) & 0xf) << 24);
  p.gate = 1;
  residual_block<T>(p, &g, eps, b - tab[i], lds, xs, nr, nx);
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
void stage_geom(int64_t d, int64_t k, int udtype, int& rows, int& slabs, bool fine) {
  const int V = udtype == GSI_BF16 ? 8 : 4;
  const int rps = kBlock / (int)(k / V);
  // at least eight row steps per workgroup, kPartSlabs slabs at most ...
  int64_t r = ceil_div(d, kPartSlabs);
  if (fine) {  // ... or, at most 64 KB of U per workgroup (a workgroup keeps 32 KB in flight, so a larger slab is a
               // long pole of the launch), as long as that needs no more than kStageSlabs slabs
    const int64_t cap = 65536 / (k * (int64_t)elem_size(udtype));
    if (r > cap) r = cap;
    if (r < ceil_div(d, kStageSlabs)) r = ceil_div(d, kStageSlabs);
  }
  if (r < 8 * rps) r = 8 * rps;
  rows = (int)(ceil_div(r, rps) * rps);
  slabs = (int)ceil_div(d, rows);
}

void stage_clear(StageArgs& a, float eps) {
  std::memset(&a, 0, sizeof(a));
  a.eps = eps;
}

void stage_add_part(StageArgs& a, const ProjTask& t, const float* E, int ncb) {
  StagePart& p = a.a[a.na++];
  p.U = t.U; p.X = t.X; p.part_c = t.part_c;
  p.d = t.d; p.k_rows = t.k | (t.s_rows << 16); p.slabs_x = t.s_slabs | (t.xdtype << 16) | (ncb << 20);
  p.x2_off = E ? (int)(reinterpret_cast<char*>(t.part_n) - reinterpret_cast<char*>(t.part_c)) : 0;
}

void stage_add_cred(StageArgs& a, const ProjTask& t, const float* E) {
  StageCRed& p = a.cr[a.ncr++];
  p.part_c = t.part_c; p.C = t.C; p.k_slabs = t.k | (t.s_slabs << 16);
  p.E = E; p.gw_off = (int)(reinterpret_cast<char*>(t.part_n) - reinterpret_cast<char*>(t.part_c));
  if (E) a.gram = 1;
}

void stage_set_res_xcd_order(StageArgs& a, int res, int r) { a.b[res].gate = (a.b[res].gate & 0xff) | (r << 8); }

int stage_add_res(StageArgs& a, const ProjTask& t, bool c_ready, const float* E, bool skip_fired_image) {
  StageRes& p = a.b[a.nb];
  p.U = t.U; p.X = t.X; p.part_c = c_ready ? nullptr : t.part_c; p.C = t.C; p.R = t.R; p.part_n = t.part_n;
  p.d = t.d; p.k_rows = t.k | (t.b_rows << 16);
  p.slabs_x = t.b_slabs | (t.s_slabs << 16) | (t.xdtype << 24);
  p.gate = 0;
  if (E) {  // the gate of this input is evaluated by its residual workgroups: entry a.nb of the gate table
    StageGate& g = a.g[a.nb];
    g.part_n = t.part_n; g.rnorm = t.rnorm; g.xnorm = t.xnorm; g.mask = t.mask; g.fired_idx = t.fired_idx;
    g.n_fired = t.n_fired; g.b_slabs = t.s_slabs; g.skip_fired_image = skip_fired_image ? 1 : 0;
    p.gate = a.nb + 1;
    a.gram = 1;
  }
  return a.nb++;
}

void stage_add_img(StageArgs& a, int res, const void* M, float* Y, const float* scale, int m) {
  StageImg& im = a.im[a.ni++];
  im.M = M; im.Y = Y; im.scale = scale; im.m = m; im.blk_res = res << 24;
}

void stage_add_gate(StageArgs& a, const ProjTask& t) {
  StageGate& g = a.g[a.ng++];
  g.part_n = t.part_n; g.rnorm = t.rnorm; g.xnorm = t.xnorm; g.mask = t.mask; g.fired_idx = t.fired_idx;
  g.n_fired = t.n_fired; g.b_slabs = t.b_slabs; g.skip_fired_image = 0;
}

hipError_t stage_launch(StageArgs& a, int dtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  int ta = 0, tb = 0, ti = 0;
  for (int i = 0; i < a.na; ++i) {
    a.a_begin[i] = ta;
    ta += (a.a[i].slabs_x & 0xffff) * std::max(1, (a.a[i].slabs_x >> 20) & 0xff);
  }
  for (int i = 0; i < a.nb; ++i) {
    a.b_begin[i] = tb;
    tb += a.b[i].slabs_x & 0xffff;
  }
  for (int i = 0; i < a.ni; ++i) {
    const int res = a.im[i].blk_res >> 24;
    a.im[i].blk_res = (res << 24) | ti;
    ti += image_blocks(a.im[i].m, a.b[res].k_rows & 0xffff, dtype, a.im[i].scale != nullptr);
    if (ti >= (1 << 24)) return hipErrorInvalidValue;
  }
  a.a_total = ta; a.b_total = tb; a.i_total = ti;
  const int grid = ta + tb + ti + (a.gram ? a.ncr * kGramBlocks : a.ncr + a.ng);
  if (grid == 0) return hipSuccess;
  if (dtype == GSI_BF16) {
    if (e0 && e1) hipExtLaunchKernelGGL((proj_stage<BF16>), dim3(grid), dim3(kBlock), 0, s, e0, e1, 0, a);
    else proj_stage<BF16><<<grid, kBlock, 0, s>>>(a);
  } else {
    if (e0 && e1) hipExtLaunchKernelGGL((proj_stage<F32>), dim3(grid), dim3(kBlock), 0, s, e0, e1, 0, a);
    else proj_stage<F32><<<grid, kBlock, 0, s>>>(a);
  }
  return hipGetLastError();
}

size_t stage_table_bytes(int n_in, int n_maps) {
  return align_up((size_t)n_in * sizeof(TabIn), 256) + align_up((size_t)n_maps * sizeof(TabMap), 256) +
         3 * align_up((size_t)(n_in + 1) * sizeof(int), 256) + align_up((size_t)(n_maps + 1) * sizeof(int), 256);
}

hipError_t stage_table_build(const TabIn* ins, int n_in, const TabMap* maps, int n_maps, int dtype, std::vector<char>& host,
                             StageTableGeom& g) {
  if (n_in <= 0 || n_in > kMaxTabIn || n_maps < 0 || n_maps > kMaxTabMaps) return hipErrorInvalidValue;
  g.n_in = n_in; g.n_maps = n_maps; g.dtype = dtype;
  g.off_maps = align_up((size_t)n_in * sizeof(TabIn), 256);
  g.off_p = g.off_maps + align_up((size_t)n_maps * sizeof(TabMap), 256);
  g.off_r = g.off_p + align_up((size_t)(n_in + 1) * sizeof(int), 256);
  g.off_c = g.off_r + align_up((size_t)(n_in + 1) * sizeof(int), 256);
  g.off_i = g.off_c + align_up((size_t)(n_in + 1) * sizeof(int), 256);
  host.assign(stage_table_bytes(n_in, n_maps), 0);
  std::memcpy(host.data(), ins, (size_t)n_in * sizeof(TabIn));
  if (n_maps) std::memcpy(host.data() + g.off_maps, maps, (size_t)n_maps * sizeof(TabMap));
  int* pb = reinterpret_cast<int*>(host.data() + g.off_p);
  int* rb = reinterpret_cast<int*>(host.data() + g.off_r);
  int* cb = reinterpret_cast<int*>(host.data() + g.off_c);
  int* ib = reinterpret_cast<int*>(host.data() + g.off_i);
  int64_t tp = 0, tr = 0, tc = 0, ti = 0;
  size_t bytes = 0;  // bases and images of the call
  for (int i = 0; i < n_in; ++i) {
    bytes += (size_t)ins[i].d * (ins[i].k_rows & 0xffff) * elem_size(dtype);
    pb[i] = (int)tp;
    rb[i] = (int)tr;
    cb[i] = (int)tc;
    tp += ins[i].slabs & 0xffff;
    tr += ins[i].slabs >> 16;
    tc += ceil_div(ins[i].k_rows & 0xffff, kWave);
  }
  for (int j = 0; j < n_maps; ++j) {
    ib[j] = (int)ti;
    ti += image_blocks(maps[j].m, maps[j].k, dtype, maps[j].scale != nullptr, kTabImgItems);
    bytes += (size_t)maps[j].m * maps[j].k * (maps[j].scale ? 1 : elem_size(dtype));
  }
  g.nt = bytes >= kStreamBytes ? 1 : 0;
  // Few partials per input (slabs x rank up to 4096 values, 32 KB with their low parts): the kGramBlocks workgroups of
  // an input each add them again rather than wait for a launch that adds them once.
  g.merge = 1;
  for (int i = 0; i < n_in; ++i)
    if ((int64_t)(ins[i].slabs & 0xffff) * (ins[i].k_rows & 0xffff) > 4096) g.merge = 0;
  pb[n_in] = (int)tp; rb[n_in] = (int)tr; cb[n_in] = (int)tc; ib[n_maps] = (int)ti;
  if (tp >= (1 << 30) || tr + ti >= (1 << 30)) return hipErrorInvalidValue;
  g.tp = (int)tp; g.tc = (int)tc; g.tr = (int)tr; g.ti = (int)ti;
  return hipSuccess;
}

hipError_t stage_table_launch(const void* table, const StageTableGeom& g, float eps, hipStream_t s, int which_timed,
                              hipEvent_t e0, hipEvent_t e1) {
  const char* base = static_cast<const char*>(table);
  const TabIn* d_ins = reinterpret_cast<const TabIn*>(base);
  const TabMap* d_maps = reinterpret_cast<const TabMap*>(base + g.off_maps);
  const int* d_pb = reinterpret_cast<const int*>(base + g.off_p);
  const int* d_rb = reinterpret_cast<const int*>(base + g.off_r);
  const int* d_cb = reinterpret_cast<const int*>(base + g.off_c);
  const int* d_ib = reinterpret_cast<const int*>(base + g.off_i);
  const int n_in = g.n_in, n_maps = g.n_maps;
  auto ev = [&](int w) { return which_timed == w && e0 && e1; };
  // 1. partial projections
  auto partial = [&](auto kern) {
    if (ev(0)) hipExtLaunchKernelGGL(kern, dim3((unsigned)g.tp), dim3(kBlock), 0, s, e0, e1, 0, d_ins, d_pb, n_in);
    else kern<<<(unsigned)g.tp, kBlock, 0, s>>>(d_ins, d_pb, n_in);
  };
  if (g.dtype == GSI_BF16) {
    if (g.nt) partial(table_partial<BF16, true>);
    else partial(table_partial<BF16, false>);
  } else {
    if (g.nt) partial(table_partial<F32, true>);
    else partial(table_partial<F32, false>);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  // 2. coefficient sums, then the shares of c^T E c
  if (!g.merge) {
    table_cred<<<(unsigned)g.tc, kBlock, 0, s>>>(d_ins, d_cb, n_in);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  if (ev(1)) hipExtLaunchKernelGGL(table_gram, dim3((unsigned)n_in * kGramBlocks), dim3(kBlock), 0, s, e0, e1, 0, d_ins, g.merge);
  else table_gram<<<(unsigned)n_in * kGramBlocks, kBlock, 0, s>>>(d_ins, g.merge);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  // 3. gates, residuals of fired inputs, image rows
  const unsigned grid = (unsigned)(g.ti + g.tr);
  auto rows = [&](auto kern) {
    if (ev(2)) hipExtLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, e0, e1, 0, d_ins, d_maps, d_ib, d_rb, n_in, n_maps, g.tr, eps);
    else kern<<<grid, kBlock, 0, s>>>(d_ins, d_maps, d_ib, d_rb, n_in, n_maps, g.tr, eps);
  };
  if (g.dtype == GSI_BF16) {
    if (g.nt) rows(table_rows<BF16, true>);
    else rows(table_rows<BF16, false>);
  } else {
    if (g.nt) rows(table_rows<F32, true>);
    else rows(table_rows<F32, false>);
  }
  return hipGetLastError();
}

hipError_t stage_table_run(void* table, const TabIn* ins, int n_in, const TabMap* maps, int n_maps, int dtype, float eps,
                           hipStream_t s, int which_timed, hipEvent_t e0, hipEvent_t e1) {
  if (n_in <= 0) return hipSuccess;
  std::vector<char> host;
  StageTableGeom g;
  if (hipError_t e = stage_table_build(ins, n_in, maps, n_maps, dtype, host, g); e != hipSuccess) return e;
  if (hipError_t e = upload_launch(host.data(), host.size(), table, s); e != hipSuccess) return e;
  return stage_table_launch(table, g, eps, s, which_timed, e0, e1);
}

}  // namespace gsi
