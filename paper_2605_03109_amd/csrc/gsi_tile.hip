// Linear maps of a decode batch (2..128 tokens per call) on the matrix cores: Algorithm 1 lines 4-7 in
// the y = M c (+ W r when the gate fires) form of Eq. (exact), and the dense baseline y = W x.
//
// The work is a skinny GEMM bound by the one pass over the weights, so the kernel is organised around
// that pass.  A work item is 128 rows of one matrix by a slice of 512 contraction columns: each of the
// eight waves owns 16 rows and requests its whole share (16 loads of 16 bytes per lane) at once, straight
// from memory into A operands of v_mfma_f32_16x16x32_bf16 (lane l holds row l%16, columns 8*(l/16)..+8
// of a 32-column step).  The B operands are the same columns of up to 32 tokens' activation vectors,
// staged once per workgroup in LDS: fp32 activations are split into a bf16 head and a bf16
// tail (the rounded remainder) and take two MFMAs, so nothing is rounded to 8 bits.  More than 32 tokens
// take further rounds against the same A registers: the weights are read once whatever the token count.
// For the W term the tokens are the fired ones, taken from the device-side list in ascending order; with
// no fired token the kernel leaves before touching the weight matrix.
// Items of one matrix that cover different column slices write partial sums to the workspace, and a
// second kernel adds them in slice order, so results do not vary from run to run.
#include "gsi_decode.h"
#include "gsi_device.h"

namespace gsi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTBlock = 512;                       // threads per workgroup
constexpr int kTWaves = kTBlock / kWave;           // 8
constexpr int kItemRows = 16 * kTWaves;            // 128 rows per item
constexpr int kSteps = 16;                         // MFMA steps per item
constexpr int kStepCols = 32;                      // contraction columns per MFMA
constexpr int kSliceCols = kSteps * kStepCols;     // 512 columns per item
constexpr int kRoundTok = 32;                      // tokens staged per round (two MFMA token tiles)
constexpr int kMaxTok = 128;                       // tokens per call
constexpr int kMaxTokTiles = kMaxTok / 16;
constexpr int kVRow = kSliceCols + 8;              // bf16 per staged token row: 16 bytes of padding keep
                                                   // the 16 lanes of a 128-bit LDS read on distinct banks
constexpr int kHalfVec = 16 * kSliceCols / 4 / kTBlock;  // float4 per thread per 16 staged tokens (4)

template <int N>
__device__ __forceinline__ int find_task(const int (&begin)[N], int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < N; ++i)
    if (i < n && b >= begin[i]) t = i;
  return t;
}

// Requests this thread's share of half a staging round: tokens [g0 + 16 * half, + 16) of the phase (token j
// is row idx ? idx[j] : j of V), columns [c0, c0 + 32 * ns).  A wave pair covers one token row per pass.
// Every load is unconditional: tokens past the count repeat the last one and columns past the slice its
// last four; what they stage is never used.
__device__ __forceinline__ void stage_issue(float4 (&v)[kHalfVec], int half, const float* __restrict__ V, int64_t ldv,
                                            const int32_t* __restrict__ idx, int g0, int count, int B, int c0, int ns,
                                            int wave) {
  const int c4 = min((int)(threadIdx.x & 127), 8 * ns - 1);
  const int j0 = g0 + 16 * half + (wave >> 1);
  int tok[kHalfVec];  // all token indices first (uniform across the wave), so that their loads overlap
  if (idx) {
#pragma unroll
    for (int i = 0; i < kHalfVec; ++i) tok[i] = idx[min(j0 + 4 * i, count - 1)];
#pragma unroll
    for (int i = 0; i < kHalfVec; ++i) tok[i] = min(max(tok[i], 0), B - 1);
  } else {
#pragma unroll
    for (int i = 0; i < kHalfVec; ++i) tok[i] = min(j0 + 4 * i, count - 1);
  }
#pragma unroll
  for (int i = 0; i < kHalfVec; ++i) v[i] = *reinterpret_cast<const float4*>(V + (int64_t)tok[i] * ldv + c0 + 4 * c4);
}

// fp32 -> bf16 head and bf16 tail of the (exact) remainder, both rounded to nearest even: x - (head + tail)
// is below 2^-17 |x|
__device__ __forceinline__ void stage_commit(const float4 (&v)[kHalfVec], int half, uint16_t (*vhi)[kVRow],
                                             uint16_t (*vlo)[kVRow], int wave) {
  const int c4 = threadIdx.x & 127;
#pragma unroll
  for (int i = 0; i < kHalfVec; ++i) {
    const int t = 16 * half + (wave >> 1) + 4 * i;
    const float x[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    uint16_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const __bf16 hi = (__bf16)x[e];
      h[e] = __builtin_bit_cast(uint16_t, hi);
      const __bf16 lo = (__bf16)(x[e] - __uint_as_float((uint32_t)h[e] << 16));
      l[e] = __builtin_bit_cast(uint16_t, lo);
    }
    *reinterpret_cast<uint2*>(&vhi[t][4 * c4]) = uint2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
    *reinterpret_cast<uint2*>(&vlo[t][4 * c4]) = uint2{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
  }
}

__global__ __launch_bounds__(kTBlock) void tile_rows(const LinBatch lb) {
  __shared__ __align__(16) uint16_t vhi[kRoundTok][kVRow];
  __shared__ __align__(16) uint16_t vlo[kRoundTok][kVRow];

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lane = threadIdx.x % kWave;
  const int li = lane & 15, lq = lane >> 4;
  const int B = lb.B;

  // item -> (map, kind, row block, column slice).  The image items come first: they are few and always have work,
  // and behind the weight items of a step in which nothing fired (which only read a count and leave) they would
  // wait for two rounds of empty workgroups to drain.
  const bool second = (int)blockIdx.x < lb.tile_split;
  const int ti = second ? find_task(lb.blk_begin2, lb.n, blockIdx.x) : find_task(lb.blk_begin, lb.n, blockIdx.x);
  const LinTask& p = lb.t[ti];
  const LinGroup& g = lb.g[p.group];
  const int m = p.m;
  const int item = blockIdx.x - (second ? lb.blk_begin2[ti] : lb.blk_begin[ti]);

  const uint16_t* A;
  const float* V;
  const int32_t* idx = nullptr;
  int K, count, slices, g_begin = 0;
  bool to_part;
  if (second) {
    // image term over all tokens, whole rank in one slice, written straight to Y; one item per round of
    // 32 tokens, so that a large batch spreads over more workgroups instead of taking rounds in turn
    A = reinterpret_cast<const uint16_t*>(p.M); V = g.C; K = g.k; slices = (B + kRoundTok - 1) / kRoundTok;
    to_part = false;
    g_begin = (item % slices) * kRoundTok;
    count = min(B, g_begin + kRoundTok);
  } else if (lb.dense) {
    A = reinterpret_cast<const uint16_t*>(p.W); V = reinterpret_cast<const float*>(g.X); K = g.d; count = B;
    slices = p.slices; to_part = true;
  } else {
    int nf = g.n_fired[0];
    nf = nf < 0 ? 0 : (nf > B ? B : nf);
    // the fired tokens' r (added to the image term), or their x (replacing it: Algorithm 1, line 7)
    A = reinterpret_cast<const uint16_t*>(p.W); V = g.wx ? reinterpret_cast<const float*>(g.X) : g.R; K = g.d;
    count = nf; idx = g.fired_idx;
    slices = p.slices; to_part = true;
  }
  if (count == 0) return;  // uniform: no fired token, no weight byte is read
  const int rb = item / slices, ks = second ? 0 : item - rb * slices;
  const int c0 = ks * kSliceCols;
  const int ns = min(kSteps, (K - c0) / kStepCols);
  const int row0 = rb * kItemRows + 16 * wave;

  // first round's activations, then the weights, so that the activations can be converted and staged while
  // the weights are still on their way
  float4 v[kHalfVec];
  stage_issue(v, 0, V, K, idx, g_begin, count, B, c0, ns, wave);
  __builtin_amdgcn_sched_barrier(0);
  uint4 w[kSteps];
  {
    // uniform base + one 32-bit lane offset (the matrix is smaller than 2 GiB); rows past m repeat the last
    const char* base = reinterpret_cast<const char*>(A + c0);
    const uint32_t voff = ((uint32_t)min(row0 + li, m - 1) * (uint32_t)K + 8u * lq) * 2u;
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
      w[s] = *reinterpret_cast<const uint4*>(base + (size_t)(min(s, ns - 1) * kStepCols * 2) + voff);
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the weight requests ahead of the wait for the activations
  stage_commit(v, 0, vhi, vlo, wave);
  if (count - g_begin > 16) {  // uniform
    stage_issue(v, 1, V, K, idx, g_begin, count, B, c0, ns, wave);
    stage_commit(v, 1, vhi, vlo, wave);
  }

  for (int g0 = g_begin; g0 < count; g0 += kRoundTok) {
    if (g0 != g_begin) {
      __syncthreads();  // the previous round's operands have been read
      stage_issue(v, 0, V, K, idx, g0, count, B, c0, ns, wave);
      stage_commit(v, 0, vhi, vlo, wave);
      if (count - g0 > 16) {
        stage_issue(v, 1, V, K, idx, g0, count, B, c0, ns, wave);
        stage_commit(v, 1, vhi, vlo, wave);
      }
    }
    __syncthreads();
    const bool two = count - g0 > 16;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      if (s < ns) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, w[s]);
        const int col = s * kStepCols + 8 * lq;
        const bf16x8 h0 = *reinterpret_cast<const bf16x8*>(&vhi[li][col]);
        const bf16x8 l0 = *reinterpret_cast<const bf16x8*>(&vlo[li][col]);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h0, acc0, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l0, acc0, 0, 0, 0);
        if (two) {
          const bf16x8 h1 = *reinterpret_cast<const bf16x8*>(&vhi[16 + li][col]);
          const bf16x8 l1 = *reinterpret_cast<const bf16x8*>(&vlo[16 + li][col]);
          acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h1, acc1, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l1, acc1, 0, 0, 0);
        }
      }
    }
    // lane holds token li of each tile, rows 4*lq .. 4*lq+3 of the wave's 16
    const int row = row0 + 4 * lq;
    if (row < m) {  // m is a multiple of 4
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int j = g0 + 16 * t + li;
        if (j < count) {
          const f32x4 a = t ? acc1 : acc0;
          float* dst = to_part ? p.part + ((int64_t)ks * B + j) * m + row : p.Y + (int64_t)j * m + row;
          *reinterpret_cast<float4*>(dst) = float4{a[0], a[1], a[2], a[3]};
        }
      }
    }
  }
}

// Y[token j] (+)= sum over column slices of the partial products of the weight term.  Four threads share an
// output (each adds a quarter of the slices in order, the four sums are then added in order): fixed order, and
// one memory round trip up to 32 slices.
constexpr int kSumParts = 4, kSumOut = 256 / kSumParts;
__global__ __launch_bounds__(256) void tile_reduce(const LinBatch lb) {
  __shared__ float4 red[kSumParts][kSumOut];
  const LinTask& p = lb.t[blockIdx.y];
  const LinGroup& g = lb.g[p.group];
  const int B = lb.B, m = p.m;
  int count = B;
  if (!lb.dense) {
    const int nf = g.n_fired[0];
    count = nf < 0 ? 0 : (nf > B ? B : nf);
  }
  const int m4 = m >> 2;
  if ((int64_t)blockIdx.x * kSumOut >= (int64_t)count * m4) return;  // uniform
  const int el = threadIdx.x % kSumOut, part = threadIdx.x / kSumOut;
  const int64_t e = (int64_t)blockIdx.x * kSumOut + el;
  const bool live = e < (int64_t)count * m4;
  const int j = live ? (int)(e / m4) : 0, r4 = live ? (int)(e - (int64_t)j * m4) : 0;
  const float4* src = reinterpret_cast<const float4*>(p.part + (int64_t)j * m) + r4;
  const int64_t slice_stride = (int64_t)B * m4;
  const int per = (p.slices + kSumParts - 1) / kSumParts;
  const int s_begin = part * per, s_end = min(p.slices, s_begin + per);
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  for (int k0 = s_begin; k0 < s_end; k0 += 8) {  // eight requests in flight; the sum keeps slice order
    float4 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = src[min(k0 + u, p.slices - 1) * slice_stride];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (k0 + u < s_end) { s.x += q[u].x; s.y += q[u].y; s.z += q[u].z; s.w += q[u].w; }
  }
  red[part][el] = s;
  __syncthreads();
  if (part != 0 || !live) return;
#pragma unroll
  for (int w = 1; w < kSumParts; ++w) {
    const float4 q = red[w][el];
    s.x += q.x; s.y += q.y; s.z += q.z; s.w += q.w;
  }
  int tok = j;
  if (!lb.dense) tok = min(max(g.fired_idx[j], 0), B - 1);
  float4* y = reinterpret_cast<float4*>(p.Y + (int64_t)tok * m) + r4;
  if (lb.dense || g.wx) *y = s;
  else {
    const float4 o = *y;
    *y = float4{o.x + s.x, o.y + s.y, o.z + s.z, o.w + s.w};
  }
}


// ================================================================================================
// Projection of a decode batch (Algorithm 1, lines 1-3): c = U^T x, r = x - U c, |r|^2, |x|^2
// ================================================================================================
constexpr int kPBlock = 256;                 // partial-projection workgroup: 4 waves, one 16-column block each
constexpr int kPCols = 64;                   // columns of U per workgroup
constexpr int kPSteps = 4;                   // 32-row steps per slab of U (a slab is 128 rows)
constexpr int kPURow = kPCols + 4;           // bf16 per staged U row: the 136-byte stride keeps the four
                                             // row groups of the column-wise 16-bit reads on distinct banks
constexpr int kPXRow = kStepCols + 8;        // bf16 per staged token row (80 bytes): conflict-free 128-bit reads

// c partials: part_c[slab][t][j] = sum over the slab's rows i of U[i][j] x_t[i].
// The contraction runs over rows of U, which are not contiguous in memory, so a 32-row x 64-column tile of
// U is staged in LDS as it is stored and the A operand (16 columns x 32 rows) is gathered column-wise with
// 16-bit reads; it then serves every token tile (two MFMAs each: bf16 head and tail of the fp32 x).
template <int XV>  // XV = token groups of 32 the call may have (1, 2 or 4): sizes the register arrays
__global__ __launch_bounds__(kPBlock) void tile_proj_partial(const ProjBatch pb) {
  __shared__ __align__(16) uint16_t us[2][kStepCols][kPURow];
  __shared__ __align__(16) uint16_t xh[2][kMaxTok][kPXRow];
  __shared__ __align__(16) uint16_t xl[2][kMaxTok][kPXRow];

  const int ti = find_task(pb.a_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  const int local = blockIdx.x - pb.a_begin[ti];
  const int cgroups = p.k / kPCols;
  // the column groups of a row slab are a_slabs workgroups apart: on the same XCD when a_slabs is a multiple of 8
  // (workgroups go to the 8 XCDs in turn), and so is the residual workgroup of the same rows
  const int slab = local % p.a_slabs, cg = local / p.a_slabs;
  const int d = p.d, k = p.k, B = pb.B;
  if (local == 0 && threadIdx.x == 0) *p.sync = 0u;  // the residual launch counts its finished workgroups here
  const int row_begin = slab * p.a_rows;
  const int steps = (min(p.a_rows, d - row_begin)) / kStepCols;  // 1..4: d and a_rows are multiples of 32
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lane = threadIdx.x % kWave, li = lane & 15, lq = lane >> 4;
  const int ntile = (B + 15) >> 4;
  const uint16_t* U = reinterpret_cast<const uint16_t*>(p.U);
  const float* X = reinterpret_cast<const float*>(p.X);

  // staging roles: U tile 32 rows x 8 chunks of 16 bytes = 256 threads; x tile B tokens x 8 float4
  const int urow = threadIdx.x >> 3, uch = threadIdx.x & 7;
  const uint16_t* usrc = U + (int64_t)(row_begin + urow) * k + cg * kPCols + 8 * uch;
  constexpr int kXV = XV;                     // float4 per thread and step: one per 32 tokens
  constexpr int kTiles = 2 * XV;              // MFMA token tiles
  const int xc4 = threadIdx.x & 7;
  const float* xsrc[kXV];
#pragma unroll
  for (int u = 0; u < kXV; ++u) {
    const int t = min((int)(threadIdx.x >> 3) + 32 * u, B - 1);  // tokens past B repeat the last one
    xsrc[u] = X + (int64_t)t * d + row_begin + 4 * xc4;
  }
  // A slab is at most four steps (128 rows): everything it reads is requested at once, then staged and
  // consumed step by step (two LDS buffers), so the slab costs one memory round trip, not four.
  uint4 ur[kPSteps];
  float4 xr[kPSteps][kXV];
#pragma unroll
  for (int s = 0; s < kPSteps; ++s) {
    const int sc = min(s, steps - 1);  // steps past the slab repeat the last one and are not consumed
    ur[s] = *reinterpret_cast<const uint4*>(usrc + (int64_t)sc * kStepCols * k);
#pragma unroll
    for (int u = 0; u < kXV; ++u) xr[s][u] = *reinterpret_cast<const float4*>(xsrc[u] + sc * kStepCols);
  }
  __builtin_amdgcn_sched_barrier(0);  // every request of the slab is issued before the first wait
  auto commit = [&](int s, int buf) {
    uint2* ud = reinterpret_cast<uint2*>(&us[buf][urow][8 * uch]);
    ud[0] = uint2{ur[s].x, ur[s].y};
    ud[1] = uint2{ur[s].z, ur[s].w};
#pragma unroll
    for (int u = 0; u < kXV; ++u) {
      {
        const int t = (threadIdx.x >> 3) + 32 * u;  // tokens past B hold a copy of the last one, never used
        const float x[4] = {xr[s][u].x, xr[s][u].y, xr[s][u].z, xr[s][u].w};
        uint16_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const __bf16 hi = (__bf16)x[e];
          h[e] = __builtin_bit_cast(uint16_t, hi);
          const __bf16 lo = (__bf16)(x[e] - __uint_as_float((uint32_t)h[e] << 16));
          l[e] = __builtin_bit_cast(uint16_t, lo);
        }
        *reinterpret_cast<uint2*>(&xh[buf][t][4 * xc4]) = uint2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
        *reinterpret_cast<uint2*>(&xl[buf][t][4 * xc4]) = uint2{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
      }
    }
  };

  f32x4 acc[kTiles];
#pragma unroll
  for (int t = 0; t < kTiles; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  commit(0, 0);
#pragma unroll
  for (int s = 0; s < kPSteps; ++s) {
    if (s < steps) {  // uniform
      const int buf = s & 1;
      __syncthreads();  // step s is staged; step s-1 (the other buffer) has been read by every wave
      // A operand: lane (column li of the wave's block, row group lq) gathers rows 8 lq .. 8 lq + 7
      uint16_t a16[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) a16[e] = us[buf][8 * lq + e][16 * wave + li];
      uint4 ap;
      ap.x = (uint32_t)a16[0] | ((uint32_t)a16[1] << 16); ap.y = (uint32_t)a16[2] | ((uint32_t)a16[3] << 16);
      ap.z = (uint32_t)a16[4] | ((uint32_t)a16[5] << 16); ap.w = (uint32_t)a16[6] | ((uint32_t)a16[7] << 16);
      const bf16x8 a = __builtin_bit_cast(bf16x8, ap);
#pragma unroll
      for (int t = 0; t < kTiles; ++t) {
        if (t < ntile) {  // uniform
          const bf16x8 h = *reinterpret_cast<const bf16x8*>(&xh[buf][16 * t + li][8 * lq]);
          const bf16x8 l = *reinterpret_cast<const bf16x8*>(&xl[buf][16 * t + li][8 * lq]);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acc[t], 0, 0, 0);
        }
      }
      if (s + 1 < kPSteps && s + 1 < steps) commit(s + 1, buf ^ 1);
    }
  }
  // lane holds token li of each tile, columns 4 lq .. 4 lq + 3 of the wave's block
#pragma unroll
  for (int t = 0; t < kTiles; ++t) {
    const int tok = 16 * t + li;
    if (t < ntile && tok < B) {
      float* dst = p.part_c + ((int64_t)slab * B + tok) * k + cg * kPCols + 16 * wave + 4 * lq;
      *reinterpret_cast<float4*>(dst) = float4{acc[t][0], acc[t][1], acc[t][2], acc[t][3]};
    }
  }
}

// C[t][j] = sum over slabs of the partial projections.  Sixteen threads share an output (each adds a sixteenth
// of the slabs in order, the sixteen sums are then added in order): fixed order, one or two memory round trips.
constexpr int kRedParts = 16, kRedOut = 256 / kRedParts;
__global__ __launch_bounds__(256) void tile_proj_reduce(const ProjBatch pb) {
  __shared__ float4 red[kRedParts][kRedOut];
  const ProjTask& p = pb.t[blockIdx.y];
  const int B = pb.B, k4 = p.k >> 2;
  const int el = threadIdx.x % kRedOut, part = threadIdx.x / kRedOut;
  const int e = blockIdx.x * kRedOut + el;
  const bool live = e < B * k4;
  const int per = (p.a_slabs + kRedParts - 1) / kRedParts;
  const int s_begin = part * per, s_end = min(p.a_slabs, s_begin + per);
  const float4* src = reinterpret_cast<const float4*>(p.part_c) + (live ? e : 0);
  const int64_t stride = (int64_t)B * k4;
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = s_begin; s0 < s_end; s0 += 8) {
    float4 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = src[min(s0 + u, p.a_slabs - 1) * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < s_end) { s.x += q[u].x; s.y += q[u].y; s.z += q[u].z; s.w += q[u].w; }
  }
  red[part][el] = s;
  __syncthreads();
  if (part == 0 && live) {
    float4 t = red[0][el];
#pragma unroll
    for (int w = 1; w < kRedParts; ++w) {
      const float4 q = red[w][el];
      t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
    }
    reinterpret_cast<float4*>(p.C)[e] = t;
  }
}

// |r|, |x| per token from the row blocks' shares, then the gate and the ordered list of fired tokens
// (Eq. (gate); Algorithm 1, line 4), by the 512 threads of one workgroup.  16 threads share a token (4 beyond
// 32 tokens): each adds its part of the shares in order, the part sums are then added in order.
// red: 512 float2 and two ints of LDS.
__device__ __forceinline__ void norms_and_gate(const ProjTask& p, int B, int do_gate, float eps, float2* red,
                                               int* wave_count) {
  const int slots = B <= 32 ? 32 : kMaxTok, parts = kTBlock / slots;
  const int t = threadIdx.x % slots, part = threadIdx.x / slots;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int per = (p.b_slabs + parts - 1) / parts;
  const int s_begin = part * per, s_end = min(p.b_slabs, s_begin + per);
  float sr = 0.f, sx = 0.f;
  const float2* src = reinterpret_cast<const float2*>(p.part_n) + min(t, B - 1);
  for (int s0 = s_begin; s0 < s_end; s0 += 8) {
    unsigned long long q[8];  // (|r|^2, |x|^2) shares, read past the caches: other workgroups of this launch wrote them
#pragma unroll
    for (int u = 0; u < 8; ++u)
      q[u] = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src + (int64_t)min(s0 + u, p.b_slabs - 1) * B),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < s_end) { sr += __uint_as_float((unsigned)q[u]); sx += __uint_as_float((unsigned)(q[u] >> 32)); }
  }
  red[part * slots + t] = float2{sr, sx};
  __syncthreads();
  // the threads of part 0 (thread index = token) finish the job; the others only keep the barriers
  const bool head = part == 0;
  sr = red[t].x;
  sx = red[t].y;
  for (int w = 1; w < parts; ++w) {
    sr += red[w * slots + t].x;
    sx += red[w * slots + t].y;
  }
  const float rn = sqrtf(sr), xn = sqrtf(sx);
  if (head && t < B) {
    p.rnorm[t] = rn;
    p.xnorm[t] = xn;
  }
  if (!do_gate) return;  // uniform
  const bool fired = head && t < B && gate_fires(rn, xn, eps);
  if (head && t < B) p.mask[t] = fired ? 1 : 0;
  const unsigned long long ballot = __ballot(fired);
  const int rank_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
  if (wave < kMaxTok / kWave && lane == 0) wave_count[wave] = __popcll(ballot);
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int wv = 0; wv < kMaxTok / kWave; ++wv) {
    const int c = wave_count[wv];
    if (wv < wave) before += c;
    total += c;
  }
  if (fired) p.fired_idx[before + rank_in_wave] = t;
  if (threadIdx.x == 0) p.n_fired[0] = total;
}

// r = x - U c for 128 rows x 32 tokens per workgroup (the weights of this product are the rows of U, which are
// contiguous: same operand flow as tile_rows), R written, and the row block's share of |r|^2 and |x|^2.
// The workgroup of an input that finishes last (a counter in the workspace, zeroed by the partial-projection
// launch) turns the shares into the norms, the gate decisions and the list of fired tokens: no launch of its own.
__global__ __launch_bounds__(kTBlock) void tile_residual(const ProjBatch pb) {
  __shared__ int s_last;
  __shared__ __align__(16) uint16_t vhi[kRoundTok][kVRow];
  __shared__ __align__(16) uint16_t vlo[kRoundTok][kVRow];
  __shared__ float red[kTWaves][kRoundTok][2];

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lane = threadIdx.x % kWave, li = lane & 15, lq = lane >> 4;
  const int B = pb.B;
  const int ti = find_task(pb.b_begin, pb.n, blockIdx.x);
  const ProjTask& p = pb.t[ti];
  const int rounds = (B + kRoundTok - 1) / kRoundTok;
  const int item = blockIdx.x - pb.b_begin[ti];
  const int nrb = p.d / kItemRows;  // row blocks; the rounds of a row block are nrb workgroups apart (same XCD)
  const int rb = item % nrb, g0 = (item / nrb) * kRoundTok;
  const int count = min(B, g0 + kRoundTok);
  const int d = p.d, k = p.k, ns = k / kStepCols;
  const int row0 = rb * kItemRows + 16 * wave;  // d is a multiple of 128: every row exists
  const uint16_t* U = reinterpret_cast<const uint16_t*>(p.U);
  const float* X = reinterpret_cast<const float*>(p.X);

  float4 v[kHalfVec];
  stage_issue(v, 0, p.C, k, nullptr, g0, count, B, 0, ns, wave);
  __builtin_amdgcn_sched_barrier(0);
  uint4 w[kSteps];
  {
    const char* base = reinterpret_cast<const char*>(U);
    const uint32_t voff = ((uint32_t)(row0 + li) * (uint32_t)k + 8u * lq) * 2u;
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
      w[s] = *reinterpret_cast<const uint4*>(base + (size_t)(min(s, ns - 1) * kStepCols * 2) + voff);
  }
  // x of the lane's outputs: token g0 + 16 t + li, rows row0 + 4 lq .. + 3
  float4 xv[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = min(g0 + 16 * t + li, B - 1);
    xv[t] = *reinterpret_cast<const float4*>(X + (int64_t)j * d + row0 + 4 * lq);
  }
  __builtin_amdgcn_sched_barrier(0);
  stage_commit(v, 0, vhi, vlo, wave);
  const bool two = count - g0 > 16;
  if (two) {
    stage_issue(v, 1, p.C, k, nullptr, g0, count, B, 0, ns, wave);
    stage_commit(v, 1, vhi, vlo, wave);
  }
  __syncthreads();
  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    if (s < ns) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, w[s]);
      const int col = s * kStepCols + 8 * lq;
      const bf16x8 h0 = *reinterpret_cast<const bf16x8*>(&vhi[li][col]);
      const bf16x8 l0 = *reinterpret_cast<const bf16x8*>(&vlo[li][col]);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h0, acc0, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l0, acc0, 0, 0, 0);
      if (two) {
        const bf16x8 h1 = *reinterpret_cast<const bf16x8*>(&vhi[16 + li][col]);
        const bf16x8 l1 = *reinterpret_cast<const bf16x8*>(&vlo[16 + li][col]);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h1, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l1, acc1, 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = g0 + 16 * t + li;
    const f32x4 a = t ? acc1 : acc0;
    const float4 x = xv[t];
    const float4 r = float4{x.x - a[0], x.y - a[1], x.z - a[2], x.w - a[3]};
    float sr = 0.f, sx = 0.f;
    if (j < count) {
      *reinterpret_cast<float4*>(p.R + (int64_t)j * d + row0 + 4 * lq) = r;
      sr = fmaf(r.x, r.x, fmaf(r.y, r.y, fmaf(r.z, r.z, r.w * r.w)));
      sx = fmaf(x.x, x.x, fmaf(x.y, x.y, fmaf(x.z, x.z, x.w * x.w)));
    }
    // the four row groups of the wave (lanes li, li+16, li+32, li+48), fixed order
    sr += __shfl_xor(sr, 16); sr += __shfl_xor(sr, 32);
    sx += __shfl_xor(sx, 16); sx += __shfl_xor(sx, 32);
    if (lq == 0) {
      red[wave][16 * t + li][0] = sr;
      red[wave][16 * t + li][1] = sx;
    }
  }
  __syncthreads();
  if (threadIdx.x < 2 * kRoundTok) {
    const int tl = threadIdx.x >> 1, c = threadIdx.x & 1;
    if (g0 + tl < count) {
      float sum = 0.f;
#pragma unroll
      for (int wv = 0; wv < kTWaves; ++wv) sum += red[wv][tl][c];
      // written through to memory (a store that is coherent across the chip), so that the workgroup that finishes
      // last can read it without anybody writing a whole L2 back: such a write-back costs about a microsecond per
      // workgroup, one after the other
      __hip_atomic_store(&p.part_n[((int64_t)rb * B + g0 + tl) * 2 + c], sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (!pb.norms) return;  // uniform
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores have completed ...
  __syncthreads();                                  // ... in every wave before the workgroup counts as done
  if (threadIdx.x == 0) {
    const unsigned done = __hip_atomic_fetch_add(p.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = done + 1u == (unsigned)(nrb * rounds);
  }
  __syncthreads();
  if (!s_last) return;  // uniform
  norms_and_gate(p, B, pb.gate, pb.eps, reinterpret_cast<float2*>(&vhi[0][0]), reinterpret_cast<int*>(&vlo[0][0]));
}

}  // namespace

int tile_slices(int64_t d) { return (int)ceil_div(d, kSliceCols); }

// ---- projection ---------------------------------------------------------------------------------
bool tile_project_shape_ok(int64_t d, int64_t k, int64_t B, int udtype) {
  return udtype == GSI_BF16 && B >= 2 && B <= kMaxTok && d % kItemRows == 0 && k % kPCols == 0 && k <= kSliceCols &&
         d < (1 << 24);
}

static int tile_slab_rows(int64_t) { return kPSteps * kStepCols; }

size_t tile_project_ws(int64_t d, int64_t k, int64_t B) {
  const int a_slabs = (int)ceil_div(d, tile_slab_rows(d));
  return align_up((size_t)a_slabs * B * k * 4, 256) + align_up((size_t)(d / kItemRows) * B * 2 * 4, 256) + 256;
}

void tile_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws) {
  t.d = (int)d;
  t.k = (int)k;
  t.a_rows = tile_slab_rows(d);
  t.a_slabs = (int)ceil_div(d, t.a_rows);
  t.a_cblocks = (int)(k / kPCols);
  t.b_rows = kItemRows;
  t.b_slabs = (int)(d / kItemRows);
  t.part_c = reinterpret_cast<float*>(ws);
  t.part_n = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + align_up((size_t)t.a_slabs * B * k * 4, 256));
  t.sync = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(t.part_n) + align_up((size_t)t.b_slabs * B * 2 * 4, 256));
  t.tile = 1;
}

hipError_t tile_project_launch(ProjBatch& pb, bool with_norms, bool with_gate, float eps, hipStream_t s) {
  if (pb.n == 0 || pb.B == 0) return hipSuccess;
  const int rounds = (int)ceil_div(pb.B, kRoundTok);
  int ta = 0, tb = 0, max_k = 0;
  for (int i = 0; i < pb.n; ++i) {
    pb.a_begin[i] = ta;
    pb.b_begin[i] = tb;
    ta += pb.t[i].a_slabs * pb.t[i].a_cblocks;
    tb += pb.t[i].b_slabs * rounds;
    if (pb.t[i].k > max_k) max_k = pb.t[i].k;
  }
  pb.b_total = tb;
  pb.norms = with_norms ? 1 : 0;
  pb.gate = with_gate ? 1 : 0;
  pb.eps = eps;
  if (pb.B <= 32) tile_proj_partial<1><<<ta, kPBlock, 0, s>>>(pb);
  else if (pb.B <= 64) tile_proj_partial<2><<<ta, kPBlock, 0, s>>>(pb);
  else tile_proj_partial<4><<<ta, kPBlock, 0, s>>>(pb);
  const dim3 rgrid((unsigned)ceil_div((int64_t)pb.B * (max_k / 4), kRedOut), (unsigned)pb.n);
  tile_proj_reduce<<<rgrid, 256, 0, s>>>(pb);
  tile_residual<<<tb, kTBlock, 0, s>>>(pb);
  return hipGetLastError();
}

// shapes the matrix-core linear kernel takes (alignments and the partial-product workspace apart: tile_rows_ok)
bool tile_rows_shape_ok(int64_t m, int64_t d, int64_t k, int64_t B, int wdtype) {
  return wdtype == GSI_BF16 && B >= 2 && B <= kMaxTok && d % kStepCols == 0 && m % 4 == 0 &&
         m * d * 2 < (1ll << 32) && (k == 0 || (k % kStepCols == 0 && k <= kSliceCols));
}

size_t tile_part_bytes(int64_t m, int64_t d, int64_t B) {
  if (B < 2 || B > kMaxTok || d % kStepCols || m % 4) return 0;
  return align_up((size_t)tile_slices(d) * B * m * sizeof(float), 256);
}

bool tile_rows_ok(const LinBatch& lb, int wdtype) {
  if (wdtype != GSI_BF16 || lb.B < 2 || lb.B > kMaxTok) return false;
  for (int i = 0; i < lb.ng; ++i) {
    const LinGroup& g = lb.g[i];
    if (g.d % kStepCols) return false;
    if (lb.dense || g.wx) {
      if (g.xdtype != GSI_F32 || reinterpret_cast<uintptr_t>(g.X) % 16) return false;
    }
    if (!lb.dense) {
      if (g.k % kStepCols || g.k > kSliceCols) return false;
      if (reinterpret_cast<uintptr_t>(g.C) % 16 || reinterpret_cast<uintptr_t>(g.R) % 16) return false;
    }
  }
  for (int i = 0; i < lb.n; ++i) {
    const LinTask& t = lb.t[i];
    if (t.m % 4 || reinterpret_cast<uintptr_t>(t.Y) % 16 || reinterpret_cast<uintptr_t>(t.W) % 16) return false;
    if ((int64_t)t.m * lb.g[t.group].d * 2 >= (1ll << 32)) return false;  // 32-bit byte offsets into a matrix
    if (!t.part || reinterpret_cast<uintptr_t>(t.part) % 16) return false;
    if (!lb.dense && reinterpret_cast<uintptr_t>(t.M) % 16) return false;
  }
  return true;
}

hipError_t tile_rows_launch(LinBatch& lb, hipStream_t s) {
  int total = 0, max_m = 0;
  for (int i = 0; i < lb.n; ++i) {
    lb.blk_begin2[i] = total;
    if (!lb.dense) total += (int)(ceil_div(lb.t[i].m, kItemRows) * ceil_div(lb.B, kRoundTok));
  }
  lb.tile_split = total;  // image items below, weight items from here on
  for (int i = 0; i < lb.n; ++i) {
    lb.t[i].slices = tile_slices(lb.g[lb.t[i].group].d);
    lb.blk_begin[i] = total;
    total += (int)ceil_div(lb.t[i].m, kItemRows) * lb.t[i].slices;
    if (lb.t[i].m > max_m) max_m = lb.t[i].m;
  }
  tile_rows<<<total, kTBlock, 0, s>>>(lb);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  const dim3 grid((unsigned)ceil_div((int64_t)lb.B * (max_m / 4), kSumOut), (unsigned)lb.n);
  tile_reduce<<<grid, 256, 0, s>>>(lb);
  return hipGetLastError();
}

}  // namespace gsi
