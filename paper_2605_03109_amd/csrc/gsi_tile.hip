// Linear maps of a decode batch (2..128 tokens per call) on the matrix cores: Algorithm 1 lines 4-7 in
// the y = M c (+ W r when the gate fires) form of Eq. (exact), and the dense baseline y = W x.
//
// The work is a skinny GEMM bound by the one pass over the weights, so the kernel is organised around
// that pass.  A work item is 128 rows of one matrix by a slice of 512 contraction columns: each of the
// eight waves owns 16 rows and requests its whole share (16 loads of 16 bytes per lane) at once, straight
// from memory into A operands of v_mfma_f32_16x16x32_bf16 (lane l holds row l%16, columns 8*(l/16)..+8
// of a 32-column step).  The B operands are the same columns of up to 32 tokens' activation vectors,
// staged once per workgroup in LDS: fp32 activations are split into a bf16 head (upper 16 bits) and a bf16
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
constexpr int kVRow = kSliceCols + 8;              // bf16 per staged token row: 16 bytes of padding keep
                                                   // the 16 lanes of a 128-bit LDS read on distinct banks
constexpr int kHalfVec = 16 * kSliceCols / 4 / kTBlock;  // float4 per thread per 16 staged tokens (4)

__device__ __forceinline__ int find_task(const int* begin, int n, int b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < kMaxTasks; ++i)
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

// fp32 -> bf16 head (truncation: exactly representable, so the remainder is exact) and bf16 tail (RNE)
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
      const uint32_t bits = __float_as_uint(x[e]);
      h[e] = (uint16_t)(bits >> 16);
      const __bf16 lo = (__bf16)(x[e] - __uint_as_float(bits & 0xffff0000u));
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

  // item -> (map, kind, row block, column slice).  Items of the weight term come first (they are the long
  // ones), then the image items.
  const bool second = (int)blockIdx.x >= lb.tile_split;
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
    A = reinterpret_cast<const uint16_t*>(p.W); V = g.R; K = g.d; count = nf; idx = g.fired_idx;
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

// Y[token j] (+)= sum over column slices, in slice order, of the partial products of the weight term
__global__ __launch_bounds__(256) void tile_reduce(const LinBatch lb) {
  const LinTask& p = lb.t[blockIdx.y];
  const LinGroup& g = lb.g[p.group];
  const int B = lb.B, m = p.m;
  int count = B;
  if (!lb.dense) {
    const int nf = g.n_fired[0];
    count = nf < 0 ? 0 : (nf > B ? B : nf);
  }
  const int m4 = m >> 2;
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)count * m4) return;
  const int j = (int)(e / m4), r4 = (int)(e - (int64_t)j * m4);
  const float4* src = reinterpret_cast<const float4*>(p.part + (int64_t)j * m) + r4;
  const int64_t slice_stride = (int64_t)B * m4;
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < p.slices; k0 += 8) {  // eight requests in flight; the sum keeps slice order
    float4 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = src[min(k0 + u, p.slices - 1) * slice_stride];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (k0 + u < p.slices) { s.x += q[u].x; s.y += q[u].y; s.z += q[u].z; s.w += q[u].w; }
  }
  int tok = j;
  if (!lb.dense) tok = min(max(g.fired_idx[j], 0), B - 1);
  float4* y = reinterpret_cast<float4*>(p.Y + (int64_t)tok * m) + r4;
  if (lb.dense) *y = s;
  else {
    const float4 o = *y;
    *y = float4{o.x + s.x, o.y + s.y, o.z + s.z, o.w + s.w};
  }
}

}  // namespace

int tile_slices(int64_t d) { return (int)ceil_div(d, kSliceCols); }

size_t tile_part_bytes(int64_t m, int64_t d, int64_t B) {
  if (B < 2 || B > kRoundTok * 4 || d % kStepCols || m % 4) return 0;
  return align_up((size_t)tile_slices(d) * B * m * sizeof(float), 256);
}

bool tile_rows_ok(const LinBatch& lb, int wdtype) {
  if (wdtype != GSI_BF16 || lb.B < 2 || lb.B > kRoundTok * 4) return false;
  for (int i = 0; i < lb.ng; ++i) {
    const LinGroup& g = lb.g[i];
    if (g.d % kStepCols) return false;
    if (lb.dense) {
      if (g.xdtype != GSI_F32 || reinterpret_cast<uintptr_t>(g.X) % 16) return false;
    } else {
      if (g.k % kStepCols || g.k > kSliceCols) return false;
      if (reinterpret_cast<uintptr_t>(g.C) % 16 || reinterpret_cast<uintptr_t>(g.R) % 16) return false;
    }
  }
  for (int i = 0; i < lb.n; ++i) {
    const LinTask& t = lb.t[i];
    if (t.m % 4 || reinterpret_cast<uintptr_t>(t.Y) % 16 || reinterpret_cast<uintptr_t>(t.W) % 16) return false;
    if (!t.part || reinterpret_cast<uintptr_t>(t.part) % 16) return false;
    if (!lb.dense && reinterpret_cast<uintptr_t>(t.M) % 16) return false;
  }
  return true;
}

hipError_t tile_rows_launch(LinBatch& lb, hipStream_t s) {
  int total = 0, max_m = 0;
  for (int i = 0; i < lb.n; ++i) {
    lb.t[i].slices = tile_slices(lb.g[lb.t[i].group].d);
    lb.blk_begin[i] = total;
    total += (int)ceil_div(lb.t[i].m, kItemRows) * lb.t[i].slices;
    if (lb.t[i].m > max_m) max_m = lb.t[i].m;
  }
  lb.tile_split = total;
  for (int i = 0; i < lb.n; ++i) {
    lb.blk_begin2[i] = total;
    if (!lb.dense) total += (int)(ceil_div(lb.t[i].m, kItemRows) * ceil_div(lb.B, kRoundTok));
  }
  tile_rows<<<total, kTBlock, 0, s>>>(lb);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  const dim3 grid((unsigned)ceil_div((int64_t)lb.B * (max_m / 4), 256), (unsigned)lb.n);
  tile_reduce<<<grid, 256, 0, s>>>(lb);
  return hipGetLastError();
}

}  // namespace gsi
