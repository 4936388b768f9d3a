// Dense contractions of libgsi on the matrix cores (gfx950 MFMA, bf16 inputs, fp32 accumulation):
// the one-time image build M = W U (Eq. (exact), Section 4 "Storage") and the prefill-sized batched
// path (hundreds of tokens per call), where the work really is a GEMM:
//     C = X U            R = X - C U^T  (+ per-token partial norms)          Algorithm 1, lines 1-3
//     Y = C M^T          Y[fired] += R[fired] W^T                            Eq. (exact)
//
// One kernel, D = A B^T with both operands K-contiguous ("NT"): A[M,K], B[N,K] row-major.  A is bf16,
// or fp32 split on the fly into a bf16 head and a bf16 tail (two MFMA passes) so that an fp32 operand
// on the main term is not rounded to 8 bits (the bf16 image already uses most of the 2e-3 budget).
//
// Workgroup tile 256 x 256 x 64, eight waves 4 x 2 (two per SIMD, so that one wave's MFMAs cover the
// other's LDS reads and staging), each wave 64 x 128 as 2 x 4 v_mfma_f32_32x32x16_bf16 fragments.
// Both operand tiles are staged in LDS as bf16 (row stride padded to 144 bytes: conflict-free 128-bit
// reads); an fp32 A operand is converted on the way in.  Global loads are whole 128-byte row segments per
// eight lanes.  LDS holds two k-tiles: tile t is multiplied while tile t + 1 is written, a unit per MFMA step,
// from registers that are asked for tile t + 2 at once; one barrier per tile.  A k-tile is 64 columns deep, or
// 32 for the head + tail form (two tiles of A per stage, two MFMA passes per step: as many MFMAs between
// barriers).  Within a k-tile the lane half l/32 takes one half of the columns, eight per MFMA step: any order
// of the contraction index is as good as another as long as both operands agree.
// What bounds the loop is LDS, not the matrix cores: a k-tile is 2048 MFMA cycles per SIMD, and its LDS
// traffic (192 KB of operand reads at 128 bytes a cycle, 64 KB of staging writes at about 75) is 2400.
// Problems with few output tiles split the contraction over blockIdx.z; the partial sums go to the workspace
// and a second kernel adds them in split order and applies the epilogue.
// Operands that are N-contiguous in memory (U as the right factor of W U and X U) are transposed
// once into the workspace.
#include <algorithm>

#include "gsi_device.h"
#include "gsi_mfma.h"

namespace gsi {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 256, BN = 256, BK = 64;      // BK: the host's unit of the contraction (K is a multiple of it)
constexpr int WTM = 64, WTN = 128;              // wave tile: the eight waves sit 4 x 2 on the workgroup tile
constexpr int kThreads = 512;
constexpr int kAF = WTM / 32, kBF = WTN / 32;   // A, B fragments per wave

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a native vector: loads and stores of it are
                                                              // instructions, not aggregate copies

// AM: how the A operand is stored and fed: 0 bf16; 1 fp32, split into bf16 head + tail (two LDS tiles, two
// MFMA passes); 2 fp32, rounded once to bf16.
// Geometry of a staged k-tile by mode.  The head + tail form keeps two tiles of A per stage, so its k-tile is 32
// columns deep (two MFMA steps of two passes each: as many MFMAs between barriers as the 64-deep tile of the
// other modes) and two stages still fit in LDS.
template <int AM>
struct Geo {
  static constexpr int BKT = AM == 1 ? 32 : 64;          // columns of a k-tile
  static constexpr int LD = BKT + 8;                     // padded LDS row stride, bf16 elements (80 or 144 bytes:
                                                         // conflict-free 128-bit reads either way)
  static constexpr int KS = BKT / 16;                    // MFMA steps per k-tile
  static constexpr int CPR = BKT / 8;                    // staging units (8 elements) per tile row
  static constexpr int RPP = kThreads / CPR;             // tile rows covered by one unit index of all threads
  static constexpr int NU = BM / RPP;                    // units of A (and of B) per thread and k-tile
  static constexpr int NP = AM == 1 ? 2 : 1;             // LDS tiles of A per stage
  static constexpr int kATile = BM * LD;                 // elements of one LDS tile of A
  static constexpr int kStage = (NP * BM + BN) * LD;     // elements of one stage
  static_assert(NU == KS, "one staging unit per MFMA step");
  static_assert(BM == BN, "A and B tiles are staged alike");
};

template <int AM>
struct Stage {
  u32x4 a[Geo<AM>::NU][AM ? 2 : 1];
  u32x4 b[Geo<AM>::NU];
};

// 8 fp32 -> 8 bf16 (RNE), and the bf16 of what is left
__device__ __forceinline__ u32x4 round8(const u32x4& x0, const u32x4& x1, u32x4* tail) {
  const float x[8] = {__uint_as_float(x0[0]), __uint_as_float(x0[1]), __uint_as_float(x0[2]), __uint_as_float(x0[3]),
                      __uint_as_float(x1[0]), __uint_as_float(x1[1]), __uint_as_float(x1[2]), __uint_as_float(x1[3])};
  uint16_t h[8], l[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const __bf16 hb = (__bf16)x[e];
    h[e] = __builtin_bit_cast(uint16_t, hb);
    const __bf16 lb = (__bf16)(x[e] - __uint_as_float((uint32_t)h[e] << 16));
    l[e] = __builtin_bit_cast(uint16_t, lb);
  }
  if (tail)
    *tail = u32x4{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16),
                  (uint32_t)l[4] | ((uint32_t)l[5] << 16), (uint32_t)l[6] | ((uint32_t)l[7] << 16)};
  return u32x4{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16),
               (uint32_t)h[4] | ((uint32_t)h[5] << 16), (uint32_t)h[6] | ((uint32_t)h[7] << 16)};
}

// requests unit u of k-tile kt of both operands (unit u of a thread: tile row tid / CPR + RPP u, columns
// 8 (tid % CPR) .. + 8; the pointers already point at that row and column of k-tile 0)
template <int AM>
__device__ __forceinline__ void issue_unit(Stage<AM>& st, int u, const char* const (&ap)[Geo<AM>::NU],
                                           const char* const (&bp)[Geo<AM>::NU], int kt) {
  constexpr int ES = AM ? 4 : 2;
  const char* p = ap[u] + (int64_t)kt * Geo<AM>::BKT * ES;
  st.a[u][0] = *reinterpret_cast<const u32x4*>(p);
  if constexpr (AM != 0) st.a[u][1] = *reinterpret_cast<const u32x4*>(p + 16);
  st.b[u] = *reinterpret_cast<const u32x4*>(bp[u] + (int64_t)kt * Geo<AM>::BKT * 2);
}
template <int AM>
__device__ __forceinline__ void issue(Stage<AM>& st, const char* const (&ap)[Geo<AM>::NU], const char* const (&bp)[Geo<AM>::NU],
                                      int kt) {
#pragma unroll
  for (int u = 0; u < Geo<AM>::NU; ++u) issue_unit<AM>(st, u, ap, bp, kt);
}

// writes unit u of the staged k-tile to the LDS stage at `stage` as bf16 (fp32 A: rounded, or head and tail tiles)
template <int AM>
__device__ __forceinline__ void commit_unit(const Stage<AM>& st, int u, uint16_t* stage, int tid) {
  using G = Geo<AM>;
  const int off = ((tid / G::CPR) + G::RPP * u) * G::LD + 8 * (tid % G::CPR);
  u32x4* d0 = reinterpret_cast<u32x4*>(stage + off);
  if constexpr (AM == 0) {
    *d0 = st.a[u][0];
  } else if constexpr (AM == 2) {
    *d0 = round8(st.a[u][0], st.a[u][1], nullptr);
  } else {
    u32x4 tail;
    *d0 = round8(st.a[u][0], st.a[u][1], &tail);
    *reinterpret_cast<u32x4*>(stage + G::kATile + off) = tail;
  }
  *reinterpret_cast<u32x4*>(stage + G::NP * G::kATile + off) = st.b[u];
}
template <int AM>
__device__ __forceinline__ void commit(const Stage<AM>& st, uint16_t* stage, int tid) {
#pragma unroll
  for (int u = 0; u < Geo<AM>::NU; ++u) commit_unit<AM>(st, u, stage, tid);
}

// The MFMA operands of one step (16 columns of the k-tile) of a wave: lane half lh takes one half of the tile's
// columns, eight per step (both operands in the same order, so the order of the contraction index does not
// matter)
template <int AM>
struct Ops {
  bf16x8 a[kAF];
  bf16x8 al[AM == 1 ? kAF : 1];
  bf16x8 b[kBF];
};
template <int AM>
__device__ __forceinline__ void read_ops(Ops<AM>& o, const uint16_t* stage, int wm, int wn, int lc, int lh, int j) {
  using G = Geo<AM>;
  const int col = (G::BKT / 2) * lh + 8 * j;
  const uint16_t* Bq = stage + G::NP * G::kATile;
#pragma unroll
  for (int n = 0; n < kBF; ++n) o.b[n] = *reinterpret_cast<const bf16x8*>(Bq + (WTN * wn + 32 * n + lc) * G::LD + col);
#pragma unroll
  for (int i = 0; i < kAF; ++i) {
    const int off = (WTM * wm + 32 * i + lc) * G::LD + col;
    o.a[i] = *reinterpret_cast<const bf16x8*>(stage + off);
    if constexpr (AM == 1) o.al[i] = *reinterpret_cast<const bf16x8*>(stage + G::kATile + off);
  }
}
template <int AM>
__device__ __forceinline__ void mma(const Ops<AM>& o, f32x16 (&acc)[kAF][kBF]) {
#pragma unroll
  for (int i = 0; i < kAF; ++i) {
#pragma unroll
    for (int n = 0; n < kBF; ++n) acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[i], o.b[n], acc[i][n], 0, 0, 0);
    if constexpr (AM == 1) {
#pragma unroll
      for (int n = 0; n < kBF; ++n) acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.al[i], o.b[n], acc[i][n], 0, 0, 0);
    }
  }
}

template <int AM, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_nt(const GemmArgs g) {
  using G = Geo<AM>;
  // two stages, each the tile(s) of A followed by the tile of B
  __shared__ __align__(16) uint16_t lds[2 * G::kStage];

  int Mrows = g.M;
  if (g.n_rows_dev) {
    const int nd = g.n_rows_dev[0];
    Mrows = nd < Mrows ? nd : Mrows;
  }
  const int tile_m = blockIdx.y;
  if (tile_m * BM >= Mrows) return;  // uniform
  // the right-hand factor of this workgroup: the only one, or the segment its column tile falls in
  int tile_n = blockIdx.x, N = g.N, epi = EPI;
  const void* Bmat = g.B;
  void* Dmat = g.D;
  int64_t ldb = g.ldb, ldd = g.ldd;
  if constexpr (EPI == EPI_MULTI) {
    int si = 0;
#pragma unroll
    for (int q = 1; q < kMaxGemmSegs; ++q)
      if (q < g.nseg && (int)blockIdx.x >= g.seg[q].tile_begin) si = q;
    const GemmSeg& sg = g.seg[si];
    tile_n = blockIdx.x - sg.tile_begin;
    N = sg.N; epi = sg.epi; Bmat = sg.B; Dmat = sg.D; ldb = sg.ldb; ldd = sg.ldd;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lc = lane & 31, lh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int ES = AM ? 4 : 2;  // bytes per element of A

  // k-tiles of this split
  const int nk = g.K / G::BKT;  // K is a multiple of 64
  const int splits = g.splits > 1 ? g.splits : 1;
  const int kt0 = (int)(((int64_t)nk * blockIdx.z) / splits), kt1 = (int)(((int64_t)nk * (blockIdx.z + 1)) / splits);

  // staging pointers: a thread's unit u is tile row tid / CPR + RPP u, 8 columns at 8 (tid % CPR); rows past the
  // end repeat the last one (their results are not stored)
  const char* ap[G::NU];
  const char* bp[G::NU];
#pragma unroll
  for (int u = 0; u < G::NU; ++u) {
    int grow = tile_m * BM + (tid / G::CPR) + G::RPP * u;
    grow = grow < Mrows ? grow : Mrows - 1;
    if (g.row_idx) grow = g.row_idx[grow];
    ap[u] = reinterpret_cast<const char*>(g.A) + ((int64_t)grow * g.lda + 8 * (tid % G::CPR)) * ES;
  }
#pragma unroll
  for (int u = 0; u < G::NU; ++u) {
    int grow = tile_n * BN + (tid / G::CPR) + G::RPP * u;
    grow = grow < N ? grow : N - 1;
    bp[u] = reinterpret_cast<const char*>(Bmat) + ((int64_t)grow * ldb + 8 * (tid % G::CPR)) * 2;
  }

  f32x16 acc[kAF][kBF];
#pragma unroll
  for (int i = 0; i < kAF; ++i)
#pragma unroll
    for (int j = 0; j < kBF; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (kt0 < kt1) {
    // Tile t is multiplied out of stage t & 1 while tile t + 1 (in registers since the tile before) is written
    // to the other stage, a unit per MFMA step, and each unit's registers are asked for tile t + 2 at once.
    // One barrier per tile, before the last step: by then every wave has written its share of the next stage
    // and has the last step's operands in registers, so the first operands of the next tile are read behind
    // the last step's MFMAs.  Past the range the last tile is requested (and staged) again and never used.
    Stage<AM> st;
    issue<AM>(st, ap, bp, kt0);
    commit<AM>(st, lds, tid);
    issue<AM>(st, ap, bp, kt0 + 1 < kt1 ? kt0 + 1 : kt0);
    __syncthreads();
    Ops<AM> o[2];
    read_ops<AM>(o[0], lds, wm, wn, lc, lh, 0);
    for (int kt = kt0; kt < kt1; ++kt) {
      uint16_t* cur = lds + ((kt - kt0) & 1) * G::kStage;
      uint16_t* nxt = lds + (((kt - kt0) & 1) ^ 1) * G::kStage;
      const int kt2 = kt + 2 < kt1 ? kt + 2 : kt1 - 1;
#pragma unroll
      for (int j = 0; j < G::KS; ++j) {
        if (j + 1 < G::KS) {
          read_ops<AM>(o[(j + 1) & 1], cur, wm, wn, lc, lh, j + 1);
        } else {
          __syncthreads();
          read_ops<AM>(o[(j + 1) & 1], nxt, wm, wn, lc, lh, 0);
        }
        mma<AM>(o[j & 1], acc);
        if (j + 1 < G::KS) {
          // a unit behind every step but the last two, which share the step before the barrier
          commit_unit<AM>(st, j, nxt, tid);
          issue_unit<AM>(st, j, ap, bp, kt2);
          if (j + 2 == G::KS) {
            commit_unit<AM>(st, j + 1, nxt, tid);
            issue_unit<AM>(st, j + 1, ap, bp, kt2);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // ---- epilogue --------------------------------------------------------------------------------------
  // Element v of lane l of fragment (i, n) is row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of the
  // fragment.  The accumulators go through LDS eight rows at a time (a private strip per wave), so that
  // what touches memory is row-contiguous: a lane then owns four consecutive columns of a row.
  __syncthreads();  // the operand tiles are no longer read
  constexpr int kSR = 8, kSLD = WTN + 4;  // strip rows, padded strip stride (floats)
  float* strip = reinterpret_cast<float*>(lds) + wave * (kSR * kSLD);
  const bool partial = g.splits > 1;
  float* const pdst = partial ? g.part + (int64_t)blockIdx.z * g.M * N : nullptr;
  const int er = lane >> 5, ec = 4 * (lane & 31);  // row parity and first column of the lane's reads
#pragma unroll
  for (int c = 0; c < WTM / kSR; ++c) {
    // strip c: rows 8 c .. 8 c + 7 of the wave tile = fragment c / 4, accumulator elements 4 (c % 4) .. + 3
    const int i = c >> 2, vbase = 4 * (c & 3);
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
      const int rl = 4 * lh + vv;
#pragma unroll
      for (int n = 0; n < kBF; ++n) strip[rl * kSLD + 32 * n + lc] = acc[i][n][vbase + vv];
    }
    // The strip is private to the wave and a wave's LDS operations execute in order, so no workgroup barrier is
    // needed (one would also wait for the stores of the round before to complete); the fence only keeps the
    // compiler from moving a lane's reads above the other lanes' writes.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int col = tile_n * BN + WTN * wn + ec;
    float4 val[kSR / 2];
    int row[kSR / 2];
#pragma unroll
    for (int q = 0; q < kSR / 2; ++q) {
      row[q] = tile_m * BM + WTM * wm + kSR * c + 2 * q + er;
      val[q] = *reinterpret_cast<const float4*>(&strip[(2 * q + er) * kSLD + ec]);
    }
    if (partial) {
#pragma unroll
      for (int q = 0; q < kSR / 2; ++q)
        if (row[q] < Mrows && col < N)  // N is a multiple of 4 here (checked on the host)
          *reinterpret_cast<float4*>(pdst + (int64_t)row[q] * N + col) = val[q];
    } else if (EPI == EPI_RESIDUAL || (EPI == EPI_MULTI && epi == EPI_RESIDUAL)) {
      // r = x - acc; R written; per row the sums of r^2 and x^2 over this wave's 128 columns
      float4 x[kSR / 2];
#pragma unroll
      for (int q = 0; q < kSR / 2; ++q) {
        x[q] = float4{0.f, 0.f, 0.f, 0.f};
        if (row[q] < Mrows && col < N) {
          if (g.xdtype == GSI_F32) {
            x[q] = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g.X) + (int64_t)row[q] * g.ldx + col);
          } else {
            const uint2 xb = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(g.X) + (int64_t)row[q] * g.ldx + col);
            x[q] = float4{bf16_lo(xb.x), bf16_hi(xb.x), bf16_lo(xb.y), bf16_hi(xb.y)};
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kSR / 2; ++q) {
        const bool live = row[q] < Mrows && col < N;
        const float4 r = float4{x[q].x - val[q].x, x[q].y - val[q].y, x[q].z - val[q].z, x[q].w - val[q].w};
        float sr = 0.f, sx = 0.f;
        if (live) {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(Dmat) + (int64_t)row[q] * ldd + col) = r;
          sr = fmaf(r.x, r.x, fmaf(r.y, r.y, fmaf(r.z, r.z, r.w * r.w)));
          sx = fmaf(x[q].x, x[q].x, fmaf(x[q].y, x[q].y, fmaf(x[q].z, x[q].z, x[q].w * x[q].w)));
        }
        sr = group_sum_rt(sr, 32);
        sx = group_sum_rt(sx, 32);
        if ((lane & 31) == 0 && row[q] < Mrows && tile_n * BN + WTN * wn < N) {
          float* pn = g.part_n + ((int64_t)(tile_n * (BN / WTN) + wn) * g.part_tokens + row[q]) * 2;
          pn[0] = sr;
          pn[1] = sx;
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < kSR / 2; ++q) {
        if (row[q] < Mrows && col < N) {
          if constexpr (EPI == EPI_STORE_BF16) {
            uint2 o;
            o.x = (uint32_t)f32_to_bf16_bits(val[q].x) | ((uint32_t)f32_to_bf16_bits(val[q].y) << 16);
            o.y = (uint32_t)f32_to_bf16_bits(val[q].z) | ((uint32_t)f32_to_bf16_bits(val[q].w) << 16);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(Dmat) + (int64_t)row[q] * ldd + col) = o;
          } else if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_MULTI) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(Dmat) + (int64_t)row[q] * ldd + col) = val[q];
          } else {  // scatter: one workgroup owns an output element, so the update is ordered
            const int drow = g.row_idx ? g.row_idx[row[q]] : row[q];
            float4* dp = reinterpret_cast<float4*>(reinterpret_cast<float*>(Dmat) + (int64_t)drow * ldd + col);
            if constexpr (EPI == EPI_SCATTER_STORE) {
              *dp = val[q];
            } else {
              const float4 o = *dp;
              *dp = float4{o.x + val[q].x, o.y + val[q].y, o.z + val[q].z, o.w + val[q].w};
            }
          }
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the strip is rewritten by the next round
    __builtin_amdgcn_wave_barrier();
  }
}

// Adds the partial sums of a split contraction in split order and applies the epilogue (store / scatter-add).
// A thread owns four consecutive columns; the blocks stride over the live rows (a device-side count for the
// scatter-add product), so the launch does not grow with rows that did not fire.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_finish(const GemmArgs g) {
  int Mrows = g.M;
  if (g.n_rows_dev) {
    const int nd = g.n_rows_dev[0];
    Mrows = nd < Mrows ? nd : Mrows;
  }
  const int n4 = g.N >> 2;
  const int64_t total = (int64_t)Mrows * n4, stride = (int64_t)g.M * g.N;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int row = (int)(e / n4), col = 4 * (int)(e - (int64_t)row * n4);
    const float* src = g.part + (int64_t)row * g.N + col;
    float4 s = float4{0.f, 0.f, 0.f, 0.f};
    for (int z0 = 0; z0 < g.splits; z0 += 8) {
      float4 q[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) q[u] = *reinterpret_cast<const float4*>(src + (int64_t)min(z0 + u, g.splits - 1) * stride);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (z0 + u < g.splits) { s.x += q[u].x; s.y += q[u].y; s.z += q[u].z; s.w += q[u].w; }
    }
    if constexpr (EPI == EPI_STORE_BF16) {
      uint2 o;
      o.x = (uint32_t)f32_to_bf16_bits(s.x) | ((uint32_t)f32_to_bf16_bits(s.y) << 16);
      o.y = (uint32_t)f32_to_bf16_bits(s.z) | ((uint32_t)f32_to_bf16_bits(s.w) << 16);
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.D) + (int64_t)row * g.ldd + col) = o;
    } else if constexpr (EPI == EPI_STORE_F32) {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.D) + (int64_t)row * g.ldd + col) = s;
    } else {
      const int drow = g.row_idx ? g.row_idx[row] : row;
      float4* dp = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.D) + (int64_t)drow * g.ldd + col);
      if constexpr (EPI == EPI_SCATTER_STORE) {
        *dp = s;
      } else {
        const float4 o = *dp;
        *dp = float4{o.x + s.x, o.y + s.y, o.z + s.z, o.w + s.w};
      }
    }
  }
}

// Ut[j][i] = U[i][j] for a bf16 matrix U[rows, cols]; 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose_bf16(const uint16_t* __restrict__ U, uint16_t* __restrict__ Ut,
                                                      int rows, int cols) {
  __shared__ uint16_t tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  for (int y = ty; y < 32; y += 8) {
    const int r = r0 + y, c = c0 + tx;
    tile[y][tx] = (r < rows && c < cols) ? U[(int64_t)r * cols + c] : (uint16_t)0;
  }
  __syncthreads();
  for (int y = ty; y < 32; y += 8) {
    const int c = c0 + y, r = r0 + tx;
    if (r < rows && c < cols) Ut[(int64_t)c * rows + r] = tile[tx][y];
  }
}

template <int AM>
hipError_t launch_epi(const GemmArgs& g, int epi, hipStream_t s) {
  const int splits = g.splits > 1 ? g.splits : 1;
  dim3 grid((unsigned)ceil_div(g.N, BN), (unsigned)ceil_div(g.M, BM), (unsigned)splits);
  if (epi == EPI_MULTI) {
    grid.x = (unsigned)(g.seg[g.nseg - 1].tile_begin + ceil_div(g.seg[g.nseg - 1].N, BN));
    gemm_nt<AM, EPI_MULTI><<<grid, kThreads, 0, s>>>(g);
    return hipGetLastError();
  }
  switch (epi) {
    case EPI_STORE_BF16: gemm_nt<AM, EPI_STORE_BF16><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_STORE_F32: gemm_nt<AM, EPI_STORE_F32><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_RESIDUAL: gemm_nt<AM, EPI_RESIDUAL><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_SCATTER_STORE: gemm_nt<AM, EPI_SCATTER_STORE><<<grid, kThreads, 0, s>>>(g); break;
    default: gemm_nt<AM, EPI_SCATTER_ADD><<<grid, kThreads, 0, s>>>(g); break;
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (splits > 1) {
    const unsigned fb = (unsigned)std::min<int64_t>(ceil_div((int64_t)g.M * (g.N / 4), 256), 4096);
    switch (epi) {
      case EPI_STORE_BF16: splitk_finish<EPI_STORE_BF16><<<fb, 256, 0, s>>>(g); break;
      case EPI_STORE_F32: splitk_finish<EPI_STORE_F32><<<fb, 256, 0, s>>>(g); break;
      case EPI_SCATTER_STORE: splitk_finish<EPI_SCATTER_STORE><<<fb, 256, 0, s>>>(g); break;
      default: splitk_finish<EPI_SCATTER_ADD><<<fb, 256, 0, s>>>(g); break;
    }
  }
  return hipGetLastError();
}

}  // namespace

int mfma_splits(int64_t M, int64_t N, int64_t K, int epi) {
  if (epi == EPI_RESIDUAL) return 1;
  // the scatter-add product runs over the fired rows only (a device-side count): size it for a quarter of them
  const int64_t m_eff = (epi == EPI_SCATTER_ADD || epi == EPI_SCATTER_STORE) ? std::max<int64_t>(BM, M / 4) : M;
  const int64_t tiles = ceil_div(m_eff, BM) * ceil_div(N, BN);
  const int64_t nk = ceil_div(K, BK);
  int s = 1;
  while (s < 8 && tiles * s < 256 && nk / (s * 2) >= 4) s *= 2;  // fill the chip, keep >= 4 k-tiles per split
  return s;
}

size_t mfma_part_bytes(int64_t M, int64_t N, int64_t K, int epi) {
  const int s = mfma_splits(M, N, K, epi);
  return s > 1 ? align_up((size_t)s * M * N * sizeof(float), 256) : 0;
}

hipError_t mfma_gemm_nt(const GemmArgs& g0, int epi, hipStream_t s) {
  if (g0.M <= 0 || (epi != EPI_MULTI && g0.N <= 0)) return hipSuccess;
  GemmArgs g = g0;
  if (epi == EPI_MULTI) {  // several right-hand factors side by side, never split
    if (g.nseg < 1 || g.nseg > kMaxGemmSegs) return hipErrorInvalidValue;
    int t = 0;
    for (int i = 0; i < g.nseg; ++i) {
      g.seg[i].tile_begin = t;
      t += (int)ceil_div(g.seg[i].N, BN);
    }
    g.N = g.seg[0].N;
    g.splits = 1;
    g.part = nullptr;
    if (g.a_f32 == 2) return launch_epi<2>(g, epi, s);
    return g.a_f32 ? launch_epi<1>(g, epi, s) : launch_epi<0>(g, epi, s);
  }
  g.splits = g.part ? mfma_splits(g.M, g.N, g.K, epi) : 1;
  if (g.a_f32 == 2) return launch_epi<2>(g, epi, s);
  return g.a_f32 ? launch_epi<1>(g, epi, s) : launch_epi<0>(g, epi, s);
}

hipError_t mfma_transpose_bf16(const void* U, void* Ut, int rows, int cols, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(cols, 32), (unsigned)ceil_div(rows, 32));
  transpose_bf16<<<grid, 256, 0, s>>>(reinterpret_cast<const uint16_t*>(U), reinterpret_cast<uint16_t*>(Ut), rows, cols);
  return hipGetLastError();
}

int mfma_res_tiles(int64_t d) { return (int)ceil_div(d, WTN); }

}  // namespace gsi
