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
// Workgroup tile 256 x 128 x 64, four waves stacked along M, each wave 64 x 128 as 2 x 4
// v_mfma_f32_32x32x16_bf16 tiles.  A wave is the only reader of its 64 rows of A, so A never goes through
// LDS: a lane loads its MFMA operands straight from memory.  The 64 columns of a k-tile are dealt so that
// the lane half l/32 owns 32 consecutive columns and step j of the tile takes their j-th group of eight
// (any order of the contraction index is as good as another as long as both operands agree), which makes a
// lane's four loads of a tile one contiguous 64-byte run and a row's two halves one 128-byte line.  The
// B tile (128 x 64) is shared by the four waves through LDS (row stride padded to 144 bytes: conflict-free
// 128-bit reads), double-buffered, loaded a tile ahead through registers like the A operands.
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

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int LDB = BK + 8;  // padded LDS row stride of the B tile, bf16 elements (144 bytes)
constexpr int kThreads = 256;
constexpr int kAF = 2, kBF = 4, kKS = BK / 16;  // A fragments, B fragments per wave; MFMA steps per k-tile

// AM: how the A operand is stored and fed: 0 bf16; 1 fp32, split into bf16 head + tail (two MFMA passes);
// 2 fp32, rounded once to bf16 (one pass)
template <int AM>
struct AOps {
  uint4 r[kAF][kKS][AM ? 2 : 1];
};

__device__ __forceinline__ void split_f32x8(const uint4& a, const uint4& b, bf16x8& hi, bf16x8& lo) {
  const float x[8] = {__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w),
                      __uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const __bf16 h = (__bf16)x[e];
    hi[e] = h;
    lo[e] = (__bf16)(x[e] - __uint_as_float((uint32_t)__builtin_bit_cast(uint16_t, h) << 16));
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a native vector: loads and stores of it are
                                                              // instructions, not aggregate copies
__device__ __forceinline__ bf16x8 round_f32x8(const uint4& a, const uint4& b) {
  const float x[8] = {__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w),
                      __uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[e];
  return r;
}

struct BOps {
  u32x4 r[4];
};

struct Tiles {
  int kt1;       // end of this split's k-tiles
  int lc, lh;    // lane % 32, lane / 32
};

// A operands of k-tile kt for the lane's rows.  Past the split's range the last tile is repeated (and not
// consumed).
template <int AM>
__device__ __forceinline__ void load_a(AOps<AM>& a, const char* const (&aptr)[kAF], int kt, const Tiles& t) {
  constexpr int ES = AM ? 4 : 2;
  const int ktc = kt < t.kt1 ? kt : t.kt1 - 1;
  const int half = t.lh;
#pragma unroll
  for (int i = 0; i < kAF; ++i)
#pragma unroll
    for (int j = 0; j < kKS; ++j) {
      const char* p = aptr[i] + ((int64_t)ktc * BK + 32 * half + 8 * j) * ES;
      a.r[i][j][0] = *reinterpret_cast<const uint4*>(p);
      if constexpr (AM != 0) a.r[i][j][1] = *reinterpret_cast<const uint4*>(p + 16);
    }
}

__device__ __forceinline__ void load_b(BOps& b, const char* const (&bptr)[4], const int (&bch)[4], int kt,
                                       const Tiles& t) {
  const int ktc = kt < t.kt1 ? kt : t.kt1 - 1;
#pragma unroll
  for (int u = 0; u < 4; ++u) b.r[u] = *reinterpret_cast<const u32x4*>(bptr[u] + ((int64_t)ktc * BK + 8 * bch[u]) * 2);
}

__device__ __forceinline__ void store_b(const BOps& b, uint16_t (*Bs)[LDB], const int (&brow)[4], const int (&bch)[4]) {
#pragma unroll
  for (int u = 0; u < 4; ++u) *reinterpret_cast<u32x4*>(&Bs[brow[u]][8 * bch[u]]) = b.r[u];
}

template <int AM>
__device__ __forceinline__ void compute(const AOps<AM>& a, const uint16_t (*Bs)[LDB], const Tiles& t,
                                        f32x16 (&acc)[kAF][kBF]) {
#pragma unroll
  for (int j = 0; j < kKS; ++j) {
    bf16x8 b[kBF];
#pragma unroll
    for (int n = 0; n < kBF; ++n) b[n] = *reinterpret_cast<const bf16x8*>(&Bs[32 * n + t.lc][32 * t.lh + 8 * j]);
#pragma unroll
    for (int i = 0; i < kAF; ++i) {
      if constexpr (AM == 2) {
        const bf16x8 av = round_f32x8(a.r[i][j][0], a.r[i][j][1]);
#pragma unroll
        for (int n = 0; n < kBF; ++n) acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b[n], acc[i][n], 0, 0, 0);
      } else if constexpr (AM == 1) {
        bf16x8 hi, lo;
        split_f32x8(a.r[i][j][0], a.r[i][j][1], hi, lo);
#pragma unroll
        for (int n = 0; n < kBF; ++n) {
          acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, b[n], acc[i][n], 0, 0, 0);
          acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, b[n], acc[i][n], 0, 0, 0);
        }
      } else {
        const bf16x8 av = __builtin_bit_cast(bf16x8, a.r[i][j][0]);
#pragma unroll
        for (int n = 0; n < kBF; ++n) acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b[n], acc[i][n], 0, 0, 0);
      }
    }
  }
}

template <int AM, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_nt(const GemmArgs g) {
  __shared__ __align__(16) uint16_t Bs[2][BN][LDB];

  int Mrows = g.M;
  if (g.n_rows_dev) {
    const int nd = g.n_rows_dev[0];
    Mrows = nd < Mrows ? nd : Mrows;
  }
  const int tile_m = blockIdx.y, tile_n = blockIdx.x;
  if (tile_m * BM >= Mrows) return;  // uniform
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lc = lane & 31, lh = lane >> 5;
  constexpr int ES = AM ? 4 : 2;  // bytes per element of A

  // k-tiles of this split
  const int nk = g.K / BK;  // K is a multiple of 64
  const int splits = g.splits > 1 ? g.splits : 1;
  const int kt0 = (int)(((int64_t)nk * blockIdx.z) / splits), kt1 = (int)(((int64_t)nk * (blockIdx.z + 1)) / splits);

  // ---- A: per-lane row pointers (rows past the end repeat the last one and are not stored) -----------
  const char* aptr[kAF];
#pragma unroll
  for (int i = 0; i < kAF; ++i) {
    int grow = tile_m * BM + wave * 64 + i * 32 + lc;
    grow = grow < Mrows ? grow : Mrows - 1;
    if (g.row_idx) grow = g.row_idx[grow];
    aptr[i] = reinterpret_cast<const char*>(g.A) + (int64_t)grow * g.lda * ES;
  }
  // ---- B: 128 rows x 8 chunks of 16 bytes per k-tile, four chunks per thread ---------------------------
  const char* bptr[4];
  int brow[4], bch[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int q = tid + kThreads * u;
    brow[u] = q >> 3;
    bch[u] = q & 7;
    int grow = tile_n * BN + brow[u];
    grow = grow < g.N ? grow : g.N - 1;
    bptr[u] = reinterpret_cast<const char*>(g.B) + (int64_t)grow * g.ldb * 2;
  }

  f32x16 acc[kAF][kBF];
#pragma unroll
  for (int i = 0; i < kAF; ++i)
#pragma unroll
    for (int j = 0; j < kBF; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (kt0 < kt1) {
    const Tiles tl{kt1, lc, lh};
    AOps<AM> a0, a1;
    BOps b;
    load_a<AM>(a0, aptr, kt0, tl);
    load_b(b, bptr, bch, kt0, tl);
    store_b(b, Bs[0], brow, bch);
    __syncthreads();
    for (int kt = kt0; kt < kt1; kt += 2) {
      // tile kt from (a0, buffer 0); tile kt+1 from (a1, buffer 1)
      __builtin_amdgcn_sched_barrier(0);
      load_a<AM>(a1, aptr, kt + 1, tl);
      load_b(b, bptr, bch, kt + 1, tl);
      __builtin_amdgcn_sched_barrier(0);
      compute<AM>(a0, Bs[0], tl, acc);
      store_b(b, Bs[1], brow, bch);
      __syncthreads();
      if (kt + 1 < kt1) {  // uniform
        __builtin_amdgcn_sched_barrier(0);
        load_a<AM>(a0, aptr, kt + 2, tl);
        load_b(b, bptr, bch, kt + 2, tl);
        __builtin_amdgcn_sched_barrier(0);
        compute<AM>(a1, Bs[1], tl, acc);
        store_b(b, Bs[0], brow, bch);
        __syncthreads();
      }
    }
  }

  // ---- epilogue: element v of lane l of tile (i, n) is row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 ----
  const int rsub = lh * 4;
  const int row_base = tile_m * BM + wave * 64, col_base = tile_n * BN;
  if (g.splits > 1) {  // partial sums of this split; the finishing kernel applies the epilogue
    float* part = g.part + (int64_t)blockIdx.z * g.M * g.N;
#pragma unroll
    for (int i = 0; i < kAF; ++i)
#pragma unroll
      for (int n = 0; n < kBF; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v / 4) + rsub + (v % 4), col = col_base + 32 * n + lc;
          if (row < Mrows && col < g.N) part[(int64_t)row * g.N + col] = acc[i][n][v];
        }
    return;
  }
  if constexpr (EPI == EPI_RESIDUAL) {
    // r = x - acc; R written; per row the sums of r^2 and x^2 over this workgroup's 128 columns (the wave
    // holds all of them for its rows: four fragments in the lane, 32 lanes per row)
#pragma unroll
    for (int i = 0; i < kAF; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row_base + i * 32 + 8 * (v / 4) + rsub + (v % 4);
        float sr = 0.f, sx = 0.f;
#pragma unroll
        for (int n = 0; n < kBF; ++n) {
          const int col = col_base + 32 * n + lc;
          if (row < Mrows && col < g.N) {
            const float x = load_act(g.X, g.xdtype, (int64_t)row * g.ldx + col);
            const float r = x - acc[i][n][v];
            reinterpret_cast<float*>(g.D)[(int64_t)row * g.ldd + col] = r;
            sr = fmaf(r, r, sr);
            sx = fmaf(x, x, sx);
          }
        }
        sr = group_sum_rt(sr, 32);
        sx = group_sum_rt(sx, 32);
        if (lc == 0 && row < Mrows) {
          float* pn = g.part_n + ((int64_t)tile_n * g.part_tokens + row) * 2;
          pn[0] = sr;
          pn[1] = sx;
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < kAF; ++i)
#pragma unroll
      for (int n = 0; n < kBF; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v / 4) + rsub + (v % 4), col = col_base + 32 * n + lc;
          if (row < Mrows && col < g.N) {
            const float val = acc[i][n][v];
            if constexpr (EPI == EPI_STORE_BF16) {
              reinterpret_cast<uint16_t*>(g.D)[(int64_t)row * g.ldd + col] = f32_to_bf16_bits(val);
            } else if constexpr (EPI == EPI_STORE_F32) {
              reinterpret_cast<float*>(g.D)[(int64_t)row * g.ldd + col] = val;
            } else {  // EPI_SCATTER_ADD: one workgroup owns an output element, so the update is ordered
              const int drow = g.row_idx ? g.row_idx[row] : row;
              float* dp = reinterpret_cast<float*>(g.D) + (int64_t)drow * g.ldd + col;
              *dp += val;
            }
          }
        }
  }
}

// Adds the partial sums of a split contraction in split order and applies the epilogue (store / scatter-add).
template <int EPI>
__global__ __launch_bounds__(256) void splitk_finish(const GemmArgs g) {
  int Mrows = g.M;
  if (g.n_rows_dev) {
    const int nd = g.n_rows_dev[0];
    Mrows = nd < Mrows ? nd : Mrows;
  }
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)Mrows * g.N) return;
  const int row = (int)(e / g.N), col = (int)(e - (int64_t)row * g.N);
  const int64_t stride = (int64_t)g.M * g.N;
  float q[8];
  float s = 0.f;
  for (int z0 = 0; z0 < g.splits; z0 += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = g.part[(int64_t)min(z0 + u, g.splits - 1) * stride + e];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (z0 + u < g.splits) s += q[u];
  }
  if constexpr (EPI == EPI_STORE_BF16) {
    reinterpret_cast<uint16_t*>(g.D)[(int64_t)row * g.ldd + col] = f32_to_bf16_bits(s);
  } else if constexpr (EPI == EPI_STORE_F32) {
    reinterpret_cast<float*>(g.D)[(int64_t)row * g.ldd + col] = s;
  } else {
    const int drow = g.row_idx ? g.row_idx[row] : row;
    reinterpret_cast<float*>(g.D)[(int64_t)drow * g.ldd + col] += s;
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
  switch (epi) {
    case EPI_STORE_BF16: gemm_nt<AM, EPI_STORE_BF16><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_STORE_F32: gemm_nt<AM, EPI_STORE_F32><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_RESIDUAL: gemm_nt<AM, EPI_RESIDUAL><<<grid, kThreads, 0, s>>>(g); break;
    default: gemm_nt<AM, EPI_SCATTER_ADD><<<grid, kThreads, 0, s>>>(g); break;
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (splits > 1) {
    const unsigned fb = (unsigned)ceil_div((int64_t)g.M * g.N, 256);
    switch (epi) {
      case EPI_STORE_BF16: splitk_finish<EPI_STORE_BF16><<<fb, 256, 0, s>>>(g); break;
      case EPI_STORE_F32: splitk_finish<EPI_STORE_F32><<<fb, 256, 0, s>>>(g); break;
      default: splitk_finish<EPI_SCATTER_ADD><<<fb, 256, 0, s>>>(g); break;
    }
  }
  return hipGetLastError();
}

}  // namespace

int mfma_splits(int64_t M, int64_t N, int64_t K, int epi) {
  if (epi == EPI_RESIDUAL) return 1;
  // the scatter-add product runs over the fired rows only (a device-side count): size it for a quarter of them
  const int64_t m_eff = epi == EPI_SCATTER_ADD ? std::max<int64_t>(BM, M / 4) : M;
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
  if (g0.M <= 0 || g0.N <= 0) return hipSuccess;
  GemmArgs g = g0;
  g.splits = g.part ? mfma_splits(g.M, g.N, g.K, epi) : 1;
  if (g.a_f32 == 2) return launch_epi<2>(g, epi, s);
  return g.a_f32 ? launch_epi<1>(g, epi, s) : launch_epi<0>(g, epi, s);
}

hipError_t mfma_transpose_bf16(const void* U, void* Ut, int rows, int cols, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(cols, 32), (unsigned)ceil_div(rows, 32));
  transpose_bf16<<<grid, 256, 0, s>>>(reinterpret_cast<const uint16_t*>(U), reinterpret_cast<uint16_t*>(Ut), rows, cols);
  return hipGetLastError();
}

int mfma_res_tiles(int64_t d) { return (int)ceil_div(d, BN); }

}  // namespace gsi
