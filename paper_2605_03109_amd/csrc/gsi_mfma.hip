// Dense contractions of libgsi on the matrix cores (gfx950 MFMA, bf16 inputs, fp32 accumulation):
// the one-time image build M = W U (Eq. (exact), Section 4 "Storage") and the prefill-sized batched
// path (hundreds of tokens per call), where the work really is a GEMM:
//     C = X U            R = X - C U^T  (+ per-token partial norms)          Algorithm 1, lines 1-3
//     Y = C M^T          Y[fired] += R[fired] W^T                            Eq. (exact)
//
// One kernel, D = A B^T with both operands K-contiguous ("NT"): A[M,K], B[N,K] row-major.  A is bf16,
// or fp32 split on the fly into a bf16 head and a bf16 tail (two MFMA passes) so that an fp32 operand
// on the main term is not rounded to 8 bits (the bf16 image already uses most of the 2e-3 budget).
// Workgroup tile 128 x 128 x 32, four waves in a 2 x 2 arrangement, each wave 64 x 64 as 2 x 2
// v_mfma_f32_32x32x16_bf16 tiles; operands staged through LDS (row stride padded to 80 bytes), global
// loads of the next k-tile in flight during the MFMAs of the current one.
// Operands that are N-contiguous in memory (U as the right factor of W U and X U) are transposed
// once into the workspace.
#include "gsi_device.h"
#include "gsi_mfma.h"

namespace gsi {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 128, BN = 128, BK = 32, LDK = 40;  // LDK: padded LDS row stride in bf16 elements
constexpr int kThreads = 256;

union Frag {
  uint4 u;
  bf16x8 v;
};

template <bool AF32, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_nt(const GemmArgs g) {
  __shared__ __align__(16) uint16_t As[2][AF32 ? 2 : 1][BM][LDK];
  __shared__ __align__(16) uint16_t Bs[2][BN][LDK];
  __shared__ float red[2][BM][2];  // residual epilogue: per wave column, per row, (|r|^2, |x|^2)

  int Mrows = g.M;
  if (g.n_rows_dev) {
    const int nd = g.n_rows_dev[0];
    Mrows = nd < Mrows ? nd : Mrows;
  }
  const int tile_m = blockIdx.y, tile_n = blockIdx.x;
  if (tile_m * BM >= Mrows) return;  // uniform
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // ---- global -> register staging -----------------------------------------------------------------
  // bf16 operand: 128 rows x 64 bytes = 512 chunks of 16 bytes, two per thread
  // fp32 operand: 128 rows x 128 bytes = 1024 chunks of 16 bytes, four per thread
  constexpr int NA = AF32 ? 4 : 2;
  const char* aptr[NA];
  int arow_l[NA], akc[NA];
#pragma unroll
  for (int u = 0; u < NA; ++u) {
    const int q = tid + kThreads * u;
    const int row = AF32 ? (q >> 3) : (q >> 2);
    const int kc = AF32 ? (q & 7) : (q & 3);
    int grow = tile_m * BM + row;
    grow = grow < Mrows ? grow : Mrows - 1;
    if (g.row_idx) grow = g.row_idx[grow];
    arow_l[u] = row;
    akc[u] = kc;
    aptr[u] = reinterpret_cast<const char*>(g.A) + ((int64_t)grow * g.lda) * (AF32 ? 4 : 2) + kc * 16;
  }
  const char* bptr[2];
  int brow_l[2], bkc[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int q = tid + kThreads * u;
    const int row = q >> 2, kc = q & 3;
    int grow = tile_n * BN + row;
    grow = grow < g.N ? grow : g.N - 1;
    brow_l[u] = row;
    bkc[u] = kc;
    bptr[u] = reinterpret_cast<const char*>(g.B) + ((int64_t)grow * g.ldb) * 2 + kc * 16;
  }
  uint4 ra[NA], rb[2];
  auto gload = [&](int kt) {
    const int64_t koffA = (int64_t)kt * BK * (AF32 ? 4 : 2), koffB = (int64_t)kt * BK * 2;
#pragma unroll
    for (int u = 0; u < NA; ++u) ra[u] = *reinterpret_cast<const uint4*>(aptr[u] + koffA);
#pragma unroll
    for (int u = 0; u < 2; ++u) rb[u] = *reinterpret_cast<const uint4*>(bptr[u] + koffB);
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < NA; ++u) {
      if constexpr (AF32) {
        const float f[4] = {__uint_as_float(ra[u].x), __uint_as_float(ra[u].y), __uint_as_float(ra[u].z),
                            __uint_as_float(ra[u].w)};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          hi[e] = f32_to_bf16_bits(f[e]);
          lo[e] = f32_to_bf16_bits(f[e] - bf16_bits_to_f32(hi[e]));
        }
        uint2 h, l;
        h.x = hi[0] | ((uint32_t)hi[1] << 16); h.y = hi[2] | ((uint32_t)hi[3] << 16);
        l.x = lo[0] | ((uint32_t)lo[1] << 16); l.y = lo[2] | ((uint32_t)lo[3] << 16);
        *reinterpret_cast<uint2*>(&As[buf][0][arow_l[u]][akc[u] * 4]) = h;
        *reinterpret_cast<uint2*>(&As[buf][AF32 ? 1 : 0][arow_l[u]][akc[u] * 4]) = l;
      } else {
        *reinterpret_cast<uint4*>(&As[buf][0][arow_l[u]][akc[u] * 8]) = ra[u];
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) *reinterpret_cast<uint4*>(&Bs[buf][brow_l[u]][bkc[u] * 8]) = rb[u];
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = g.K / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      Frag a[2], al[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i].u = *reinterpret_cast<const uint4*>(&As[buf][0][wm * 64 + i * 32 + fr][ks * 16 + fk]);
        if constexpr (AF32) al[i].u = *reinterpret_cast<const uint4*>(&As[buf][AF32 ? 1 : 0][wm * 64 + i * 32 + fr][ks * 16 + fk]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j].u = *reinterpret_cast<const uint4*>(&Bs[buf][wn * 64 + j * 32 + fr][ks * 16 + fk]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
          if constexpr (AF32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i].v, b[j].v, acc[i][j], 0, 0, 0);
        }
    }
    if (kt + 1 < nk) lstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: element v of lane l of tile (i, j) is row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 ----
  const int col_l = lane & 31, rsub = (lane >> 5) * 4;
  if constexpr (EPI == EPI_RESIDUAL) {
    // r = x - acc; R written; per row the sums of r^2 and x^2 over this workgroup's 128 columns
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rl = wm * 64 + i * 32 + 8 * (v / 4) + rsub + (v % 4);
        const int row = tile_m * BM + rl;
        float sr = 0.f, sx = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int col = tile_n * BN + wn * 64 + j * 32 + col_l;
          if (row < Mrows && col < g.N) {
            const float x = load_act(g.X, g.xdtype, (int64_t)row * g.ldx + col);
            const float r = x - acc[i][j][v];
            reinterpret_cast<float*>(g.D)[(int64_t)row * g.ldd + col] = r;
            sr = fmaf(r, r, sr);
            sx = fmaf(x, x, sx);
          }
        }
        sr = group_sum_rt(sr, 32);
        sx = group_sum_rt(sx, 32);
        if (col_l == 0) {
          red[wn][rl][0] = sr;
          red[wn][rl][1] = sx;
        }
      }
    }
    __syncthreads();
    if (tid < BM) {
      const int row = tile_m * BM + tid;
      if (row < Mrows) {
        float* pn = g.part_n + ((int64_t)tile_n * g.part_tokens + row) * 2;
        pn[0] = red[0][tid][0] + red[1][tid][0];
        pn[1] = red[0][tid][1] + red[1][tid][1];
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = tile_m * BM + wm * 64 + i * 32 + 8 * (v / 4) + rsub + (v % 4);
          const int col = tile_n * BN + wn * 64 + j * 32 + col_l;
          if (row < Mrows && col < g.N) {
            const float val = acc[i][j][v];
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

template <bool AF32>
hipError_t launch_epi(const GemmArgs& g, int epi, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(g.N, BN), (unsigned)ceil_div(g.M, BM));
  switch (epi) {
    case EPI_STORE_BF16: gemm_nt<AF32, EPI_STORE_BF16><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_STORE_F32: gemm_nt<AF32, EPI_STORE_F32><<<grid, kThreads, 0, s>>>(g); break;
    case EPI_RESIDUAL: gemm_nt<AF32, EPI_RESIDUAL><<<grid, kThreads, 0, s>>>(g); break;
    default: gemm_nt<AF32, EPI_SCATTER_ADD><<<grid, kThreads, 0, s>>>(g); break;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t mfma_gemm_nt(const GemmArgs& g, int epi, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  return g.a_f32 ? launch_epi<true>(g, epi, s) : launch_epi<false>(g, epi, s);
}

hipError_t mfma_transpose_bf16(const void* U, void* Ut, int rows, int cols, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(cols, 32), (unsigned)ceil_div(rows, 32));
  transpose_bf16<<<grid, 256, 0, s>>>(reinterpret_cast<const uint16_t*>(U), reinterpret_cast<uint16_t*>(Ut), rows, cols);
  return hipGetLastError();
}

int mfma_res_tiles(int64_t d) { return (int)ceil_div(d, BN); }

}  // namespace gsi
