// Single-token weight-streaming kernel of libgsi: the W r correction of Eq. (exact) for the maps whose
// gate fired (Algorithm 1, lines 4 and 7), and the dense baseline y = W x, for one decode token.
//
// A persistent grid of two 512-thread workgroups per CU (sixteen waves per CU).  Structure of one launch:
//   1. gate of every input group: one wave per group reads the count of fired tokens the projection launch
//      published (Eq. (gate)), or -- a stack of one set of inputs -- evaluates the gate itself from the residual
//      launch's slab shares and publishes it; every workgroup does the same arithmetic on the same words, so the
//      decision is uniform across the grid without communication.  If nothing fired the kernel ends here: no byte
//      of W is read;
//   2. once per fired group: the residual vector is staged in LDS, then the rows of W of the group's
//      maps are dealt round-robin over all waves of the grid (neighbouring waves stream neighbouring
//      rows), one row per wave in units of eight 16-byte loads per lane, fp32 FMA against the staged
//      vector, a DPP wave reduction, and one lane adds the result to the image term y = M c that the
//      preceding launch wrote (every output element is updated by exactly one lane).
// The dense baseline runs the same code with every group "fired", x in place of r and a plain store.
#include <hip/hip_ext.h>

#include <cstring>

#include "gsi_decode.h"
#include "gsi_device.h"
#include "gsi_wstream.h"

namespace gsi {
namespace {

constexpr int kBlock = 512;  // waves of a workgroup share one staged activation vector
constexpr int kWaves = kBlock / kWave;
constexpr int kWgsPerCu = 2;  // persistent grid: workgroups per CU

// LONG: an input of the launch is longer than kMaxLinD elements (its vector is staged a block of columns at a time)
template <class T, bool DENSE, bool TAIL, bool NT, bool LONG>
__global__ __launch_bounds__(kBlock) void stream_rows(const LinBatch lb) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  extern __shared__ __align__(16) float xs[];  // one activation vector (r of a fired input, or x)

  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform by construction
  const int gw = blockIdx.x * kWaves + wave;  // this wave's index in the grid
  const int GW = gridDim.x * kWaves;
  const int ng = lb.ng, n = lb.n;

  // ---- 1. gates: one wave per group in every workgroup reads the group's published count ---------------------
  __shared__ unsigned s_fired_g[kMaxTasks];
  if constexpr (!DENSE) {
    for (int gi = wave; gi < ng; gi += kWaves) {  // wave gi evaluates the gate of group gi
      const LinGroup& g = lb.g[gi];
      bool f;
      if (g.part_n) {  // not yet published: the same sums, in the same order, as the gate workgroup of the staged kernel
        float tr, tx;
        wave_norm_sums(g.part_n, g.b_slabs, 1, 0, tr, tx);
        const float rn = sqrtf(tr), xn = sqrtf(tx);
        f = gate_fires(rn, xn, lb.eps);
        if (blockIdx.x == 0 && lane == 0) {  // identical arithmetic in every workgroup: one of them publishes
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
    __syncthreads();
  }
  unsigned fired_mask = 0;
  if constexpr (DENSE) {
    fired_mask = (1u << ng) - 1u;
  } else {
    for (int gi = 0; gi < ng; ++gi) fired_mask |= s_fired_g[gi] << gi;
    fired_mask = __builtin_amdgcn_readfirstlane(fired_mask);
    if (fired_mask == 0) return;  // the common case: nothing fired, no byte of W is read
  }

  // ---- 2. rows of W of fired maps (every map in the dense baseline) -------------------------------------
  bool staged = false;
  for (int gi = 0; gi < ng; ++gi) {
    if (!((fired_mask >> gi) & 1u)) continue;  // uniform across the grid
    const LinGroup& g = lb.g[gi];
    const int d_all = g.d;
    const bool whole_all = DENSE || g.wx;  // the product takes x (and replaces y) rather than r (added to y)
    // A vector longer than the LDS holds is taken in blocks of kMaxLinD columns: every block streams its columns of
    // every row and adds to what the blocks before left in y (the same lane owns an output element in every block).
    // (Without LONG the loop is one pass over the whole vector, known at compile time.)
    for (int c0 = 0; c0 < (LONG ? d_all : 1); c0 += kMaxLinD) {
    const int d = LONG ? min(kMaxLinD, d_all - c0) : d_all;
    const bool whole = LONG ? whole_all && c0 == 0 : whole_all;

    // stage the activation vector (readers of the previous vector are past the barrier)
    if (staged) __syncthreads();
    staged = true;
    if (whole_all && g.xdtype != GSI_F32) {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) xs[idx] = load_act(g.X, g.xdtype, c0 + idx);
    } else {
      const float4* src = reinterpret_cast<const float4*>((whole_all ? reinterpret_cast<const float*>(g.X) : g.R) + c0);
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

    int first = gw;  // rows of the group's maps are dealt round-robin, map after map
    for (int ti = 0; ti < n; ++ti) {
      const LinTask& t = lb.t[ti];
      if (t.group != gi) continue;  // uniform
      const int m = t.m;
      stream_map_rows<T, TAIL, false, NT>(reinterpret_cast<const S*>(t.W) + c0, t.Y, m, d, d_all, xs, whole, first, GW,
                                          lane);
      // continue the deal: the next map starts with the wave after the one that took this map's last row
      first = (first - m % GW + GW) % GW;
    }
    }
  }
}

// The same streaming for ALL fired inputs of a call, descriptors in device memory.
template <class T, bool TAIL, bool NT, bool LONG>
__global__ __launch_bounds__(kBlock) void stream_fired(const FiredIn* __restrict__ ins, const FiredMap* __restrict__ maps,
                                                       int n_in) {
  using S = typename T::storage;
  extern __shared__ __align__(16) float xs[];  // one activation vector (r of a fired input, or x)
  __shared__ unsigned char s_f[kMaxFiredIn];
  __shared__ unsigned s_any;

  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int gw = blockIdx.x * kWaves + wave;
  const int GW = gridDim.x * kWaves;

  // ---- 1. which inputs fired: every workgroup reads the same published counts, so the decision is uniform
  if (threadIdx.x == 0) s_any = 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < n_in; i += kBlock) {
    const bool f = ins[i].n_fired[0] > 0;
    s_f[i] = f ? 1 : 0;
    if (f) s_any = 1u;  // every writer stores the same value
  }
  __syncthreads();
  if (s_any == 0u) return;  // the common case: nothing fired, no byte of W is read

  // ---- 2. rows of W of the fired inputs' maps, dealt round-robin over all waves of the grid, map after map
  bool staged = false;
  int first = gw;
  for (int i = 0; i < n_in; ++i) {
    if (!__builtin_amdgcn_readfirstlane((int)s_f[i])) continue;  // uniform across the grid
    const FiredIn* in = ins + i;
    const int d_all = __builtin_amdgcn_readfirstlane(in->d);
    const int flags = __builtin_amdgcn_readfirstlane(in->flags);
    const int xdtype = flags >> 1;
    const bool whole_all = (flags & kFiredWx) != 0;  // the product takes x (and replaces y) rather than r (added to y)
    const int mb = __builtin_amdgcn_readfirstlane(in->map_begin), me = __builtin_amdgcn_readfirstlane(in->map_end);
    // (a vector longer than the LDS holds: blocks of kMaxLinD columns, as in stream_rows)
    for (int c0 = 0; c0 < (LONG ? d_all : 1); c0 += kMaxLinD) {
    const int d = LONG ? min(kMaxLinD, d_all - c0) : d_all;
    const bool whole = LONG ? whole_all && c0 == 0 : whole_all;
    if (staged) __syncthreads();  // readers of the previous vector are done
    staged = true;
    if (whole_all && xdtype != GSI_F32) {
      for (int idx = threadIdx.x; idx < d; idx += kBlock) xs[idx] = load_act(in->X, xdtype, c0 + idx);
    } else {
      const float4* src = reinterpret_cast<const float4*>((whole_all ? reinterpret_cast<const float*>(in->X) : in->R) + c0);
      float4* dst = reinterpret_cast<float4*>(xs);
      const int n4 = d / 4;
      int q = threadIdx.x;
      for (; q + 3 * kBlock < n4; q += 4 * kBlock) {  // four independent loads per thread and trip
        const float4 a = src[q], b = src[q + kBlock], c = src[q + 2 * kBlock], e = src[q + 3 * kBlock];
        dst[q] = a;
        dst[q + kBlock] = b;
        dst[q + 2 * kBlock] = c;
        dst[q + 3 * kBlock] = e;
      }
      for (; q < n4; q += kBlock) dst[q] = src[q];
    }
    __syncthreads();
    int fst = first;  // every block of columns deals the rows alike: the same lane owns an output element throughout
    for (int j = mb; j < me; ++j) {
      const FiredMap* mp = maps + j;
      const int m = __builtin_amdgcn_readfirstlane(mp->m);
      stream_map_rows<T, TAIL, false, NT>(reinterpret_cast<const S*>(mp->W) + c0, mp->Y, m, d, d_all, xs, whole, fst, GW,
                                          lane);
      fst = (fst - m % GW + GW) % GW;  // the next map starts with the wave after this map's last row
    }
    if (!LONG || c0 + kMaxLinD >= d_all) first = fst;
    }
  }
}

constexpr int kUploadBytes = 3840;
struct UploadArgs {
  uint4 v[kUploadBytes / 16];
};
// copies its own arguments to device memory (descriptor tables of a call; see gsi_decode.h)
__global__ __launch_bounds__(256) void upload_table(const UploadArgs a, uint4* __restrict__ dst, int n16) {
  for (int i = threadIdx.x; i < n16; i += 256) dst[i] = a.v[i];
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

template <class T, bool DENSE, bool TAIL, bool NT, bool LONG>
hipError_t launch_one(const LinBatch& lb, unsigned grid, size_t smem, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  static const hipError_t attr =  // the kernel may use more than the default 64 KB of dynamic LDS
      hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_rows<T, DENSE, TAIL, NT, LONG>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (kMaxLinD + kMaxSumK) * (int)sizeof(float));
  if (attr != hipSuccess) return attr;
  if (e0 && e1) {  // the events take the dispatch's own start and stop timestamps
    hipExtLaunchKernelGGL((stream_rows<T, DENSE, TAIL, NT, LONG>), dim3(grid), dim3(kBlock), smem, s, e0, e1, 0, lb);
  } else {
    stream_rows<T, DENSE, TAIL, NT, LONG><<<grid, kBlock, smem, s>>>(lb);
  }
  return hipGetLastError();
}

template <class T, bool DENSE>
hipError_t launch_shape(const LinBatch& lb, bool tail, bool nt, bool lng, unsigned grid, size_t smem, hipStream_t s,
                        hipEvent_t e0, hipEvent_t e1) {
  switch ((tail ? 4 : 0) | (nt ? 2 : 0) | (lng ? 1 : 0)) {
    case 0: return launch_one<T, DENSE, false, false, false>(lb, grid, smem, s, e0, e1);
    case 1: return launch_one<T, DENSE, false, false, true>(lb, grid, smem, s, e0, e1);
    case 2: return launch_one<T, DENSE, false, true, false>(lb, grid, smem, s, e0, e1);
    case 3: return launch_one<T, DENSE, false, true, true>(lb, grid, smem, s, e0, e1);
    case 4: return launch_one<T, DENSE, true, false, false>(lb, grid, smem, s, e0, e1);
    case 5: return launch_one<T, DENSE, true, false, true>(lb, grid, smem, s, e0, e1);
    case 6: return launch_one<T, DENSE, true, true, false>(lb, grid, smem, s, e0, e1);
    default: return launch_one<T, DENSE, true, true, true>(lb, grid, smem, s, e0, e1);
  }
}

template <class T>
hipError_t launch_dtype(const LinBatch& lb, bool tail, bool nt, bool lng, unsigned grid, size_t smem, hipStream_t s,
                        hipEvent_t e0, hipEvent_t e1) {
  return lb.dense ? launch_shape<T, true>(lb, tail, nt, lng, grid, smem, s, e0, e1)
                  : launch_shape<T, false>(lb, tail, nt, lng, grid, smem, s, e0, e1);
}

}  // namespace

size_t fired_table_bytes(int n_in, int n_maps) {
  return align_up((size_t)n_in * sizeof(FiredIn), 256) + align_up((size_t)n_maps * sizeof(FiredMap), 256);
}

hipError_t upload_launch(const void* src, size_t bytes, void* dst, hipStream_t s) {
  if (bytes % 16) return hipErrorInvalidValue;
  const char* p = static_cast<const char*>(src);
  char* q = static_cast<char*>(dst);
  while (bytes > 0) {
    const size_t n = bytes < (size_t)kUploadBytes ? bytes : (size_t)kUploadBytes;
    UploadArgs a;
    std::memcpy(&a, p, n);
    upload_table<<<1, 256, 0, s>>>(a, reinterpret_cast<uint4*>(q), (int)(n / 16));
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    p += n;
    q += n;
    bytes -= n;
  }
  return hipSuccess;
}

template <class T, bool TAIL, bool NT, bool LONG>
static hipError_t launch_fired(const FiredIn* ins, const FiredMap* maps, int n_in, unsigned grid, size_t smem,
                               hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_fired<T, TAIL, NT, LONG>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLinD * (int)sizeof(float));
  if (attr != hipSuccess) return attr;
  if (e0 && e1) hipExtLaunchKernelGGL((stream_fired<T, TAIL, NT, LONG>), dim3(grid), dim3(kBlock), smem, s, e0, e1, 0, ins, maps, n_in);
  else stream_fired<T, TAIL, NT, LONG><<<grid, kBlock, smem, s>>>(ins, maps, n_in);
  return hipGetLastError();
}

template <class T>
static hipError_t launch_fired_shape(const FiredIn* ins, const FiredMap* maps, const FiredGeom& g, hipStream_t s,
                                     hipEvent_t e0, hipEvent_t e1) {
  switch ((g.tail ? 4 : 0) | (g.nt ? 2 : 0) | (g.long_d ? 1 : 0)) {
    case 0: return launch_fired<T, false, false, false>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 1: return launch_fired<T, false, false, true>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 2: return launch_fired<T, false, true, false>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 3: return launch_fired<T, false, true, true>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 4: return launch_fired<T, true, false, false>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 5: return launch_fired<T, true, false, true>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    case 6: return launch_fired<T, true, true, false>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
    default: return launch_fired<T, true, true, true>(ins, maps, g.n_in, g.grid, g.smem, s, e0, e1);
  }
}

hipError_t stream_fired_geom(int n_in, const FiredIn* host_ins, const FiredMap* host_maps, int wdtype, FiredGeom& g) {
  if (n_in <= 0 || n_in > kMaxFiredIn) return hipErrorInvalidValue;
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  int64_t rows = 0;
  size_t maxd = 0, bytes = 0;
  bool tail = false;
  for (int i = 0; i < n_in; ++i) {
    if ((size_t)host_ins[i].d > maxd) maxd = (size_t)host_ins[i].d;
    if ((host_ins[i].d / V) % (kWave * kLU)) tail = true;
    for (int j = host_ins[i].map_begin; j < host_ins[i].map_end; ++j) {
      rows += host_maps[j].m;
      bytes += (size_t)host_maps[j].m * host_ins[i].d * elem_size(wdtype);
    }
  }
  if (maxd > (size_t)kMaxStreamD) return hipErrorInvalidValue;
  g.long_d = maxd > (size_t)kMaxLinD ? 1 : 0;
  if (g.long_d) maxd = kMaxLinD;  // longer vectors are staged a block of columns at a time
  int64_t grid = (int64_t)kWgsPerCu * num_cus();
  if (grid > ceil_div(rows, kWaves)) grid = ceil_div(rows, kWaves);
  if (grid < 1) grid = 1;
  g.n_in = n_in; g.wdtype = wdtype; g.tail = tail ? 1 : 0; g.grid = (unsigned)grid; g.smem = maxd * sizeof(float);
  g.nt = bytes >= kStreamBytes ? 1 : 0;  // (all maps of the call: which of them fire is not known here)
  return hipSuccess;
}

hipError_t stream_fired_run(const void* table, const FiredGeom& g, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  const FiredIn* ins = static_cast<const FiredIn*>(table);
  const FiredMap* maps = reinterpret_cast<const FiredMap*>(static_cast<const char*>(table) + fired_table_bytes(g.n_in, 0));
  return g.wdtype == GSI_BF16 ? launch_fired_shape<BF16>(ins, maps, g, s, e0, e1)
                              : launch_fired_shape<F32>(ins, maps, g, s, e0, e1);
}

hipError_t stream_fired_launch(const void* table, int n_in, const FiredIn* host_ins, const FiredMap* host_maps,
                               int wdtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (n_in <= 0) return hipSuccess;
  FiredGeom g;
  if (hipError_t e = stream_fired_geom(n_in, host_ins, host_maps, wdtype, g); e != hipSuccess) return e;
  return stream_fired_run(table, g, s, e0, e1);
}

size_t stream_smem_bytes(const LinBatch& lb) {
  size_t maxd = 0;
  for (int i = 0; i < lb.ng; ++i)
    if ((size_t)lb.g[i].d > maxd) maxd = (size_t)lb.g[i].d;
  if (maxd > (size_t)kMaxLinD) maxd = kMaxLinD;  // longer vectors are staged a block of columns at a time
  return maxd * sizeof(float);
}

hipError_t stream_rows_launch(LinBatch& lb, int wdtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  // persistent grid: a few workgroups per CU, never more waves than rows
  int64_t rows = 0;
  size_t bytes = 0;
  bool tail = false;
  for (int i = 0; i < lb.n; ++i) {
    rows += lb.t[i].m;
    bytes += (size_t)lb.t[i].m * lb.g[lb.t[i].group].d * elem_size(wdtype);
    if ((lb.g[lb.t[i].group].d / V) % (kWave * kLU)) tail = true;
  }
  const bool nt = bytes >= kStreamBytes;
  bool lng = false;
  for (int i = 0; i < lb.ng; ++i)
    if (lb.g[i].d > kMaxLinD) lng = true;
  int64_t grid = (int64_t)kWgsPerCu * num_cus();
  if (grid > ceil_div(rows, kWaves)) grid = ceil_div(rows, kWaves);
  if (grid < 1) grid = 1;
  const size_t smem = stream_smem_bytes(lb);
  return wdtype == GSI_BF16 ? launch_dtype<BF16>(lb, tail, nt, lng, (unsigned)grid, smem, s, e0, e1)
                            : launch_dtype<F32>(lb, tail, nt, lng, (unsigned)grid, smem, s, e0, e1);
}

}  // namespace gsi
