// The fused single-token kernel of libgsi: Algorithm 1 (lines 1-7) for ONE token over a chunk of up to four
// inputs and the linear maps that read them, in ONE launch, with the basis read once (Section 7.3 of the paper
// asks for the gate fused with the product and the basis kept on chip).
//
// A grid of one 1024-thread workgroup per CU, all co-resident.  Per chunk:
//   loads     every wave requests all of its operands at once and keeps them in registers: a "basis wave" holds
//             one item of a basis (16 loads of 16 bytes per lane = 16 * rpw consecutive rows of U, rpw = rows
//             per 64-lane load) and the matching x; an "image wave" holds up to 16 loads of image rows.  Image
//             waves never read memory again before they consume these registers, so their loads stay in
//             flight across the exchanges below (loads return in order within a wave).
//   phase 1   basis waves: partial c of their item (Alg. 1 line 1), published as (value, tag) words;
//   reduce    each workgroup sums a few columns of c over all items in a fixed order and publishes them; every
//             workgroup then fetches the finished c into LDS;
//   phase 2   basis waves: r = x - U c on their rows out of the SAME registers (line 2), R written, the
//             item's |r|^2, |x|^2 published; image waves: y = M c of their rows (line 5);
//   gate      every workgroup sums the published norms in a fixed order and applies Eq. (gate) -- identical
//             arithmetic everywhere, so the decision is uniform across the grid; workgroup 0 writes
//             rnorm / xnorm / mask / fired_idx / n_fired.  Nothing fired: the chunk ends here;
//   slow path the residual (or x) of each fired input is staged in LDS and the rows of W of its maps are
//             streamed by all waves of the grid (line 7; gsi_wstream.h).
//
// Exchanges between workgroups use no grid barrier: every exchanged float travels as one 8-byte word
// (value, tag) written with one chip-coherent store, tag = a launch counter that never repeats, and a reader
// simply re-reads a word until its tag is the current one.  The words live in a static device array of the
// library (zero at load, written by this kernel only), so a tag can never be met by accident.  Every wait is
// bounded (one second): on expiry the wave gives up, the launch still ends, a counter records it, and the
// outputs of that launch are not valid.  Launches that overlap in time on one device are not supported.
//
// All sums have a fixed order that depends on the shapes only (never on how items fall on workgroups), so a
// result does not depend on what else shares the launch.
#include <hip/hip_ext.h>

#include <mutex>

#include "gsi_device.h"
#include "gsi_fused.h"
#include "gsi_wstream.h"

namespace gsi {
namespace {

using u64 = unsigned long long;

constexpr size_t kStateBytes = 256;
constexpr size_t kCSlotBytes = (size_t)kFusedMaxCols * 8;
constexpr size_t kNSlotBytes = (size_t)kFusedMaxItems * 2 * 8;
constexpr size_t kPcBytes = (size_t)8 << 20;        // partial projections: items * k words
constexpr size_t kStaticWsBytes = (size_t)8 << 20;  // general-purpose part (the entry point without a workspace)
constexpr size_t kOffC = kStateBytes;
constexpr size_t kOffN = kOffC + kCSlotBytes;
constexpr size_t kOffP = kOffN + kNSlotBytes;
constexpr size_t kOffWs = kOffP + kPcBytes;
constexpr size_t kScratchBytes = kOffWs + kStaticWsBytes;
constexpr long long kSpinTicks = 100000000ll;  // bound of a wait, in ticks of the 100 MHz wall clock

// The library's static scratch.  Host code never uses this name as an address: see scratch_ptr().
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct FState {
  unsigned epoch;     // tags handed out so far
  unsigned exit;      // workgroups of the running launch that have finished
  unsigned wg_done;   // workgroups whose stores of a fired chunk have completed
  unsigned timeouts;  // waits that expired, ever
};

__device__ __forceinline__ u64 ld64(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st64(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 pack(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }
__device__ __forceinline__ void st_f32(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_f32(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_u32(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u32(unsigned* p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned add_u32(unsigned* p, unsigned v) { return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Words base[q * stride], q < cnt (<= N), of the current tag: all requested at once, then re-read until valid.
// out[q] = 0 for q >= cnt.  The wait is bounded; once any wave of the workgroup has given up, nobody waits.
template <int N>
__device__ __forceinline__ void poll_strided(const u64* base, int64_t stride, int cnt, unsigned tag, float (&out)[N],
                                             volatile unsigned* abort_flag) {
  u64 v[N];
#pragma unroll
  for (int q = 0; q < N; ++q) v[q] = q < cnt ? ld64(base + q * stride) : ((u64)tag << 32);
  bool pending = false;
#pragma unroll
  for (int q = 0; q < N; ++q) pending |= (unsigned)(v[q] >> 32) != tag;
  if (pending) {
    const long long t0 = wall_clock64();
    while (pending && !*abort_flag) {
      pending = false;
#pragma unroll
      for (int q = 0; q < N; ++q)
        if ((unsigned)(v[q] >> 32) != tag) {
          v[q] = ld64(base + q * stride);
          pending |= (unsigned)(v[q] >> 32) != tag;
        }
      if (pending && wall_clock64() - t0 > kSpinTicks) *abort_flag = 1u;
    }
  }
#pragma unroll
  for (int q = 0; q < N; ++q) out[q] = __uint_as_float((unsigned)v[q]);
}

template <class T>
__global__ __launch_bounds__(kFusedBlock) void fused_token(const FusedArgs a, unsigned char* __restrict__ sc) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  extern __shared__ __align__(16) float smem[];
  float* cs = smem;                  // finished coefficients of the chunk's inputs, [n_in][k]
  float* xsave = smem + kFusedMaxCols;               // x of the rows a basis wave holds, [wave][64]
  float* xs = smem + kFusedMaxCols + kFusedBlock;    // the staged vector of the slow path
  __shared__ unsigned s_epoch, s_abort, s_done, s_fired[kFusedMaxIn];

  FState* st = reinterpret_cast<FState*>(sc);
  u64* cslot = reinterpret_cast<u64*>(sc + kOffC);
  u64* nslot = reinterpret_cast<u64*>(sc + kOffN);
  u64* pc = reinterpret_cast<u64*>(sc + kOffP);
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int b = blockIdx.x, G = gridDim.x;
  if (threadIdx.x == 0) {
    s_epoch = ld_u32(&st->epoch);
    s_abort = 0;
    s_done = 0;
  }
  __syncthreads();
  const unsigned epoch0 = s_epoch;
  int fired_chunks = 0;

  for (int ci = 0; ci < a.n_chunks; ++ci) {
    const FusedChunk& ch = a.c[ci];
    const unsigned tag = epoch0 + (unsigned)ci + 1u;
    const int k = ch.k, lsh = ch.lsh, lpr = 1 << lsh, rpw = kWave >> lsh;
    const int kshift = __builtin_ctz(k);
    const int cc = lane & (lpr - 1), rg = lane >> lsh;  // 16-byte chunk of the row, row of the load
    const bool uwave = wave < ch.u_waves;

    // ---- loads: everything this wave needs from the basis / the images, requested at once ---------------
    // Per load q (uniform over the wave): the matrix, its first row of this load and its row count.  A load
    // without work reads the first bytes of the exchange state instead (one cache line, no memory traffic).
    int it = -1, ii = 0;                   // basis wave: its item and the item's input
    const S* base[kFusedLoads];
    int rowq[kFusedLoads], lim[kFusedLoads];
    float* yq[kFusedLoads];                // image wave: output of the load's rows
    int inq[kFusedLoads];                  // ... and the input its map reads
#pragma unroll
    for (int q = 0; q < kFusedLoads; ++q) {
      base[q] = nullptr;
      rowq[q] = 0;
      lim[q] = 0;
      yq[q] = nullptr;
      inq[q] = 0;
    }
    if (uwave) {
      const int cand = wave * G + b;
      if (cand < ch.n_items) {
        it = cand;
#pragma unroll
        for (int i = 1; i < kFusedMaxIn; ++i)
          if (i < ch.n_in && it >= ch.in[i].item0) ii = i;
        const FusedIn& in = ch.in[ii];
        const int row0 = (it - in.item0) * (kFusedLoads * rpw);
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) {
          base[q] = reinterpret_cast<const S*>(in.U);
          rowq[q] = row0 + q * rpw;
          lim[q] = in.d;
        }
      }
    } else {
      const int v = wave - ch.u_waves;
      const int wb = b * ch.wg_units;
      const int we = min(wb + ch.wg_units, ch.n_units);
      const int ub = min(wb + v * ch.wave_units, we);
      const int ue = min(ub + ch.wave_units, we);
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        const int u = ub + q;
        int jj = 0;
#pragma unroll
        for (int j = 1; j < kFusedMaxMap; ++j)
          if (j < ch.n_mp && u >= ch.mp[j].unit0) jj = j;
        const FusedMap& mp = ch.mp[jj];
        if (u < ue) {
          base[q] = reinterpret_cast<const S*>(mp.M);
          rowq[q] = (u - mp.unit0) * rpw;
          lim[q] = mp.m;
          yq[q] = mp.Y;
          inq[q] = mp.in;
        }
      }
    }
    uint4 raw[kFusedLoads];
    float xv[kFusedLoads];
#pragma unroll
    for (int q = 0; q < kFusedLoads; ++q) {
      const int r = min(rowq[q] + rg, lim[q] - 1);  // clamped: the loads are unconditional
      const S* p = base[q] ? base[q] + (int64_t)r * k + cc * V : reinterpret_cast<const S*>(sc);
      raw[q] = *reinterpret_cast<const uint4*>(p);
    }
    if (it >= 0) {
      const float* X = reinterpret_cast<const float*>(ch.in[ii].X);
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) xv[q] = X[min(rowq[q] + rg, lim[q] - 1)];
    }

    // ---- phase 1: partial c of the item (fixed order: loads ascending, then the row groups of the wave) ----
    if (it >= 0) {
      float acc[V];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        float w[V];
        T::widen(raw[q], w);
        const float x = rowq[q] + rg < lim[q] ? xv[q] : 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] = fmaf(w[e], x, acc[e]);
      }
      for (int off = lpr; off < kWave; off <<= 1) {
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += __shfl_xor(acc[e], off, kWave);
      }
      if (cc == 0) {  // x is needed once more, by the lane that forms the row's residual: parked in LDS
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) xsave[wave * kWave + q * rpw + rg] = xv[q];
      }
      if (rg == 0) {
        u64* dst = pc + (int64_t)it * k + cc * V;
#pragma unroll
        for (int e = 0; e < V; ++e) st64(dst + e, pack(acc[e], tag));
      }
    }

    if (uwave) {
      // ---- reduce: this workgroup's columns of c, one wave per column, items in ascending order per lane ----
      const int ncol = ch.n_in << kshift;
      for (int col = wave; col < ch.wg_cols; col += ch.u_waves) {
        const int cg = b * ch.wg_cols + col;
        if (cg < ncol) {
          const int i = cg >> kshift, j = cg & (k - 1);
          const FusedIn& in = ch.in[i];
          const int P = in.n_items;
          const u64* base = pc + (int64_t)in.item0 * k + j;
          float s = 0.f;
          for (int p0 = 0; p0 < P; p0 += kWave * 8) {
            float v[8];
            const int left = P - p0 - lane;
            poll_strided<8>(base + (int64_t)(p0 + lane) * k, (int64_t)kWave * k, left > 0 ? (left + kWave - 1) / kWave : 0,
                            tag, v, &s_abort);
#pragma unroll
            for (int q = 0; q < 8; ++q) s += v[q];
          }
          s = group_sum<kWave>(s);
          if (lane == 0) {
            st64(cslot + cg, pack(s, tag));
            in.C[j] = s;
          }
        }
      }
      // ---- the finished c of every input of the chunk -> LDS
      const int nth = ch.u_waves * kWave;
      for (int s0 = wave * kWave + lane; s0 < ncol; s0 += nth * 4) {
        float v[4];
        const int left = ncol - s0;
        poll_strided<4>(cslot + s0, nth, (left + nth - 1) / nth, tag, v, &s_abort);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (s0 + q * nth < ncol) cs[s0 + q * nth] = v[q];
      }
    }
    __syncthreads();

    // ---- phase 2: residual rows (basis waves) and image rows (image waves) out of the registers ----------
    if (it >= 0) {
      const FusedIn& in = ch.in[ii];
      float cv[V];
      lds_vec<V>(cs + (ii << kshift) + cc * V, cv);
      float ar = 0.f, ax = 0.f;
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        float w[V];
        T::widen(raw[q], w);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) s = fmaf(w[e], cv[e], s);
        s = group_sum_rt(s, lpr);
        const int r = rowq[q] + rg;
        if (r < lim[q] && cc == 0) {
          const float x = xsave[wave * kWave + q * rpw + rg];
          const float res = x - s;
          st_f32(in.R + r, res);
          ar = fmaf(res, res, ar);
          ax = fmaf(x, x, ax);
        }
      }
      ar = group_sum<kWave>(ar);
      ax = group_sum<kWave>(ax);
      if (lane == 0) {
        st64(nslot + 2 * it, pack(ar, tag));
        st64(nslot + 2 * it + 1, pack(ax, tag));
      }
    } else if (!uwave) {
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        if (yq[q]) {  // uniform over the wave
          float w[V], cv[V];
          T::widen(raw[q], w);
          lds_vec<V>(cs + (inq[q] << kshift) + cc * V, cv);
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < V; ++e) s = fmaf(w[e], cv[e], s);
          s = group_sum_rt(s, lpr);
          const int r = rowq[q] + rg;
          if (cc == 0 && r < lim[q]) st_f32(yq[q] + r, s);
        }
      }
    }

    // ---- gate: one wave per input, the items' norms in ascending order per lane -----------------------------
    if (uwave) {
      for (int i = wave; i < ch.n_in; i += ch.u_waves) {
        const FusedIn& in = ch.in[i];
        const int P = in.n_items;
        const u64* base = nslot + 2 * (int64_t)in.item0;
        float sr = 0.f, sx = 0.f;
        for (int p0 = 0; p0 < P; p0 += kWave * 4) {
          float vr[4], vx[4];
          const int left = P - p0 - lane;
          const int cnt = left > 0 ? (left + kWave - 1) / kWave : 0;
          poll_strided<4>(base + 2 * (int64_t)(p0 + lane), 2 * kWave, cnt, tag, vr, &s_abort);
          poll_strided<4>(base + 2 * (int64_t)(p0 + lane) + 1, 2 * kWave, cnt, tag, vx, &s_abort);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            sr += vr[q];
            sx += vx[q];
          }
        }
        const float rn = sqrtf(group_sum<kWave>(sr)), xn = sqrtf(group_sum<kWave>(sx));
        const bool f = gate_fires(rn, xn, a.eps);
        if (lane == 0) {
          s_fired[i] = f ? 1u : 0u;
          if (b == 0) {  // what the norm and gate kernels would write
            in.rnorm[0] = rn;
            in.xnorm[0] = xn;
            if (in.n_fired) {  // null in a projection-only launch
              in.mask[0] = f ? 1 : 0;
              if (f) in.fired_idx[0] = 0;
              in.n_fired[0] = f ? 1 : 0;
            }
          }
        }
      }
    }
    __syncthreads();
    unsigned fired_mask = 0;
    for (int i = 0; i < ch.n_in; ++i) fired_mask |= s_fired[i] << i;
    if (s_abort) fired_mask = 0;  // a wait expired: this launch's results are void, end it quickly
    fired_mask = __builtin_amdgcn_readfirstlane(fired_mask);
    if (fired_mask == 0) continue;  // the common case: nothing fired, no byte of W is read

    // ---- slow path: rows of W of the fired inputs' maps --------------------------------------------------
    // The image rows and residuals this phase reads were written by other workgroups: wait until every
    // workgroup's stores of this chunk have completed (they were issued before the gate, so this is short).
    ++fired_chunks;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane == 0) {
      const unsigned old = atomicAdd(&s_done, 1u);
      if (old == (unsigned)(kFusedWaves * fired_chunks - 1)) add_u32(&st->wg_done, 1u);
    }
    if (threadIdx.x == 0) {
      const unsigned want = (unsigned)G * (unsigned)fired_chunks;
      const long long t0 = wall_clock64();
      while (ld_u32(&st->wg_done) < want && !s_abort)
        if (wall_clock64() - t0 > kSpinTicks) s_abort = 1u;
    }
    __syncthreads();
    const int GW = G * kFusedWaves, gw = b * kFusedWaves + wave;
    for (int gi = 0; gi < ch.n_in; ++gi) {
      if (!((fired_mask >> gi) & 1u)) continue;  // uniform across the grid
      const FusedIn& in = ch.in[gi];
      const int dd = in.d;
      const bool whole = in.wx != 0;  // y = W x (Algorithm 1, line 7) replaces y; else W r is added to M c
      if (whole) {
        const float* X = reinterpret_cast<const float*>(in.X);
        for (int idx = threadIdx.x; idx < dd; idx += kFusedBlock) xs[idx] = X[idx];
      } else {
        for (int idx = threadIdx.x; idx < dd; idx += 4 * kFusedBlock) {
          float v[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = idx + q * kFusedBlock < dd ? ld_f32(in.R + idx + q * kFusedBlock) : 0.f;
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (idx + q * kFusedBlock < dd) xs[idx + q * kFusedBlock] = v[q];
        }
      }
      __syncthreads();
      const bool tail = ((dd / V) % (kWave * kLU)) != 0;
      int first = gw;  // rows of the input's maps are dealt round-robin, map after map
      for (int j = 0; j < ch.n_mp; ++j) {
        const FusedMap& mp = ch.mp[j];
        if (mp.in != gi) continue;  // uniform
        if (tail) stream_map_rows<T, true, true>(reinterpret_cast<const S*>(mp.W), mp.Y, mp.m, dd, xs, whole, first, GW, lane);
        else stream_map_rows<T, false, true>(reinterpret_cast<const S*>(mp.W), mp.Y, mp.m, dd, xs, whole, first, GW, lane);
        first = (first - mp.m % GW + GW) % GW;
      }
      __syncthreads();  // the staged vector is free again
    }
  }

  // ---- the last workgroup to finish leaves the exchange state ready for the next launch -----------------
  __syncthreads();
  if (threadIdx.x == 0) {
    if (s_abort) add_u32(&st->timeouts, 1u);
    const unsigned old = add_u32(&st->exit, 1u);
    if (old == (unsigned)G - 1u) {
      st_u32(&st->exit, 0u);
      st_u32(&st->wg_done, 0u);
      st_u32(&st->epoch, epoch0 + (unsigned)a.n_chunks);
    }
  }
}

int num_cus() {
  int dev = 0, cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) return 0;
  return cu;
}

// Device address of the static scratch array on the current device: asked of the runtime once per device
// (each device holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_scratch[kMaxDevices];
int g_cus[kMaxDevices];

hipError_t scratch_ptr(unsigned char** out, int* cus) {
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch[dev]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch[dev] = static_cast<unsigned char*>(p);
    g_cus[dev] = num_cus();
  }
  *out = g_scratch[dev];
  if (cus) *cus = g_cus[dev];
  return hipSuccess;
}

template <class T>
hipError_t launch_as(const FusedArgs& a, unsigned grid, size_t smem, unsigned char* sc, hipStream_t s, hipEvent_t e0,
                     hipEvent_t e1) {
  static const hipError_t attr =  // more than the default 64 KB of dynamic LDS
      hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_token<T>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (kFusedMaxCols + kFusedBlock + kFusedMaxD) * (int)sizeof(float));
  if (attr != hipSuccess) return attr;
  if (e0 && e1) {  // the events take the dispatch's own start and stop timestamps
    hipExtLaunchKernelGGL((fused_token<T>), dim3(grid), dim3(kFusedBlock), smem, s, e0, e1, 0, a, sc);
  } else {
    fused_token<T><<<grid, kFusedBlock, smem, s>>>(a, sc);
  }
  return hipGetLastError();
}

bool pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }

}  // namespace

bool fused_input_ok(int64_t d, int64_t k, int udtype, const void* U, const void* X, int xdtype, const float* C,
                    const float* R, bool wx) {
  (void)X; (void)C; (void)R; (void)wx;  // element alignment (checked by the caller) is all they need
  if (xdtype != GSI_F32) return false;
  const int V = udtype == GSI_BF16 ? 8 : 4;
  if (udtype != GSI_BF16 && udtype != GSI_F32) return false;
  if (k % V || !pow2(k / V) || k / V > kWave || k / V < 8 || k > kFusedMaxCols) return false;  // 8..64 lanes per row
  if (d < 1 || d > (1 << 24)) return false;
  return reinterpret_cast<uintptr_t>(U) % 16 == 0;
}

bool fused_map_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M) {
  (void)k;
  const int V = wdtype == GSI_BF16 ? 8 : 4;
  if (m < 1 || m > (1 << 24) || d % V || d > kFusedMaxD) return false;
  return reinterpret_cast<uintptr_t>(W) % 16 == 0 && reinterpret_cast<uintptr_t>(M) % 16 == 0;
}

bool fused_plan(FusedChunk& ch, int dtype) {
  unsigned char* sc = nullptr;
  int G = 0;
  if (scratch_ptr(&sc, &G) != hipSuccess || G < 1) return false;
  const int V = dtype == GSI_BF16 ? 8 : 4;
  const int k = ch.k;
  if (ch.n_in < 1 || ch.n_in > kFusedMaxIn || ch.n_mp < 0 || ch.n_mp > kFusedMaxMap) return false;
  if (k % V || !pow2(k / V) || k / V > kWave) return false;
  const int lpr = k / V, rpw = kWave / lpr;
  ch.lsh = __builtin_ctz(lpr);
  if ((int64_t)ch.n_in * k > kFusedMaxCols) return false;
  int64_t items = 0, units = 0;
  for (int i = 0; i < ch.n_in; ++i) {
    ch.in[i].item0 = (int)items;
    ch.in[i].n_items = (int)ceil_div(ch.in[i].d, kFusedLoads * rpw);
    items += ch.in[i].n_items;
  }
  for (int j = 0; j < ch.n_mp; ++j) {
    ch.mp[j].unit0 = (int)units;
    ch.mp[j].n_units = (int)ceil_div(ch.mp[j].m, rpw);
    units += ch.mp[j].n_units;
  }
  if (items > kFusedMaxItems || (size_t)items * k * 8 > kPcBytes || units > (1 << 28)) return false;
  ch.n_items = (int)items;
  ch.n_units = (int)units;
  ch.wg_cols = (int)ceil_div((int64_t)ch.n_in * k, G);
  ch.wg_units = (int)ceil_div(units, G);
  const int need_u = (int)std::max<int64_t>(1, ceil_div(items, G));
  if (ch.n_mp == 0) {
    if (need_u > kFusedWaves) return false;
    ch.u_waves = kFusedWaves;
    ch.wave_units = 0;
    return true;
  }
  // basis waves: as many as the items need, and two or more when the image rows leave room (they also
  // carry the exchanges); image waves: the rest
  for (int uw = std::max(need_u, 2); uw >= need_u; --uw) {
    if (uw >= kFusedWaves) continue;
    const int per = (int)ceil_div(ch.wg_units, kFusedWaves - uw);
    if (per <= kFusedLoads) {
      ch.u_waves = uw;
      ch.wave_units = per;
      return true;
    }
  }
  return false;
}

hipError_t fused_launch(const FusedArgs& a, int dtype, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (a.n_chunks < 1) return hipSuccess;
  unsigned char* sc = nullptr;
  int G = 0;
  if (hipError_t e = scratch_ptr(&sc, &G); e != hipSuccess) return e;
  if (G < 1) return hipErrorInvalidDevice;
  size_t maxd = 0;
  for (int c = 0; c < a.n_chunks; ++c)
    for (int j = 0; j < a.c[c].n_mp; ++j) maxd = std::max<size_t>(maxd, (size_t)a.c[c].in[a.c[c].mp[j].in].d);
  const size_t smem = ((size_t)kFusedMaxCols + kFusedBlock + maxd) * sizeof(float);
  return dtype == GSI_BF16 ? launch_as<BF16>(a, (unsigned)G, smem, sc, s, e0, e1)
                           : launch_as<F32>(a, (unsigned)G, smem, sc, s, e0, e1);
}

hipError_t fused_timeouts(unsigned* count) {
  unsigned char* sc = nullptr;
  if (hipError_t e = scratch_ptr(&sc, nullptr); e != hipSuccess) return e;
  if (hipError_t e = hipDeviceSynchronize(); e != hipSuccess) return e;
  FState h;
  if (hipError_t e = hipMemcpy(&h, sc, sizeof(h), hipMemcpyDeviceToHost); e != hipSuccess) return e;
  *count = h.timeouts;
  return hipSuccess;
}

hipError_t static_workspace(void** ptr, size_t* bytes) {
  unsigned char* sc = nullptr;
  if (hipError_t e = scratch_ptr(&sc, nullptr); e != hipSuccess) return e;
  *ptr = sc + kOffWs;
  *bytes = kStaticWsBytes;
  return hipSuccess;
}

}  // namespace gsi
