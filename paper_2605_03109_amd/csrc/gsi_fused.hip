// The fused single-token kernel of libgsi: Algorithm 1 (lines 1-7) for ONE token over a chunk of up to four
// inputs and the linear maps that read them, in ONE launch, with the basis read once (Section 7.3 of the paper
// asks for the gate fused with the product and the basis kept on chip).
//
// A grid of one 1024-thread workgroup (16 waves) per CU, all co-resident.  Per chunk:
//   loads     every wave requests all of its operands at once and keeps them in registers.  Workgroup g of the
//             first n_groups workgroups is a "basis workgroup": its waves 0-7 each hold one item of basis group g
//             (8 loads of 16 bytes per lane = 8 * rpw consecutive rows of U, rpw = rows per 64-lane load, and the
//             matching x), its waves 8-15 hold image rows (up to 8 loads each).  The other workgroups hold image
//             rows in waves 1-15; their wave 0 holds nothing and serves the exchanges.  Image waves never read
//             memory again before they consume their registers, so their loads stay in flight across the
//             exchanges below (loads return in order within a wave);
//   phase 1   basis waves: partial c of their item (Alg. 1 line 1); the eight partials of the group are added in
//             LDS in wave order and published as (value, tag) words;
//   reduce    each workgroup sums a few columns of c over all groups in a fixed order and publishes them; every
//             workgroup then fetches the finished c into LDS;
//   phase 2   basis waves: r = x - U c on their rows out of the SAME registers (line 2), R written, the group's
//             |r|^2, |x|^2 added in LDS and published; image waves: y = M c of their rows (line 5);
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
// All sums have a fixed order that depends on the shapes only (never on what else shares the launch): items
// and groups are cut from each input by its own row count.
#include <hip/hip_ext.h>

#include <mutex>

#include "gsi_device.h"
#include "gsi_fused.h"
#include "gsi_wstream.h"

namespace gsi {
namespace {

using u64 = unsigned long long;

constexpr size_t kStateBytes = 256;
// Words that every workgroup reads (the finished c, the groups' norms) are published in kCopies copies, and a
// workgroup reads copy (its index mod kCopies): when all 256 workgroups re-read the same few kilobytes, the
// memory channels that hold them serve every request one after another and an exchange takes microseconds.
constexpr int kCopies = 16;
constexpr size_t kCSlotBytes = (size_t)kCopies * kFusedMaxCols * 8;
constexpr size_t kNSlotBytes = (size_t)2 * kCopies * kFusedMaxGroups * 2 * 8;  // two sets, by chunk parity
constexpr size_t kPcBytes = (size_t)kFusedMaxGroups * 512 * 8;  // partial projections: groups * k words
constexpr size_t kStaticWsBytes = (size_t)8 << 20;              // general-purpose part (the entry point without a workspace)
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
  unsigned wg_done;   // workgroups whose stores of a fired chunk have completed, ever (wraps)
  unsigned timeouts;  // waits that expired, ever
  unsigned pad;
};

__device__ __forceinline__ u64 ld64(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st64(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 pack(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }
__device__ __forceinline__ void st_f32(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_f32(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_u32(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u32(unsigned* p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned add_u32(unsigned* p, unsigned v) { return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// A value that is the same in every lane of the wave, moved to a scalar register.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <class P>
__device__ __forceinline__ P* uni(P* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<P*>(((unsigned long long)hi << 32) | lo);
}

// 16 (or 4) bytes at base + voff through a buffer descriptor: the base is uniform over the wave, the offset a
// 32-bit register per lane, and an offset at or beyond `bytes` reads zeros instead of memory.
__device__ __forceinline__ uint4 buf_load16(const void* base, unsigned bytes, unsigned voff) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)bytes, 0x00020000);
  return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0));
}
__device__ __forceinline__ float buf_load4(const void* base, unsigned bytes, unsigned voff) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)bytes, 0x00020000);
  return __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, 0, 0));
}

// Words base[q * qstride + c], q < nq (<= NQ), c < NC, of the current tag: all requested at once, then re-read
// until valid.  out = 0 for q >= nq.  The wait is bounded; once any wave of the workgroup has given up, nobody waits.
template <int NQ, int NC>
__device__ __forceinline__ void poll_words(const u64* base, int64_t qstride, int nq, unsigned tag, float (&out)[NQ][NC],
                                           volatile unsigned* abort_flag) {
  u64 v[NQ][NC];
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int c = 0; c < NC; ++c) v[q][c] = q < nq ? ld64(base + q * qstride + c) : ((u64)tag << 32);
  bool pending = false;
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int c = 0; c < NC; ++c) pending |= (unsigned)(v[q][c] >> 32) != tag;
  if (pending) {
    const long long t0 = wall_clock64();
    while (pending && !*abort_flag) {
      pending = false;
#pragma unroll
      for (int q = 0; q < NQ; ++q)
#pragma unroll
        for (int c = 0; c < NC; ++c)
          if ((unsigned)(v[q][c] >> 32) != tag) {
            v[q][c] = ld64(base + q * qstride + c);
            pending |= (unsigned)(v[q][c] >> 32) != tag;
          }
      if (pending && wall_clock64() - t0 > kSpinTicks) *abort_flag = 1u;
    }
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int c = 0; c < NC; ++c) out[q][c] = __uint_as_float((unsigned)v[q][c]);
}

template <class T>
__global__ __launch_bounds__(kFusedBlock) void fused_token(const FusedArgs a, unsigned char* __restrict__ sc) {
  constexpr int V = T::kVec;
  using S = typename T::storage;
  constexpr int GI = kFusedGroup;
  constexpr int SW = kFusedWaves - 1;  // the service wave
  extern __shared__ __align__(16) float smem[];
  float* cs = smem;                                // finished coefficients of the chunk's inputs, [n_in][k]
  float* xsave = smem + kFusedMaxCols;             // x of the rows a basis wave holds, [wave][64]
  float* red = smem + kFusedMaxCols + kFusedBlock; // partial c of the group's items, [GI][k]; later the staged
  float* xs = red;                                 // vector of the slow path
  __shared__ __align__(16) FusedArgs s_a;          // the arguments, fetched once by all lanes together
  __shared__ unsigned s_epoch, s_done0, s_abort, s_done, s_fired[kFusedMaxIn];
  __shared__ float s_nred[GI][2];
  // what each image wave's loads are (written when they are requested, read back in phase 2): output row
  // pointer, first row, rows of the map (low 24 bits) and the map's input (high 8 bits)
  __shared__ __align__(16) uint4 s_img[kFusedWaves][kFusedLoads];

  FState* st = reinterpret_cast<FState*>(sc);
  u64* cslot = reinterpret_cast<u64*>(sc + kOffC);
  u64* nslot = reinterpret_cast<u64*>(sc + kOffN);
  u64* pc = reinterpret_cast<u64*>(sc + kOffP);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int b = blockIdx.x, G = gridDim.x;
  {
    // (descriptor fields are needed in long dependent chains: one parallel fetch into LDS instead of a scalar
    // load, and its memory latency, per link of the chain)
    const uint4* src = reinterpret_cast<const uint4*>(&a);
    uint4* dst = reinterpret_cast<uint4*>(&s_a);
    for (int i = threadIdx.x; i < (int)(sizeof(FusedArgs) / 16); i += kFusedBlock) dst[i] = src[i];
  }
  if (threadIdx.x == 0) {
    // Both words change only after every workgroup of this launch has published something, which each does
    // after this read: workgroup 0 advances the epoch when it ends, and it cannot end before it has read
    // every workgroup's words; wg_done is first added to after a gate, which needs every workgroup's norms.
    s_epoch = ld_u32(&st->epoch);
    s_done0 = ld_u32(&st->wg_done);
    s_abort = 0;
    s_done = 0;
  }
  __syncthreads();
  const unsigned epoch0 = (unsigned)uni((int)s_epoch);
  const unsigned done0 = (unsigned)uni((int)s_done0);
  const int n_chunks = uni(s_a.n_chunks);
  const float eps = __int_as_float(uni(__float_as_int(s_a.eps)));
  int fired_chunks = 0;

  // What this wave holds of the chunk whose operands are in its registers (set when they are requested):
  int h_ii = 0, h_row0 = 0, h_dlim = 0;  // basis wave: the group's input, the item's first row, the input's rows
  int h_ub = 0, h_ue = 0;                // image wave: its units [ub, ue)
  uint4 raw[kFusedLoads];
  float xv[kFusedLoads];

  // ---- loads of a chunk: everything this wave needs from the basis / the images, requested at once.  The
  // address of every load first (a load without work reads the first bytes of the exchange state: one cache
  // line, no memory traffic), then all loads in one run, unconditionally.
  // (ldc == n_chunks: nothing left to request; the loads still run, on the idle line, so that the registers
  // are written on every path -- else they would count as live, and be spilled, across the slow path)
  auto issue_loads = [&](int ldc) {
    {
      int lane = __lane_id();
      asm volatile("" : "+v"(lane));
      const bool real = ldc < n_chunks;
      const FusedChunk& nx = s_a.c[real ? ldc : 0];
      const int k = uni(nx.k), lsh = uni(nx.lsh), n_in = uni(nx.n_in), n_mp = uni(nx.n_mp), NG = uni(nx.n_groups);
      const int lpr = 1 << lsh, rpw = kWave >> lsh;
      const int cc = lane & (lpr - 1), rg = lane >> lsh;
      const bool bwg = b < NG;
      // Loads go through buffer descriptors: a base that is uniform over the wave, a 32-bit byte offset per lane,
      // and rows past the end of a matrix read zeros.  A load without work reads the first 16 bytes of the
      // exchange state (one cache line, no memory traffic).
      const unsigned rowb = (unsigned)k * (unsigned)sizeof(S);  // bytes of a row
      const void* lb[kFusedLoads];   // per load: base, size (uniform over the wave) and the lane's byte offset
      unsigned ln[kFusedLoads], lo[kFusedLoads];
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        lb[q] = reinterpret_cast<const void*>(sc);
        ln[q] = 16u;
        lo[q] = 0u;
      }
      const void* X = reinterpret_cast<const void*>(sc);
      unsigned xbytes = 0u, r0 = 0u;
      if (!real) {
      } else if (bwg && wave < GI) {
        int ii = 0;
#pragma unroll
        for (int i = 1; i < kFusedMaxIn; ++i)
          if (i < n_in && b >= nx.in[i].group0) ii = i;
        h_ii = uni(ii);
        const FusedIn& in = nx.in[h_ii];
        h_row0 = uni(((b - in.group0) * GI + wave) * (kFusedLoads * rpw));
        h_dlim = uni(in.d);
        const void* U = uni(in.U);
        X = uni(in.X);
        xbytes = (unsigned)h_dlim * 4u;
        r0 = (unsigned)(h_row0 + rg);
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) {
          lb[q] = U;
          ln[q] = (unsigned)h_dlim * rowb;
          lo[q] = (r0 + (unsigned)(q * rpw)) * rowb + (unsigned)(cc * V) * (unsigned)sizeof(S);
        }
      } else if (wave != SW) {
        const int slot = bwg ? b * (SW - GI) + (wave - GI) : NG * (SW - GI) + (b - NG) * SW + wave;
        h_ub = uni(min(slot * nx.wave_units, nx.n_units));
        h_ue = uni(min(h_ub + nx.wave_units, nx.n_units));
        // the first unit of every map, fetched at once; the map of a unit = the last whose first unit is <= it
        int u0[kFusedMaxMap];
        {
          const int4 a0 = *reinterpret_cast<const int4*>(&nx.unit0[0]), a1 = *reinterpret_cast<const int4*>(&nx.unit0[4]);
          u0[0] = uni(a0.x); u0[1] = uni(a0.y); u0[2] = uni(a0.z); u0[3] = uni(a0.w);
          u0[4] = uni(a1.x); u0[5] = uni(a1.y); u0[6] = uni(a1.z); u0[7] = uni(a1.w);
        }
        int jq[kFusedLoads];
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) {
          const int u = h_ub + q;
          int jj = 0;
#pragma unroll
          for (int j = 1; j < kFusedMaxMap; ++j) jj += u >= u0[j] ? 1 : 0;
          jq[q] = jj;
        }
        // the descriptors of those maps: all requested from LDS before the first is used
        uint4 md[kFusedLoads];  // {M, Y} of load q's map
        int2 mm[kFusedLoads];   // {m, in}
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) {
          const FusedMap& mp = nx.mp[jq[q]];
          const uint2 pm = *reinterpret_cast<const uint2*>(&mp.M), py = *reinterpret_cast<const uint2*>(&mp.Y);
          md[q] = make_uint4(pm.x, pm.y, py.x, py.y);
          mm[q] = *reinterpret_cast<const int2*>(&mp.m);
        }
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) {
          if (h_ub + q < h_ue) {  // uniform over the wave
            const int row = (h_ub + q - u0[jq[q]]) * rpw;
            const int m = uni(mm[q].x);
            lb[q] = reinterpret_cast<const void*>(((unsigned long long)(unsigned)uni((int)md[q].y) << 32) | (unsigned)uni((int)md[q].x));
            ln[q] = (unsigned)m * rowb;
            lo[q] = (unsigned)(row + rg) * rowb + (unsigned)(cc * V) * (unsigned)sizeof(S);
            if (lane == 0) s_img[wave][q] = make_uint4(md[q].z, md[q].w, (unsigned)row, (unsigned)m | ((unsigned)mm[q].y << 24));
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) raw[q] = buf_load16(lb[q], ln[q], lo[q]);
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) xv[q] = buf_load4(X, xbytes, (r0 + (unsigned)(q * rpw)) * 4u);
    }
  };

  // ---- gate of a chunk (the service wave): the groups' norms of every input, in ascending order per lane ----
  auto gate_chunk = [&](int gc, int lane) {
    const FusedChunk& ch = s_a.c[gc];
    const unsigned tag = epoch0 + (unsigned)gc + 1u;
    const int n_in = uni(ch.n_in);
    const u64* nbase = nslot + ((int64_t)(gc & 1) * kCopies + (b % kCopies)) * kFusedMaxGroups * 2;
    float v[kFusedMaxIn][2][2];
#pragma unroll
    for (int i = 0; i < kFusedMaxIn; ++i) {  // all inputs requested before the first is waited for
      const int P = i < n_in ? ch.in[i < n_in ? i : 0].n_groups : 0;
      const int g0 = ch.in[i < n_in ? i : 0].group0;
      const int left = P - lane;
      poll_words<2, 2>(nbase + 2 * ((int64_t)g0 + lane), 2 * kWave, left > 0 ? (left + kWave - 1) / kWave : 0, tag, v[i],
                       &s_abort);
    }
#pragma unroll
    for (int i = 0; i < kFusedMaxIn; ++i) {
      if (i < n_in) {
        const FusedIn& in = ch.in[i];
        const float sr = v[i][0][0] + v[i][1][0];
        const float sx = v[i][0][1] + v[i][1][1];
        const float rn = sqrtf(group_sum<kWave>(sr)), xn = sqrtf(group_sum<kWave>(sx));
        const bool f = gate_fires(rn, xn, eps);
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
  };

  // ---- slow path of a chunk whose gate fired: rows of W of the fired inputs' maps ------------------------------
  // The image rows and residuals this phase reads were written by other workgroups: wait until every workgroup's
  // stores of the chunk have completed (they were issued long before, so this is short).
  auto slow_path = [&](int fc, unsigned fired_mask) {
    int lane = __lane_id();
    asm volatile("" : "+v"(lane));
    const int tid = wave * kWave + lane;
    const FusedChunk& ch = s_a.c[fc];
    const int n_in = uni(ch.n_in), n_mp = uni(ch.n_mp);
    ++fired_chunks;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane == 0) {
      const unsigned old = atomicAdd(&s_done, 1u);
      if (old == (unsigned)(kFusedWaves * fired_chunks - 1)) add_u32(&st->wg_done, 1u);
    }
    if (tid == 0) {
      const unsigned want = (unsigned)G * (unsigned)fired_chunks;
      const long long t0 = wall_clock64();
      while (ld_u32(&st->wg_done) - done0 < want && !s_abort)
        if (wall_clock64() - t0 > kSpinTicks) s_abort = 1u;
    }
    __syncthreads();
    const int GW = G * kFusedWaves, gw = b * kFusedWaves + wave;
    for (int gi = 0; gi < n_in; ++gi) {
      if (!((fired_mask >> gi) & 1u)) continue;  // uniform across the grid
      const FusedIn& in = ch.in[gi];
      const int dd = uni(in.d);
      const bool whole = uni(in.wx) != 0;  // y = W x (Algorithm 1, line 7) replaces y; else W r is added to M c
      int tid2 = wave * kWave + __lane_id();  // (recomputed: see the note on `lane` in the main loop)
      asm volatile("" : "+v"(tid2));
      if (whole) {
        const float* X = reinterpret_cast<const float*>(in.X);
        for (int idx = tid2; idx < dd; idx += kFusedBlock) xs[idx] = X[idx];
      } else {
        for (int idx = tid2; idx < dd; idx += 4 * kFusedBlock) {
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
      for (int j = 0; j < n_mp; ++j) {
        const FusedMap& mp = ch.mp[j];
        if (uni(mp.in) != gi) continue;  // uniform
        const int m = uni(mp.m);
        const S* W = reinterpret_cast<const S*>(mp.W);
        float* Y = mp.Y;
        if (tail) stream_map_rows<T, true, true>(W, Y, m, dd, dd, xs, whole, first, GW, lane);
        else stream_map_rows<T, false, true>(W, Y, m, dd, dd, xs, whole, first, GW, lane);
        first = (first - m % GW + GW) % GW;
      }
      __syncthreads();  // the staged vector is free again
    }
  };

  // Chunks run in order, and the exchanges of neighbouring chunks overlap: the operands of chunk ci + 1 are
  // requested as soon as phase 2 of chunk ci has consumed the registers, and the gate of chunk ci is decided
  // together with the coefficient exchange of chunk ci + 1 (its slow path, if the gate fired, then runs after
  // phase 2 of chunk ci + 1, when the registers are free again).  The norms travel in two sets of words, by
  // chunk parity, because a chunk's norms are still being read when the next chunk's are written.
  issue_loads(0);
  for (int ci = 0; ci < n_chunks; ++ci) {
    // (the lane number passes through an empty asm statement so that nothing derived from it is computed once
    // before the loop and then kept, or spilled, across this long body)
    int lane = __lane_id();
    asm volatile("" : "+v"(lane));
    const int tid = wave * kWave + lane;
    const FusedChunk& ch = s_a.c[ci];
    const unsigned tag = epoch0 + (unsigned)ci + 1u;
    const int k = uni(ch.k), lsh = uni(ch.lsh), n_in = uni(ch.n_in), NG = uni(ch.n_groups);
    const int lpr = 1 << lsh, rpw = kWave >> lsh;
    const int kshift = __builtin_ctz(k);
    const int cc = lane & (lpr - 1), rg = lane >> lsh;  // 16-byte chunk of the row, row of the load
    const bool bwg = b < NG;                            // basis workgroup: holds basis group b
    const bool bwave = bwg && wave < GI;                // holds an item of the group
    const bool iwave = wave != SW && !bwave;            // holds image rows

    // ---- phase 1: partial c of the item (fixed order: loads ascending, then the row groups of the wave),
    //      then of the group (waves ascending)
    if (bwave) {
      float acc[V];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        float w[V];
        T::widen(raw[q], w);
        const float x = h_row0 + q * rpw + rg < h_dlim ? xv[q] : 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] = fmaf(w[e], x, acc[e]);
      }
      for (int off = lpr; off < kWave; off <<= 1) {
#pragma unroll
        for (int e = 0; e < V; ++e)
          acc[e] += __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ off) << 2, __float_as_int(acc[e])));
      }
      if (cc == 0) {  // x is needed once more, by the lane that forms the row's residual: parked in LDS
#pragma unroll
        for (int q = 0; q < kFusedLoads; ++q) xsave[wave * kWave + q * rpw + rg] = xv[q];
      }
      if (rg == 0) {
#pragma unroll
        for (int e = 0; e < V; ++e) red[wave * k + cc * V + e] = acc[e];
      }
    }
    __syncthreads();
    if (bwg && tid < k) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < GI; ++w) s += red[w * k + tid];
      st64(pc + (int64_t)b * k + tid, pack(s, tag));
    }

    if (wave == SW) {
      // ---- reduce: this workgroup's columns of c, four neighbouring columns at a time, groups ascending per lane
      const int ncol = n_in << kshift;
      const int nquad = ch.wg_cols >> 2;
      for (int qi = 0; qi < nquad; ++qi) {
        const int cg = b * ch.wg_cols + 4 * qi;
        if (cg < ncol) {
          const int i = cg >> kshift, j = cg & (k - 1);
          const FusedIn& in = ch.in[i];
          const int P = in.n_groups;
          float v[2][4];
          const int left = P - lane;
          poll_words<2, 4>(pc + ((int64_t)in.group0 + lane) * k + j, (int64_t)kWave * k,
                           left > 0 ? (left + kWave - 1) / kWave : 0, tag, v, &s_abort);
          float s[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) s[c] = group_sum<kWave>(v[0][c] + v[1][c]);
          {  // lane -> (copy, column): 16 copies x 4 columns
            const int c4 = lane & 3;
            const float mine = c4 == 0 ? s[0] : c4 == 1 ? s[1] : c4 == 2 ? s[2] : s[3];
            st64(cslot + (int64_t)(lane >> 2) * kFusedMaxCols + cg + c4, pack(mine, tag));
            if (lane < 4) in.C[j + lane] = mine;
          }
        }
      }
      // ---- the gate of the previous chunk (its norms were published after its phase 2)
      if (ci > 0) gate_chunk(ci - 1, lane);
      // ---- the finished c of every input of the chunk -> LDS
      for (int s0 = lane; s0 < ncol; s0 += kWave * 16) {
        float v[16][1];
        const int left = ncol - s0;
        poll_words<16, 1>(cslot + (int64_t)(b % kCopies) * kFusedMaxCols + s0, kWave, (left + kWave - 1) / kWave, tag, v,
                          &s_abort);
#pragma unroll
        for (int q = 0; q < 16; ++q)
          if (s0 + q * kWave < ncol) cs[s0 + q * kWave] = v[q][0];
      }
    }
    __syncthreads();
    unsigned fired_prev = 0;  // the gate of chunk ci - 1
    if (ci > 0) {
      const int pn = uni(s_a.c[ci - 1].n_in);
      for (int i = 0; i < pn; ++i) fired_prev |= s_fired[i] << i;
      if (s_abort) fired_prev = 0;  // a wait expired: this launch's results are void, end it quickly
      fired_prev = (unsigned)uni((int)fired_prev);
    }

    // ---- phase 2: residual rows (basis waves) and image rows (image waves) out of the registers ----------
    if (bwave) {
      // (the registers pass through an empty asm statement: else the widened values of phase 1 are kept for
      // this phase, twice the registers the raw words take)
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) asm volatile("" : "+v"(raw[q].x), "+v"(raw[q].y), "+v"(raw[q].z), "+v"(raw[q].w));
      const FusedIn& in = ch.in[h_ii];
      float* R = uni(in.R);
      float cv[V];
      lds_vec<V>(cs + (h_ii << kshift) + cc * V, cv);
      float ar = 0.f, ax = 0.f;
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        float w[V];
        T::widen(raw[q], w);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) s = fmaf(w[e], cv[e], s);
        s = group_sum_rt(s, lpr);
        const int r = h_row0 + q * rpw + rg;
        if (r < h_dlim && cc == 0) {
          const float x = xsave[wave * kWave + q * rpw + rg];
          const float res = x - s;
          st_f32(R + r, res);
          ar = fmaf(res, res, ar);
          ax = fmaf(x, x, ax);
        }
      }
      ar = group_sum<kWave>(ar);
      ax = group_sum<kWave>(ax);
      if (lane == 0) {
        s_nred[wave][0] = ar;
        s_nred[wave][1] = ax;
      }
    } else if (iwave) {
      uint4 dq[kFusedLoads];
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) dq[q] = s_img[wave][q];  // (same address in every lane)
#pragma unroll
      for (int q = 0; q < kFusedLoads; ++q) {
        if (h_ub + q < h_ue) {  // uniform over the wave
          float* Y = reinterpret_cast<float*>(((unsigned long long)(unsigned)uni((int)dq[q].y) << 32) | (unsigned)uni((int)dq[q].x));
          const int row = uni((int)dq[q].z), m = uni((int)(dq[q].w & 0xffffffu)), in = uni((int)(dq[q].w >> 24));
          float w[V], cv[V];
          T::widen(raw[q], w);
          lds_vec<V>(cs + (in << kshift) + cc * V, cv);
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < V; ++e) s = fmaf(w[e], cv[e], s);
          s = group_sum_rt(s, lpr);
          const int r = row + rg;
          if (cc == 0 && r < m) st_f32(Y + r, s);
        }
      }
    }
    __syncthreads();
    if (bwg && tid < 2 * kCopies) {  // the group's |r|^2, |x|^2: waves ascending; thread -> (copy, which)
      const int which = tid & 1;
      float sn = 0.f;
#pragma unroll
      for (int w = 0; w < GI; ++w) sn += s_nred[w][which];
      st64(nslot + (((int64_t)(ci & 1) * kCopies + (tid >> 1)) * kFusedMaxGroups + b) * 2 + which, pack(sn, tag));
    }

    // the registers are free: the slow path of the previous chunk, if its gate fired (the common case: it did
    // not, and no byte of W is read), then the request for the next chunk's operands
    if (fired_prev != 0) slow_path(ci - 1, fired_prev);
    issue_loads(ci + 1);
  }

  // ---- the gate (and slow path) of the last chunk
  {
    int lane = __lane_id();
    asm volatile("" : "+v"(lane));
    if (wave == SW) gate_chunk(n_chunks - 1, lane);
    __syncthreads();
    unsigned fired_last = 0;
    const int pn = uni(s_a.c[n_chunks - 1].n_in);
    for (int i = 0; i < pn; ++i) fired_last |= s_fired[i] << i;
    if (s_abort) fired_last = 0;
    fired_last = (unsigned)uni((int)fired_last);
    if (fired_last != 0) slow_path(n_chunks - 1, fired_last);
  }

  // ---- the next launch gets fresh tags (see the note where the epoch is read)
  __syncthreads();
  if (wave == 0 && __lane_id() == 0) {
    if (s_abort) add_u32(&st->timeouts, 1u);
    if (b == 0) st_u32(&st->epoch, epoch0 + (unsigned)n_chunks);
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
  if (k % V || !pow2(k / V) || k / V > kWave || k / V < 8 || k > 512) return false;
  const int lpr = k / V, rpw = kWave / lpr;
  ch.lsh = __builtin_ctz(lpr);
  if ((int64_t)ch.n_in * k > kFusedMaxCols) return false;
  int64_t groups = 0, units = 0;
  for (int i = 0; i < ch.n_in; ++i) {
    ch.in[i].group0 = (int)groups;
    ch.in[i].n_groups = (int)ceil_div(ch.in[i].d, (int64_t)kFusedGroup * kFusedLoads * rpw);
    if (ch.in[i].n_groups > 2 * kWave) return false;  // a wave sums a column over at most two groups per lane
    groups += ch.in[i].n_groups;
  }
  for (int j = 0; j < ch.n_mp; ++j) {
    ch.mp[j].unit0 = (int)units;
    ch.mp[j].n_units = (int)ceil_div(ch.mp[j].m, rpw);
    units += ch.mp[j].n_units;
  }
  for (int j = 0; j < kFusedMaxMap; ++j) ch.unit0[j] = j < ch.n_mp ? ch.mp[j].unit0 : 0x7fffffff;
  if (groups > G || groups > kFusedMaxGroups || units > (1 << 28)) return false;
  ch.n_groups = (int)groups;
  ch.n_units = (int)units;
  ch.wg_cols = 4 * (int)ceil_div((int64_t)ch.n_in * k, 4 * (int64_t)G);
  if (ch.wg_cols / 4 > kFusedGroup) return false;
  // image waves: seven in a basis workgroup, fifteen in the others (the last wave of every workgroup holds
  // nothing: it serves the exchanges)
  const int64_t slots = groups * (kFusedWaves - 1 - kFusedGroup) + (G - groups) * (kFusedWaves - 1);
  ch.wave_units = slots > 0 ? (int)ceil_div(units, slots) : 0;
  if (units > 0 && (slots < 1 || ch.wave_units > kFusedLoads)) return false;
  return true;
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
  // cs | xsave | the larger of the group's partials [8][k] and the staged vector of the slow path
  const size_t smem = ((size_t)kFusedMaxCols + kFusedBlock + std::max<size_t>(maxd, (size_t)kFusedGroup * 512)) * sizeof(float);
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

