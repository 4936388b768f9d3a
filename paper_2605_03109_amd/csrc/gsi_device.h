// Device-side helpers shared by the HIP kernels of libgsi (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gsi {

constexpr int kWave = 64;

// ---- storage formats -------------------------------------------------------------------------
// bfloat16 is the upper half of an IEEE binary32 word: widening is a shift, exact.
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct F32 {
  using storage = float;
  static constexpr int kVec = 4;  // elements per 16-byte load
  __device__ static __forceinline__ float load(const float* p, int64_t i) { return p[i]; }
  __device__ static __forceinline__ void store(float* p, int64_t i, float v) { p[i] = v; }
  // 16-byte vector load of kVec consecutive elements
  __device__ static __forceinline__ void load_vec(const float* p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  // widen 16 raw bytes (as loaded) to kVec floats
  __device__ static __forceinline__ void widen(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
};

struct BF16 {
  using storage = uint16_t;
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const uint16_t* p, int64_t i) { return bf16_bits_to_f32(p[i]); }
  __device__ static __forceinline__ void store(uint16_t* p, int64_t i, float v) { p[i] = f32_to_bf16_bits(v); }
  __device__ static __forceinline__ void load_vec(const uint16_t* p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
  __device__ static __forceinline__ void widen(const uint4& v, float (&f)[8]) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
};

// OCP E4M3 bytes (images only): the hardware conversion widens two codes of a 32-bit word at a time, exactly.
struct FP8 {
  using storage = uint8_t;
  static constexpr int kVec = 16;
  __device__ static __forceinline__ void widen(const uint4& v, float (&f)[16]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[q], false);
      const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[q], true);
      f[4 * q + 0] = lo[0]; f[4 * q + 1] = lo[1];
      f[4 * q + 2] = hi[0]; f[4 * q + 3] = hi[1];
    }
  }
};

// 16 bytes that are read once and not again soon (a streamed operand): a non-temporal load, which the caches
// may drop first
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// activation element of runtime dtype (0 = fp32, 1 = bf16)
__device__ __forceinline__ float load_act(const void* p, int dtype, int64_t i) {
  return dtype == 0 ? reinterpret_cast<const float*>(p)[i]
                    : bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(p)[i]);
}

// ---- cross-lane reductions ---------------------------------------------------------------------
// Sums over aligned groups of `width` consecutive lanes (width a power of two <= 64); every lane of a
// group ends with the group's total.  Steps inside a row of 16 lanes are DPP adds (no LDS round
// trip); rows are combined through four lane reads.  The order of additions is fixed, so results
// are identical run to run and between kernels.
template <int ctrl>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, false));
}

// Branch-free for a run-time width: every step is executed, steps beyond the width add zero.
__device__ __forceinline__ float group_sum_rt(float v, int width) {
  float t;
  t = dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
  v += width >= 2 ? t : 0.f;
  t = dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2
  v += width >= 4 ? t : 0.f;
  t = dpp_move<0x141>(v);  // row_half_mirror: lane i <-> 7 - i of each half row
  v += width >= 8 ? t : 0.f;
  t = dpp_move<0x140>(v);  // row_mirror: lane i <-> 15 - i of each row
  v += width >= 16 ? t : 0.f;
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  const float lo = r0 + r1, hi = r2 + r3;
  const float half = (threadIdx.x & 32) ? hi : lo;
  return width >= 64 ? lo + hi : (width >= 32 ? half : v);
}

template <int width>
__device__ __forceinline__ float group_sum(float v) {
  return group_sum_rt(v, width);
}

// ---- gate -----------------------------------------------------------------------------------------
// fast path iff rho < eps (Algorithm 1, line 4); x = 0 never fires.  IEEE division and square root.
__device__ __forceinline__ bool gate_fires(float rnorm, float xnorm, float eps) {
  return (xnorm > 0.f) && (rnorm / xnorm >= eps);
}

// Sums over the residual kernel's slab shares part_n[slab][B][2] of token t: lane l adds slabs
// l, l + 64, ... in order, then a butterfly over the wave.  Every lane gets both sums; the order
// depends on nslab only, so every kernel that calls this gets the same bits.
// per-lane part of the sums below (lets a caller put the loads of several inputs in flight together)
__device__ __forceinline__ void wave_norm_partial(const float* __restrict__ part_n, int nslab, float& ar, float& ax) {
  const int lane = threadIdx.x % kWave;
  ar = 0.f;
  ax = 0.f;
  for (int s = lane; s < nslab; s += kWave) {
    const float2 v = *reinterpret_cast<const float2*>(part_n + (int64_t)s * 2);
    ar += v.x;
    ax += v.y;
  }
}

__device__ __forceinline__ void wave_norm_sums(const float* __restrict__ part_n, int nslab, int B, int t, float& sr,
                                               float& sx) {
  const int lane = threadIdx.x % kWave;
  float ar = 0.f, ax = 0.f;
  for (int s = lane; s < nslab; s += kWave) {
    const float2 v = *reinterpret_cast<const float2*>(part_n + ((int64_t)s * B + t) * 2);
    ar += v.x;
    ax += v.y;
  }
  sr = group_sum<kWave>(ar);
  sx = group_sum<kWave>(ax);
}

}  // namespace gsi
