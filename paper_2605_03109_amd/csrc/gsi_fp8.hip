// The cached image in 8-bit floating point (Section 7, "Combination with quantization": half the bytes on the
// fast path).  A one-time step after the image build, not a hot kernel: one wave per row finds the row's
// largest magnitude, takes the smallest power of two that brings it to at most 448 (the largest E4M3 value) and
// writes the E4M3 code nearest to every scaled element, ties to the even code.  Scaling by a power of two is
// exact, so the codes depend on the stored image alone.
#include <algorithm>

#include "gsi_device.h"
#include "gsi_internal.h"

namespace gsi {
namespace {

constexpr int kBlock = 256;
constexpr int kRowsPerBlock = kBlock / kWave;

// E4M3 code of t (|t| <= 448 or NaN): sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0 is
// subnormal (multiples of 2^-9), S.1111.111 is NaN, there is no infinity.
__device__ __forceinline__ uint32_t e4m3_code(float t) {
  const uint32_t u = __float_as_uint(t);
  const uint32_t sign = (u >> 24) & 0x80u;
  const uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return 0x7fu;                    // NaN
  if (a >= 0x43e00000u) return sign | 0x7eu;            // 448 and beyond: the largest finite code
  if (a < 0x3c800000u) {                                // below 2^-6: subnormal codes, steps of 2^-9
    const float r = rintf(__uint_as_float(a) * 512.0f); // exact product, round half to even: 0 .. 8 (8 = 2^-6)
    return sign | (uint32_t)r;
  }
  // normal: keep 3 mantissa bits, round half to even on the 20 dropped ones; a carry walks into the exponent
  uint32_t q = a >> 20;
  const uint32_t rem = a & 0xfffffu;
  q += (rem > 0x80000u || (rem == 0x80000u && (q & 1u))) ? 1u : 0u;
  return sign | (q - (120u << 3));                      // exponent bias 127 -> 7
}

template <class T>
__global__ __launch_bounds__(kBlock) void quantize_rows(const typename T::storage* __restrict__ M, int64_t m, int64_t k,
                                                        uint8_t* __restrict__ M8, float* __restrict__ scale) {
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kWave;
  if (row >= m) return;  // whole waves leave; there is no barrier below
  const typename T::storage* src = M + row * k;
  float amax = 0.f;
  for (int64_t j = lane; j < k; j += kWave) {
    const float v = fabsf(T::load(src, j));
    amax = (v > amax && v <= 3.4028234663852886e38f) ? v : amax;  // elements that are not finite take no part
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) {
    const float other = __shfl_xor(amax, o, kWave);
    amax = other > amax ? other : amax;
  }
  // amax = g * 2^q, 1 <= g < 2: the scale exponent is q - 8 when g <= 1.75 and q - 7 otherwise
  int e = 0;
  if (amax > 0.f) {
    int q;
    const float g = frexpf(amax, &q);                    // g in [0.5, 1)
    e = (g <= 0.875f) ? q - 9 : q - 8;
    e = e < -126 ? -126 : (e > 127 ? 127 : e);
  }
  if (lane == 0) scale[row] = __uint_as_float((uint32_t)(e + 127) << 23);
  uint8_t* dst = M8 + row * k;
  for (int64_t j = lane; j < k; j += kWave) {
    // two exact power-of-two factors: a single one would leave the normal range for large |e|
    const int e1 = -e / 2, e2 = -e - e1;
    const float t = T::load(src, j) * __uint_as_float((uint32_t)(e1 + 127) << 23) * __uint_as_float((uint32_t)(e2 + 127) << 23);
    dst[j] = (uint8_t)e4m3_code(t);
  }
}

// out[i,j] = scale_i * value(M8[i,j]) in the weights' storage type (exact: a 4-bit significand times a power of
// two, unless a row scale below 2^-117 pushes it under the normal range).  Used by calls of several tokens, whose
// kernels read the image as a matrix-core operand in the weights' type.
template <class T>
__global__ __launch_bounds__(kBlock) void expand_rows(const uint8_t* __restrict__ M8, const float* __restrict__ scale,
                                                      int64_t m, int64_t k, typename T::storage* __restrict__ out) {
  const int64_t n = m * k;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < n; e += (int64_t)gridDim.x * kBlock) {
    const auto pair = __builtin_amdgcn_cvt_pk_f32_fp8((int)M8[e], false);
    T::store(out, e, pair[0] * scale[e / k]);
  }
}

}  // namespace

hipError_t expand_image_fp8(const uint8_t* M8, const float* scale, int64_t m, int64_t k, void* out, int out_dtype,
                            hipStream_t s) {
  const unsigned blocks = (unsigned)std::min<int64_t>(ceil_div(m * k, kBlock), 8192);
  if (out_dtype == GSI_BF16)
    expand_rows<BF16><<<blocks, kBlock, 0, s>>>(M8, scale, m, k, reinterpret_cast<uint16_t*>(out));
  else
    expand_rows<F32><<<blocks, kBlock, 0, s>>>(M8, scale, m, k, reinterpret_cast<float*>(out));
  return hipGetLastError();
}

hipError_t quantize_image_fp8(const void* M, int mdtype, int64_t m, int64_t k, uint8_t* M8, float* scale,
                              hipStream_t s) {
  const unsigned blocks = (unsigned)ceil_div(m, kRowsPerBlock);
  if (mdtype == GSI_BF16)
    quantize_rows<BF16><<<blocks, kBlock, 0, s>>>(reinterpret_cast<const uint16_t*>(M), m, k, M8, scale);
  else
    quantize_rows<F32><<<blocks, kBlock, 0, s>>>(reinterpret_cast<const float*>(M), m, k, M8, scale);
  return hipGetLastError();
}

}  // namespace gsi
