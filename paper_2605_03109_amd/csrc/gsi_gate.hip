// Gate of Eq. (gate) / Algorithm 1 line 4 with order-preserving stream compaction on the device.
//
// One workgroup walks the B tokens in chunks of 1024.  Per chunk: every lane decides its token,
// wave ballots give the in-wave rank, a 16-entry LDS table gives the rank of the wave, and a running
// base carries the count across chunks.  The fired list therefore comes out in ascending token
// order without atomics, and the count is written last.
#include "gsi_device.h"
#include "gsi_internal.h"

namespace gsi {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / kWave;

__global__ __launch_bounds__(kBlock) void gate_kernel(const float* __restrict__ rnorm,
                                                      const float* __restrict__ xnorm, int64_t B, float eps,
                                                      uint8_t* __restrict__ mask, int32_t* __restrict__ fired_idx,
                                                      int32_t* __restrict__ n_fired) {
  __shared__ int wave_count[kWaves];
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  int base = 0;
  for (int64_t t0 = 0; t0 < B; t0 += kBlock) {
    const int64_t t = t0 + threadIdx.x;
    bool fired = false;
    if (t < B) {
      const float xn = xnorm[t], rn = rnorm[t];
      // fast path iff rho < eps; x = 0 never fires.  IEEE division, so both sides of a parity check
      // see the same ratio up to fp32 rounding of the norms.
      fired = (xn > 0.f) && (rn / xn >= eps);
      mask[t] = fired ? 1 : 0;
    }
    const unsigned long long ballot = __ballot(fired);
    const int rank_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_count[wave] = __popcll(ballot);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const int c = wave_count[w];
      if (w < wave) before += c;
      total += c;
    }
    if (fired) fired_idx[base + before + rank_in_wave] = (int32_t)t;
    base += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) n_fired[0] = base;
}

}  // namespace

hipError_t launch_gate(const float* rnorm, const float* xnorm, int64_t B, float eps, uint8_t* mask,
                       int32_t* fired_idx, int32_t* n_fired, hipStream_t s) {
  gate_kernel<<<1, kBlock, 0, s>>>(rnorm, xnorm, B, eps, mask, fired_idx, n_fired);
  return hipGetLastError();
}

}  // namespace gsi
