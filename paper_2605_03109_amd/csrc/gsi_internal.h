// Host-side declarations shared by the translation units of libgsi.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/gsi.h"

namespace gsi {

inline size_t elem_size(int dtype) { return dtype == GSI_BF16 ? 2 : 4; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- generic kernels: any shape, element-wise access ---------------------------------------------
hipError_t generic_build_image(const void* W, const void* U, void* M, int64_t m, int64_t d, int64_t k, int wdtype,
                               hipStream_t s);
hipError_t generic_build_gram(const void* U, int64_t d, int64_t k, int udtype, float* E, hipStream_t s);
hipError_t generic_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype,
                           float* C, float* R, float* rnorm, float* xnorm, hipStream_t s);
hipError_t generic_gated_linear(const void* W, const void* M, const float* C, const float* R,
                                const int32_t* fired_idx, const int32_t* n_fired, int64_t m, int64_t d, int64_t k,
                                int64_t B, int wdtype, float* Y, hipStream_t s, const void* X = nullptr,
                                int xdtype = 0);  // X: fired tokens get y = W x
hipError_t generic_dense_linear(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int wdtype,
                                int xdtype, float* Y, hipStream_t s);

// ---- the image in 8-bit floating point (gsi_fp8.hip) ---------------------------------------------------
hipError_t quantize_image_fp8(const void* M, int mdtype, int64_t m, int64_t k, uint8_t* M8, float* scale,
                              hipStream_t s);
// out[m,k] (out_dtype) = scale_i * value(M8[i,j])
hipError_t expand_image_fp8(const uint8_t* M8, const float* scale, int64_t m, int64_t k, void* out, int out_dtype,
                            hipStream_t s);

// ---- gate + stream compaction (one kernel for every shape) ----------------------------------------
hipError_t launch_gate(const float* rnorm, const float* xnorm, int64_t B, float eps, uint8_t* mask,
                       int32_t* fired_idx, int32_t* n_fired, hipStream_t s);

}  // namespace gsi
