// Host entry points of the rank-1 basis extension (gsi_extend.hip).
#pragma once
#include "gsi_internal.h"

namespace gsi {

struct ExtState {  // verdicts of one extension step, in the workspace
  int cand;        // the token is a candidate: |x| > 0, |r| / |x| >= tau, k < K
  int ext;         // ... and its re-orthogonalised residual does not vanish: the basis grows
  int kc;          // the column that is written
  float inv;       // 1 / |r2|
};

struct ExtMap {
  const void* W;   // [m, d]
  void* M;         // [m, K]
  int64_t m;
};

size_t extend_ws_bytes(int64_t d, int64_t K);
hipError_t extend_basis(void* U, int64_t d, int64_t K, int udtype, int32_t* k_cur, const float* R, const float* rnorm,
                        const float* xnorm, float tau, const ExtMap* maps, int n_maps, float* gram, int32_t* extended,
                        void* ws, hipStream_t s);

}  // namespace gsi
