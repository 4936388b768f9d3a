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

struct ExtIn {  // one basis of a call
  void* U;               // [d, K]
  const float* R;        // [d] residual of the token against the current basis
  const float* rnorm;    // [1]
  const float* xnorm;    // [1]
  int32_t* k_cur;        // [1] columns in use
  int32_t* extended;     // [1] or null
  float* gram;           // [K, K] or null
  char* ws;              // extend_ws_bytes(d, K) bytes of this basis' own
  int64_t d, K;
  int slabs, rows_per_slab, wgs, uvec;  // geometry (extend_fill)
};

struct ExtMapRec {  // one map that reads a basis of the call
  const void* W;  // [m, d]
  void* M;        // [m, K]
  int64_t m;
  int in;         // index of its basis in the call
  int vec;        // rows of W take 16-byte loads (extend_fill_map)
};

size_t extend_ws_bytes(int64_t d, int64_t K);
// bytes of the record table of a call with n bases and n_maps maps (0 for one basis: its record travels in the
// kernel arguments)
size_t extend_table_bytes(int n, int n_maps);
void extend_fill(ExtIn& in, int udtype);
void extend_fill_map(ExtMapRec& mp, int64_t d, int udtype);
// One extension step of n bases of one storage type (maps: all their maps, in any order).  table: device memory of
// extend_table_bytes(n, n_maps) bytes, 256-byte aligned (unused for n == 1).
hipError_t extend_many(const ExtIn* in, int n, const ExtMapRec* maps, int n_maps, int udtype, float tau, void* table,
                       hipStream_t s);

}  // namespace gsi
