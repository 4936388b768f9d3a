// Task tables and host entry points of the decode-time kernels (see gsi_decode.hip).
#pragma once
#include "gsi_internal.h"

namespace gsi {

constexpr int kMaxTasks = 8;        // tasks per launch (passed by value in the kernel arguments)
constexpr int kTokTile = 4;         // tokens processed together by the projection / image kernels
constexpr int kMaxSlabRows = 256;   // rows of U per workgroup, upper bound
constexpr int kTargetSlabs = 128;   // row slabs per input the slab height aims for
constexpr int kMaxK = 512;          // largest rank the vector projection kernels take
constexpr int kRowsPerBlock = 16;   // output rows per workgroup in the linear-map kernels
constexpr int kMaxLinD = 16384;     // floats of LDS the linear-map kernels may use for one vector

struct ProjTask {
  const void* U;
  const void* X;
  float* C;
  float* R;
  float* rnorm;
  float* xnorm;
  uint8_t* mask;       // gate outputs, used only when the gate is fused into the norm kernel
  int32_t* fired_idx;
  int32_t* n_fired;
  float* part_c;       // [nslab][B][k]
  float* part_n;       // [nslab][B][2]
  int d, k, nslab, slab_rows;
  int udtype, xdtype;
};

struct ProjBatch {
  ProjTask t[kMaxTasks];
  int blk_begin[kMaxTasks];
  int n, B;
};

struct LinTask {
  const void* W;
  const void* M;
  const float* C;
  const float* R;
  const void* X;       // dense baseline only
  const int32_t* fired_idx;
  const int32_t* n_fired;
  float* Y;
  int m, d, k, xdtype;
};

struct LinBatch {
  LinTask t[kMaxTasks];
  int blk_begin[kMaxTasks];
  int n, B;
};

// eligibility of the vector kernels for a shape / alignment (else the generic kernels run)
bool decode_project_ok(int64_t d, int64_t k, int udtype, const void* U);
bool decode_linear_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M);

int decode_slab_rows(int64_t d, int64_t k, int udtype);
size_t decode_project_ws(int64_t d, int64_t k, int64_t B, int udtype);
// fills d, k, slab geometry and the two workspace pointers of a task whose other fields are set
void decode_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws);

hipError_t decode_project_launch(ProjBatch& pb, int udtype, bool with_gate, float eps, hipStream_t s);
hipError_t decode_gated_launch(LinBatch& lb, int wdtype, hipStream_t s);
hipError_t decode_dense_launch(LinBatch& lb, int wdtype, hipStream_t s);

}  // namespace gsi
