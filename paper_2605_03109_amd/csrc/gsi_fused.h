// The fused single-token kernel of libgsi: Algorithm 1 for ONE token over a group of inputs and their maps in
// one launch (gsi_fused.hip).  Host-side description of a launch.
#pragma once
#include "gsi_internal.h"

namespace gsi {

constexpr int kFusedBlock = 1024;       // threads of a workgroup (16 waves), one workgroup per CU
constexpr int kFusedWaves = kFusedBlock / 64;
constexpr int kFusedLoads = 8;          // 16-byte loads per lane a wave holds in registers
constexpr int kFusedMaxIn = 4;          // inputs of a chunk
constexpr int kFusedMaxMap = 8;         // maps of a chunk
constexpr int kFusedMaxChunks = 4;      // chunks of a launch (the kernel arguments hold them by value)
constexpr int kFusedMaxCols = 2048;     // projection coefficients of a chunk (sum of k over its inputs)
constexpr int kFusedGroup = 8;          // items (= waves) whose partial results one workgroup combines
constexpr int kFusedMaxGroups = 512;    // basis groups of a chunk (one per workgroup at most)
constexpr int kFusedMaxD = 16384;       // floats of LDS the staged vector of the slow path may take

struct FusedIn {
  const void* U;
  const void* X;
  float* C;
  float* R;
  float* rnorm;
  float* xnorm;
  uint8_t* mask;
  int32_t* fired_idx;
  int32_t* n_fired;
  int d, xdtype, wx;
  int group0, n_groups;  // basis groups of this input: [group0, group0 + n_groups) of the chunk
  int pad;
};

struct FusedMap {
  const void* W;
  const void* M;
  float* Y;
  int m, in;
  int unit0, n_units;  // image units (one 16-byte load per lane: 64 / lanes-per-row rows) of this map
};

struct FusedChunk {
  FusedIn in[kFusedMaxIn];
  FusedMap mp[kFusedMaxMap];
  int n_in, n_mp;
  int k, lsh;       // rank (shared by the inputs of a chunk), log2 of the lanes that hold one row
  int n_groups;     // basis groups (kFusedGroup items each); workgroup g < n_groups holds group g
  int n_units;      // image units
  int wave_units;   // image units per image wave (<= kFusedLoads)
  int wg_cols;      // coefficients reduced by one workgroup (a multiple of 4)
  int unit0[kFusedMaxMap];  // first image unit of every map (copy of mp[].unit0, contiguous; INT_MAX past n_mp)
};

struct FusedArgs {
  FusedChunk c[kFusedMaxChunks];
  int n_chunks;
  float eps;
  int pad[2];
};
static_assert(sizeof(FusedArgs) % 16 == 0, "the kernel copies its arguments in 16-byte pieces");
static_assert(sizeof(FusedArgs) <= 4096, "kernel arguments are limited to 4 KB");

// Can this input / map take the fused kernel at all (dtype, rank, alignment)?
bool fused_input_ok(int64_t d, int64_t k, int udtype, const void* U, const void* X, int xdtype, const float* C,
                    const float* R, bool wx);
bool fused_map_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M);

// Completes the geometry of a chunk whose inputs and maps (pointers, d, m, in, wx, xdtype) and k are filled in.
// Returns false when the chunk exceeds what one launch can hold (registers, scratch); nothing is launched then.
bool fused_plan(FusedChunk& ch, int dtype);

// Launches the chunks of `a` (all of one storage dtype) on the current device.
// e0 / e1 (optional): events that take the start / stop timestamps of the kernel's dispatch.
hipError_t fused_launch(const FusedArgs& a, int dtype, hipStream_t s, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);

// Number of waits inside fused launches on the current device that ran into their time limit since the
// library was loaded (0 in normal operation).  Synchronises the device.
hipError_t fused_timeouts(unsigned* count);

// Device address and size of the general-purpose part of the library's static scratch array on the current
// device (used by the entry point that takes no workspace).
hipError_t static_workspace(void** ptr, size_t* bytes);

}  // namespace gsi
