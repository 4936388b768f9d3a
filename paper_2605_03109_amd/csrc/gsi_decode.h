// Task tables and host entry points of the decode-time kernels (gsi_project.hip, gsi_linear.hip).
//
// Every kernel is launched over a small table of tasks passed by value in the kernel arguments, so
// the projections of several inputs, or the linear maps of several weights, share one launch.
#pragma once
#include <vector>

#include "gsi_internal.h"

namespace gsi {

constexpr int kMaxTasks = 16;       // inputs (projection tasks, input groups of the linear kernels) per launch
constexpr int kMaxLinTasks = 24;    // maps (linear tasks, image tasks) per launch
constexpr int kTokTile = 4;         // tokens processed together by the projection / image kernels
constexpr int kColBlock = 64;       // columns of U per workgroup in the partial projection
constexpr int kPartSlabs = 32;      // row slabs of U per input in the partial projection, upper bound (= partials per c_j)
constexpr int kMaxResSlabs = 512;   // row slabs per input in the residual kernel, upper bound
constexpr int kMaxK = 512;          // largest rank the vector projection kernels take
constexpr int kRowsPerBlock = 16;   // output rows per workgroup in the batched-token linear kernels
constexpr int kMaxLinD = 16384;     // floats of LDS one activation vector may take in the linear kernels
constexpr int kMaxStreamD = 65536;  // longest input of the single-token weight-streaming kernels (blocks of kMaxLinD columns)
constexpr int kStageMaxRows = 2048; // rows of U per workgroup in the single-token staged kernel (their activations sit in LDS)
constexpr int kMaxSumK = 2048;      // floats of LDS all projection coefficients of a launch may take

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
  float* part_c;       // [a_slabs][B][k]  partial projections, one per row slab
  float* part_n;       // [b_slabs][B][2]  partial |r|^2, |x|^2, one per residual slab
  unsigned* sync;      // decode batch on the matrix cores: finished residual workgroups of this input
  int d, k;
  int a_rows, a_slabs, a_cblocks;  // partial projection: rows per slab, slabs, column blocks
  int b_rows, b_slabs;             // residual: rows per slab, slabs
  int udtype, xdtype;
  int tile;                        // decode batch on the matrix cores (gsi_tile.hip) with its own slab geometry
  int b_perm;                      // residual slabs per partial-projection slab when the residual launch walks its
                                   // slabs in the XCD order of the partial projection, else 0 (filled at launch)
  int s_rows, s_slabs;             // single token (gsi_stage.hip): rows per slab and slabs of the partial projection
};

struct ProjBatch {
  ProjTask t[kMaxTasks];
  int a_begin[kMaxTasks];  // first workgroup of each task in the partial-projection launch
  int b_begin[kMaxTasks];  // ... in the residual launch
  int n, B;
  int b_total;             // workgroups of the residual launch that are residual slabs
  int norms, gate;         // decode batch on the matrix cores: the residual launch finishes with the norms (+ gate)
  float eps;
};
static_assert(sizeof(ProjBatch) <= 4096, "kernel arguments are limited to 4 KB");

// One image map y = M c of a single-token launch (gsi_image.h)
struct ImgTask {
  const void* M;
  float* Y;
  const float* part_c;  // partial projections [a_slabs][1][k] of the map's input, or null ...
  const float* C;       // ... then the finished coefficients C[k]
  const float* scale;   // E4M3 image: row scales [m]; null for an image in the weights' dtype
  int m, k, a_slabs, blk_begin;
};

struct ImgBatch {
  ImgTask t[kMaxLinTasks];
  int n, total;         // tasks, workgroups
};

// One input group as seen by the linear kernels: its projection outputs and its gate.
struct LinGroup {
  const float* C;
  const float* R;
  const void* X;                 // dense baseline, and the W x form of the slow path (xdtype)
  const int32_t* fired_idx;
  const int32_t* n_fired;
  int wx;                        // fired tokens get y = W x (Algorithm 1, line 7) instead of M c + W r
  int d, k, xdtype;
  // single token, gate not yet published (a stack of one set of inputs leaves it to the weight kernel and saves a
  // launch): the residual launch's slab shares of the norms and where the gate's outputs go; else part_n is null
  int b_slabs;
  const float* part_n;
  float* rnorm;
  float* xnorm;
  uint8_t* mask;
  int32_t* fired_idx_out;
  int32_t* n_fired_out;
};

struct LinTask {
  const void* W;
  const void* M;
  float* Y;
  float* part;   // several-token matrix-core kernel: partial products [slices][B][m] of the weight term
  int m, group;
  int slices;    // ... column slices of the weight term (filled at launch)
};

struct LinBatch {
  LinGroup g[kMaxTasks];
  LinTask t[kMaxLinTasks];
  int blk_begin[kMaxLinTasks];     // several-token kernels: first workgroup of each task
  int blk_begin2[kMaxLinTasks];    // matrix-core kernel: first image-term workgroup of each task
  int tile_split;                  // ... first image-term workgroup of the launch
  int n, ng, B;
  int dense;                 // y = W x, no image term
  float eps;                 // for groups whose gate the single-token kernel evaluates itself
};
static_assert(sizeof(LinBatch) <= 4096, "kernel arguments are limited to 4 KB");

// eligibility of the vector kernels for a shape / alignment (else the generic kernels run)
bool decode_project_ok(int64_t d, int64_t k, int udtype, const void* U);
// (B: tokens of the call; a single token's kernels take inputs of up to kMaxStreamD elements, and so does a decode
// batch of 2..128 tokens whose shape the matrix-core kernel takes)
bool decode_linear_ok(int64_t m, int64_t d, int64_t k, int wdtype, const void* W, const void* M, int64_t B = 2);

size_t decode_project_ws(int64_t d, int64_t k, int64_t B, int udtype);
// fills d, k, slab geometry and the two workspace pointers of a task whose other fields are set
void decode_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws);

// partial projection + residual (+ norms, + gate): with_norms = false leaves the norms to the
// single-token linear kernel (which reads part_n itself)
// `img` (single token only): image maps whose workgroups ride in the residual launch
hipError_t decode_project_launch(ProjBatch& pb, int udtype, bool with_norms, bool with_gate, float eps,
                                 hipStream_t s, ImgBatch* img = nullptr);
// stand-alone image launch for one token: y = M c with c read from C (tasks' C set, part_c null)
hipError_t decode_image_launch(ImgBatch& ib, int wdtype, hipStream_t s);
// norms (and gate) of tasks whose part_n / b_slabs / rnorm / xnorm (mask, fired_idx, n_fired) are set
hipError_t decode_norms_launch(const ProjBatch& pb, bool with_gate, float eps, hipStream_t s);
// can a set of tasks share one single-token launch (LDS budget)?
// (wdtype: a decode batch whose maps all take the matrix-core kernel needs no LDS vector and always fits)
bool decode_linear_fits(const LinBatch& lb, int wdtype);
// e0 / e1 (optional): events that take the start / stop timestamps of the single-token kernel's dispatch
hipError_t decode_linear_launch(LinBatch& lb, int wdtype, hipStream_t s, hipEvent_t e0 = nullptr,
                                hipEvent_t e1 = nullptr);

// several tokens on the matrix cores (gsi_tile.hip): workspace of one map's partial products (0 when the
// shape does not take this path), eligibility of a filled batch, launch
size_t tile_part_bytes(int64_t m, int64_t d, int64_t B);
// ... and the projection of a decode batch: shape eligibility, workspace, geometry of a task, launches
bool tile_project_shape_ok(int64_t d, int64_t k, int64_t B, int udtype);
size_t tile_project_ws(int64_t d, int64_t k, int64_t B);
void tile_project_fill(ProjTask& t, int64_t d, int64_t k, int64_t B, void* ws);
hipError_t tile_project_launch(ProjBatch& pb, bool with_norms, bool with_gate, float eps, hipStream_t s);
bool tile_rows_shape_ok(int64_t m, int64_t d, int64_t k, int64_t B, int wdtype);
bool tile_rows_ok(const LinBatch& lb, int wdtype);
hipError_t tile_rows_launch(LinBatch& lb, hipStream_t s);

// ---- single token: projection, residual, image rows and gate as stages of one kernel (gsi_stage.hip) -------
// A launch carries up to five kinds of workgroups, each kind working on a different set of independent inputs:
// partial projections, the sums of the partials, residual slabs and image rows, gates.  Consecutive sets overlap
// and nothing inside a launch waits for anything else in it.
struct StagePart {        // partial projection c = U^T x of one input over row slabs
  const void* U;
  const void* X;
  float* part_c;          // [slabs][k]
  int d;
  int k_rows;             // k | rows per slab << 16
  int slabs_x;            // slabs | xdtype << 16 | column blocks << 20 (0 or 1: whole rows)
  int x2_off;             // single-pass gate: byte offset from part_c of the slab shares of |x|^2 (doubles); else 0
};

struct StageCRed {        // c = sum of the partials in fixed slab order, one workgroup per input ...
  const float* part_c;
  float* C;
  const float* E;         // ... or, single-pass gate (E = U^T U - I, [k][k] fp32): kGramBlocks workgroups per input,
                          //     each adds the partials, takes a block of rows of E and writes its share of c^T E c
                          //     to gw[slabs + block]; block 0 also writes C and |c|^2 to gw[slabs + kGramBlocks]
  int k_slabs;            // k | slabs << 16
  int gw_off;             // byte offset from part_c of the doubles gw
};
constexpr int kGramBlocks = 16;
// doubles of the single-pass gate per input: slab shares of |x|^2, block shares of c^T E c, shares of |c|^2.
// With this gate the partial projections are kept to double precision (a second array of low parts behind the
// first, [slabs][k] each): |x|^2 - |c|^2 cancels to 1/400 of either term at the threshold 0.05, and an error of c
// enters it in first order (the explicit residual feels it only in second order).
constexpr int kStageSlabs = 128;  // row slabs per input of the staged kernel when a sum stage adds the partials
constexpr int kC2Shares = 8;       // shares of |c|^2 (one per 64 columns)
constexpr int kGateDoubles = kStageSlabs + kGramBlocks + kC2Shares;

struct StageRes {         // r = x - U c, and the slab shares of |r|^2, |x|^2, of one input over row slabs
  const void* U;
  const void* X;
  const float* part_c;    // null: c is read from C; else c is the sum of these partials and slab 0 writes C
  float* C;
  float* R;
  float* part_n;          // [b_slabs][2]; unused with the single-pass gate
  int d;
  int k_rows;             // k | b_rows << 16
  int slabs_x;            // b_slabs | slabs of the partial projection << 16 | xdtype << 24
  int gate;               // bits 0-7: single-pass gate: 1 + index of this input's StageGate, evaluated by every
                          // residual workgroup (r is formed only if the gate fires); else 0.  bits 8-15: r > 0: the
                          // slabs are walked in the XCD order of the partial projection, r of them per partial slab
};

struct StageImg {         // image rows y = M c of one map
  const void* M;
  float* Y;
  const float* scale;     // E4M3 image: row scales; else null
  int m;                  // rows
  int blk_res;            // first workgroup | index of the input among the launch's StageRes << 24
};

struct StageGate {        // |r|, |x| from the slab shares and Eq. (gate) of one input
  const float* part_n;    // single-pass gate: the input's kGateDoubles doubles instead
  float* rnorm;
  float* xnorm;
  uint8_t* mask;
  int32_t* fired_idx;
  int32_t* n_fired;
  int b_slabs;            // single-pass gate: slabs of the partial projection
  int skip_fired_image;   // single-pass gate: image rows of this input are left to the weight kernel when it fires
};

struct StageArgs {
  StagePart a[kMaxTasks];
  StageCRed cr[kMaxTasks];
  StageRes b[kMaxTasks];
  StageImg im[kMaxLinTasks];
  StageGate g[kMaxTasks];
  int a_begin[kMaxTasks];  // first workgroup of each partial-projection task (relative to the role's first)
  int b_begin[kMaxTasks];
  int na, ncr, nb, ni, ng;
  int a_total, b_total, i_total;  // workgroups per role; grid order: residual slabs, partial projections, image
                                  // rows, coefficient sums and gates (one workgroup each; kGramBlocks per sum
                                  // with the single-pass gate, whose gates have no workgroups of their own)
  int gram;                       // the launch's inputs use the single-pass gate
  float eps;
};
static_assert(sizeof(StageArgs) <= 4096, "kernel arguments are limited to 4 KB");

// rows per slab and slabs of the single-token partial projection.  fine: slabs of at most 64 KB (up to kStageSlabs
// of them) for calls whose partials are added by a sum stage; else kPartSlabs slabs at most, because every
// residual and image workgroup then adds the partials itself
void stage_geom(int64_t d, int64_t k, int udtype, int& rows, int& slabs, bool fine = false);
void stage_clear(StageArgs& a, float eps);
// E (single-pass gate): the input's cached U^T U - I, else null
// ncb: column blocks (a power of two; k / ncb at least 64 columns): more, narrower workgroups for small calls
void stage_add_part(StageArgs& a, const ProjTask& t, const float* E = nullptr, int ncb = 1);
void stage_add_cred(StageArgs& a, const ProjTask& t, const float* E = nullptr);
// returns its index; single-pass gate: the residual workgroups evaluate and publish the gate themselves
int stage_add_res(StageArgs& a, const ProjTask& t, bool c_ready, const float* E = nullptr, bool skip_fired_image = false);
void stage_add_img(StageArgs& a, int res, const void* M, float* Y, const float* scale, int m);
// residual task `res` walks its slabs in the XCD order of the partial projection (r residual slabs per partial slab)
void stage_set_res_xcd_order(StageArgs& a, int res, int r);
void stage_add_gate(StageArgs& a, const ProjTask& t);
// e0 / e1 (optional): events that take the start / stop timestamps of the dispatch
hipError_t stage_launch(StageArgs& a, int dtype, hipStream_t s, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);

// ---- single token, many inputs, single-pass gate: the stages as three launches over a table in device memory ----
// A call with more inputs than one launch's arguments describe runs each stage ONCE for all its inputs: partial
// projections; coefficient sums with the shares of c^T E c; image rows and (behind the gate) residuals.  Launches
// that each move hundreds of megabytes amortise their fixed cost and their ramp and tail, which a pipeline of
// 16-input launches pays a dozen times.  The descriptors are uploaded like those of the weight-streaming launch.
struct TabIn {
  const void* U;
  const void* X;
  float* C;
  float* R;
  const float* E;
  float* rnorm;
  float* xnorm;
  uint8_t* mask;
  int32_t* fired_idx;
  int32_t* n_fired;
  float* part_c;         // [s_slabs][k], followed at gw_off bytes by the doubles of the single-pass gate
  int d;
  int k_rows;            // k | rows per slab of the partial projection << 16
  int slabs;             // slabs of the partial projection | residual slabs << 16
  int r_rows_x;          // rows per residual slab | xdtype << 16 | W x form of the slow path << 20
  int gw_off;
  int pad;
};
struct TabMap {          // everything an image workgroup needs, so that its loads of M wait for one table entry only
  const void* M;
  float* Y;
  const float* scale;    // E4M3 image: row scales; else null
  const float* C;        // the input's coefficients
  const double* gw;      // W x form of the slow path: the input's gate doubles (a fired input's rows are skipped); else null
  int m, k;              // rows, rank
  int slabs;             // slabs of the input's partial projection (layout of gw)
  int in;                // index of the input
};
constexpr int kTabImgItems = 8;   // items per image workgroup of the table launch (32 KB of M; 16 KB and 64 KB measured the same)
constexpr int kMaxTabIn = 1024, kMaxTabMaps = 2048;  // (the first-workgroup tables are searched in LDS)
size_t stage_table_bytes(int n_in, int n_maps);
struct StageTableGeom {   // what the host needs to launch over a table that is already in device memory
  int n_in, n_maps, dtype;
  int nt;                 // bases and images together exceed kStreamBytes: non-temporal loads
  int merge;              // the launch of the c^T E c shares adds the partial projections itself (few partials per
                          // input: no launch for the coefficient sums)
  int tp, tc, tr, ti;     // workgroups: partial projections, coefficient sums, residual slabs, image rows
  size_t off_maps, off_p, off_r, off_c, off_i;  // byte offsets of the sections of the table
};
// ins / maps: host arrays -> the table's bytes (host) and its geometry
hipError_t stage_table_build(const TabIn* ins, int n_in, const TabMap* maps, int n_maps, int dtype, std::vector<char>& host,
                             StageTableGeom& g);
// which_timed: 0, 1, 2 = the launch whose dispatch the events time, else -1
hipError_t stage_table_launch(const void* table, const StageTableGeom& g, float eps, hipStream_t s, int which_timed = -1,
                              hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);
// build + upload to `table` (device memory of stage_table_bytes(n_in, n_maps)) + launch
hipError_t stage_table_run(void* table, const TabIn* ins, int n_in, const TabMap* maps, int n_maps, int dtype, float eps,
                           hipStream_t s, int which_timed = -1, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);

// ---- single token, many inputs: weight streaming over a table in device memory (gsi_stream.hip) -----------
// One launch streams the rows of W of every fired input of a call, however many inputs and maps the call has.
// The descriptors do not fit the kernel arguments, so they are uploaded to the workspace first (by small kernels
// that copy their own arguments: no host-to-device copy is enqueued, which a captured graph would replay from
// host memory that no longer holds them).
struct FiredIn {
  const float* R;
  const void* X;               // W x form of the slow path (xdtype)
  const int32_t* n_fired;
  int d;
  int flags;                   // kFiredWx | xdtype << 1
  int map_begin, map_end;      // this input's maps in the table of FiredMap
};
constexpr int kFiredWx = 1;
struct FiredMap {
  const void* W;
  float* Y;
  int m, pad;
};
constexpr int kMaxFiredIn = 4096;  // inputs per launch (a flag per input in LDS)
size_t fired_table_bytes(int n_in, int n_maps);
// uploads `bytes` (a multiple of 16) from host memory `src` to device memory `dst` through kernel arguments
hipError_t upload_launch(const void* src, size_t bytes, void* dst, hipStream_t s);
// table: n_in FiredIn followed (at fired_table_bytes(n_in, 0)) by the FiredMap of all inputs, in device memory
hipError_t stream_fired_launch(const void* table, int n_in, const FiredIn* host_ins, const FiredMap* host_maps,
                               int wdtype, hipStream_t s, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);
// bytes one launch (or one step's fast path) must stream before its loads go non-temporal: twice the 256 MB
// memory-side cache, so that operands a caller walks again within a step or two keep their cache hits
constexpr size_t kStreamBytes = (size_t)512 << 20;
struct FiredGeom {        // launch shape of the weight-streaming kernel over a table in device memory
  int n_in, wdtype, tail;
  int nt;                 // non-temporal weight loads
  int long_d;             // an input is longer than kMaxLinD elements (staged a block of columns at a time)
  unsigned grid;
  size_t smem;
};
hipError_t stream_fired_geom(int n_in, const FiredIn* host_ins, const FiredMap* host_maps, int wdtype, FiredGeom& g);
hipError_t stream_fired_run(const void* table, const FiredGeom& g, hipStream_t s, hipEvent_t e0 = nullptr,
                            hipEvent_t e1 = nullptr);

// single-token persistent kernel (gsi_stream.hip)
size_t stream_smem_bytes(const LinBatch& lb);
hipError_t stream_rows_launch(LinBatch& lb, int wdtype, hipStream_t s, hipEvent_t e0 = nullptr,
                              hipEvent_t e1 = nullptr);

}  // namespace gsi
