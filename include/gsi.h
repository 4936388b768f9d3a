/*
 * gsi.h -- C ABI of libgsi: the gated subspace linear layer on one AMD MI355X (gfx950).
 *
 * The operation (paper, Section 3 "The gated residual passthrough" and Section 4, Algorithm 1):
 * an activation x in R^d is split by an orthonormal basis U in R^{d x k} (the paper's V_k) into
 *      c = U^T x          (the paper's g)                       Eq. (decompose), Alg. 1 line 1
 *      r = x - U c                                              Eq. (decompose), Alg. 1 line 2
 *      rho = |r| / |x|                                          Eq. (gate),      Alg. 1 line 3
 * and a linear map y = W x, W in R^{m x d}, is evaluated through the cached image M = W U as
 *      y = M c                      when rho <  eps  (fast path: k columns are read)
 *      y = M c + W r  ( = W x )     when rho >= eps  (gate fires; Eq. (exact))
 *
 * Conventions common to every call
 *   - All matrices are dense, row-major and contiguous:  W[m,d]  U[d,k]  M[m,k]  X[B,d]  C[B,k]
 *     R[B,d]  Y[B,m]; B is the number of tokens in the call, tokens are independent.
 *   - EVERY pointer argument is a DEVICE pointer (HBM of the current HIP device) unless the comment
 *     says "host".  The caller owns every buffer, including the scratch workspace `ws`, whose
 *     minimum size is returned by gsi_workspace_bytes(); the library allocates nothing, frees
 *     nothing and keeps no state apart from a thread-local error string.
 *   - Storage dtypes (enum below): weights, images and bases share `wdtype`; activations have
 *     `xdtype`.  c, r, norms and y are always fp32; all accumulation is fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call only enqueues
 *     work: it never synchronises and never reads a device result on the host (the fired-token
 *     count stays in device memory).  Calls on one stream execute in order.
 *   - Return value: GSI_OK (0) or a negative gsi error code; gsi_last_error() then describes it.
 *     Arguments are validated on the host before anything is launched; on error nothing was enqueued.
 *   - B == 0 is a valid no-op.  Shapes must satisfy 1 <= k <= d, m >= 1.  Pointers must be aligned
 *     to their element size; shapes/pointers that additionally allow 16-byte vector access take the
 *     fast kernels, everything else a slower generic kernel with the same results up to rounding order.
 *   - What the fast kernels take (measured: the generic ones are 3x to 30x slower): 16-byte aligned pointers;
 *     a rank of 8 * 2^j columns in bf16 (8 .. 512), 4 * 2^j in fp32 (another rank: pad U and M with zero columns
 *     up to such a rank, which changes no result); inputs of up to 65536 elements, a multiple
 *     of 8 (bf16) / 4 (fp32), for one token per call; for 2 .. 128 tokens per call bf16 storage, fp32
 *     activations, d a multiple of 128, k a multiple of 64 (else the vector kernels up to d = 16384, d a
 *     multiple of 32 for the maps); more than 128 tokens: bf16 storage, d and k multiples of 64.
 */
#ifndef GSI_H
#define GSI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum gsi_status {
  GSI_OK = 0,
  GSI_ERR_NULL = -1,      /* a required pointer is NULL                               */
  GSI_ERR_SHAPE = -2,     /* k < 1, k > d, m < 1, B < 0, bad descriptor index, ...    */
  GSI_ERR_DTYPE = -3,     /* unknown or unsupported dtype code                        */
  GSI_ERR_ALIGN = -4,     /* pointer not aligned to its element size                  */
  GSI_ERR_WORKSPACE = -5, /* ws is NULL or smaller than gsi_workspace_bytes()         */
  GSI_ERR_HIP = -6        /* the HIP runtime refused a launch                         */
};

enum gsi_dtype { GSI_F32 = 0, GSI_BF16 = 1 };
/* storage of a quantised image only (gsi_quantize_image_fp8, GSI_MAP_IMAGE_FP8); never a wdtype/xdtype */
enum { GSI_FP8_E4M3 = 2 };

/* selector for gsi_workspace_bytes() */
enum gsi_call {
  GSI_CALL_BUILD_IMAGE = 0,
  GSI_CALL_PROJECT = 1,
  GSI_CALL_GATE = 2,
  GSI_CALL_GATED_LINEAR = 3,
  GSI_CALL_DENSE_LINEAR = 4,
  GSI_CALL_LAYER_STACK = 5
};

/* One-time image build, M = W U (Eq. (exact); Section 4 "Storage": computed once per weight and
 * kept beside W).  W[m,d], U[d,k] in `wdtype`; M[m,k] written in `wdtype` (one rounding of the fp32
 * accumulator when bf16).  ws: gsi_workspace_bytes(GSI_CALL_BUILD_IMAGE, m, d, k, 0). */
int gsi_build_image(const void* W, const void* U, void* M, int64_t m, int64_t d, int64_t k, int wdtype,
                    void* ws, size_t ws_bytes, void* stream);

/* One-time companion of a basis for GSI_INPUT_GATE_SINGLE_PASS: E[k,k] (fp32, row-major) = U^T U - I, the
 * departure of the STORED basis U[d,k] (`udtype`) from orthonormality (Definition "Activation basis and residual
 * ratio" assumes V_k^T V_k = I; storage rounding breaks it by about 1e-3 in bf16).  Accumulated in fp64, rounded
 * once to fp32.  Any shape with 1 <= k <= d; no workspace. */
int gsi_build_gram(const void* U, int64_t d, int64_t k, int udtype, float* E, void* stream);

/* The cached image in 8-bit floating point (Section 7 "Combination with quantization": half the fast-path
 * bytes).  The paper names no format; this library stores OCP E4M3 codes (1 sign, 4 exponent bits with bias 7,
 * 3 mantissa bits, largest finite value 448, no infinities) with one power-of-two scale per output row:
 *   scale[i] = the smallest 2^e (e in [-126, 127]) with max_j |M[i,j]| / 2^e <= 448, 1 for a zero row;
 *   M8[i,j]  = the E4M3 code nearest to M[i,j] / scale[i], ties to the even code (the division is exact).
 * M[m,k] in `mdtype` (GSI_F32 or GSI_BF16: an image as gsi_build_image wrote it), M8[m,k] bytes, scale[m] fp32.
 * NaN elements give the NaN code 0x7F.  No workspace. */
int gsi_quantize_image_fp8(const void* M, int mdtype, int64_t m, int64_t k, uint8_t* M8, float* scale, void* stream);

/* Projection, residual and the two norms of Algorithm 1 lines 1-3 for B tokens.
 * U[d,k] in `udtype`, X[B,d] in `xdtype`.  Outputs (fp32): C[B,k] = X U, R[B,d] = X - C U^T (formed
 * explicitly), rnorm[B] = |r_t|_2, xnorm[B] = |x_t|_2.  ws: GSI_CALL_PROJECT with (m ignored). */
int gsi_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype,
                float* C, float* R, float* rnorm, float* xnorm, void* ws, size_t ws_bytes, void* stream);

/* Gate of Eq. (gate) / Algorithm 1 line 4 with on-device stream compaction.
 * fired_t = (xnorm_t > 0) and (rnorm_t / xnorm_t >= eps)   [fast path iff rho < eps].
 * mask[B] (1 = fired), fired_idx[0..n_fired) = fired token indices in ascending order (entries past
 * n_fired are left untouched; the buffer must hold B ints), n_fired[0] = their count. */
int gsi_gate(const float* rnorm, const float* xnorm, int64_t B, float eps, uint8_t* mask,
             int32_t* fired_idx, int32_t* n_fired, void* stream);

/* Gated linear map: Y[t,:] = M C[t,:] for every token, plus W R[t,:] for t in fired_idx[0..n_fired).
 * Tokens that did not fire never touch W; when n_fired == 0 no byte of W is read.  W[m,d], M[m,k]
 * in `wdtype`; C, R fp32; fired_idx / n_fired are the device outputs of gsi_gate; Y[B,m] fp32
 * (`ydtype` must be GSI_F32).  ws: GSI_CALL_GATED_LINEAR (partial products of the several-token kernels).
 * Arithmetic by call size (bf16 weights): one token -- fp32 FMA on widened weights; 2..128 tokens -- MFMA
 * with c and r fed as bf16 head + tail (nothing rounded to 8 bits); more than 128 tokens -- MFMA GEMM with
 * c as head + tail and r rounded once to bf16 (its term is scaled by the residual ratio). */
int gsi_gated_linear(const void* W, const void* M, const float* C, const float* R, const int32_t* fired_idx,
                     const int32_t* n_fired, int64_t m, int64_t d, int64_t k, int64_t B, int wdtype, void* Y,
                     int ydtype, void* ws, size_t ws_bytes, void* stream);

/* Dense baseline Y[t,:] = W X[t,:] (what the method is measured against; Section 3.1 "standard
 * linear-layer computation").  Same kernels as the fired path of gsi_gated_linear.  Y fp32.
 * ws: GSI_CALL_DENSE_LINEAR (0 bytes for a single token). */
int gsi_dense_linear(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int wdtype, int xdtype,
                     float* Y, void* ws, size_t ws_bytes, void* stream);

/* Online basis maintenance: one DGKS rank-1 extension of a basis of fixed capacity, with the matching append to the
 * cached images (Section 5.3 "The cascade initialization", Section 5.4 "Time-dimension tracking": a token whose
 * residual ratio exceeds a threshold extends the basis by one orthonormal vector; Section 7 "Online basis
 * adaptation").  The paper gives no threshold, capacity or eviction rule; here the basis lives in U[d,K] (`udtype`)
 * whose columns from k on are ZERO (a zero column changes neither c, r nor y, so every other call runs on it
 * unchanged at rank K; the vector kernels and plans take ranks of 8 * 2^j columns in bf16, 4 * 2^j in fp32, so pick
 * K among those), k_cur[0] is a device counter of the columns in use, and nothing is ever evicted.
 * Inputs: the residual R[d], rnorm[1], xnorm[1] of ONE token against the current basis, as gsi_project or
 * gsi_layer_stack wrote them (with GSI_INPUT_GATE_SINGLE_PASS, R exists only for a token that fired).
 *   candidate iff xnorm > 0, rnorm / xnorm >= tau (compared like the gate) and k_cur < K;
 *   s = U^T r, r2 = r - U s (classical Gram-Schmidt's re-orthogonalisation pass); if |r2| > 0:
 *   column k_cur of U = r2 / |r2| rounded to `udtype`; for each map, column k_cur of M[m,K] = W u for the STORED u
 *   (rounded to `udtype`, which must also be the maps' dtype), so that M = W U keeps holding (Eq. (exact));
 *   if `gram` (the E[K,K] of gsi_build_gram) is not NULL its row and column k_cur become U^T u - e_k;
 *   k_cur[0] += 1.  extended[0] (may be NULL) = 1 if the basis grew, else 0.
 * Everything is decided on the device; a token that does not extend the basis costs a few empty launches and no pass
 * over U or W.  maps: HOST array.  ws: gsi_extend_basis_workspace_bytes(d, K).  The cascade of Section 5.3 is this
 * call on a basis array that was initialised with the previous layer's columns. */
typedef struct gsi_extend_map {
  const void* W;      /* [m,d] udtype */
  void* M;            /* [m,K] udtype; column k_cur is written */
  int64_t m;
} gsi_extend_map;
int gsi_extend_basis(void* U, int64_t d, int64_t K, int udtype, int32_t* k_cur, const float* R, const float* rnorm,
                     const float* xnorm, float tau, const gsi_extend_map* maps, int32_t n_maps, float* gram,
                     int32_t* extended, void* ws, size_t ws_bytes, void* stream);
size_t gsi_extend_basis_workspace_bytes(int64_t d, int64_t K);

/* The same step for n bases in ONE set of launches (Section 5.4 "Time-dimension tracking": every basis of a model
 * sees every token).  Each basis is extended exactly as gsi_extend_basis would extend it, bit for bit, on its own
 * verdict; a token after which no basis grows costs seven nearly empty launches for the whole call instead of seven
 * per basis.  descs: HOST array, one entry per basis with the arguments of gsi_extend_basis (maps: HOST array of
 * n_maps entries, may be NULL when n_maps is 0; gram and extended may be NULL); all bases of a call share one
 * udtype; n <= 65535 and at most 65535 maps in all.  tau as in gsi_extend_basis, one value for the call.
 * ws: gsi_extend_many_workspace_bytes(descs, n) bytes, 256-byte aligned (the call copies its descriptor table there).
 * Two bases of one call must not share U, k_cur, maps' M or gram. */
typedef struct gsi_extend_desc {
  void* U;                     /* [d,K] udtype, columns k_cur.. zero                      */
  int64_t d, K;
  int32_t udtype;
  int32_t n_maps;
  int32_t* k_cur;              /* device, [1]                                              */
  const float* R;              /* device, [d]: residual of the token against this basis    */
  const float* rnorm;          /* device, [1]                                              */
  const float* xnorm;          /* device, [1]                                              */
  const gsi_extend_map* maps;  /* HOST array of the maps that read this basis              */
  float* gram;                 /* device, [K,K] or NULL                                    */
  int32_t* extended;           /* device, [1] or NULL                                      */
} gsi_extend_desc;
int gsi_extend_many(const gsi_extend_desc* descs, int32_t n, float tau, void* ws, size_t ws_bytes, void* stream);
size_t gsi_extend_many_workspace_bytes(const gsi_extend_desc* descs, int32_t n);

/* Descriptors for gsi_layer_stack (host structs holding device pointers). */
typedef struct gsi_input_desc {
  const void* U;      /* basis of this input, [d,k], udtype                                     */
  const void* X;      /* tokens [B,d], xdtype; when src_map >= 0 this must be maps[src_map].Y   */
  int64_t d, k;
  int32_t udtype, xdtype;
  float* C;           /* outputs of the projection, as in gsi_project                           */
  float* R;
  float* rnorm;
  float* xnorm;
  uint8_t* mask;      /* outputs of the gate, as in gsi_gate                                    */
  int32_t* fired_idx;
  int32_t* n_fired;
  int32_t src_map;    /* -1: X is an external buffer; j >= 0: X is the output Y of maps[j]      */
  int32_t flags;      /* 0, or a combination of the GSI_INPUT_* flags below                     */
  const float* gram;  /* [k,k] fp32, E = U^T U - I from gsi_build_gram; read only with           */
                      /* GSI_INPUT_GATE_SINGLE_PASS, may be NULL otherwise                       */
} gsi_input_desc;

/* gsi_input_desc.flags.  By default a fired token gets y = M c + W r (Eq. (exact)).  With
 * GSI_INPUT_SLOW_PATH_WX the maps of this input give a fired token y = W x instead, the slow path as
 * Algorithm 1 (line 7) prints it: equal in exact arithmetic, but free of the stored image's rounding, so
 * that a fired token equals the dense product of gsi_dense_stack.  Tokens that did not fire are not
 * affected.  gsi_gated_linear has no x and always uses the default form. */
enum { GSI_INPUT_SLOW_PATH_WX = 1, GSI_INPUT_FUSED_KERNEL = 2, GSI_INPUT_GATE_SINGLE_PASS = 4 };

/* GSI_INPUT_GATE_SINGLE_PASS (single-token calls, B == 1, on the vector kernels; otherwise ignored and the
 * residual is formed as usual): the residual ratio of Eq. (rho) is evaluated in ONE pass over the basis.  For
 * c = U^T x and any stored U,  |x - U c|^2 = |x|^2 - |c|^2 + c^T E c  with  E = U^T U - I  (gsi_build_gram; E is
 * zero only for an exactly orthonormal basis, which a basis rounded to bf16 is not), so the gate needs U once and
 * the k x k matrix E instead of U a second time.  The two large terms and the final combination are accumulated
 * in fp64.  rnorm, xnorm, mask, fired_idx, n_fired and C are written as always (rnorm from the formula);
 * R is written ONLY when the gate fires (an un-fired token's r is never needed); with GSI_INPUT_SLOW_PATH_WX as
 * well R is not written at all and the maps of a fired input skip their image rows: fast-path tokens read M,
 * slow-path tokens read W, merged in one output (Section 7.3 "Kernel-level implementation"). */

/* GSI_INPUT_FUSED_KERNEL (single-token calls, B == 1; ignored otherwise): this input and the maps that read
 * it are processed by the fused kernel -- projection, residual, gate, image rows and, if the gate fires, the
 * rows of W in ONE launch that reads the basis once and keeps it in registers between c = U^T x and r = x - U c
 * (Section 7.3 "Kernel-level implementation": gate fused with the product, basis kept on chip).  Up to four
 * such inputs of one rank share a chunk, up to four chunks a launch; workgroups exchange partial sums through
 * a static device array of the library, so calls that use this flag must not overlap in time on one device
 * (same stream, or ordered streams).  Shapes the kernel does not take (rank not 8..64 sixteen-byte pieces per
 * row, k > 512, more than eight maps on an input, E4M3 images, activations not fp32, d above 16384 with maps)
 * silently take the separate kernels.  Results equal the default path's up to the order of the fp32 sums.
 * Every wait inside the kernel is bounded (one second); gsi_fused_timeouts() counts waits that expired. */

typedef struct gsi_map_desc {
  const void* W;      /* [m,d] wdtype, d = inputs[input_id].d                                   */
  const void* M;      /* [m,k] wdtype, k = inputs[input_id].k; E4M3 bytes with GSI_MAP_IMAGE_FP8 */
  float* Y;           /* [B,m] fp32                                                             */
  int64_t m;
  int32_t wdtype;
  int32_t input_id;   /* which input this map reads                                             */
  const float* M_scale; /* [m] row scales of an FP8 image (gsi_quantize_image_fp8), else unused  */
  int32_t flags;      /* 0, or GSI_MAP_IMAGE_FP8                                                */
  int32_t reserved;   /* 0                                                                      */
} gsi_map_desc;

/* gsi_map_desc.flags.  GSI_MAP_IMAGE_FP8: M and M_scale are the outputs of gsi_quantize_image_fp8 and the
 * image term is y_i = M_scale[i] * sum_j value(M[i,j]) c_j (fp32 accumulation).  The codes are read as they are
 * (half the image bytes) by single-token calls (B == 1) on the vector kernels: k a multiple of 16 and at most
 * 512, M aligned to 16 bytes, and the shapes and alignments of W, U, C, R that those kernels need.  Every other
 * call first expands the image, exactly, to `wdtype` in the workspace (gsi_layer_stack_workspace_bytes accounts
 * for it) and then runs the map as one with an ordinary image: same results, no saving in bytes. */
enum { GSI_MAP_IMAGE_FP8 = 1 };

/* A chain of per-layer linear maps sharing their inputs' projections (Section 1: every linear map
 * of a block that reads the same input shares one basis, one projection and one gate).  For each
 * input: gsi_project + gsi_gate once; for each map: gsi_gated_linear on its input's c, r and fired
 * list.  `maps` and `inputs` are HOST arrays (read during the call only).  Inputs with src_map >= 0
 * are processed after the map that produces them.  Results are identical to issuing the separate
 * calls in that order.  ws: gsi_layer_stack_workspace_bytes(). */
int gsi_layer_stack(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                    int64_t B, float eps, void* ws, size_t ws_bytes, void* stream);

/* gsi_layer_stack for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and therefore cannot provide a workspace: identical to gsi_layer_stack,
 * with the scratch memory taken from a static device array of the library instead of `ws`.  The call allocates
 * nothing on the device and frees nothing.  Limit: the array holds 8 MiB
 * of workspace; a call whose gsi_layer_stack_workspace_bytes() exceeds that returns GSI_ERR_WORKSPACE and enqueues
 * nothing (single-token calls need kilobytes; decode batches of a few tokens fit; prefill-sized batches do not).
 * Every call on a device shares that device's array and finds the previous call's contents in it (the kernels
 * write what they read, nothing needs clearing); calls that overlap in time on one device race on it and are
 * not supported -- issue them on one stream or order the streams. */
int gsi_layer_stack_static(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                           int64_t B, float eps, void* stream);

/* A single-token call of gsi_layer_stack marshalled ONCE.  gsi_layer_stack turns its host descriptors into device
 * tables on every call (a dozen small launches that read their arguments from host memory: tens of microseconds for a
 * 32-layer stack); a decode loop that calls the same layers with the same buffers token after token can build the
 * tables once and then only launch the kernels.
 *   gsi_stack_plan_build validates exactly like gsi_layer_stack(..., B = 1, ...), writes the tables to `plan_mem`
 *   (DEVICE memory of at least gsi_stack_plan_bytes(n_maps, n_inputs) bytes, 256-byte aligned, owned by the caller)
 *   and fills `plan` (a small HOST struct, opaque).  Nothing of the method runs.  Only calls that the table launches
 *   serve whole can be planned (GSI_ERR_SHAPE otherwise): every input external (src_map = -1), with
 *   GSI_INPUT_GATE_SINGLE_PASS (optionally GSI_INPUT_SLOW_PATH_WX) and a 16-byte aligned gram, one dtype throughout,
 *   shapes and alignments of the vector kernels, at most 1024 inputs and 2048 maps.
 *   gsi_stack_plan_run enqueues the call: the same kernels on the same tables as gsi_layer_stack would use, hence the
 *   same bits.  The plan refers to every buffer of the descriptors, to `ws` and to `plan_mem`: all must stay valid
 *   and unmoved; `ws` is in use while a run is in flight, as with gsi_layer_stack.  eps is given per run. */
typedef struct gsi_stack_plan {
  uint64_t opaque[24];
} gsi_stack_plan;
size_t gsi_stack_plan_bytes(int32_t n_maps, int32_t n_inputs);
int gsi_stack_plan_build(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                         void* ws, size_t ws_bytes, void* plan_mem, size_t plan_bytes, gsi_stack_plan* plan, void* stream);
int gsi_stack_plan_run(const gsi_stack_plan* plan, float eps, void* stream);

/* Instrumented variant for measurements (not part of the method): identical to gsi_layer_stack; in addition the
 * two HIP events (hipEvent_t passed as void*, created by the caller with timing enabled) take the start and stop
 * timestamps of the dispatch of ONE of the single-token launches of the call, so hipEventElapsedTime(begin, end)
 * is that launch's execution time as a profiler reports it.  which_kernel: 0 = the projection-side launches, in the
 * order the call enqueues them: the launches of the staged kernel (a set of up to 16 inputs per stage), or, for a
 * call that runs every stage once over descriptor tables, its three timed launches (partial projections; shares of
 * c^T E c; image rows with gates and residuals -- the coefficient sums in between are not counted), or the fused
 * kernel of inputs with GSI_INPUT_FUSED_KERNEL; 1 = the weight-streaming launches (rows of W of the fired inputs'
 * maps).  launch_index counts the launches of that kind from 0.  If the call makes fewer launches of that kind
 * (always so for B != 1) it is still enqueued in full, the events are not recorded and GSI_ERR_SHAPE is returned. */
int gsi_layer_stack_timed(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                          int64_t B, float eps, void* ws, size_t ws_bytes, void* stream, int which_kernel,
                          int launch_index, void* ev_begin, void* ev_end);

/* Dense baseline for a whole stack: Y = W X for every map, all maps in one launch (Section 3.1,
 * the computation the method replaces).  Uses only W, Y, m, wdtype, input_id of each map and X, d,
 * xdtype of each input (src_map must be -1).  ws: device workspace of at least
 * gsi_dense_stack_workspace_bytes(...) bytes (0 for a single token: ws may then be NULL). */
int gsi_dense_stack(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                    int64_t B, void* ws, size_t ws_bytes, void* stream);

/* Minimum workspace size in bytes for one call (arguments that a call does not have are ignored). */
size_t gsi_workspace_bytes(int which_call, int64_t m, int64_t d, int64_t k, int64_t B);
size_t gsi_layer_stack_workspace_bytes(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                                       int32_t n_inputs, int64_t B);
size_t gsi_dense_stack_workspace_bytes(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                                       int32_t n_inputs, int64_t B);

/* Number of bounded waits inside fused-kernel launches (GSI_INPUT_FUSED_KERNEL) on the current device that
 * expired since the library was loaded: 0 in normal operation; the outputs of a launch in which a wait expired
 * are not valid.  count: HOST pointer.  Synchronises the device. */
int gsi_fused_timeouts(uint32_t* count);

/* Thread-local description of the last error returned on this thread ("" if none). */
const char* gsi_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int gsi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GSI_H */
