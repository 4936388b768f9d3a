// C ABI of libgsi: argument validation, workspace accounting and kernel selection.
// Every entry point only enqueues work on the caller's stream; nothing here synchronises,
// allocates or reads device memory.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "gsi_decode.h"
#include "gsi_extend.h"
#include "gsi_fused.h"
#include "gsi_internal.h"
#include "gsi_mfma.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(GSI_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr int64_t kDecodeMaxB = 128;  // above this token count the slab-partial scheme is not used

bool dtype_ok(int dt) { return dt == GSI_F32 || dt == GSI_BF16; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

#define GSI_REQUIRE_PTR(p)                                                        \
  do {                                                                            \
    if ((p) == nullptr) return fail(GSI_ERR_NULL, "%s: %s is NULL", __func__, #p); \
  } while (0)
#define GSI_REQUIRE_ALIGNED(p, a)                                                                       \
  do {                                                                                                  \
    if (!aligned((p), (a))) return fail(GSI_ERR_ALIGN, "%s: %s is not %zu-byte aligned", __func__, #p, (size_t)(a)); \
  } while (0)

int check_shape(const char* fn, int64_t m, int64_t d, int64_t k, int64_t B) {
  if (d < 1) return fail(GSI_ERR_SHAPE, "%s: d = %lld < 1", fn, (long long)d);
  if (k < 1 || k > d) return fail(GSI_ERR_SHAPE, "%s: need 1 <= k <= d, got k = %lld, d = %lld", fn, (long long)k, (long long)d);
  if (m < 1) return fail(GSI_ERR_SHAPE, "%s: m = %lld < 1", fn, (long long)m);
  if (B < 0) return fail(GSI_ERR_SHAPE, "%s: B = %lld < 0", fn, (long long)B);
  // index arithmetic inside the kernels is 64-bit, but token/row counters of a launch are 32-bit
  if (m > (1ll << 30) || d > (1ll << 30) || B > (1ll << 30))
    return fail(GSI_ERR_SHAPE, "%s: dimension above 2^30", fn);
  return GSI_OK;
}

int check_ws(const char* fn, const void* ws, size_t have, size_t need) {
  if (need == 0) return GSI_OK;
  if (ws == nullptr) return fail(GSI_ERR_WORKSPACE, "%s: workspace is NULL, %zu bytes needed", fn, need);
  if (have < need) return fail(GSI_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, have, need);
  if (!aligned(ws, 256)) return fail(GSI_ERR_ALIGN, "%s: workspace is not 256-byte aligned", fn);
  return GSI_OK;
}

}  // namespace

extern "C" {

const char* gsi_last_error(void) { return g_err; }

int gsi_fused_timeouts(uint32_t* count) {
  GSI_REQUIRE_PTR(count);
  unsigned n = 0;
  if (hipError_t e = gsi::fused_timeouts(&n); e != hipSuccess) return hip_fail(e, "gsi_fused_timeouts");
  *count = n;
  return GSI_OK;
}

int gsi_version(void) { return 100; }

// ---- eligibility of the matrix-core paths (bf16 operands, K dimensions multiples of 64) -----------------
static bool mfma_image_ok(int64_t m, int64_t d, int64_t k) {
  return d % 64 == 0 && k % 4 == 0 && m < (1ll << 30) && k < (1ll << 30) && m * k < (1ll << 31);
}
static bool mfma_batch_ok(int64_t d, int64_t k, int64_t B) {
  return B > kDecodeMaxB && d % 64 == 0 && k % 64 == 0 && B < (1ll << 30) && B * d < (1ll << 31);
}
static size_t mfma_project_ws(int64_t d, int64_t k, int64_t B) {
  return gsi::align_up((size_t)k * d * 2, 256) + gsi::align_up((size_t)gsi::mfma_res_tiles(d) * B * 2 * 4, 256) +
         gsi::mfma_part_bytes(B, k, d, gsi::EPI_STORE_F32);
}
// workspace of one linear map of a call with B tokens: partial products of the decode-batch kernel, or of
// the split contraction of the prefill-sized W term (dense = 1: of the dense product)
static size_t map_part_bytes(int64_t m, int64_t d, int64_t B, int dense) {
  if (B > kDecodeMaxB)
    return d % 64 == 0 ? gsi::mfma_part_bytes(B, m, d, dense ? gsi::EPI_STORE_F32 : gsi::EPI_SCATTER_ADD) : 0;
  return gsi::tile_part_bytes(m, d, B);
}

size_t gsi_workspace_bytes(int which_call, int64_t m, int64_t d, int64_t k, int64_t B) {
  switch (which_call) {
    case GSI_CALL_BUILD_IMAGE:
      // the transposed basis of the matrix-core build (bf16 operands); generic kernels need none
      if (m < 1 || d < 1 || k < 1 || k > d || !mfma_image_ok(m, d, k)) return 0;
      return gsi::align_up((size_t)k * d * 2, 256) + gsi::mfma_part_bytes(m, k, d, gsi::EPI_STORE_BF16);
    case GSI_CALL_PROJECT: {
      if (d < 1 || k < 1 || k > d || B < 1) return 0;
      if (B > kDecodeMaxB) return mfma_batch_ok(d, k, B) ? mfma_project_ws(d, k, B) : 0;
      // the slab partials of the vector projection kernels; sized for the wider of the two dtypes so
      // that the query does not depend on the dtype (generic kernels need none)
      size_t need = 0;
      for (int dt = 0; dt < 2; ++dt) {
        if (!gsi::decode_project_ok(d, k, dt, nullptr)) continue;
        const size_t w = gsi::decode_project_ws(d, k, B, dt);
        if (w > need) need = w;
      }
      return need;
    }
    case GSI_CALL_GATED_LINEAR:
    case GSI_CALL_DENSE_LINEAR:
      // partial products of the matrix-core kernels
      if (m < 1 || d < 1 || B < 1) return 0;
      return map_part_bytes(m, d, B, which_call == GSI_CALL_DENSE_LINEAR);
    default:
      return 0;
  }
}

int gsi_build_image(const void* W, const void* U, void* M, int64_t m, int64_t d, int64_t k, int wdtype, void* ws,
                    size_t ws_bytes, void* stream) {
  GSI_REQUIRE_PTR(W);
  GSI_REQUIRE_PTR(U);
  GSI_REQUIRE_PTR(M);
  if (!dtype_ok(wdtype)) return fail(GSI_ERR_DTYPE, "gsi_build_image: unknown wdtype %d", wdtype);
  if (int rc = check_shape("gsi_build_image", m, d, k, 0)) return rc;
  const size_t es = gsi::elem_size(wdtype);
  GSI_REQUIRE_ALIGNED(W, es);
  GSI_REQUIRE_ALIGNED(U, es);
  GSI_REQUIRE_ALIGNED(M, es);
  if (int rc = check_ws("gsi_build_image", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_BUILD_IMAGE, m, d, k, 0)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (wdtype == GSI_BF16 && mfma_image_ok(m, d, k) && aligned(W, 16) && aligned(U, 2) && aligned(M, 8)) {
    // matrix cores: M = W (U^T)^T with the basis transposed once into the workspace
    e = gsi::mfma_transpose_bf16(U, ws, (int)d, (int)k, s);
    if (e == hipSuccess) {
      gsi::GemmArgs g;
      std::memset(&g, 0, sizeof(g));
      g.A = W; g.lda = d; g.a_f32 = 0;
      g.B = ws; g.ldb = d;
      g.D = M; g.ldd = k;
      g.M = (int)m; g.N = (int)k; g.K = (int)d;
      if (gsi::mfma_part_bytes(m, k, d, gsi::EPI_STORE_BF16))
        g.part = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + gsi::align_up((size_t)k * d * 2, 256));
      e = gsi::mfma_gemm_nt(g, gsi::EPI_STORE_BF16, s);
    }
  } else {
    e = gsi::generic_build_image(W, U, M, m, d, k, wdtype, s);
  }
  if (e != hipSuccess) return hip_fail(e, "gsi_build_image");
  return GSI_OK;
}

int gsi_build_gram(const void* U, int64_t d, int64_t k, int udtype, float* E, void* stream) {
  GSI_REQUIRE_PTR(U);
  GSI_REQUIRE_PTR(E);
  if (!dtype_ok(udtype)) return fail(GSI_ERR_DTYPE, "gsi_build_gram: unknown udtype %d", udtype);
  if (int rc = check_shape("gsi_build_gram", 1, d, k, 0)) return rc;
  GSI_REQUIRE_ALIGNED(U, gsi::elem_size(udtype));
  GSI_REQUIRE_ALIGNED(E, 4);
  if (k > 65535 * 16) return fail(GSI_ERR_SHAPE, "gsi_build_gram: k = %lld is too large", (long long)k);
  hipError_t e = gsi::generic_build_gram(U, d, k, udtype, E, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "gsi_build_gram");
  return GSI_OK;
}

size_t gsi_extend_basis_workspace_bytes(int64_t d, int64_t K) {
  return d >= 1 && K >= 1 ? gsi::extend_ws_bytes(d, K) : 0;
}

// argument checks of one basis of an extension call; appends its record and those of its maps
static int add_extend_desc(const char* fn, int idx, const gsi_extend_desc& e, char* ws, std::vector<gsi::ExtIn>& ins,
                           std::vector<gsi::ExtMapRec>& mps) {
  if (!e.U || !e.k_cur || !e.R || !e.rnorm || !e.xnorm)
    return fail(GSI_ERR_NULL, "%s: a pointer (U, k_cur, R, rnorm, xnorm) of basis %d is NULL", fn, idx);
  if (!dtype_ok(e.udtype)) return fail(GSI_ERR_DTYPE, "%s: unknown udtype %d (basis %d)", fn, e.udtype, idx);
  if (int rc = check_shape(fn, 1, e.d, e.K, 0)) return rc;
  if (e.n_maps < 0) return fail(GSI_ERR_SHAPE, "%s: n_maps = %d < 0 (basis %d)", fn, e.n_maps, idx);
  if (e.n_maps > 0 && !e.maps) return fail(GSI_ERR_NULL, "%s: maps of basis %d is NULL", fn, idx);
  if (e.K > (int64_t)65535 * 64 || e.d > (1ll << 31) - 1)
    return fail(GSI_ERR_SHAPE, "%s: d = %lld, K = %lld is too large (basis %d)", fn, (long long)e.d, (long long)e.K, idx);
  const size_t es = gsi::elem_size(e.udtype);
  if (!aligned(e.U, es) || !aligned(e.k_cur, 4) || !aligned(e.R, 4) || !aligned(e.rnorm, 4) || !aligned(e.xnorm, 4) ||
      (e.gram && !aligned(e.gram, 4)) || (e.extended && !aligned(e.extended, 4)))
    return fail(GSI_ERR_ALIGN, "%s: a pointer of basis %d is not aligned to its element size", fn, idx);
  gsi::ExtIn in;
  std::memset(&in, 0, sizeof(in));
  in.U = e.U; in.R = e.R; in.rnorm = e.rnorm; in.xnorm = e.xnorm; in.k_cur = e.k_cur; in.extended = e.extended;
  in.gram = e.gram; in.ws = ws; in.d = e.d; in.K = e.K;
  gsi::extend_fill(in, e.udtype);
  for (int j = 0; j < e.n_maps; ++j) {
    const gsi_extend_map& mp = e.maps[j];
    if (!mp.W) return fail(GSI_ERR_NULL, "%s: maps[%d].W of basis %d is NULL", fn, j, idx);
    if (!mp.M) return fail(GSI_ERR_NULL, "%s: maps[%d].M of basis %d is NULL", fn, j, idx);
    if (mp.m < 1 || mp.m > (1ll << 30))
      return fail(GSI_ERR_SHAPE, "%s: maps[%d].m = %lld out of range (basis %d)", fn, j, (long long)mp.m, idx);
    if (!aligned(mp.W, es) || !aligned(mp.M, es))
      return fail(GSI_ERR_ALIGN, "%s: maps[%d] of basis %d is not aligned to its element size", fn, j, idx);
    gsi::ExtMapRec r;
    std::memset(&r, 0, sizeof(r));
    r.W = mp.W; r.M = mp.M; r.m = mp.m; r.in = (int)ins.size();
    gsi::extend_fill_map(r, e.d, e.udtype);
    mps.push_back(r);
  }
  ins.push_back(in);
  return GSI_OK;
}

int gsi_extend_basis(void* U, int64_t d, int64_t K, int udtype, int32_t* k_cur, const float* R, const float* rnorm,
                     const float* xnorm, float tau, const gsi_extend_map* maps, int32_t n_maps, float* gram,
                     int32_t* extended, void* ws, size_t ws_bytes, void* stream) {
  const char* fn = "gsi_extend_basis";
  if (!(tau >= 0.f)) return fail(GSI_ERR_SHAPE, "%s: tau must be a number >= 0", fn);
  gsi_extend_desc e;
  std::memset(&e, 0, sizeof(e));
  e.U = U; e.d = d; e.K = K; e.udtype = udtype; e.k_cur = k_cur; e.R = R; e.rnorm = rnorm; e.xnorm = xnorm;
  e.maps = maps; e.n_maps = n_maps; e.gram = gram; e.extended = extended;
  std::vector<gsi::ExtIn> ins;
  std::vector<gsi::ExtMapRec> mps;
  if (int rc = add_extend_desc(fn, 0, e, static_cast<char*>(ws), ins, mps)) return rc;
  if (int rc = check_ws(fn, ws, ws_bytes, gsi_extend_basis_workspace_bytes(d, K))) return rc;
  hipError_t err = gsi::extend_many(ins.data(), 1, mps.data(), (int)mps.size(), udtype, tau, nullptr,
                                    static_cast<hipStream_t>(stream));
  if (err != hipSuccess) return hip_fail(err, fn);
  return GSI_OK;
}

size_t gsi_extend_many_workspace_bytes(const gsi_extend_desc* descs, int32_t n) {
  if (!descs || n < 1) return 0;
  int64_t n_maps = 0;
  size_t need = 0;
  for (int i = 0; i < n; ++i) {
    if (descs[i].d < 1 || descs[i].K < 1 || descs[i].n_maps < 0) return 0;
    n_maps += descs[i].n_maps;
    need += gsi::align_up(gsi::extend_ws_bytes(descs[i].d, descs[i].K), 256);
  }
  return gsi::extend_table_bytes(n, (int)n_maps) + need;
}

int gsi_extend_many(const gsi_extend_desc* descs, int32_t n, float tau, void* ws, size_t ws_bytes, void* stream) {
  const char* fn = "gsi_extend_many";
  if (n < 0 || n > 65535) return fail(GSI_ERR_SHAPE, "%s: n = %d out of range (0 .. 65535)", fn, n);
  if (n == 0) return GSI_OK;
  GSI_REQUIRE_PTR(descs);
  if (!(tau >= 0.f)) return fail(GSI_ERR_SHAPE, "%s: tau must be a number >= 0", fn);
  int64_t n_maps = 0;
  for (int i = 0; i < n; ++i) {
    if (descs[i].n_maps < 0) return fail(GSI_ERR_SHAPE, "%s: n_maps = %d < 0 (basis %d)", fn, descs[i].n_maps, i);
    if (descs[i].udtype != descs[0].udtype)
      return fail(GSI_ERR_DTYPE, "%s: the bases of one call share one storage type (basis %d: %d, basis 0: %d)", fn, i,
                  descs[i].udtype, descs[0].udtype);
    n_maps += descs[i].n_maps;
  }
  if (n_maps > 65535) return fail(GSI_ERR_SHAPE, "%s: %lld maps in one call (at most 65535)", fn, (long long)n_maps);
  const size_t need = gsi_extend_many_workspace_bytes(descs, n);
  if (need == 0) return fail(GSI_ERR_SHAPE, "%s: a basis has d < 1 or K < 1", fn);
  if (int rc = check_ws(fn, ws, ws_bytes, need)) return rc;
  if (!aligned(ws, 256)) return fail(GSI_ERR_ALIGN, "%s: ws is not aligned to 256 bytes", fn);
  std::vector<gsi::ExtIn> ins;
  std::vector<gsi::ExtMapRec> mps;
  ins.reserve(n);
  mps.reserve((size_t)n_maps);
  char* p = static_cast<char*>(ws) + gsi::extend_table_bytes(n, (int)n_maps);
  for (int i = 0; i < n; ++i) {
    if (int rc = add_extend_desc(fn, i, descs[i], p, ins, mps)) return rc;
    p += gsi::align_up(gsi::extend_ws_bytes(descs[i].d, descs[i].K), 256);
  }
  hipError_t err = gsi::extend_many(ins.data(), n, mps.data(), (int)mps.size(), descs[0].udtype, tau, ws,
                                    static_cast<hipStream_t>(stream));
  if (err != hipSuccess) return hip_fail(err, fn);
  return GSI_OK;
}

int gsi_quantize_image_fp8(const void* M, int mdtype, int64_t m, int64_t k, uint8_t* M8, float* scale, void* stream) {
  GSI_REQUIRE_PTR(M);
  GSI_REQUIRE_PTR(M8);
  GSI_REQUIRE_PTR(scale);
  if (!dtype_ok(mdtype)) return fail(GSI_ERR_DTYPE, "gsi_quantize_image_fp8: mdtype %d is neither GSI_F32 nor GSI_BF16", mdtype);
  if (m < 1 || k < 1) return fail(GSI_ERR_SHAPE, "gsi_quantize_image_fp8: m = %lld, k = %lld", (long long)m, (long long)k);
  GSI_REQUIRE_ALIGNED(M, gsi::elem_size(mdtype));
  GSI_REQUIRE_ALIGNED(scale, 4);
  hipError_t e = gsi::quantize_image_fp8(M, mdtype, m, k, M8, scale, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "gsi_quantize_image_fp8");
  return GSI_OK;
}

// argument checks shared by the stand-alone entry points and by gsi_layer_stack
static int check_project_args(const char* fn, const void* U, const void* X, int64_t d, int64_t k, int64_t B,
                              int udtype, int xdtype, const float* C, const float* R, const float* rnorm,
                              const float* xnorm) {
  if (!dtype_ok(udtype) || !dtype_ok(xdtype))
    return fail(GSI_ERR_DTYPE, "%s: unknown dtype (udtype %d, xdtype %d)", fn, udtype, xdtype);
  if (int rc = check_shape(fn, 1, d, k, B)) return rc;
  if (B == 0) return GSI_OK;
  if (!U || !X || !C || !R || !rnorm || !xnorm)
    return fail(GSI_ERR_NULL, "%s: a projection pointer (U, X, C, R, rnorm, xnorm) is NULL", fn);
  if (!aligned(U, gsi::elem_size(udtype)) || !aligned(X, gsi::elem_size(xdtype)) || !aligned(C, 4) ||
      !aligned(R, 4) || !aligned(rnorm, 4) || !aligned(xnorm, 4))
    return fail(GSI_ERR_ALIGN, "%s: a projection pointer is not aligned to its element size", fn);
  return GSI_OK;
}

static int check_gate_args(const char* fn, const float* rnorm, const float* xnorm, int64_t B, float eps,
                           const uint8_t* mask, const int32_t* fired_idx, const int32_t* n_fired) {
  if (B < 0 || B > (1ll << 30)) return fail(GSI_ERR_SHAPE, "%s: B = %lld out of range", fn, (long long)B);
  if (!(eps == eps)) return fail(GSI_ERR_SHAPE, "%s: eps is NaN", fn);
  if (!n_fired) return fail(GSI_ERR_NULL, "%s: n_fired is NULL", fn);
  if (!aligned(n_fired, 4)) return fail(GSI_ERR_ALIGN, "%s: n_fired is not 4-byte aligned", fn);
  if (B > 0) {
    if (!rnorm || !xnorm || !mask || !fired_idx)
      return fail(GSI_ERR_NULL, "%s: a gate pointer (rnorm, xnorm, mask, fired_idx) is NULL", fn);
    if (!aligned(rnorm, 4) || !aligned(xnorm, 4) || !aligned(fired_idx, 4))
      return fail(GSI_ERR_ALIGN, "%s: a gate pointer is not 4-byte aligned", fn);
  }
  return GSI_OK;
}

static int check_gated_args(const char* fn, const void* W, const void* M, const float* C, const float* R,
                            const int32_t* fired_idx, const int32_t* n_fired, int64_t m, int64_t d, int64_t k,
                            int64_t B, int wdtype, const void* Y, int ydtype) {
  if (!dtype_ok(wdtype)) return fail(GSI_ERR_DTYPE, "%s: unknown wdtype %d", fn, wdtype);
  if (ydtype != GSI_F32) return fail(GSI_ERR_DTYPE, "%s: ydtype must be GSI_F32, got %d", fn, ydtype);
  if (int rc = check_shape(fn, m, d, k, B)) return rc;
  if (B == 0) return GSI_OK;
  if (!W || !M || !C || !R || !fired_idx || !n_fired || !Y)
    return fail(GSI_ERR_NULL, "%s: a pointer (W, M, C, R, fired_idx, n_fired, Y) is NULL", fn);
  const size_t es = gsi::elem_size(wdtype);
  if (!aligned(W, es) || !aligned(M, es) || !aligned(C, 4) || !aligned(R, 4) || !aligned(fired_idx, 4) ||
      !aligned(n_fired, 4) || !aligned(Y, 4))
    return fail(GSI_ERR_ALIGN, "%s: a pointer is not aligned to its element size", fn);
  return GSI_OK;
}

static bool project_vector_path(int64_t d, int64_t k, int64_t B, int udtype, const void* U) {
  return B <= kDecodeMaxB && gsi::decode_project_ok(d, k, udtype, U);
}

static void fill_proj_task(gsi::ProjTask& t, const void* U, const void* X, int64_t d, int64_t k, int64_t B,
                           int udtype, int xdtype, float* C, float* R, float* rnorm, float* xnorm, void* ws) {
  t.U = U; t.X = X; t.C = C; t.R = R; t.rnorm = rnorm; t.xnorm = xnorm;
  t.udtype = udtype; t.xdtype = xdtype;
  gsi::decode_project_fill(t, d, k, B, ws);
}

// Prefill-sized projection on the matrix cores: C = X U, R = X - C U^T with per-tile partial norms, then
// the norm (+ gate) kernel.  `gate` may be null (norms only).
// `img` (optional): image terms Y = C M^T of maps that read this input; they need c only, so they ride in the
// residual's launch as further right-hand factors of the same left operand.
struct ImageRider {
  const void* M;
  float* Y;
  int64_t m;
};
static hipError_t mfma_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int xdtype, float* C,
                               float* R, float* rnorm, float* xnorm, uint8_t* mask, int32_t* fired_idx,
                               int32_t* n_fired, bool with_gate, float eps, void* ws, hipStream_t s,
                               const ImageRider* img = nullptr, int n_img = 0) {
  void* Ut = ws;
  float* part_n = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + gsi::align_up((size_t)k * d * 2, 256));
  hipError_t e = gsi::mfma_transpose_bf16(U, Ut, (int)d, (int)k, s);
  if (e != hipSuccess) return e;
  gsi::GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.A = X; g.lda = d; g.a_f32 = xdtype == GSI_F32;
  g.B = Ut; g.ldb = d;
  g.D = C; g.ldd = k;
  g.M = (int)B; g.N = (int)k; g.K = (int)d;
  if (gsi::mfma_part_bytes(B, k, d, gsi::EPI_STORE_F32))
    g.part = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + gsi::align_up((size_t)k * d * 2, 256) +
                                      gsi::align_up((size_t)gsi::mfma_res_tiles(d) * B * 2 * 4, 256));
  e = gsi::mfma_gemm_nt(g, gsi::EPI_STORE_F32, s);
  if (e != hipSuccess) return e;
  std::memset(&g, 0, sizeof(g));
  g.A = C; g.lda = k; g.a_f32 = 1;
  g.B = U; g.ldb = k;
  g.D = R; g.ldd = d;
  g.M = (int)B; g.N = (int)d; g.K = (int)k;
  g.X = X; g.xdtype = xdtype; g.ldx = d; g.part_n = part_n; g.part_tokens = (int)B;
  if (n_img > 0) {
    g.nseg = 1 + n_img;
    g.seg[0] = gsi::GemmSeg{U, k, R, d, (int)d, 0, gsi::EPI_RESIDUAL};
    for (int q = 0; q < n_img; ++q) g.seg[1 + q] = gsi::GemmSeg{img[q].M, k, img[q].Y, img[q].m, (int)img[q].m, 0, gsi::EPI_STORE_F32};
    e = gsi::mfma_gemm_nt(g, gsi::EPI_MULTI, s);
  } else {
    e = gsi::mfma_gemm_nt(g, gsi::EPI_RESIDUAL, s);
  }
  if (e != hipSuccess) return e;
  gsi::ProjBatch pb;
  std::memset(&pb, 0, sizeof(pb));
  pb.n = 1;
  pb.B = (int)B;
  pb.t[0].part_n = part_n; pb.t[0].b_slabs = gsi::mfma_res_tiles(d);
  pb.t[0].rnorm = rnorm; pb.t[0].xnorm = xnorm;
  pb.t[0].mask = mask; pb.t[0].fired_idx = fired_idx; pb.t[0].n_fired = n_fired;
  return gsi::decode_norms_launch(pb, with_gate, eps, s);
}

static bool mfma_project_path(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype,
                              const float* C, const float* R) {
  return udtype == GSI_BF16 && mfma_batch_ok(d, k, B) && aligned(U, 16) && aligned(X, 16) && aligned(C, 16) &&
         aligned(R, 16) && (xdtype == GSI_F32 || xdtype == GSI_BF16);
}

// Prefill-sized gated map on the matrix cores: Y = C M^T for every token, then Y[fired] += R[fired] W^T
// over the compacted list (row tiles beyond the device-side count exit at once).
static hipError_t mfma_gated(const void* W, const void* M, const float* C, const float* R, const int32_t* fired_idx,
                             const int32_t* n_fired, int64_t m, int64_t d, int64_t k, int64_t B, float* Y,
                             float* part, hipStream_t s, const void* Xwx = nullptr, int xdtype = 0,
                             bool image_done = false) {
  gsi::GemmArgs g;
  hipError_t e = hipSuccess;
  if (!image_done) {
    std::memset(&g, 0, sizeof(g));
    g.A = C; g.lda = k; g.a_f32 = 1;
    g.B = M; g.ldb = k;
    g.D = Y; g.ldd = m;
    g.M = (int)B; g.N = (int)m; g.K = (int)k;
    e = gsi::mfma_gemm_nt(g, gsi::EPI_STORE_F32, s);
    if (e != hipSuccess) return e;
  }
  std::memset(&g, 0, sizeof(g));
  // r enters rounded once to bf16: its term is scaled by the residual ratio, so the rounding (2^-9 relative)
  // adds a few 1e-4 of |y| at most, beside the 1.7e-3 that the bf16 image already costs
  g.A = R; g.lda = d; g.a_f32 = 2;
  if (Xwx) {  // fired tokens get y = W x, fed exactly as the dense product feeds x
    g.A = Xwx;
    g.a_f32 = xdtype == GSI_F32 ? 1 : 0;
  }
  g.B = W; g.ldb = d;
  g.D = Y; g.ldd = m;
  g.M = (int)B; g.N = (int)m; g.K = (int)d;
  g.row_idx = fired_idx; g.n_rows_dev = n_fired;
  g.part = gsi::mfma_part_bytes(B, m, d, gsi::EPI_SCATTER_ADD) ? part : nullptr;
  return gsi::mfma_gemm_nt(g, Xwx ? gsi::EPI_SCATTER_STORE : gsi::EPI_SCATTER_ADD, s);
}

static bool mfma_gated_path(const void* W, const void* M, const float* C, const float* R, int64_t d, int64_t k,
                            int64_t B, int wdtype, int64_t m, const void* Y) {
  return wdtype == GSI_BF16 && mfma_batch_ok(d, k, B) && aligned(W, 16) && aligned(M, 16) && aligned(C, 16) &&
         aligned(R, 16) && m % 4 == 0 && B * m < (1ll << 31) && aligned(Y, 16);
}

// Prefill-sized dense baseline on the matrix cores: Y = X W^T
static bool mfma_dense_path(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int wdtype,
                            const void* Y) {
  return wdtype == GSI_BF16 && B > kDecodeMaxB && d % 64 == 0 && m % 4 == 0 && B * m < (1ll << 31) &&
         aligned(W, 16) && aligned(X, 16) && aligned(Y, 16);
}
static hipError_t mfma_dense(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int xdtype, float* Y,
                             float* part, hipStream_t s) {
  gsi::GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.A = X; g.lda = d; g.a_f32 = xdtype == GSI_F32;
  g.B = W; g.ldb = d;
  g.D = Y; g.ldd = m;
  g.M = (int)B; g.N = (int)m; g.K = (int)d;
  g.part = gsi::mfma_part_bytes(B, m, d, gsi::EPI_STORE_F32) ? part : nullptr;
  return gsi::mfma_gemm_nt(g, gsi::EPI_STORE_F32, s);
}

static void clear(gsi::LinBatch& lb, int64_t B) {
  std::memset(&lb, 0, sizeof(lb));
  lb.B = (int)B;
}

// A decode batch (2..128 tokens) over an input longer than the linear kernels' LDS vector runs on the matrix-core
// kernel only: what that kernel needs beyond decode_linear_ok (reads_x: the product reads x, dense or W x form).
static bool long_batch_ok(int64_t d, int64_t B, const void* Y, bool reads_x, const void* X, int xdtype) {
  if (B == 1 || d <= gsi::kMaxLinD) return true;
  return aligned(Y, 16) && (!reads_x || (xdtype == GSI_F32 && aligned(X, 16)));
}

// Adds map `mp` (reading group description `gd`) to the batch, flushing first when the batch is full or
// its LDS budget would be exceeded.  `gkey` identifies the input so maps of one input share a group slot.
namespace {
struct LinBatcher {
  gsi::LinBatch lb;
  int gkeys[gsi::kMaxTasks];
  int wdtype;
  hipStream_t s;
  int64_t B;
  hipEvent_t e0 = nullptr, e1 = nullptr;  // optional dispatch-timestamp events for the launches of this batcher
  gsi::ImgBatch sib;                      // single token: image maps y = M c not yet written by an earlier launch
  int* n_launches = nullptr;               // the launch whose count equals timed_index gets the events
  int timed_index = -1;
  float eps = 0.f;                          // for groups whose gate the single-token kernel evaluates
  void reset(int64_t B_, int dense) {
    B = B_;
    clear(lb, B_);
    lb.dense = dense;
    lb.eps = eps;
    std::memset(&sib, 0, sizeof(sib));
  }
  hipError_t flush() {
    if (lb.n == 0) return hipSuccess;
    if (sib.n > 0)  // the image term first: the weight-streaming launch adds W r to it
      if (hipError_t ei = gsi::decode_image_launch(sib, wdtype, s); ei != hipSuccess) return ei;
    const bool timed = n_launches && (*n_launches)++ == timed_index;
    hipError_t e = gsi::decode_linear_launch(lb, wdtype, s, timed ? e0 : nullptr, timed ? e1 : nullptr);
    reset(B, lb.dense);
    return e;
  }
  hipError_t add(int gkey, const gsi::LinGroup& gd, const void* W, const void* M, float* Y, int64_t m,
                 bool need_image = false, float* part = nullptr, const float* mscale = nullptr) {
    for (int attempt = 0; attempt < 2; ++attempt) {
      int gi = -1;
      for (int i = 0; i < lb.ng; ++i)
        if (gkeys[i] == gkey) gi = i;
      gsi::LinBatch trial = lb;
      if (gi < 0) {
        if (trial.ng == gsi::kMaxTasks) gi = -2;
        else { gi = trial.ng++; trial.g[gi] = gd; }
      }
      if (gi >= 0 && trial.n < gsi::kMaxLinTasks) {
        gsi::LinTask& t = trial.t[trial.n++];
        t.W = W; t.M = M; t.Y = Y; t.m = (int)m; t.group = gi; t.part = part; t.slices = 0;
        if (gsi::decode_linear_fits(trial, wdtype)) {
          if (gi == lb.ng) gkeys[gi] = gkey;
          lb = trial;
          if (need_image) {  // as many image tasks as linear tasks at most, so this never overflows
            gsi::ImgTask& it = sib.t[sib.n++];
            it.M = M; it.Y = Y; it.part_c = nullptr; it.C = gd.C; it.m = (int)m; it.k = gd.k; it.a_slabs = 0;
            it.scale = mscale;
          }
          return hipSuccess;
        }
      }
      if (hipError_t e = flush(); e != hipSuccess) return e;  // start a new launch and try once more
    }
    return hipErrorInvalidValue;  // a single map that passed decode_linear_ok always fits an empty batch
  }
};
}  // namespace

int gsi_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype, float* C,
                float* R, float* rnorm, float* xnorm, void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_project_args("gsi_project", U, X, d, k, B, udtype, xdtype, C, R, rnorm, xnorm)) return rc;
  if (B == 0) return GSI_OK;
  if (int rc = check_ws("gsi_project", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_PROJECT, 0, d, k, B))) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (project_vector_path(d, k, B, udtype, U)) {
    gsi::ProjBatch pb;
    std::memset(&pb, 0, sizeof(pb));
    pb.n = 1;
    pb.B = (int)B;
    fill_proj_task(pb.t[0], U, X, d, k, B, udtype, xdtype, C, R, rnorm, xnorm, ws);
    e = gsi::decode_project_launch(pb, udtype, true, false, 0.f, s);
  } else if (mfma_project_path(U, X, d, k, B, udtype, xdtype, C, R)) {
    e = mfma_project(U, X, d, k, B, xdtype, C, R, rnorm, xnorm, nullptr, nullptr, nullptr, false, 0.f, ws, s);
  } else {
    e = gsi::generic_project(U, X, d, k, B, udtype, xdtype, C, R, rnorm, xnorm, s);
  }
  if (e != hipSuccess) return hip_fail(e, "gsi_project");
  return GSI_OK;
}

int gsi_gate(const float* rnorm, const float* xnorm, int64_t B, float eps, uint8_t* mask, int32_t* fired_idx,
             int32_t* n_fired, void* stream) {
  if (int rc = check_gate_args("gsi_gate", rnorm, xnorm, B, eps, mask, fired_idx, n_fired)) return rc;
  // B == 0 still launches: the count must read 0 afterwards.
  hipError_t e = gsi::launch_gate(rnorm, xnorm, B, eps, mask, fired_idx, n_fired, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "gsi_gate");
  return GSI_OK;
}

int gsi_gated_linear(const void* W, const void* M, const float* C, const float* R, const int32_t* fired_idx,
                     const int32_t* n_fired, int64_t m, int64_t d, int64_t k, int64_t B, int wdtype, void* Y,
                     int ydtype, void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_gated_args("gsi_gated_linear", W, M, C, R, fired_idx, n_fired, m, d, k, B, wdtype, Y, ydtype))
    return rc;
  if (B == 0) return GSI_OK;
  if (int rc = check_ws("gsi_gated_linear", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_GATED_LINEAR, m, d, k, B)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (!mfma_gated_path(W, M, C, R, d, k, B, wdtype, m, Y) && gsi::decode_linear_ok(m, d, k, wdtype, W, M, B) &&
      aligned(C, 16) && aligned(R, 16) && long_batch_ok(d, B, Y, false, nullptr, 0)) {
    LinBatcher bt;
    bt.wdtype = wdtype; bt.s = s;
    bt.reset(B, 0);
    gsi::LinGroup gd;
    std::memset(&gd, 0, sizeof(gd));
    gd.C = C; gd.R = R; gd.fired_idx = fired_idx; gd.n_fired = n_fired;
    gd.d = (int)d; gd.k = (int)k;
    e = bt.add(0, gd, W, M, (float*)Y, m, B == 1, gsi::tile_part_bytes(m, d, B) ? (float*)ws : nullptr);
    if (e == hipSuccess) e = bt.flush();
  } else if (mfma_gated_path(W, M, C, R, d, k, B, wdtype, m, Y)) {
    e = mfma_gated(W, M, C, R, fired_idx, n_fired, m, d, k, B, (float*)Y, (float*)ws, s);
  } else {
    e = gsi::generic_gated_linear(W, M, C, R, fired_idx, n_fired, m, d, k, B, wdtype, (float*)Y, s);
  }
  if (e != hipSuccess) return hip_fail(e, "gsi_gated_linear");
  return GSI_OK;
}

int gsi_dense_linear(const void* W, const void* X, int64_t m, int64_t d, int64_t B, int wdtype, int xdtype,
                     float* Y, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(wdtype) || !dtype_ok(xdtype))
    return fail(GSI_ERR_DTYPE, "gsi_dense_linear: unknown dtype (wdtype %d, xdtype %d)", wdtype, xdtype);
  if (int rc = check_shape("gsi_dense_linear", m, d, 1, B)) return rc;
  if (B == 0) return GSI_OK;
  GSI_REQUIRE_PTR(W);
  GSI_REQUIRE_PTR(X);
  GSI_REQUIRE_PTR(Y);
  GSI_REQUIRE_ALIGNED(W, gsi::elem_size(wdtype));
  GSI_REQUIRE_ALIGNED(X, gsi::elem_size(xdtype));
  GSI_REQUIRE_ALIGNED(Y, 4);
  if (int rc = check_ws("gsi_dense_linear", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_DENSE_LINEAR, m, d, 0, B)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (mfma_dense_path(W, X, m, d, B, wdtype, Y)) {
    e = mfma_dense(W, X, m, d, B, xdtype, Y, (float*)ws, s);
  } else if (gsi::decode_linear_ok(m, d, 0, wdtype, W, nullptr, B) && aligned(X, 16) &&
             long_batch_ok(d, B, Y, true, X, xdtype)) {
    gsi::LinBatch lb;
    clear(lb, B);
    lb.n = lb.ng = 1;
    lb.dense = 1;
    lb.g[0].X = X; lb.g[0].xdtype = xdtype; lb.g[0].d = (int)d;
    lb.t[0].W = W; lb.t[0].Y = Y; lb.t[0].m = (int)m; lb.t[0].group = 0;
    lb.t[0].part = gsi::tile_part_bytes(m, d, B) ? (float*)ws : nullptr;
    e = gsi::decode_linear_launch(lb, wdtype, s);
  } else {
    e = gsi::generic_dense_linear(W, X, m, d, B, wdtype, xdtype, Y, s);
  }
  if (e != hipSuccess) return hip_fail(e, "gsi_dense_linear");
  return GSI_OK;
}

// the W x form of the slow path reads x with 16-byte loads in the vector kernels
static bool wx_vector_ok(const gsi_input_desc& in) {
  return !(in.flags & GSI_INPUT_SLOW_PATH_WX) || aligned(in.X, 16);
}

// Is the E4M3 image of this map read as codes?  Only by the single-token vector kernels; every other call
// expands it (exactly) to the weights' type in the workspace first and runs the map with an ordinary image.
static bool fp8_codes_read(const gsi_map_desc& mp, const gsi_input_desc& in, int64_t B) {
  return B == 1 && aligned(mp.M, 16) && in.k % 16 == 0 && in.k <= gsi::kMaxK &&
         project_vector_path(in.d, in.k, B, in.udtype, in.U) &&
         gsi::decode_linear_ok(mp.m, in.d, in.k, mp.wdtype, mp.W, nullptr, B) && aligned(in.C, 16) && aligned(in.R, 16) &&
         wx_vector_ok(in);
}
static size_t fp8_expand_bytes(const gsi_map_desc& mp, const gsi_input_desc& in, int64_t B) {
  if (!(mp.flags & GSI_MAP_IMAGE_FP8) || B < 1 || mp.m < 1 || in.k < 1 || fp8_codes_read(mp, in, B)) return 0;
  return gsi::align_up((size_t)mp.m * in.k * gsi::elem_size(mp.wdtype), 256);
}

// single token: the descriptor table of the weight-streaming launch sits at the start of the workspace
// (and behind it the table of the staged launches of a call with many inputs and the single-pass gate)
static size_t stack_table_bytes(int32_t n_maps, int32_t n_inputs, int64_t B) {
  return B == 1 && n_maps > 0 && n_inputs > 0
             ? gsi::fired_table_bytes(n_inputs, n_maps) + gsi::stage_table_bytes(n_inputs, n_maps)
             : 0;
}

size_t gsi_layer_stack_workspace_bytes(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                                       int32_t n_inputs, int64_t B) {
  if (!inputs || n_inputs < 0) return 0;
  // projections of independent inputs share a launch, so every input has its own region
  size_t need = stack_table_bytes(maps ? n_maps : 0, n_inputs, B);
  for (int i = 0; i < n_inputs; ++i)
    need += gsi::align_up(gsi_workspace_bytes(GSI_CALL_PROJECT, 0, inputs[i].d, inputs[i].k, B), 256);
  // and so do the maps of a decode batch (partial products of the weight term)
  if (maps)
    for (int j = 0; j < n_maps; ++j) {
      const int id = maps[j].input_id;
      if (id >= 0 && id < n_inputs) need += map_part_bytes(maps[j].m, inputs[id].d, B, 0);
    }
  // E4M3 images that are not read as codes are expanded to the weights' type
  if (maps)
    for (int j = 0; j < n_maps; ++j) {
      const int id = maps[j].input_id;
      if (id >= 0 && id < n_inputs) need += fp8_expand_bytes(maps[j], inputs[id], B);
    }
  return need;
}

// What gsi_stack_plan_build leaves in the caller's gsi_stack_plan: the launch shapes of a single-token call whose
// descriptor tables sit in the caller's device memory.
struct PlanRec {
  uint32_t magic;
  int32_t has_fired;
  gsi::StageTableGeom sg;
  gsi::FiredGeom fg;
  void* stage_table;
  void* fired_table;
};
static_assert(sizeof(PlanRec) <= sizeof(gsi_stack_plan), "gsi_stack_plan is too small");
constexpr uint32_t kPlanMagic = 0x47534950u;
// building a plan: the tables go to `dev` instead of the workspace and nothing else is launched
struct PlanBuild {
  PlanRec* rec;
  char* dev;
  int n_in_done = 0, n_maps_done = 0;
};

static int layer_stack_impl(const char* fn, const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                            int32_t n_inputs, int64_t B, float eps, void* ws, size_t ws_bytes, void* stream,
                            hipEvent_t ev_begin, hipEvent_t ev_end, int which = -1, int launch_index = 0,
                            int* n_launches = nullptr, PlanBuild* plan = nullptr);

int gsi_layer_stack(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                    int64_t B, float eps, void* ws, size_t ws_bytes, void* stream) {
  return layer_stack_impl("gsi_layer_stack", maps, n_maps, inputs, n_inputs, B, eps, ws, ws_bytes, stream, nullptr,
                          nullptr);
}

int gsi_layer_stack_static(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                           int64_t B, float eps, void* stream) {
  const char* fn = "gsi_layer_stack_static";
  void* ws = nullptr;
  size_t have = 0;
  if (hipError_t e = gsi::static_workspace(&ws, &have); e != hipSuccess) return hip_fail(e, fn);
  if (n_maps < 0 || n_inputs < 0) return fail(GSI_ERR_SHAPE, "%s: negative count", fn);
  if (n_maps > 0) GSI_REQUIRE_PTR(maps);
  if (n_inputs > 0) GSI_REQUIRE_PTR(inputs);
  for (int j = 0; j < n_maps; ++j)
    if (maps[j].input_id < 0 || maps[j].input_id >= n_inputs)
      return fail(GSI_ERR_SHAPE, "%s: maps[%d].input_id = %d out of range", fn, j, maps[j].input_id);
  const size_t need = B > 0 ? gsi_layer_stack_workspace_bytes(maps, n_maps, inputs, n_inputs, B) : 0;
  if (need > have)
    return fail(GSI_ERR_WORKSPACE,
                "%s: this call needs %zu bytes of scratch, the library's static array holds %zu; use gsi_layer_stack "
                "with a workspace",
                fn, need, have);
  return layer_stack_impl(fn, maps, n_maps, inputs, n_inputs, B, eps, ws, have, stream, nullptr, nullptr);
}

int gsi_layer_stack_timed(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                          int64_t B, float eps, void* ws, size_t ws_bytes, void* stream, int which_kernel,
                          int launch_index, void* ev_begin, void* ev_end) {
  if (!ev_begin || !ev_end) return fail(GSI_ERR_NULL, "gsi_layer_stack_timed: an event is NULL");
  if (which_kernel < 0 || which_kernel > 1)
    return fail(GSI_ERR_SHAPE, "gsi_layer_stack_timed: which_kernel = %d is not 0 or 1", which_kernel);
  if (launch_index < 0) return fail(GSI_ERR_SHAPE, "gsi_layer_stack_timed: launch_index = %d < 0", launch_index);
  int n = 0;
  const int rc = layer_stack_impl("gsi_layer_stack_timed", maps, n_maps, inputs, n_inputs, B, eps, ws, ws_bytes, stream,
                                  static_cast<hipEvent_t>(ev_begin), static_cast<hipEvent_t>(ev_end), which_kernel,
                                  launch_index, &n);
  if (rc != GSI_OK) return rc;
  if (launch_index >= n)
    return fail(GSI_ERR_SHAPE, "gsi_layer_stack_timed: the call made %d launches of kind %d, none has index %d (the call "
                "itself was enqueued in full)", n, which_kernel, launch_index);
  return GSI_OK;
}

size_t gsi_dense_stack_workspace_bytes(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                                       int32_t n_inputs, int64_t B) {
  if (!maps || !inputs || n_maps < 0 || n_inputs < 0) return 0;
  size_t need = 0;  // partial products of the several-token matrix-core kernel, one region per map
  for (int j = 0; j < n_maps; ++j) {
    const int id = maps[j].input_id;
    if (id >= 0 && id < n_inputs) need += map_part_bytes(maps[j].m, inputs[id].d, B, 1);
  }
  return need;
}

int gsi_dense_stack(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                    int64_t B, void* ws, size_t ws_bytes, void* stream) {
  const char* fn = "gsi_dense_stack";
  if (n_maps < 0 || n_inputs < 0) return fail(GSI_ERR_SHAPE, "%s: negative count", fn);
  if (n_maps > 0) GSI_REQUIRE_PTR(maps);
  if (n_inputs > 0) GSI_REQUIRE_PTR(inputs);
  if (B < 0) return fail(GSI_ERR_SHAPE, "%s: B = %lld < 0", fn, (long long)B);
  for (int j = 0; j < n_maps; ++j) {
    const gsi_map_desc& mp = maps[j];
    if (mp.input_id < 0 || mp.input_id >= n_inputs)
      return fail(GSI_ERR_SHAPE, "%s: maps[%d].input_id = %d out of range", fn, j, mp.input_id);
    const gsi_input_desc& in = inputs[mp.input_id];
    if (in.src_map != -1) return fail(GSI_ERR_SHAPE, "%s: chained inputs are not supported", fn);
    if (!dtype_ok(mp.wdtype) || !dtype_ok(in.xdtype)) return fail(GSI_ERR_DTYPE, "%s: unknown dtype", fn);
    if (int rc = check_shape(fn, mp.m, in.d, 1, B)) return rc;
    if (B > 0) {
      if (!mp.W || !in.X || !mp.Y) return fail(GSI_ERR_NULL, "%s: W, X or Y of maps[%d] is NULL", fn, j);
      if (!aligned(mp.W, gsi::elem_size(mp.wdtype)) || !aligned(in.X, gsi::elem_size(in.xdtype)) || !aligned(mp.Y, 4))
        return fail(GSI_ERR_ALIGN, "%s: a pointer of maps[%d] is not aligned to its element size", fn, j);
    }
  }
  if (B == 0) return GSI_OK;
  if (int rc = check_ws(fn, ws, ws_bytes, gsi_dense_stack_workspace_bytes(maps, n_maps, inputs, n_inputs, B)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::vector<float*> part(n_maps, nullptr);
  {
    size_t off = 0;
    for (int j = 0; j < n_maps; ++j) {
      const size_t pb = map_part_bytes(maps[j].m, inputs[maps[j].input_id].d, B, 1);
      if (pb) part[j] = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + off);
      off += pb;
    }
  }
  std::vector<char> done(n_maps, 0);
  for (int j = 0; j < n_maps; ++j) {  // prefill-sized batches: one matrix-core product per map
    const gsi_map_desc& mp = maps[j];
    const gsi_input_desc& in = inputs[mp.input_id];
    if (!mfma_dense_path(mp.W, in.X, mp.m, in.d, B, mp.wdtype, mp.Y)) continue;
    if (hipError_t e = mfma_dense(mp.W, in.X, mp.m, in.d, B, in.xdtype, mp.Y, part[j], s); e != hipSuccess)
      return hip_fail(e, fn);
    done[j] = 1;
  }
  for (int dt = 0; dt < 2; ++dt) {
    LinBatcher bt;
    bt.wdtype = dt; bt.s = s;
    bt.reset(B, 1);
    for (int j = 0; j < n_maps; ++j) {
      const gsi_map_desc& mp = maps[j];
      const gsi_input_desc& in = inputs[mp.input_id];
      if (done[j] || mp.wdtype != dt || !gsi::decode_linear_ok(mp.m, in.d, 0, mp.wdtype, mp.W, nullptr, B) ||
          !aligned(in.X, 16) || !long_batch_ok(in.d, B, mp.Y, true, in.X, in.xdtype))
        continue;
      gsi::LinGroup gd;
      std::memset(&gd, 0, sizeof(gd));
      gd.X = in.X; gd.xdtype = in.xdtype; gd.d = (int)in.d;
      if (hipError_t e = bt.add(mp.input_id, gd, mp.W, nullptr, mp.Y, mp.m, false, part[j]); e != hipSuccess)
        return hip_fail(e, fn);
      done[j] = 1;
    }
    if (hipError_t e = bt.flush(); e != hipSuccess) return hip_fail(e, fn);
  }
  for (int j = 0; j < n_maps; ++j) {
    if (done[j]) continue;
    const gsi_map_desc& mp = maps[j];
    const gsi_input_desc& in = inputs[mp.input_id];
    hipError_t e = gsi::generic_dense_linear(mp.W, in.X, mp.m, in.d, B, mp.wdtype, in.xdtype, mp.Y, s);
    if (e != hipSuccess) return hip_fail(e, fn);
  }
  return GSI_OK;
}

static int layer_stack_impl(const char* fn, const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                            int32_t n_inputs, int64_t B, float eps, void* ws, size_t ws_bytes, void* stream,
                            hipEvent_t ev_begin, hipEvent_t ev_end, int which, int launch_index, int* n_launches,
                            PlanBuild* plan) {
  int n_stage_launches = 0, n_stream_launches = 0;  // counted for the timed variant
  if (n_maps < 0 || n_inputs < 0) return fail(GSI_ERR_SHAPE, "%s: negative count", fn);
  if (n_maps > 0) GSI_REQUIRE_PTR(maps);
  if (n_inputs > 0) GSI_REQUIRE_PTR(inputs);
  if (B < 0) return fail(GSI_ERR_SHAPE, "%s: B = %lld < 0", fn, (long long)B);
  for (int j = 0; j < n_maps; ++j) {
    const int id = maps[j].input_id;
    if (id < 0 || id >= n_inputs) return fail(GSI_ERR_SHAPE, "%s: maps[%d].input_id = %d out of range", fn, j, id);
  }
  for (int i = 0; i < n_inputs; ++i) {
    const int sm = inputs[i].src_map;
    if (sm < -1 || sm >= n_maps) return fail(GSI_ERR_SHAPE, "%s: inputs[%d].src_map = %d out of range", fn, i, sm);
    if (sm >= 0) {
      if (inputs[i].X != (const void*)maps[sm].Y)
        return fail(GSI_ERR_SHAPE, "%s: inputs[%d].X must be maps[%d].Y", fn, i, sm);
      if (inputs[i].xdtype != GSI_F32 || inputs[i].d != maps[sm].m)
        return fail(GSI_ERR_SHAPE, "%s: inputs[%d] does not match the output of maps[%d]", fn, i, sm);
    }
  }
  // validate everything before the first launch
  for (int i = 0; i < n_inputs; ++i) {
    const gsi_input_desc& in = inputs[i];
    if (in.flags & ~(GSI_INPUT_SLOW_PATH_WX | GSI_INPUT_FUSED_KERNEL | GSI_INPUT_GATE_SINGLE_PASS))
      return fail(GSI_ERR_SHAPE, "%s: inputs[%d].flags = %d has unknown bits", fn, i, in.flags);
    if (in.flags & GSI_INPUT_GATE_SINGLE_PASS) {
      if (!in.gram) return fail(GSI_ERR_NULL, "%s: inputs[%d].gram is NULL with GSI_INPUT_GATE_SINGLE_PASS", fn, i);
      if (!aligned(in.gram, 4)) return fail(GSI_ERR_ALIGN, "%s: inputs[%d].gram is not aligned to 4 bytes", fn, i);
    }
    if (int rc = check_project_args(fn, in.U, in.X, in.d, in.k, B, in.udtype, in.xdtype, in.C, in.R, in.rnorm,
                                    in.xnorm))
      return rc;
    if (int rc = check_gate_args(fn, in.rnorm, in.xnorm, B, eps, in.mask, in.fired_idx, in.n_fired)) return rc;
  }
  for (int j = 0; j < n_maps; ++j) {
    const gsi_map_desc& mp = maps[j];
    const gsi_input_desc& in = inputs[mp.input_id];
    if (mp.flags & ~GSI_MAP_IMAGE_FP8)
      return fail(GSI_ERR_SHAPE, "%s: maps[%d].flags = %d has unknown bits", fn, j, mp.flags);
    const bool fp8 = (mp.flags & GSI_MAP_IMAGE_FP8) != 0;
    // (an E4M3 image is bytes: the alignment rule of the weights' type does not apply to it)
    if (int rc = check_gated_args(fn, mp.W, fp8 ? mp.W : mp.M, in.C, in.R, in.fired_idx, in.n_fired, mp.m, in.d, in.k, B,
                                  mp.wdtype, mp.Y, GSI_F32))
      return rc;
    if (fp8 && B > 0) {
      if (!mp.M) return fail(GSI_ERR_NULL, "%s: maps[%d].M is NULL", fn, j);
      if (!mp.M_scale) return fail(GSI_ERR_NULL, "%s: maps[%d].M_scale is NULL", fn, j);
      if (!aligned(mp.M_scale, 4)) return fail(GSI_ERR_ALIGN, "%s: maps[%d].M_scale is not aligned to 4 bytes", fn, j);
    }
  }
  if (int rc = check_ws(fn, ws, ws_bytes, gsi_layer_stack_workspace_bytes(maps, n_maps, inputs, n_inputs, B)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);

  // Bookkeeping of the call lives in thread-local vectors that keep their capacity from call to call: after the
  // first call of a thread the enqueue path allocates no host memory for them.
  struct Scratch {
    std::vector<size_t> ws_off;
    std::vector<float*> part;
    std::vector<int> mode, mode_separate, part_ncb, ready, mready;
    std::vector<gsi::ProjTask> ptask;
    std::vector<char> map_fused, in_done, map_done, img_done, gate_inline;
  };
  static thread_local Scratch sc;
  std::vector<size_t>& ws_off = sc.ws_off;
  std::vector<float*>& part = sc.part;
  ws_off.assign(n_inputs, 0);
  part.assign(n_maps, nullptr);
  {
    size_t off = stack_table_bytes(n_maps, n_inputs, B);
    for (int i = 0; i < n_inputs; ++i) {
      ws_off[i] = off;
      off += gsi::align_up(gsi_workspace_bytes(GSI_CALL_PROJECT, 0, inputs[i].d, inputs[i].k, B), 256);
    }
    for (int j = 0; j < n_maps; ++j) {
      const size_t pb = map_part_bytes(maps[j].m, inputs[maps[j].input_id].d, B, 0);
      if (pb) part[j] = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + off);
      off += pb;
    }
  }

  // E4M3 images that no kernel of this call reads as codes (several tokens, or shapes the single-token vector
  // kernels do not take) are expanded, exactly, to the weights' type in the workspace first; their maps then run
  // as maps with an ordinary image.
  std::vector<gsi_map_desc> expanded;
  if (B > 0) {
    size_t off = stack_table_bytes(n_maps, n_inputs, B);
    for (int i = 0; i < n_inputs; ++i)
      off += gsi::align_up(gsi_workspace_bytes(GSI_CALL_PROJECT, 0, inputs[i].d, inputs[i].k, B), 256);
    for (int j = 0; j < n_maps; ++j) off += map_part_bytes(maps[j].m, inputs[maps[j].input_id].d, B, 0);
    for (int j = 0; j < n_maps; ++j) {
      const gsi_input_desc& in = inputs[maps[j].input_id];
      const size_t bytes = fp8_expand_bytes(maps[j], in, B);
      if (!bytes) continue;
      if (expanded.empty()) expanded.assign(maps, maps + n_maps);
      void* tmp = reinterpret_cast<char*>(ws) + off;
      off += bytes;
      if (hipError_t e = gsi::expand_image_fp8(reinterpret_cast<const uint8_t*>(maps[j].M), maps[j].M_scale, maps[j].m,
                                               in.k, tmp, maps[j].wdtype, s);
          e != hipSuccess)
        return hip_fail(e, fn);
      expanded[j].M = tmp;
      expanded[j].M_scale = nullptr;
      expanded[j].flags &= ~GSI_MAP_IMAGE_FP8;
    }
    if (!expanded.empty()) maps = expanded.data();
  }

  // How each input is processed.  kVecInline: vector projection kernels, norms and gate evaluated
  // inside the single-token linear kernel (possible when B == 1 and every map reading the input takes
  // that kernel).  kVecGate: vector projection kernels followed by the fused norm + gate kernel.
  // kGeneric: generic projection kernels and the stand-alone gate kernel.
  enum { kGeneric = 0, kVecGate = 1, kVecInline = 2 };
  std::vector<int>& mode = sc.mode;
  std::vector<gsi::ProjTask>& ptask = sc.ptask;
  mode.assign(n_inputs, kGeneric);
  ptask.resize(n_inputs);
  for (int i = 0; i < n_inputs; ++i) {
    const gsi_input_desc& in = inputs[i];
    std::memset(&ptask[i], 0, sizeof(gsi::ProjTask));
    if (B == 0 || !project_vector_path(in.d, in.k, B, in.udtype, in.U)) continue;
    mode[i] = kVecGate;
    fill_proj_task(ptask[i], in.U, in.X, in.d, in.k, B, in.udtype, in.xdtype, in.C, in.R, in.rnorm, in.xnorm,
                   reinterpret_cast<char*>(ws) + ws_off[i]);
    ptask[i].mask = in.mask; ptask[i].fired_idx = in.fired_idx; ptask[i].n_fired = in.n_fired;
    if (B != 1) continue;
    int readers = 0;
    bool all_stream = true;
    for (int j = 0; j < n_maps; ++j) {
      if (maps[j].input_id != i) continue;
      ++readers;
      if (!gsi::decode_linear_ok(maps[j].m, in.d, in.k, maps[j].wdtype, maps[j].W, maps[j].M, B) ||
          !aligned(in.C, 16) || !aligned(in.R, 16) || !wx_vector_ok(in))
        all_stream = false;
    }
    if (readers > 0 && all_stream) mode[i] = kVecInline;
  }

  if (plan) {  // a plan holds the table launches of ONE set of independent inputs and nothing else
    if (B != 1 || n_inputs < 1 || n_maps < 1 || n_inputs > gsi::kMaxTabIn || n_inputs > gsi::kMaxFiredIn ||
        n_maps > gsi::kMaxTabMaps)
      return fail(GSI_ERR_SHAPE, "%s: a plan takes a single-token call of 1..%d inputs and 1..%d maps", fn,
                  std::min(gsi::kMaxTabIn, gsi::kMaxFiredIn), gsi::kMaxTabMaps);
    for (int i = 0; i < n_inputs; ++i) {
      const gsi_input_desc& in = inputs[i];
      if (in.src_map >= 0 || mode[i] != kVecInline || !(in.flags & GSI_INPUT_GATE_SINGLE_PASS) ||
          (in.flags & GSI_INPUT_FUSED_KERNEL) || !aligned(in.gram, 16) || in.udtype != inputs[0].udtype)
        return fail(GSI_ERR_SHAPE,
                    "%s: inputs[%d] cannot be planned (needs an external X, GSI_INPUT_GATE_SINGLE_PASS with a 16-byte "
                    "aligned gram, shapes and alignments of the vector kernels, one dtype for all inputs)", fn, i);
    }
    for (int j = 0; j < n_maps; ++j) {
      const gsi_map_desc& mp = maps[j];
      const gsi_input_desc& in = inputs[mp.input_id];
      if (mp.wdtype != in.udtype || in.d > gsi::kMaxStreamD ||
          mfma_gated_path(mp.W, mp.M, in.C, in.R, in.d, in.k, B, mp.wdtype, mp.m, mp.Y))
        return fail(GSI_ERR_SHAPE, "%s: maps[%d] cannot be planned", fn, j);
    }
  }

  // Single token: an input that asks for the fused kernel (GSI_INPUT_FUSED_KERNEL; gsi_fused.hip) and whose
  // basis, activations and maps all suit it is processed, with its maps, by that kernel alone.
  enum { kFusedMode = 3, kFusedDone = 4 };
  std::vector<int>& mode_separate = sc.mode_separate;  // what the separate kernels would do with each input
  mode_separate = mode;
  std::vector<char>& map_fused = sc.map_fused;
  map_fused.assign(n_maps, 0);
  if (B == 1) {
    for (int i = 0; i < n_inputs; ++i) {
      const gsi_input_desc& in = inputs[i];
      if (!(in.flags & GSI_INPUT_FUSED_KERNEL) ||
          !gsi::fused_input_ok(in.d, in.k, in.udtype, in.U, in.X, in.xdtype, in.C, in.R,
                               (in.flags & GSI_INPUT_SLOW_PATH_WX) != 0))
        continue;
      bool ok = true;
      int readers = 0;
      for (int j = 0; j < n_maps && ok; ++j) {
        if (maps[j].input_id != i) continue;
        ++readers;
        ok = maps[j].wdtype == in.udtype && !(maps[j].flags & GSI_MAP_IMAGE_FP8) &&
             gsi::fused_map_ok(maps[j].m, in.d, in.k, maps[j].wdtype, maps[j].W, maps[j].M);
      }
      if (ok && readers <= gsi::kFusedMaxMap) mode[i] = kFusedMode;
    }
  }

  // Schedule in waves: an input is ready when its producer map has been enqueued, a map when its
  // input has.  Ready inputs (maps) of one dtype that take the same kernels share a launch.
  std::vector<char>&in_done = sc.in_done, &map_done = sc.map_done, &img_done = sc.img_done;
  std::vector<char>& gate_inline = sc.gate_inline;  // the weight kernel evaluates this input's gate
  std::vector<int>& part_ncb = sc.part_ncb;         // column blocks of this input's partial projection
  in_done.assign(n_inputs, 0);
  map_done.assign(n_maps, 0);
  img_done.assign(n_maps, 0);
  gate_inline.assign(n_inputs, 0);
  part_ncb.assign(n_inputs, 1);
  int remaining = n_inputs + n_maps;
  while (remaining > 0) {
    int progressed = 0;
    std::vector<int>& ready = sc.ready;
    ready.clear();
    for (int i = 0; i < n_inputs; ++i)
      if (!in_done[i] && (inputs[i].src_map < 0 || map_done[inputs[i].src_map])) ready.push_back(i);
    // fused chunks: ready inputs of one dtype and rank are packed, with their maps, into chunks as long as a
    // chunk fits one launch's registers and scratch; up to kFusedMaxChunks chunks share a launch
    if (B == 1) {
      gsi::FusedArgs fa;
      std::memset(&fa, 0, sizeof(fa));
      fa.eps = eps;
      int fa_dt = -1;
      gsi::FusedChunk cur;
      std::memset(&cur, 0, sizeof(cur));
      int cur_dt = -1;
      auto flush = [&]() -> hipError_t {
        if (fa.n_chunks == 0) return hipSuccess;
        const bool timed = which == 0 && n_stage_launches == launch_index;
        ++n_stage_launches;
        hipError_t e = gsi::fused_launch(fa, fa_dt, s, timed ? ev_begin : nullptr, timed ? ev_end : nullptr);
        fa.n_chunks = 0;
        return e;
      };
      auto close_chunk = [&]() -> hipError_t {
        if (cur.n_in == 0) return hipSuccess;
        if (fa.n_chunks > 0 && fa_dt != cur_dt)
          if (hipError_t e = flush(); e != hipSuccess) return e;
        fa.c[fa.n_chunks++] = cur;
        fa_dt = cur_dt;
        std::memset(&cur, 0, sizeof(cur));
        if (fa.n_chunks == gsi::kFusedMaxChunks) return flush();
        return hipSuccess;
      };
      auto append = [&](gsi::FusedChunk& ch, int i) -> bool {  // input i and its maps; false when they do not fit
        const gsi_input_desc& in = inputs[i];
        if (ch.n_in == gsi::kFusedMaxIn) return false;
        if (ch.n_in > 0 && ch.k != (int)in.k) return false;
        ch.k = (int)in.k;
        const int slot = ch.n_in++;
        gsi::FusedIn& fi = ch.in[slot];
        fi.U = in.U; fi.X = in.X; fi.C = in.C; fi.R = in.R; fi.rnorm = in.rnorm; fi.xnorm = in.xnorm;
        fi.mask = in.mask; fi.fired_idx = in.fired_idx; fi.n_fired = in.n_fired;
        fi.d = (int)in.d; fi.xdtype = in.xdtype; fi.wx = (in.flags & GSI_INPUT_SLOW_PATH_WX) ? 1 : 0;
        for (int j = 0; j < n_maps; ++j) {
          if (maps[j].input_id != i) continue;
          if (ch.n_mp == gsi::kFusedMaxMap) return false;
          gsi::FusedMap& fm = ch.mp[ch.n_mp++];
          fm.W = maps[j].W; fm.M = maps[j].M; fm.Y = maps[j].Y; fm.m = (int)maps[j].m; fm.in = slot;
        }
        return gsi::fused_plan(ch, in.udtype);
      };
      for (int i : ready) {
        if (mode[i] != kFusedMode) continue;
        gsi::FusedChunk trial = cur;
        bool ok = (cur.n_in == 0 || cur_dt == inputs[i].udtype) && append(trial, i);
        if (!ok) {
          if (hipError_t e = close_chunk(); e != hipSuccess) return hip_fail(e, fn);
          std::memset(&trial, 0, sizeof(trial));
          ok = append(trial, i);
        }
        if (!ok) {  // too large for the fused kernel even alone: the separate kernels take it
          mode[i] = mode_separate[i];
          continue;
        }
        cur = trial;
        cur_dt = inputs[i].udtype;
        mode[i] = kFusedDone;
        for (int j = 0; j < n_maps; ++j)
          if (maps[j].input_id == i) { map_fused[j] = 1; img_done[j] = 1; }
      }
      if (hipError_t e = close_chunk(); e != hipSuccess) return hip_fail(e, fn);
      if (hipError_t e = flush(); e != hipSuccess) return hip_fail(e, fn);
    }
    // several tokens, or a single token whose maps do not all take the weight-streaming kernel: vector projection
    // kernels followed by the norm + gate kernel
    for (int dt = 0; dt < 2; ++dt) {
      gsi::ProjBatch pb;
      std::memset(&pb, 0, sizeof(pb));
      pb.B = (int)B;
      auto flush = [&]() -> hipError_t {
        if (pb.n == 0) return hipSuccess;
        hipError_t e = gsi::decode_project_launch(pb, dt, true, true, eps, s);
        std::memset(&pb, 0, sizeof(pb));
        pb.B = (int)B;
        return e;
      };
      for (int i : ready) {
        if (mode[i] != kVecGate || inputs[i].udtype != dt) continue;
        pb.t[pb.n++] = ptask[i];
        if (pb.n == gsi::kMaxTasks)
          if (hipError_t e = flush(); e != hipSuccess) return hip_fail(e, fn);
      }
      if (hipError_t e = flush(); e != hipSuccess) return hip_fail(e, fn);
    }
    // single token: the staged kernel.  Launch g holds the partial projections of set g (up to kMaxTasks
    // independent inputs), the coefficient sums of set g - 1, the residuals and image rows of set g - 2 and the
    // gates of set g - 3.  A call of one set skips the sum stage (its residual and image workgroups add the
    // partials themselves: the same function, the same bits).
    // With the single-pass gate (GSI_INPUT_GATE_SINGLE_PASS and a 16-byte aligned E) the stages are: partial
    // projections and shares of |x|^2 of set g; coefficient sums and shares of c^T E c of set g - 1; image rows
    // and, behind the gate their workgroups evaluate, residuals of set g - 2.
    for (int pass = 0; pass < 4 && B == 1; ++pass) {
      const int dt = pass & 1;
      const bool sp = pass >= 2;
      auto single_pass = [&](int i) {
        return (inputs[i].flags & GSI_INPUT_GATE_SINGLE_PASS) && aligned(inputs[i].gram, 16);
      };
      std::vector<int> list;
      for (int i : ready)
        if (mode[i] == kVecInline && inputs[i].udtype == dt && single_pass(i) == sp) list.push_back(i);
      if (list.empty()) continue;
      const int nsets = (int)gsi::ceil_div((int64_t)list.size(), gsi::kMaxTasks);
      for (int g = 0; g < nsets; ++g) {  // the largest input of a set goes first so that its workgroups start first
        auto first = list.begin() + (size_t)g * gsi::kMaxTasks;
        auto last = (g + 1 == nsets) ? list.end() : first + gsi::kMaxTasks;
        std::stable_sort(first, last, [&](int x, int y) {
          return inputs[x].d * inputs[x].k > inputs[y].d * inputs[y].k;
        });
      }
      auto set_size = [&](int g) {
        return (g < 0 || g >= nsets) ? 0 : std::min<int>(gsi::kMaxTasks, (int)list.size() - g * gsi::kMaxTasks);
      };
      auto member = [&](int g, int q) { return list[(size_t)g * gsi::kMaxTasks + q]; };
      const int sum_stage = (sp || nsets > 1) ? 1 : 0;
      // One set, explicit gate, and few enough maps for the weight kernel whose descriptors are kernel arguments:
      // that kernel evaluates and publishes the gates itself, which saves the gate launch.
      // (the whole call must be that small, so that none of its maps takes the weight launch over a table)
      const bool inline_gate = !sp && nsets == 1 && !plan && n_maps <= gsi::kMaxLinTasks && n_inputs <= gsi::kMaxTasks;
      if (inline_gate)
        for (int i : list) gate_inline[i] = 1;
      if (sum_stage)  // the partials are added once per input: finer slabs
        for (int i : list) gsi::stage_geom(inputs[i].d, inputs[i].k, dt, ptask[i].s_rows, ptask[i].s_slabs, true);
      if (sp && (nsets > 1 || plan) && (int)list.size() <= gsi::kMaxTabIn && n_maps > 0 && n_maps <= gsi::kMaxTabMaps) {
        // many inputs: every stage once, over a descriptor table in the workspace (three launches)
        std::vector<gsi::TabIn> tin(list.size());
        std::vector<gsi::TabMap> tmp;
        for (size_t q = 0; q < list.size(); ++q) {
          const int i = list[q];
          const gsi_input_desc& in = inputs[i];
          const gsi::ProjTask& pt = ptask[i];
          gsi::TabIn& t = tin[q];
          std::memset(&t, 0, sizeof(t));
          t.U = in.U; t.X = in.X; t.C = in.C; t.R = in.R; t.E = in.gram; t.rnorm = in.rnorm; t.xnorm = in.xnorm;
          t.mask = in.mask; t.fired_idx = in.fired_idx; t.n_fired = in.n_fired; t.part_c = pt.part_c;
          t.d = pt.d;
          t.k_rows = pt.k | (pt.s_rows << 16);
          // residual slabs of at least 256 rows: nearly all of their workgroups only evaluate the gate and leave
          const int rps = 256 / (pt.k / (dt == GSI_BF16 ? 8 : 4));
          int r_rows = pt.b_rows;
          if (r_rows < 256) r_rows = (int)(gsi::ceil_div(256, rps) * rps);
          const int r_slabs = (int)gsi::ceil_div(pt.d, r_rows);
          t.slabs = pt.s_slabs | (r_slabs << 16);
          t.r_rows_x = r_rows | (in.xdtype << 16) | ((in.flags & GSI_INPUT_SLOW_PATH_WX) ? 1 << 20 : 0);
          t.gw_off = (int)(reinterpret_cast<char*>(pt.part_n) - reinterpret_cast<char*>(pt.part_c));
          for (int j = 0; j < n_maps; ++j) {
            if (maps[j].input_id != i || maps[j].wdtype != dt || img_done[j]) continue;
            gsi::TabMap tm;
            std::memset(&tm, 0, sizeof(tm));
            tm.M = maps[j].M; tm.Y = maps[j].Y;
            tm.scale = (maps[j].flags & GSI_MAP_IMAGE_FP8) ? maps[j].M_scale : nullptr;
            tm.C = in.C;
            tm.gw = (in.flags & GSI_INPUT_SLOW_PATH_WX) ? reinterpret_cast<const double*>(pt.part_n) : nullptr;
            tm.m = (int)maps[j].m; tm.k = pt.k; tm.slabs = pt.s_slabs; tm.in = (int)q;
            tmp.push_back(tm);
            img_done[j] = 1;
          }
        }
        const int wt = (which == 0 && launch_index >= n_stage_launches && launch_index < n_stage_launches + 3)
                           ? launch_index - n_stage_launches : -1;
        n_stage_launches += 3;
        if (plan) {  // the table goes to the plan's memory; its launches are the plan's to make
          std::vector<char> host;
          if (hipError_t e = gsi::stage_table_build(tin.data(), (int)tin.size(), tmp.data(), (int)tmp.size(), dt, host,
                                                    plan->rec->sg);
              e != hipSuccess)
            return hip_fail(e, fn);
          plan->rec->stage_table = plan->dev + gsi::fired_table_bytes(n_inputs, n_maps);
          if (hipError_t e = gsi::upload_launch(host.data(), host.size(), plan->rec->stage_table, s); e != hipSuccess)
            return hip_fail(e, fn);
          plan->n_in_done += (int)tin.size();
          continue;
        }
        void* table = reinterpret_cast<char*>(ws) + gsi::fired_table_bytes(n_inputs, n_maps);
        if (hipError_t e = gsi::stage_table_run(table, tin.data(), (int)tin.size(), tmp.data(), (int)tmp.size(), dt, eps,
                                                s, wt, ev_begin, ev_end);
            e != hipSuccess)
          return hip_fail(e, fn);
        continue;
      }
      for (int g = 0; g < nsets + 2 + sum_stage - (sp || inline_gate ? 1 : 0); ++g) {
        gsi::StageArgs a;
        gsi::stage_clear(a, eps);
        {  // a set with few slabs splits the columns of its bases so that the launch still fills the chip
          int total = 0;
          for (int q = 0; q < set_size(g); ++q) total += ptask[member(g, q)].s_slabs;
          for (int q = 0; q < set_size(g); ++q) {
            const int i = member(g, q);
            int ncb = 1;
            while (total * ncb < 384 && inputs[i].k / (ncb * 2) >= 64 && (inputs[i].k / (ncb * 2)) % 64 == 0) ncb *= 2;
            part_ncb[i] = ncb;
            gsi::stage_add_part(a, ptask[i], sp ? inputs[i].gram : nullptr, ncb);
          }
        }
        if (sum_stage)
          for (int q = 0; q < set_size(g - 1); ++q) {
            const int i = member(g - 1, q);
            gsi::stage_add_cred(a, ptask[i], sp ? inputs[i].gram : nullptr);
          }
        const int gr = g - 1 - sum_stage;
        for (int q = 0; q < set_size(gr); ++q) {
          const int i = member(gr, q);
          const bool wx = (inputs[i].flags & GSI_INPUT_SLOW_PATH_WX) != 0;
          const int res = gsi::stage_add_res(a, ptask[i], sum_stage != 0, sp ? inputs[i].gram : nullptr, sp && wx);
          // One set without a sum stage: the launch before this one was the partial projections alone, in the same
          // task order.  If both launches start this input on the same XCD, the residual slabs follow the XCD order
          // of the partial slabs (second read of the basis out of the L2 that holds it).
          if (nsets == 1 && !sum_stage) {
            int a_off = 0, b_off = 0;
            for (int q2 = 0; q2 < q; ++q2) {
              const gsi::ProjTask& t2 = ptask[member(gr, q2)];
              a_off += t2.s_slabs * part_ncb[member(gr, q2)];
              b_off += t2.b_slabs;
            }
            const gsi::ProjTask& t = ptask[i];
            if (t.s_slabs % 8 == 0 && t.b_slabs % t.s_slabs == 0 && a_off % 8 == b_off % 8 &&
                (int64_t)t.s_slabs * t.s_rows == t.d && (int64_t)t.b_slabs * t.b_rows == t.d && t.b_slabs / t.s_slabs < 256)
              gsi::stage_set_res_xcd_order(a, res, t.b_slabs / t.s_slabs);
          }
          for (int j = 0; j < n_maps && a.ni < gsi::kMaxLinTasks; ++j) {
            if (maps[j].input_id != i || maps[j].wdtype != dt || img_done[j]) continue;
            gsi::stage_add_img(a, res, maps[j].M, maps[j].Y,
                               (maps[j].flags & GSI_MAP_IMAGE_FP8) ? maps[j].M_scale : nullptr, (int)maps[j].m);
            img_done[j] = 1;
          }
        }
        if (!sp && !inline_gate)
          for (int q = 0; q < set_size(gr - 1); ++q) gsi::stage_add_gate(a, ptask[member(gr - 1, q)]);
        const bool timed = which == 0 && n_stage_launches == launch_index;
        ++n_stage_launches;
        if (hipError_t e = gsi::stage_launch(a, dt, s, timed ? ev_begin : nullptr, timed ? ev_end : nullptr);
            e != hipSuccess)
          return hip_fail(e, fn);
      }
    }
    for (int i : ready) {
      const gsi_input_desc& in = inputs[i];
      if (mode[i] == kGeneric) {
        if (B > 0 && mfma_project_path(in.U, in.X, in.d, in.k, B, in.udtype, in.xdtype, in.C, in.R)) {
          // image terms of this input's maps that take the matrix-core path ride in the residual's launch
          ImageRider riders[gsi::kMaxGemmSegs - 1];
          int n_riders = 0;
          for (int j = 0; j < n_maps && n_riders < gsi::kMaxGemmSegs - 1; ++j) {
            const gsi_map_desc& mp = maps[j];
            if (mp.input_id != i || img_done[j]) continue;
            if (!mfma_gated_path(mp.W, mp.M, in.C, in.R, in.d, in.k, B, mp.wdtype, mp.m, mp.Y) || !wx_vector_ok(in))
              continue;
            riders[n_riders++] = ImageRider{mp.M, mp.Y, mp.m};
            img_done[j] = 1;
          }
          hipError_t e = mfma_project(in.U, in.X, in.d, in.k, B, in.xdtype, in.C, in.R, in.rnorm, in.xnorm, in.mask,
                                      in.fired_idx, in.n_fired, true, eps, reinterpret_cast<char*>(ws) + ws_off[i], s,
                                      riders, n_riders);
          if (e != hipSuccess) return hip_fail(e, fn);
        } else {
          if (B > 0) {
            hipError_t e = gsi::generic_project(in.U, in.X, in.d, in.k, B, in.udtype, in.xdtype, in.C, in.R,
                                                in.rnorm, in.xnorm, s);
            if (e != hipSuccess) return hip_fail(e, fn);
          }
          hipError_t e = gsi::launch_gate(in.rnorm, in.xnorm, B, eps, in.mask, in.fired_idx, in.n_fired, s);
          if (e != hipSuccess) return hip_fail(e, fn);
        }
      }
      in_done[i] = 1;
      --remaining;
      ++progressed;
    }

    std::vector<int>& mready = sc.mready;
    mready.clear();
    for (int j = 0; j < n_maps; ++j)
      if (!map_done[j] && in_done[maps[j].input_id] == 1) mready.push_back(j);
    // single token, more inputs or maps than one launch's arguments describe: one weight-streaming launch over
    // a descriptor table uploaded to the workspace
    for (int dt = 0; dt < 2 && B == 1; ++dt) {
      auto eligible = [&](int j) {
        const gsi_map_desc& mp = maps[j];
        const gsi_input_desc& in = inputs[mp.input_id];
        return !map_done[j] && !map_fused[j] && mp.wdtype == dt && in.d <= gsi::kMaxStreamD &&
               !mfma_gated_path(mp.W, mp.M, in.C, in.R, in.d, in.k, B, mp.wdtype, mp.m, mp.Y) &&
               gsi::decode_linear_ok(mp.m, in.d, in.k, mp.wdtype, mp.W, mp.M, B) && aligned(in.C, 16) &&
               aligned(in.R, 16) && wx_vector_ok(in);
      };
      std::vector<int> order;  // inputs in order of first appearance
      std::vector<int> slot(n_inputs, -1);
      int n_el = 0;
      for (int j : mready) {
        if (!eligible(j)) continue;
        ++n_el;
        if (slot[maps[j].input_id] < 0) {
          slot[maps[j].input_id] = (int)order.size();
          order.push_back(maps[j].input_id);
        }
      }
      if (((n_el <= gsi::kMaxLinTasks && (int)order.size() <= gsi::kMaxTasks) && !plan) ||
          (int)order.size() > gsi::kMaxFiredIn || n_el == 0)
        continue;  // the launch below, with its descriptors in the kernel arguments, takes them
      std::vector<gsi::FiredIn> fin(order.size());
      std::vector<gsi::FiredMap> fmp;
      fmp.reserve(n_el);
      gsi::ImgBatch sib;  // image maps y = M c not yet written by an earlier launch
      std::memset(&sib, 0, sizeof(sib));
      for (size_t q = 0; q < order.size(); ++q) {
        const gsi_input_desc& in = inputs[order[q]];
        gsi::FiredIn& f = fin[q];
        f.R = in.R; f.X = in.X; f.n_fired = in.n_fired; f.d = (int)in.d;
        f.flags = ((in.flags & GSI_INPUT_SLOW_PATH_WX) ? gsi::kFiredWx : 0) | (in.xdtype << 1);
        f.map_begin = (int)fmp.size();
        for (int j : mready) {
          if (maps[j].input_id != order[q] || !eligible(j)) continue;
          const gsi_map_desc& mp = maps[j];
          fmp.push_back(gsi::FiredMap{mp.W, mp.Y, (int)mp.m, 0});
          if (!img_done[j]) {
            if (sib.n == gsi::kMaxLinTasks) {
              if (hipError_t e = gsi::decode_image_launch(sib, dt, s); e != hipSuccess) return hip_fail(e, fn);
              std::memset(&sib, 0, sizeof(sib));
            }
            gsi::ImgTask& it = sib.t[sib.n++];
            it.M = mp.M; it.Y = mp.Y; it.part_c = nullptr; it.C = in.C; it.m = (int)mp.m; it.k = (int)in.k;
            it.a_slabs = 0; it.scale = (mp.flags & GSI_MAP_IMAGE_FP8) ? mp.M_scale : nullptr;
            img_done[j] = 1;
          }
          map_done[j] = 2;
        }
        f.map_end = (int)fmp.size();
      }
      if (sib.n > 0 && !plan)
        if (hipError_t e = gsi::decode_image_launch(sib, dt, s); e != hipSuccess) return hip_fail(e, fn);
      const size_t in_bytes = gsi::fired_table_bytes((int)fin.size(), 0);
      const size_t bytes = gsi::fired_table_bytes((int)fin.size(), (int)fmp.size());
      std::vector<char> table(bytes, 0);
      std::memcpy(table.data(), fin.data(), fin.size() * sizeof(gsi::FiredIn));
      std::memcpy(table.data() + in_bytes, fmp.data(), fmp.size() * sizeof(gsi::FiredMap));
      if (plan) {
        if (sib.n > 0 || plan->rec->has_fired)
          return fail(GSI_ERR_SHAPE, "%s: the call cannot be planned (its maps do not share one weight-streaming launch)", fn);
        if (hipError_t e = gsi::stream_fired_geom((int)fin.size(), fin.data(), fmp.data(), dt, plan->rec->fg);
            e != hipSuccess)
          return hip_fail(e, fn);
        plan->rec->fired_table = plan->dev;
        plan->rec->has_fired = 1;
        if (hipError_t e = gsi::upload_launch(table.data(), bytes, plan->dev, s); e != hipSuccess) return hip_fail(e, fn);
        plan->n_maps_done += (int)fmp.size();
        continue;
      }
      if (hipError_t e = gsi::upload_launch(table.data(), bytes, ws, s); e != hipSuccess) return hip_fail(e, fn);
      const bool timed = which == 1 && n_stream_launches == launch_index;
      ++n_stream_launches;
      if (hipError_t e = gsi::stream_fired_launch(ws, (int)fin.size(), fin.data(), fmp.data(), dt, s,
                                                  timed ? ev_begin : nullptr, timed ? ev_end : nullptr);
          e != hipSuccess)
        return hip_fail(e, fn);
    }
    for (int dt = 0; dt < 2; ++dt) {
      LinBatcher bt;
      bt.wdtype = dt; bt.s = s;
      if (which == 1) { bt.e0 = ev_begin; bt.e1 = ev_end; bt.n_launches = &n_stream_launches; bt.timed_index = launch_index; }
      bt.eps = eps;
      bt.reset(B, 0);
      for (int j : mready) {
        const gsi_map_desc& mp = maps[j];
        const gsi_input_desc& in = inputs[mp.input_id];
        if (map_done[j] || map_fused[j] || mp.wdtype != dt || B == 0) continue;
        if (mfma_gated_path(mp.W, mp.M, in.C, in.R, in.d, in.k, B, mp.wdtype, mp.m, mp.Y) && wx_vector_ok(in))
          continue;  // matrix cores below
        if (!gsi::decode_linear_ok(mp.m, in.d, in.k, mp.wdtype, mp.W, mp.M, B) || !aligned(in.C, 16) ||
            !aligned(in.R, 16) || !wx_vector_ok(in) ||
            !long_batch_ok(in.d, B, mp.Y, (in.flags & GSI_INPUT_SLOW_PATH_WX) != 0, in.X, in.xdtype))
          continue;
        gsi::LinGroup gd;
        std::memset(&gd, 0, sizeof(gd));
        gd.C = in.C; gd.R = in.R; gd.fired_idx = in.fired_idx; gd.n_fired = in.n_fired;
        gd.d = (int)in.d; gd.k = (int)in.k;
        gd.wx = (in.flags & GSI_INPUT_SLOW_PATH_WX) ? 1 : 0;
        gd.X = in.X; gd.xdtype = in.xdtype;
        if (gate_inline[mp.input_id]) {
          const gsi::ProjTask& pt = ptask[mp.input_id];
          gd.part_n = pt.part_n; gd.b_slabs = pt.b_slabs; gd.rnorm = in.rnorm; gd.xnorm = in.xnorm; gd.mask = in.mask;
          gd.fired_idx_out = in.fired_idx; gd.n_fired_out = in.n_fired;
        }
        if (hipError_t e = bt.add(mp.input_id, gd, mp.W, mp.M, mp.Y, mp.m, B == 1 && !img_done[j], part[j],
                                  (mp.flags & GSI_MAP_IMAGE_FP8) ? mp.M_scale : nullptr);
            e != hipSuccess)
          return hip_fail(e, fn);
        map_done[j] = 2;
      }
      if (hipError_t e = bt.flush(); e != hipSuccess) return hip_fail(e, fn);
    }
    for (int j : mready) {
      const gsi_map_desc& mp = maps[j];
      const gsi_input_desc& in = inputs[mp.input_id];
      if (map_done[j] != 2 && !map_fused[j] && B > 0) {
        hipError_t e;
        const bool wx = (in.flags & GSI_INPUT_SLOW_PATH_WX) != 0;
        if (mfma_gated_path(mp.W, mp.M, in.C, in.R, in.d, in.k, B, mp.wdtype, mp.m, mp.Y) && wx_vector_ok(in))
          e = mfma_gated(mp.W, mp.M, in.C, in.R, in.fired_idx, in.n_fired, mp.m, in.d, in.k, B, mp.Y, part[j], s,
                         wx ? in.X : nullptr, in.xdtype, img_done[j] != 0);
        else
          e = gsi::generic_gated_linear(mp.W, mp.M, in.C, in.R, in.fired_idx, in.n_fired, mp.m, in.d, in.k, B,
                                        mp.wdtype, mp.Y, s, wx ? in.X : nullptr, in.xdtype);
        if (e != hipSuccess) return hip_fail(e, fn);
      }
      map_done[j] = 1;
      --remaining;
      ++progressed;
    }
    if (!progressed) return fail(GSI_ERR_SHAPE, "%s: src_map dependencies form a cycle", fn);
  }
  if (n_launches) *n_launches = which == 0 ? n_stage_launches : n_stream_launches;
  if (plan && (plan->n_in_done != n_inputs || plan->n_maps_done != n_maps))
    return fail(GSI_ERR_SHAPE, "%s: the call cannot be planned (%d of %d inputs and %d of %d maps take the table launches)",
                fn, plan->n_in_done, n_inputs, plan->n_maps_done, n_maps);
  return GSI_OK;
}

size_t gsi_stack_plan_bytes(int32_t n_maps, int32_t n_inputs) {
  if (n_maps < 1 || n_inputs < 1) return 0;
  return gsi::fired_table_bytes(n_inputs, n_maps) + gsi::stage_table_bytes(n_inputs, n_maps);
}

int gsi_stack_plan_build(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                         void* ws, size_t ws_bytes, void* plan_mem, size_t plan_bytes, gsi_stack_plan* plan, void* stream) {
  const char* fn = "gsi_stack_plan_build";
  GSI_REQUIRE_PTR(plan);
  GSI_REQUIRE_PTR(plan_mem);
  std::memset(plan, 0, sizeof(*plan));
  if (!aligned(plan_mem, 256)) return fail(GSI_ERR_ALIGN, "%s: plan_mem is not aligned to 256 bytes", fn);
  if (plan_bytes < gsi_stack_plan_bytes(n_maps, n_inputs) || gsi_stack_plan_bytes(n_maps, n_inputs) == 0)
    return fail(GSI_ERR_WORKSPACE, "%s: plan_mem holds %zu bytes, the plan needs %zu", fn, plan_bytes,
                gsi_stack_plan_bytes(n_maps, n_inputs));
  PlanRec rec;
  std::memset(&rec, 0, sizeof(rec));
  PlanBuild pb;
  pb.rec = &rec;
  pb.dev = static_cast<char*>(plan_mem);
  if (int rc = layer_stack_impl(fn, maps, n_maps, inputs, n_inputs, 1, 0.f, ws, ws_bytes, stream, nullptr, nullptr, -1, 0,
                                nullptr, &pb))
    return rc;
  rec.magic = kPlanMagic;
  std::memcpy(plan, &rec, sizeof(rec));
  return GSI_OK;
}

int gsi_stack_plan_run(const gsi_stack_plan* plan, float eps, void* stream) {
  const char* fn = "gsi_stack_plan_run";
  GSI_REQUIRE_PTR(plan);
  PlanRec rec;
  std::memcpy(&rec, plan, sizeof(rec));
  if (rec.magic != kPlanMagic || !rec.stage_table || !rec.has_fired)
    return fail(GSI_ERR_SHAPE, "%s: not a plan that gsi_stack_plan_build filled", fn);
  if (!(eps >= 0.f)) return fail(GSI_ERR_SHAPE, "%s: eps must be a number >= 0", fn);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipError_t e = gsi::stage_table_launch(rec.stage_table, rec.sg, eps, s); e != hipSuccess) return hip_fail(e, fn);
  if (hipError_t e = gsi::stream_fired_run(rec.fired_table, rec.fg, s); e != hipSuccess) return hip_fail(e, fn);
  return GSI_OK;
}

}  // extern "C"
