// C ABI of libgsi: argument validation, workspace accounting and kernel selection.
// Every entry point only enqueues work on the caller's stream; nothing here synchronises,
// allocates or reads device memory.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "gsi_internal.h"

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

int gsi_version(void) { return 100; }

size_t gsi_workspace_bytes(int which_call, int64_t m, int64_t d, int64_t k, int64_t B) {
  (void)m; (void)d; (void)k; (void)B;
  switch (which_call) {
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
  hipError_t e = gsi::generic_build_image(W, U, M, m, d, k, wdtype, s);
  if (e != hipSuccess) return hip_fail(e, "gsi_build_image");
  return GSI_OK;
}

int gsi_project(const void* U, const void* X, int64_t d, int64_t k, int64_t B, int udtype, int xdtype, float* C,
                float* R, float* rnorm, float* xnorm, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(udtype) || !dtype_ok(xdtype))
    return fail(GSI_ERR_DTYPE, "gsi_project: unknown dtype (udtype %d, xdtype %d)", udtype, xdtype);
  if (int rc = check_shape("gsi_project", 1, d, k, B)) return rc;
  if (B == 0) return GSI_OK;
  GSI_REQUIRE_PTR(U);
  GSI_REQUIRE_PTR(X);
  GSI_REQUIRE_PTR(C);
  GSI_REQUIRE_PTR(R);
  GSI_REQUIRE_PTR(rnorm);
  GSI_REQUIRE_PTR(xnorm);
  GSI_REQUIRE_ALIGNED(U, gsi::elem_size(udtype));
  GSI_REQUIRE_ALIGNED(X, gsi::elem_size(xdtype));
  GSI_REQUIRE_ALIGNED(C, 4);
  GSI_REQUIRE_ALIGNED(R, 4);
  GSI_REQUIRE_ALIGNED(rnorm, 4);
  GSI_REQUIRE_ALIGNED(xnorm, 4);
  if (int rc = check_ws("gsi_project", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_PROJECT, 0, d, k, B))) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = gsi::generic_project(U, X, d, k, B, udtype, xdtype, C, R, rnorm, xnorm, s);
  if (e != hipSuccess) return hip_fail(e, "gsi_project");
  return GSI_OK;
}

int gsi_gate(const float* rnorm, const float* xnorm, int64_t B, float eps, uint8_t* mask, int32_t* fired_idx,
             int32_t* n_fired, void* stream) {
  if (B < 0 || B > (1ll << 30)) return fail(GSI_ERR_SHAPE, "gsi_gate: B = %lld out of range", (long long)B);
  if (!(eps == eps)) return fail(GSI_ERR_SHAPE, "gsi_gate: eps is NaN");
  GSI_REQUIRE_PTR(n_fired);
  GSI_REQUIRE_ALIGNED(n_fired, 4);
  if (B > 0) {
    GSI_REQUIRE_PTR(rnorm);
    GSI_REQUIRE_PTR(xnorm);
    GSI_REQUIRE_PTR(mask);
    GSI_REQUIRE_PTR(fired_idx);
    GSI_REQUIRE_ALIGNED(rnorm, 4);
    GSI_REQUIRE_ALIGNED(xnorm, 4);
    GSI_REQUIRE_ALIGNED(fired_idx, 4);
  }
  // B == 0 still launches: the count must read 0 afterwards.
  hipError_t e = gsi::launch_gate(rnorm, xnorm, B, eps, mask, fired_idx, n_fired, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "gsi_gate");
  return GSI_OK;
}

int gsi_gated_linear(const void* W, const void* M, const float* C, const float* R, const int32_t* fired_idx,
                     const int32_t* n_fired, int64_t m, int64_t d, int64_t k, int64_t B, int wdtype, void* Y,
                     int ydtype, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(wdtype)) return fail(GSI_ERR_DTYPE, "gsi_gated_linear: unknown wdtype %d", wdtype);
  if (ydtype != GSI_F32) return fail(GSI_ERR_DTYPE, "gsi_gated_linear: ydtype must be GSI_F32, got %d", ydtype);
  if (int rc = check_shape("gsi_gated_linear", m, d, k, B)) return rc;
  if (B == 0) return GSI_OK;
  GSI_REQUIRE_PTR(W);
  GSI_REQUIRE_PTR(M);
  GSI_REQUIRE_PTR(C);
  GSI_REQUIRE_PTR(R);
  GSI_REQUIRE_PTR(fired_idx);
  GSI_REQUIRE_PTR(n_fired);
  GSI_REQUIRE_PTR(Y);
  const size_t es = gsi::elem_size(wdtype);
  GSI_REQUIRE_ALIGNED(W, es);
  GSI_REQUIRE_ALIGNED(M, es);
  GSI_REQUIRE_ALIGNED(C, 4);
  GSI_REQUIRE_ALIGNED(R, 4);
  GSI_REQUIRE_ALIGNED(fired_idx, 4);
  GSI_REQUIRE_ALIGNED(n_fired, 4);
  GSI_REQUIRE_ALIGNED(Y, 4);
  if (int rc = check_ws("gsi_gated_linear", ws, ws_bytes, gsi_workspace_bytes(GSI_CALL_GATED_LINEAR, m, d, k, B)))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = gsi::generic_gated_linear(W, M, C, R, fired_idx, n_fired, m, d, k, B, wdtype, (float*)Y, s);
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
  hipError_t e = gsi::generic_dense_linear(W, X, m, d, B, wdtype, xdtype, Y, s);
  if (e != hipSuccess) return hip_fail(e, "gsi_dense_linear");
  return GSI_OK;
}

size_t gsi_layer_stack_workspace_bytes(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs,
                                       int32_t n_inputs, int64_t B) {
  if (!maps || !inputs || n_maps < 0 || n_inputs < 0) return 0;
  size_t need = 0;
  for (int i = 0; i < n_inputs; ++i) {
    const size_t w = gsi_workspace_bytes(GSI_CALL_PROJECT, 0, inputs[i].d, inputs[i].k, B);
    if (w > need) need = w;
  }
  for (int j = 0; j < n_maps; ++j) {
    const int id = maps[j].input_id;
    if (id < 0 || id >= n_inputs) continue;
    const size_t w = gsi_workspace_bytes(GSI_CALL_GATED_LINEAR, maps[j].m, inputs[id].d, inputs[id].k, B);
    if (w > need) need = w;
  }
  return need;
}

int gsi_layer_stack(const gsi_map_desc* maps, int32_t n_maps, const gsi_input_desc* inputs, int32_t n_inputs,
                    int64_t B, float eps, void* ws, size_t ws_bytes, void* stream) {
  if (n_maps < 0 || n_inputs < 0) return fail(GSI_ERR_SHAPE, "gsi_layer_stack: negative count");
  if (n_maps > 0) GSI_REQUIRE_PTR(maps);
  if (n_inputs > 0) GSI_REQUIRE_PTR(inputs);
  if (B < 0) return fail(GSI_ERR_SHAPE, "gsi_layer_stack: B = %lld < 0", (long long)B);
  for (int j = 0; j < n_maps; ++j) {
    const int id = maps[j].input_id;
    if (id < 0 || id >= n_inputs)
      return fail(GSI_ERR_SHAPE, "gsi_layer_stack: maps[%d].input_id = %d out of range", j, id);
  }
  for (int i = 0; i < n_inputs; ++i) {
    const int sm = inputs[i].src_map;
    if (sm < -1 || sm >= n_maps)
      return fail(GSI_ERR_SHAPE, "gsi_layer_stack: inputs[%d].src_map = %d out of range", i, sm);
    if (sm >= 0) {
      if (inputs[i].X != (const void*)maps[sm].Y)
        return fail(GSI_ERR_SHAPE, "gsi_layer_stack: inputs[%d].X must be maps[%d].Y", i, sm);
      if (inputs[i].xdtype != GSI_F32 || inputs[i].d != maps[sm].m)
        return fail(GSI_ERR_SHAPE, "gsi_layer_stack: inputs[%d] does not match the output of maps[%d]", i, sm);
    }
  }
  if (int rc = check_ws("gsi_layer_stack", ws, ws_bytes,
                        gsi_layer_stack_workspace_bytes(maps, n_maps, inputs, n_inputs, B)))
    return rc;

  // Schedule: an input is ready when its producer map has been enqueued; a map when its input has.
  std::vector<char> in_done(n_inputs, 0), map_done(n_maps, 0);
  int remaining = n_inputs + n_maps;
  while (remaining > 0) {
    int progressed = 0;
    for (int i = 0; i < n_inputs; ++i) {
      if (in_done[i]) continue;
      const gsi_input_desc& in = inputs[i];
      if (in.src_map >= 0 && !map_done[in.src_map]) continue;
      if (int rc = gsi_project(in.U, in.X, in.d, in.k, B, in.udtype, in.xdtype, in.C, in.R, in.rnorm, in.xnorm, ws,
                               ws_bytes, stream))
        return rc;
      if (int rc = gsi_gate(in.rnorm, in.xnorm, B, eps, in.mask, in.fired_idx, in.n_fired, stream)) return rc;
      in_done[i] = 1;
      --remaining;
      ++progressed;
    }
    for (int j = 0; j < n_maps; ++j) {
      if (map_done[j] || !in_done[maps[j].input_id]) continue;
      const gsi_map_desc& mp = maps[j];
      const gsi_input_desc& in = inputs[mp.input_id];
      if (int rc = gsi_gated_linear(mp.W, mp.M, in.C, in.R, in.fired_idx, in.n_fired, mp.m, in.d, in.k, B,
                                    mp.wdtype, mp.Y, GSI_F32, ws, ws_bytes, stream))
        return rc;
      map_done[j] = 1;
      --remaining;
      ++progressed;
    }
    if (!progressed) return fail(GSI_ERR_SHAPE, "gsi_layer_stack: src_map dependencies form a cycle");
  }
  return GSI_OK;
}

}  // extern "C"
