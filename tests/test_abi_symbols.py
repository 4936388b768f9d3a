"""The C-ABI library loads on a machine without a GPU and exports every symbol include/gsi.h declares."""
import ctypes
import os
import re

from conftest import ROOT

HEADER = os.path.join(ROOT, "include", "gsi.h")
LIB = os.path.join(ROOT, "paper_2605_03109_amd", "libgsi.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gsi_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for required in ("gsi_build_image", "gsi_project", "gsi_gate", "gsi_gated_linear", "gsi_layer_stack",
                     "gsi_dense_linear", "gsi_workspace_bytes", "gsi_last_error"):
        assert required in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "libgsi.so is not built: run python -m paper_2605_03109_amd.build"
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in gsi.h but not exported"


def test_binding_lists_the_same_symbols():
    from paper_2605_03109_amd import gsi

    assert sorted(gsi.EXPORTS) == declared_functions()
    assert gsi.version() >= 100


def test_host_side_validation_needs_no_gpu():
    """Argument errors are detected on the host before any launch, so they can be checked here."""
    from paper_2605_03109_amd import gsi

    lib = gsi.lib
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert lib.gsi_build_image(None, one, one, 4, 4, 2, gsi.GSI_F32, None, 0, None) == gsi.GSI_ERR_NULL
    assert b"W is NULL" in lib.gsi_last_error()
    assert lib.gsi_build_image(one, one, one, 4, 4, 5, gsi.GSI_F32, None, 0, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_build_image(one, one, one, 4, 4, 0, gsi.GSI_F32, None, 0, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_build_image(one, one, one, 0, 4, 2, gsi.GSI_F32, None, 0, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_build_image(one, one, one, 4, 4, 2, 7, None, 0, None) == gsi.GSI_ERR_DTYPE
    odd = ctypes.c_void_p(257)
    assert lib.gsi_build_image(odd, one, one, 4, 4, 2, gsi.GSI_F32, None, 0, None) == gsi.GSI_ERR_ALIGN
    assert lib.gsi_project(one, one, 8, 9, 1, 0, 0, one, one, one, one, None, 0, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_project(one, one, 8, 2, -1, 0, 0, one, one, one, one, None, 0, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_project(one, one, 8, 2, 0, 0, 0, None, None, None, None, None, 0, None) == gsi.GSI_OK  # B = 0
    assert lib.gsi_gated_linear(one, one, one, one, one, one, 4, 4, 2, 1, 0, one, gsi.GSI_BF16, None, 0, None) \
        == gsi.GSI_ERR_DTYPE
    assert lib.gsi_gate(one, one, 3, ctypes.c_float(0.05), one, one, None, None) == gsi.GSI_ERR_NULL
    assert lib.gsi_gate(one, one, -1, ctypes.c_float(0.05), one, one, one, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_dense_linear(one, None, 4, 4, 1, 0, 0, one, None, 0, None) == gsi.GSI_ERR_NULL
    # descriptor tables: bad input id, dependency cycle
    mp = (gsi.MapDesc * 1)()
    inp = (gsi.InputDesc * 1)()
    mp[0].input_id = 3
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_SHAPE
    mp[0].input_id, mp[0].Y, mp[0].m, mp[0].W, mp[0].M = 0, 256, 8, 256, 256
    inp[0].src_map, inp[0].X, inp[0].d, inp[0].k, inp[0].xdtype = 0, 256, 8, 2, 0
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_NULL
    for f in ("U", "C", "R", "rnorm", "xnorm", "mask", "fired_idx", "n_fired"):
        setattr(inp[0], f, 256)
    # (a single-token call keeps a small descriptor table in the workspace)
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_WORKSPACE
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), one, 1 << 20, None) == gsi.GSI_ERR_SHAPE
    assert b"cycle" in lib.gsi_last_error()
    # unknown bits in an input's flags are refused before anything runs
    inp[0].flags = 8
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_SHAPE
    assert b"flags" in lib.gsi_last_error()
    # the single-pass gate needs its cached matrix
    inp[0].flags = gsi.INPUT_GATE_SINGLE_PASS
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_NULL
    assert b"gram" in lib.gsi_last_error()
    inp[0].flags = 0
    assert lib.gsi_build_gram(one, 8, 9, gsi.GSI_F32, one, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_build_gram(one, 8, 2, gsi.GSI_F32, None, None) == gsi.GSI_ERR_NULL
    assert lib.gsi_build_gram(one, 8, 2, 5, one, None) == gsi.GSI_ERR_DTYPE
    # the rank-1 basis extension
    em = (gsi.ExtendMap * 1)()
    args = lambda **kw: [kw.get("U", one), kw.get("d", 8), kw.get("K", 4), kw.get("dt", gsi.GSI_F32), kw.get("kc", one), one,
                         one, one, ctypes.c_float(kw.get("tau", 0.1)), em, kw.get("n", 0), None, None, kw.get("ws", one),
                         kw.get("wsn", 1 << 20), None]
    assert lib.gsi_extend_basis(*args(U=None)) == gsi.GSI_ERR_NULL
    assert lib.gsi_extend_basis(*args(kc=None)) == gsi.GSI_ERR_NULL
    assert lib.gsi_extend_basis(*args(K=9)) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_extend_basis(*args(dt=3)) == gsi.GSI_ERR_DTYPE
    assert lib.gsi_extend_basis(*args(tau=-1.0)) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_extend_basis(*args(n=1)) == gsi.GSI_ERR_NULL      # maps[0].W is NULL
    assert lib.gsi_extend_basis(*args(ws=None, wsn=0)) == gsi.GSI_ERR_WORKSPACE
    assert lib.gsi_extend_basis_workspace_bytes(4096, 256) > 0 and lib.gsi_extend_basis_workspace_bytes(0, 4) == 0
    # ... and the same step for several bases in one call
    ed = (gsi.ExtendDesc * 2)()
    for e in ed:
        e.U, e.d, e.K, e.udtype, e.n_maps = 256, 8, 4, gsi.GSI_F32, 0
        e.k_cur = e.R = e.rnorm = e.xnorm = 256
    tau = ctypes.c_float(0.1)
    need = lib.gsi_extend_many_workspace_bytes(ed, 2)
    assert need > 2 * lib.gsi_extend_basis_workspace_bytes(8, 4)  # two workspaces + the descriptor table
    assert lib.gsi_extend_many(ed, 0, tau, None, 0, None) == gsi.GSI_OK
    assert lib.gsi_extend_many(None, 2, tau, one, need, None) == gsi.GSI_ERR_NULL
    assert lib.gsi_extend_many(ed, 2, tau, None, 0, None) == gsi.GSI_ERR_WORKSPACE
    assert lib.gsi_extend_many(ed, 2, tau, odd, need, None) == gsi.GSI_ERR_ALIGN
    assert lib.gsi_extend_many(ed, 2, ctypes.c_float(-1.0), one, need, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_extend_many(ed, 70000, tau, one, need, None) == gsi.GSI_ERR_SHAPE
    ed[1].udtype = gsi.GSI_BF16
    assert lib.gsi_extend_many(ed, 2, tau, one, need, None) == gsi.GSI_ERR_DTYPE
    assert b"share one storage type" in lib.gsi_last_error()
    ed[1].udtype = gsi.GSI_F32
    ed[1].k_cur = None
    assert lib.gsi_extend_many(ed, 2, tau, one, need, None) == gsi.GSI_ERR_NULL
    assert b"basis 1" in lib.gsi_last_error()
    ed[1].k_cur = 256
    ed[1].K = 9
    assert lib.gsi_extend_many_workspace_bytes(ed, 2) > 0
    assert lib.gsi_extend_many(ed, 2, tau, one, 1 << 20, None) == gsi.GSI_ERR_SHAPE
    ed[1].K = 0
    assert lib.gsi_extend_many_workspace_bytes(ed, 2) == 0
    # a dense stack of several tokens needs its workspace
    inp[0].src_map = -1
    mp[0].m, inp[0].d, inp[0].k = 64, 64, 32
    need = lib.gsi_dense_stack_workspace_bytes(mp, 1, inp, 1, 4)
    assert need > 0 and lib.gsi_dense_stack_workspace_bytes(mp, 1, inp, 1, 1) == 0
    assert lib.gsi_dense_stack(mp, 1, inp, 1, 4, None, 0, None) == gsi.GSI_ERR_WORKSPACE
    # the 8-bit image: quantiser arguments, and maps that carry one
    assert lib.gsi_quantize_image_fp8(one, gsi.GSI_BF16, 4, 4, one, None, None) == gsi.GSI_ERR_NULL
    assert lib.gsi_quantize_image_fp8(one, 2, 4, 4, one, one, None) == gsi.GSI_ERR_DTYPE
    assert lib.gsi_quantize_image_fp8(one, gsi.GSI_F32, 0, 4, one, one, None) == gsi.GSI_ERR_SHAPE
    assert lib.gsi_quantize_image_fp8(odd, gsi.GSI_F32, 4, 4, one, one, None) == gsi.GSI_ERR_ALIGN
    mp[0].flags = 4
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 1, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_SHAPE
    assert b"maps[0].flags" in lib.gsi_last_error()
    mp[0].flags = gsi.MAP_IMAGE_FP8
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 2, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_NULL
    assert b"M_scale" in lib.gsi_last_error()
    mp[0].M_scale = 258
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 2, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_ALIGN
    mp[0].M_scale = 256
    # several tokens: the image is expanded to the weights' type in the workspace, which the query accounts for
    mp[0].flags = 0
    plain = lib.gsi_layer_stack_workspace_bytes(mp, 1, inp, 1, 4)
    mp[0].flags = gsi.MAP_IMAGE_FP8
    assert lib.gsi_layer_stack_workspace_bytes(mp, 1, inp, 1, 4) == plain + 64 * 32 * 4
    assert lib.gsi_layer_stack(mp, 1, inp, 1, 4, ctypes.c_float(0.05), None, 0, None) == gsi.GSI_ERR_WORKSPACE
