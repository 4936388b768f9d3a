"""GPU parity: libgsi (through the C ABI) against the fp64 CPU oracle on the same seeded inputs."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle.gsi_oracle as O  # noqa: E402
from paper_2605_03109_amd import workload as wl  # noqa: E402


@pytest.fixture(scope="module")
def gsi():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2605_03109_amd import gsi as g

    return g


@pytest.fixture(scope="module")
def pu(gsi):
    import parity_util

    return parity_util


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------------
# config 0: GPT-2-small MLP up-projection, fp32, 16 decode tokens one at a time, 4 fired
# ------------------------------------------------------------------------------------------------
def test_gpt2_mlp_up_fp32_decode(gsi, pu):
    w = wl.gpt2_mlp_up()
    g = w.groups[0]
    say(f"case {w.name}: d={g.d} k={g.k} m={g.maps[0][1]} T={w.T}")
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    worst = pu.check_group(w, g, [(t, t + 1) for t in range(w.T)], dg, og)
    ref = og.run()
    assert ref["n"] == 4
    worst_b = pu.check_group(w, g, [(0, w.T)], dg, og)  # the same 16 tokens as one batch
    say(f"  worst rel-L2 {max(worst, worst_b):.3e}")
    assert max(worst, worst_b) <= 1e-5


# ------------------------------------------------------------------------------------------------
# odd / tiny shapes (generic kernels), both dtypes
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("wdtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,k,m,T,nf", [(12, 3, 5, 4, 2), (33, 7, 10, 5, 1), (100, 100, 9, 3, 0), (257, 19, 65, 70, 9),
                                        (64, 8, 16, 3, 3), (1, 1, 1, 2, 0)])
def test_small_and_odd_shapes(gsi, pu, wdtype, d, k, m, T, nf):
    w = wl.tiny(d, k, m, T, nf, seed=1000 + d + k, wdtype=wdtype)
    say(f"case tiny d={d} k={k} m={m} T={T} nf={nf} {wdtype}")
    pu.check_group(w, w.groups[0], [(0, T)] + [(t, t + 1) for t in range(min(T, 3))])


# ------------------------------------------------------------------------------------------------
# mid-size shapes that span several tiles and ragged tails, aligned for the vector kernels
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("wdtype", ["bf16", "f32"])
@pytest.mark.parametrize("d,k,m,T,nf", [(1024, 64, 520, 9, 3), (776, 72, 1000, 5, 2), (4096, 256, 1032, 6, 2),
                                        (2048, 128, 264, 33, 7), (4096, 512, 512, 3, 1), (8192, 32, 300, 2, 1),
                                        (16384, 512, 520, 3, 1), (16384, 64, 264, 3, 1), (4160, 128, 264, 4, 2),
                                        (16384, 64, 264, 4, 1)])  # (the last: four tokens through the d = 16384 LDS limit)
def test_mid_shapes(gsi, pu, wdtype, d, k, m, T, nf):
    w = wl.tiny(d, k, m, T, nf, seed=2000 + d + k + m, wdtype=wdtype)
    say(f"case mid d={d} k={k} m={m} T={T} nf={nf} {wdtype}")
    worst = pu.check_group(w, w.groups[0], [(0, T), (0, 1), (T - 1, T)])
    say(f"  worst rel-L2 {worst:.3e}")


# ------------------------------------------------------------------------------------------------
# at and beyond the limits of the vector kernels: inputs of up to 65536 elements take them for the projection
# (32 slabs of 2048 rows), longer ones and ranks above 512 the generic kernels; the linear maps of an input longer
# than 16384 elements take the generic kernels too
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,m,T,nf,wdtype", [(32768, 64, 264, 4, 2, "bf16"), (65536, 8, 40, 3, 1, "bf16"),
                                               (69632, 16, 24, 3, 1, "bf16"), (2048, 1024, 64, 3, 1, "bf16"),
                                               (20480, 128, 136, 5, 2, "bf16"), (32768, 32, 72, 3, 1, "f32"),
                                               (32768, 256, 520, 20, 6, "bf16")])
def test_shapes_at_and_beyond_the_vector_kernels_limits(gsi, pu, d, k, m, T, nf, wdtype):
    w = wl.tiny(d, k, m, T, nf, seed=2300 + d + k + m, wdtype=wdtype)
    say(f"case limits d={d} k={k} m={m} T={T} nf={nf} {wdtype}")
    g = w.groups[0]
    dg = pu.DeviceGroup(w, g)
    worst = pu.check_group(w, g, [(0, T), (0, 1), (T - 1, T)], dg)
    say(f"  worst rel-L2 {worst:.3e}")
    # the same tokens as one batch through gsi_layer_stack: the bits of the separate calls, and the dense product
    sep = pu.run_separate_calls(dg, w.eps)
    st = gsi.layer_stack([{"U": dg.U, "X": dg.X}], [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}], T, w.eps)
    torch.cuda.synchronize()
    for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired"):
        assert torch.equal(st.inputs_t[0][key], sep[key]), key
    assert torch.equal(st.maps_t[0]["Y"], sep["Y"]["w"])
    Yd = gsi.dense_linear(dg.W["w"], dg.X).cpu().numpy().astype(np.float64)
    og = pu.OracleGroup(w, g)
    assert pu.rel_l2_rows(Yd, O.dense_linear(og.W["w"], og.X)).max() <= 2e-5


# ------------------------------------------------------------------------------------------------
# decode batches (2..128 tokens a call): one to eight token tiles, fired counts from none to all,
# ragged row and token tails, the long fc_out-shaped contraction
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,m,T,nf", [(4096, 256, 1032, 64, 10), (2048, 128, 520, 128, 128), (1024, 96, 260, 17, 0),
                                        (16384, 256, 528, 16, 3), (1024, 64, 512, 100, 40), (4096, 512, 256, 2, 1),
                                        (1024, 32, 36, 33, 20)])
def test_decode_batches(gsi, pu, d, k, m, T, nf):
    w = wl.tiny(d, k, m, T, nf, seed=2500 + d + k + m + T, wdtype="bf16")
    say(f"case batch d={d} k={k} m={m} T={T} nf={nf}")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    worst = pu.check_group(w, g, [(0, T), (0, min(T, 5)), (T // 2, T)], dg, og)
    name = g.maps[0][0]
    Yd = gsi.dense_linear(dg.W[name], dg.X).cpu().numpy().astype(np.float64)
    dense_err = pu.rel_l2_rows(Yd, O.dense_linear(og.W[name], og.X)).max()
    say(f"  worst rel-L2 {worst:.3e}, dense {dense_err:.3e}")
    assert dense_err <= 2e-5


# ------------------------------------------------------------------------------------------------
# degenerate gates
# ------------------------------------------------------------------------------------------------
def test_all_fire_equals_dense_and_none_fire_is_static_projection(gsi, pu):
    w = wl.tiny(512, 64, 384, 8, 3, seed=31, wdtype="bf16")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    C, R, rn, xn = gsi.project(dg.U, dg.X)
    name = g.maps[0][0]
    # eps = 0: every token fires and y must equal the dense product W x (Eq. (exact))
    mask, idx, n = gsi.gate(rn, xn, 0.0)
    assert int(n.item()) == 8 and mask.cpu().numpy().all()
    Y = gsi.gated_linear(dg.W[name], dg.M[name], C, R, idx, n).cpu().numpy().astype(np.float64)
    Yd = O.dense_linear(og.W[name], og.X)
    assert pu.rel_l2_rows(Y, Yd).max() <= 2e-3
    Ydense = gsi.dense_linear(dg.W[name], dg.X).cpu().numpy().astype(np.float64)
    assert pu.rel_l2_rows(Ydense, Yd).max() <= 2e-5
    # eps > 1: no token fires, y = (W U) U^T x for every token
    mask, idx, n = gsi.gate(rn, xn, 1.5)
    assert int(n.item()) == 0 and not mask.cpu().numpy().any()
    Y = gsi.gated_linear(dg.W[name], dg.M[name], C, R, idx, n).cpu().numpy().astype(np.float64)
    ref = og.run()
    Ys = O.gated_linear(og.W[name], og.M[name], ref["C"], ref["R"], np.zeros(8, dtype=np.uint8))
    assert pu.rel_l2_rows(Y, Ys).max() <= 2e-3


def test_zero_token_and_full_rank_basis(gsi, pu):
    # x = 0: rho := 0, not fired, y = 0
    w = wl.tiny(256, 32, 300, 4, 2, seed=41, wdtype="f32")
    g = w.groups[0]
    g.X[1, :] = 0.0
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    res = pu.run_separate_calls(dg, w.eps)
    assert res["mask"].cpu().numpy()[1] == 0
    assert float(res["xnorm"][1]) == 0.0 and float(res["rnorm"][1]) == 0.0
    assert not res["Y"]["w"][1].cpu().numpy().any()
    pu.check_group(w, g, [(0, 4)], dg, og)
    # k = d: r = 0 up to rounding, nothing fires at eps = 0.05, y = W x
    w2 = wl.tiny(64, 64, 300, 3, 0, seed=43, wdtype="f32")
    dg2, og2 = pu.DeviceGroup(w2, w2.groups[0]), pu.OracleGroup(w2, w2.groups[0])
    res2 = pu.run_separate_calls(dg2, w2.eps)
    assert int(res2["n_fired"].item()) == 0
    Y = res2["Y"]["w"].cpu().numpy().astype(np.float64)
    assert pu.rel_l2_rows(Y, O.dense_linear(og2.W["w"], og2.X)).max() <= 1e-5


def test_empty_batch(gsi):
    U = torch.zeros((16, 4), device="cuda")
    X = torch.zeros((0, 16), device="cuda")
    C, R, rn, xn = gsi.project(U, X)
    assert C.shape == (0, 4)
    n = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    mask, idx, n = gsi.gate(rn, xn, 0.05, n_fired=n)
    assert int(n.item()) == 0  # the count is written even for an empty batch
    W = torch.zeros((8, 16), device="cuda")
    M = torch.zeros((8, 4), device="cuda")
    Y = gsi.gated_linear(W, M, C, R, idx, n)
    assert Y.shape == (0, 8)


def test_gate_compaction_many_tokens(gsi):
    # ragged: B not a multiple of the 256-token chunk, ties exactly at eps, zeros
    rng = np.random.default_rng(5)
    B = 1000
    eps = np.float32(0.05)
    xn = rng.random(B).astype(np.float32) + 0.5
    rho = rng.random(B).astype(np.float32) * 0.1
    rn = (rho * xn).astype(np.float32)
    xn[17] = 0.0
    rn[17] = 0.0
    rn[100] = eps  # rho == eps exactly with xn = 1
    xn[100] = 1.0
    mask, idx, n = gsi.gate(torch.from_numpy(rn).cuda(), torch.from_numpy(xn).cuda(), float(eps))
    with np.errstate(divide="ignore", invalid="ignore"):
        exp = (xn > 0) & ((rn / xn) >= eps)  # same fp32 division as the kernel: bit-exact expectation
    assert np.array_equal(mask.cpu().numpy().astype(bool), exp)
    assert exp[100] and not exp[17]
    nn = int(n.item())
    assert nn == exp.sum()
    assert np.array_equal(idx.cpu().numpy()[:nn], np.nonzero(exp)[0])
    # and against the oracle outside the band
    m_or, idx_or, n_or = O.gate(rn.astype(np.float64), xn.astype(np.float64), float(eps))
    rho64 = O.residual_ratio(rn.astype(np.float64), xn.astype(np.float64))
    decided = np.abs(rho64 - float(eps)) >= 1e-4
    assert np.array_equal(mask.cpu().numpy()[decided], m_or[decided])


# ------------------------------------------------------------------------------------------------
# layer stack: equals the separate calls bit for bit, and the oracle within the bars
# ------------------------------------------------------------------------------------------------
def _stack_for(gsi, pu, w, B):
    dgs = [pu.DeviceGroup(w, g) for g in w.groups]
    inputs, maps, names = [], [], []
    for gi, dg in enumerate(dgs):
        inputs.append({"U": dg.U, "X": dg.X})
        for name in dg.W:
            maps.append({"W": dg.W[name], "M": dg.M[name], "input_id": gi})
            names.append((gi, name))
    return dgs, inputs, maps, names


def test_layer_stack_block_decode(gsi, pu):
    w = wl.transformer_block("blk", d=512, ffn=2048, k=64, T=12, fire_rate=0.25, p=1.5, seed=77)
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, 1)
    ogs = [pu.OracleGroup(w, g) for g in w.groups]
    T = w.T
    # whole-buffer stack object, advanced one decode token at a time
    full_inputs = [{"U": dg.U, "X": dg.X} for dg in dgs]
    st = gsi.LayerStack(full_inputs, maps, T, w.eps)
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()
    for gi, (dg, og) in enumerate(zip(dgs, ogs)):
        ref = og.run()
        assert ref["n"] == 3
        sep = pu.run_separate_calls(dg, w.eps)  # all T tokens as one batch
        ti = st.inputs_t[gi]
        # per-token decode through the stack vs one batched call: same kernels per token => same bits
        for key in ("C", "R", "rnorm", "xnorm", "mask"):
            a, b = ti[key].cpu().numpy(), sep[key].cpu().numpy()
            assert np.allclose(a, b, rtol=1e-5, atol=1e-5), key
        res = dict(C=ti["C"], R=ti["R"], rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                   n_fired=sep["n_fired"], fired_idx=sep["fired_idx"])
        mask = pu.check_projection(res, ref, w.eps)
        for j, (g2, name) in enumerate(names):
            if g2 != gi:
                continue
            pu.check_outputs(st.maps_t[j]["Y"], og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype, ref, mask)


def test_layer_stack_equals_separate_calls_bitwise(gsi, pu):
    w = wl.transformer_block("blk", d=256, ffn=1024, k=32, T=7, fire_rate=0.3, p=1.5, seed=78)
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, w.T)
    st = gsi.layer_stack(inputs, maps, w.T, w.eps)
    torch.cuda.synchronize()
    for gi, dg in enumerate(dgs):
        sep = pu.run_separate_calls(dg, w.eps)
        ti = st.inputs_t[gi]
        for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired"):
            assert torch.equal(ti[key], sep[key]), key
        n = int(sep["n_fired"].item())
        assert torch.equal(ti["fired_idx"][:n], sep["fired_idx"][:n])
        for j, (g2, name) in enumerate(names):
            if g2 == gi:
                assert torch.equal(st.maps_t[j]["Y"], sep["Y"][name]), name


@pytest.mark.parametrize("wx", [False, True])
def test_many_inputs_in_one_single_token_call(gsi, pu, wx):
    """Five blocks (20 inputs, 30 maps) in ONE call per token: more inputs than one launch of the staged kernel
    holds, so the stages of the two sets (partial projections, coefficient sums, residuals and image rows, gates)
    share launches, and the weight rows of all fired inputs are streamed by ONE launch over a descriptor table in
    the workspace.  The result must equal block-by-block calls (one set: no sum stage; descriptors in the kernel
    arguments)
    bit for bit -- on a workspace that starts out filled with ones, and again on the second pass over the tokens."""
    L, T = 5, 6
    ws_blocks = [wl.transformer_block(f"blk{l}", d=512, ffn=2048, k=64, T=T, fire_rate=0.34, p=1.5, seed=500 + l)
                 for l in range(L)]
    inputs, maps, per_block = [], [], []
    for w in ws_blocks:
        dgs, bi, bm, _ = _stack_for(gsi, pu, w, 1)
        if wx:
            bi = [dict(i, flags=gsi.INPUT_SLOW_PATH_WX) for i in bi]
        base = len(inputs)
        inputs += bi
        maps += [dict(m, input_id=m["input_id"] + base) for m in bm]
        per_block.append((bi, bm))
    eps = ws_blocks[0].eps
    say(f"case {len(inputs)} inputs / {len(maps)} maps in one call per token")
    st = gsi.LayerStack(inputs, maps, T, eps)
    st.refresh(token_offset=0, B=1)
    st.ws.fill_(0xFF)
    for rep in range(2):
        for t in range(T):
            st.refresh(token_offset=t, B=1)
            st.run()
    torch.cuda.synchronize()
    n_in = n_mp = 0
    for bi, bm in per_block:
        ref = gsi.LayerStack(bi, bm, T, eps)
        for t in range(T):
            ref.refresh(token_offset=t, B=1)
            ref.run()
        torch.cuda.synchronize()
        for a in ref.inputs_t:
            b = st.inputs_t[n_in]
            for key in ("C", "R", "rnorm", "xnorm", "mask"):
                assert torch.equal(a[key], b[key]), (n_in, key)
            n_in += 1
        for a in ref.maps_t:
            assert torch.equal(a["Y"], st.maps_t[n_mp]["Y"]), n_mp
            n_mp += 1
    # and against the oracle for the first and the last block
    for l in (0, L - 1):
        w = ws_blocks[l]
        for gi, g in enumerate(w.groups):
            og = pu.OracleGroup(w, g)
            ref = og.run()
            ti = st.inputs_t[4 * l + gi]
            res = dict(C=ti["C"], R=ti["R"], rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                       n_fired=torch.tensor([int(ti["mask"].sum().item())], dtype=torch.int32),
                       fired_idx=torch.nonzero(ti["mask"]).flatten().to(torch.int32))
            pu.check_projection(res, ref, eps)


def test_layer_stack_true_chain(gsi, pu):
    """Two maps chained: the second input is the first map's output (src_map = 0)."""
    rng = np.random.default_rng(3)
    d0, k0, m0, k1, m1, B = 256, 32, 384, 48, 200, 5
    w = wl.tiny(d0, k0, m0, B, 2, seed=91, wdtype="bf16")
    g = w.groups[0]
    dg = pu.DeviceGroup(w, g)
    U1 = wl.store(wl.make_basis64(m0, k1, 92), "bf16")
    W1 = wl.make_weight(m1, m0, 93, "bf16")
    U1d, W1d = gsi.to_device(U1, "bf16"), gsi.to_device(W1, "bf16")
    M1d = gsi.build_image(W1d, U1d)
    inputs = [{"U": dg.U, "X": dg.X}, {"U": U1d, "src_map": 0}]
    maps = [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}, {"W": W1d, "M": M1d, "input_id": 1}]
    st = gsi.layer_stack(inputs, maps, B, w.eps)
    torch.cuda.synchronize()
    # oracle on the device's own intermediate (the chain input is whatever map 0 produced, in fp32)
    Y0 = st.maps_t[0]["Y"].cpu().numpy()
    U1_64, W1_64 = O.widen(U1, "bf16"), O.widen(W1, "bf16")
    C, R, rn, xn = O.project(U1_64, Y0.astype(np.float64))
    mask, idx, n = O.gate(rn, xn, w.eps)
    ref = dict(C=C, R=R, rnorm=rn, xnorm=xn, rho=O.residual_ratio(rn, xn), mask=mask, idx=idx, n=n)
    ti = st.inputs_t[1]
    m_gpu = pu.check_projection(ti, ref, w.eps)
    pu.check_outputs(st.maps_t[1]["Y"], W1_64, O.build_image(W1_64, U1_64), gsi.bits_of(M1d), "bf16", ref, m_gpu,
                     m_small=128)


def test_run_to_run_determinism(gsi, pu):
    w = wl.tiny(2048, 128, 520, 6, 2, seed=55, wdtype="bf16")
    dg = pu.DeviceGroup(w, w.groups[0])
    a = pu.run_separate_calls(dg, w.eps)
    b = pu.run_separate_calls(dg, w.eps)
    for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired"):
        assert torch.equal(a[key], b[key])
    assert torch.equal(a["Y"]["w"], b["Y"]["w"])
    M2 = gsi.build_image(dg.W["w"], dg.U)
    assert torch.equal(M2.view(torch.int16), dg.M["w"].view(torch.int16))


def test_workspace_too_small_is_an_error_not_a_crash(gsi):
    need = gsi.workspace_bytes(gsi.CALL_PROJECT, 0, 4096, 256, 1)
    if need == 0:
        pytest.skip("projection needs no workspace in this build")
    U = torch.zeros((4096, 256), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((1, 4096), device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(gsi.GsiError) as ei:
        gsi.project(U, X, ws=small)
    assert ei.value.code == gsi.GSI_ERR_WORKSPACE


# ------------------------------------------------------------------------------------------------
# full-size GPT-J-shaped block in the launch configuration the benchmark times:
# one gsi_layer_stack call per decode token (B = 1), four inputs, six maps, k = 256, bf16
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("k,T,fused", [(256, 6, False), (64, 3, False), (128, 3, False), (512, 3, False), (256, 3, True)])
def test_gptj_block_full_size_decode(gsi, pu, k, T, fused):
    w = wl.gptj_block(T=T, k=k, fire_rate=0.34)  # 2 of 6 (1 of 3) tokens fire per input (seeded positions)
    say(f"case {w.name}: T={T} k={k}, full shapes, {'fused kernel' if fused else 'separate kernels'}")
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, 1)
    flags = gsi.INPUT_FUSED_KERNEL if fused else 0
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X, "flags": flags} for dg in dgs], maps, T, w.eps)
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()
    n_fired_total = 0
    for gi, (g, dg) in enumerate(zip(w.groups, dgs)):
        say(f"  input {g.name}: d={g.d}")
        og = pu.OracleGroup(w, g)
        ref = og.run()
        n_fired_total += ref["n"]
        ti = st.inputs_t[gi]
        mask_dev = ti["mask"].cpu().numpy()
        res = dict(C=ti["C"], R=ti["R"], rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                   n_fired=torch.tensor([int(mask_dev.sum())], dtype=torch.int32),
                   fired_idx=torch.from_numpy(np.nonzero(mask_dev)[0].astype(np.int32)))
        mask = pu.check_projection(res, ref, w.eps)
        assert np.array_equal(mask.astype(bool), g.fired_design)
        for j, (g2, name) in enumerate(names):
            if g2 != gi:
                continue
            pu.check_image(gsi.bits_of(dg.M[name]), og.M[name], og.W[name], og.U, w.wdtype)
            e, es = pu.check_outputs(st.maps_t[j]["Y"], og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype,
                                     ref, mask)
            say(f"    map {name}: rel-L2 vs exact-image oracle {e:.3e}, vs stored-image oracle {es:.3e}")
        del og
    assert n_fired_total == (8 if T == 6 else 4)
    if k != 256 or fused:
        return
    # the dense baseline the benchmark divides by: same descriptors, y = W x
    st.refresh(token_offset=0, B=1)
    st.run_dense()
    torch.cuda.synchronize()
    for j, (gi, name) in enumerate(names):
        g = w.groups[gi]
        W64 = O.widen(dict((n, W) for n, _, W in g.maps)[name], w.wdtype)
        yd = O.dense_linear(W64, O.widen(g.X[:1], w.xdtype))
        y = st.maps_t[j]["Y"][:1].cpu().numpy().astype(np.float64)
        assert pu.rel_l2_rows(y, yd).max() <= 2e-5, name


def test_timed_stack_and_dense_stack_match_plain_calls(gsi, pu):
    """gsi_layer_stack_timed == gsi_layer_stack bit for bit; gsi_dense_stack == gsi_dense_linear per map."""
    import ctypes as ct

    w = wl.transformer_block("blk", d=512, ffn=2048, k=64, T=3, fire_rate=0.34, p=1.5, seed=79)
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, 1)
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X} for dg in dgs], maps, w.T, w.eps)
    hip = ct.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ct.POINTER(ct.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ct.POINTER(ct.c_float), ct.c_void_p, ct.c_void_p]
    e0, e1 = ct.c_void_p(), ct.c_void_p()
    assert hip.hipEventCreate(ct.byref(e0)) == 0 and hip.hipEventCreate(ct.byref(e1)) == 0
    for t in range(w.T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()
    plain = [m["Y"].clone() for m in st.maps_t]
    plain_c = [i["C"].clone() for i in st.inputs_t]
    # the events bracket one launch: the staged projection kernel's first (partial projections) and second
    # (residuals, image rows) launch, the weight-streaming launch (which evaluates the gates of a one-set call)
    for which, index in ((0, 0), (0, 1), (1, 0)):
        for m in st.maps_t:
            m["Y"].zero_()
        for t in range(w.T):
            st.refresh(token_offset=t, B=1)
            st.run_timed(e0, e1, which=which, index=index)
        torch.cuda.synchronize()
        ms = ct.c_float()
        assert hip.hipEventElapsedTime(ct.byref(ms), e0, e1) == 0 and 0.0 < ms.value < 50.0, (which, index)
        for a, m in zip(plain, st.maps_t):
            assert torch.equal(a, m["Y"])
        for a, i in zip(plain_c, st.inputs_t):
            assert torch.equal(a, i["C"])
    with pytest.raises(gsi.GsiError):  # the call makes two launches of the staged kernel: there is no third
        st.run_timed(e0, e1, which=0, index=2)
    torch.cuda.synchronize()
    # dense stack, one token and a batch
    for B in (1, 3):
        st.refresh(token_offset=0, B=B)
        st.run_dense()
        torch.cuda.synchronize()
        for j, (gi, name) in enumerate(names):
            Yd = gsi.dense_linear(dgs[gi].W[name], dgs[gi].X[:B].contiguous())
            assert torch.equal(st.maps_t[j]["Y"][:B], Yd), (B, name)


# ------------------------------------------------------------------------------------------------
# prefill-sized batches (matrix-core path): several hundred tokens per call, ragged tails in every
# dimension of the 128 x 128 tiles, fp32 and bf16 activations
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,m,T,nf,xdtype", [(1024, 64, 520, 300, 60, "f32"), (2048, 128, 1000, 200, 41, "bf16"),
                                               (512, 32, 384, 129, 0, "f32"), (1024, 256, 300, 257, 257, "bf16"),
                                               (512, 64, 264, 1100, 100, "bf16")])
def test_prefill_sized_batch(gsi, pu, d, k, m, T, nf, xdtype):
    w = wl.tiny(d, k, m, T, nf, seed=4000 + d + k + T, wdtype="bf16", xdtype=xdtype)
    say(f"case prefill d={d} k={k} m={m} T={T} nf={nf} x={xdtype}")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    worst = pu.check_group(w, g, [(0, T)], dg, og)
    ref = og.run()
    assert ref["n"] == nf
    say(f"  worst rel-L2 {worst:.3e}")
    # the stack gives the same bits as the separate calls
    st = gsi.layer_stack([{"U": dg.U, "X": dg.X}], [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}], T, w.eps)
    sep = pu.run_separate_calls(dg, w.eps)
    torch.cuda.synchronize()
    for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired"):
        assert torch.equal(st.inputs_t[0][key], sep[key]), key
    assert torch.equal(st.maps_t[0]["Y"], sep["Y"]["w"])


# ------------------------------------------------------------------------------------------------
# full-size ragged decode batch: fc_in 16384x4096 and fc_out 4096x16384, k = 256, 64 tokens with a
# per-token Bernoulli(0.15) gate design, as one batch, a short batch and a window inside it
# ------------------------------------------------------------------------------------------------
def test_ffn_pair_full_size_ragged_batch(gsi, pu):
    w = wl.ffn_pair(T=64)
    for g in w.groups:
        say(f"case {w.name} input {g.name}: d={g.d} k={g.k} m={g.maps[0][1]} T={w.T} fired={int(g.fired_design.sum())}")
        dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
        worst = pu.check_group(w, g, [(0, 64), (0, 4), (20, 36)], dg, og)
        ref = og.run()
        assert np.array_equal(ref["mask"].astype(bool), g.fired_design)
        say(f"  worst rel-L2 {worst:.3e}")
        del dg, og
    # both maps in one stack call equal the separate calls bit for bit
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, w.T)
    st = gsi.layer_stack(inputs, maps, w.T, w.eps)
    torch.cuda.synchronize()
    for gi, dg in enumerate(dgs):
        sep = pu.run_separate_calls(dg, w.eps)
        for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired"):
            assert torch.equal(st.inputs_t[gi][key], sep[key]), key
        for j, (g2, name) in enumerate(names):
            if g2 == gi:
                assert torch.equal(st.maps_t[j]["Y"], sep["Y"][name]), name


# ------------------------------------------------------------------------------------------------
# full-size prefill batch: T = 2048 tokens (bf16 activations), k = 512, 20 % of the tokens of every
# input fired, the six maps of a GPT-J-shaped block in one stack call.  The projection is checked on
# every token; images and outputs on 1024 sampled rows of every map (a row of y depends on that row of W
# and M only, so the oracle computes exactly the sampled ones; the 2e-3 bar is statistical -- one bf16
# rounding per image element -- and the worst of 2048 tokens over 256 sampled rows would already brush it).
# ------------------------------------------------------------------------------------------------
def test_prefill_block_full_size_sampled(gsi, pu):
    T, k = 2048, 512
    w = wl.transformer_block("prefill_block_bf16", 4096, 16384, k, T, 0.20, 1.5, wl.BASE_SEED + 4000, xdtype="bf16")
    say(f"case {w.name}: T={T} k={k}, full shapes, sampled rows")
    dgs, inputs, maps, names = _stack_for(gsi, pu, w, T)
    st = gsi.layer_stack(inputs, maps, T, w.eps)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for gi, (g, dg) in enumerate(zip(w.groups, dgs)):
        U64, X64 = O.widen(g.U, w.wdtype), O.widen(g.X, w.xdtype)
        C, R, rn, xn = O.project(U64, X64)
        mask_o, idx_o, n_o = O.gate(rn, xn, w.eps)
        ref = dict(X=X64, C=C, R=R, rnorm=rn, xnorm=xn, rho=O.residual_ratio(rn, xn), mask=mask_o, idx=idx_o, n=n_o)
        assert n_o == int(round(0.2 * T)) and np.array_equal(mask_o.astype(bool), g.fired_design)
        ti = st.inputs_t[gi]
        res = {key: ti[key] for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired", "fired_idx")}
        mask = pu.check_projection(res, ref, w.eps)
        say(f"  input {g.name}: d={g.d}, {n_o} fired, projection and gate match on all tokens")
        for j, (g2, name) in enumerate(names):
            if g2 != gi:
                continue
            Wst = dict((n, W) for n, _, W in g.maps)[name]
            rows = np.sort(rng.choice(Wst.shape[0], size=1024, replace=False))
            W64 = O.widen(Wst[rows], w.wdtype)
            M64 = O.build_image(W64, U64)
            Mdev = gsi.bits_of(dg.M[name])[rows]
            pu.check_image(Mdev, M64, W64, U64, w.wdtype)
            Ys = st.maps_t[j]["Y"][:, torch.from_numpy(rows).to(st.maps_t[j]["Y"].device)]
            e, es = pu.check_outputs(Ys, W64, M64, Mdev, w.wdtype, ref, mask)
            say(f"    map {name}: 1024 sampled rows, rel-L2 vs exact-image oracle {e:.3e}, vs stored-image oracle {es:.3e}")
        del U64, X64, C, R, ref


# ------------------------------------------------------------------------------------------------
# the slow path as Algorithm 1 prints it (flag on the input): a fired token gets y = W x, free of the
# stored image's rounding; tokens that did not fire keep y = M c.  Checked for one token per call, a
# decode batch and a prefill-sized batch; with every token fired the stack equals the dense stack.
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,m,T,nf,B", [(1024, 64, 520, 12, 4, 1), (2048, 128, 528, 48, 9, 48), (1024, 64, 512, 300, 60, 300),
                                          (776, 72, 100, 9, 3, 9)])
def test_slow_path_wx_flag(gsi, pu, d, k, m, T, nf, B):
    w = wl.tiny(d, k, m, T, nf, seed=5200 + d + k + T, wdtype="bf16")
    say(f"case slow path W x: d={d} k={k} m={m} T={T} nf={nf} B={B}")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    ref = og.run()
    maps = [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}]
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X, "flags": gsi.INPUT_SLOW_PATH_WX}], maps, T, w.eps)
    for t0 in range(0, T, B):
        st.refresh(token_offset=t0, B=min(B, T - t0))
        st.run()
    torch.cuda.synchronize()
    mask = st.inputs_t[0]["mask"].cpu().numpy()
    assert np.array_equal(mask.astype(bool), g.fired_design)
    Y = st.maps_t[0]["Y"].cpu().numpy().astype(np.float64)
    fired = mask.astype(bool)
    # fired tokens: the dense product, to fp32-accumulation accuracy (no image in it)
    e_f = pu.rel_l2_rows(Y[fired], O.dense_linear(og.W["w"], og.X[fired]))
    assert e_f.max() <= 2e-5, e_f.max()
    # the whole output against Algorithm 1 evaluated with the device's stored image
    Mdev = O.widen(gsi.bits_of(dg.M["w"]), w.wdtype)
    e = pu.rel_l2_rows(Y, O.gated_linear_alg1(og.W["w"], Mdev, ref["C"], og.X, mask))
    assert e.max() <= 2e-5, e.max()
    say(f"  fired rows vs W x {e_f.max():.3e}, all rows vs Algorithm 1 with the stored image {e.max():.3e}")
    # eps = 0: every token fires, and the stack gives the dense stack's bits
    st0 = gsi.LayerStack([{"U": dg.U, "X": dg.X, "flags": gsi.INPUT_SLOW_PATH_WX}], maps, T, 0.0)
    for t0 in range(0, T, B):
        st0.refresh(token_offset=t0, B=min(B, T - t0))
        st0.run()
    torch.cuda.synchronize()
    y_all = st0.maps_t[0]["Y"].clone()
    for t0 in range(0, T, B):
        st0.refresh(token_offset=t0, B=min(B, T - t0))
        st0.run_dense()
    torch.cuda.synchronize()
    assert torch.equal(y_all, st0.maps_t[0]["Y"])


# ------------------------------------------------------------------------------------------------
# The cached image in 8-bit E4M3 with power-of-two row scales (Section 7, "Combination with quantization").
# The quantiser decides integers (codes): it is fed matrices from the seeded generator, never an image
# built on the device, and must give the oracle's codes and scales bit for bit.
# ------------------------------------------------------------------------------------------------
def _fp8_test_matrix(m, k, seed):
    """fp32 matrix with rows of very different size, exact ties between codes, tiny and special entries."""
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((m, k)) * np.exp(rng.uniform(-30, 30, (m, 1))) * np.exp(rng.uniform(-6, 0, (m, k)))
    M = M.astype(np.float32)
    grid = np.array([(mm / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + mm / 8.0) * 2.0 ** (e - 7)
                     for e in range(16) for mm in range(8) if not (e == 15 and mm == 7)])
    mid = 0.5 * (grid[:-1] + grid[1:])
    if m >= 8 and k >= 16:
        # rows whose maximum is exactly 448 * 2^j: the midpoints between neighbouring codes are then ties
        for r, j in ((1, 0), (2, -7), (3, 9)):
            row = rng.choice(mid, k) * rng.choice([-1.0, 1.0], k)
            row[0] = 448.0
            M[r] = (row * 2.0 ** j).astype(np.float32)
        M[4] = 0.0                                    # zero row: scale 1, codes 0
        M[5, :] = 0.0
        M[5, 3] = -1.0e-30                            # one tiny element alone
        M[6, :4] = [np.inf, -np.inf, np.nan, 3.0]     # not finite: no part in the scale, saturate / NaN code
        M[7] = np.float32(224.0) * rng.choice([-1.0, 1.0], k)   # maximum on a power-of-two boundary
    return M


@pytest.mark.parametrize("m,k,dt", [(8, 16, "f32"), (37, 50, "f32"), (256, 256, "bf16"), (1000, 512, "f32"),
                                    (4100, 64, "bf16"), (5, 1, "f32")])
def test_fp8_quantizer_bit_exact(gsi, m, k, dt):
    say(f"case fp8 quantizer: m={m} k={k} stored {dt}")
    M = _fp8_test_matrix(m, k, 8800 + m + k)
    if dt == "bf16":
        bits = wl.f32_to_bf16_bits(M)
        Md = gsi.to_device(bits, "bf16")
        M64 = O.widen(bits, "bf16")
    else:
        Md = gsi.to_device(M, "f32")
        M64 = O.widen(M, "f32")
    M8, scale = gsi.quantize_image_fp8(Md)
    torch.cuda.synchronize()
    codes_o, scale_o = O.quantize_image_fp8(M64)
    assert np.array_equal(scale.cpu().numpy().astype(np.float64), scale_o)
    got = M8.cpu().numpy()
    bad = np.argwhere(got != codes_o)
    assert bad.size == 0, f"{bad.shape[0]} codes differ, first at {bad[0]}: {got[tuple(bad[0])]:#x} vs {codes_o[tuple(bad[0])]:#x} for {M64[tuple(bad[0])]!r}"


def test_fp8_image_decodes_every_code(gsi):
    """y_i = scale_i * value(code i): the image kernel's widening of all 256 codes, bit for bit."""
    say("case fp8 decode table")
    d, k, m = 64, 16, 256
    U = np.zeros((d, k), dtype=np.float32)
    U[np.arange(k), np.arange(k)] = 1.0
    X = np.zeros((1, d), dtype=np.float32)
    X[0, 0] = 1.0                                     # c = e_0, r = 0: the gate stays shut
    M8 = np.zeros((m, k), dtype=np.uint8)
    M8[:, 0] = np.arange(256, dtype=np.uint8)
    scale = (2.0 ** ((np.arange(m) % 5) - 2)).astype(np.float32)
    dev = torch.device("cuda")
    maps = [{"W": torch.zeros((m, d), dtype=torch.bfloat16, device=dev), "M": torch.from_numpy(M8).to(dev),
             "M_scale": torch.from_numpy(scale).to(dev), "input_id": 0}]
    st = gsi.layer_stack([{"U": gsi.to_device(wl.f32_to_bf16_bits(U), "bf16"), "X": gsi.to_device(X, "f32")}], maps, 1, 0.05)
    torch.cuda.synchronize()
    assert int(st.inputs_t[0]["n_fired"].item()) == 0
    y = st.maps_t[0]["Y"].cpu().numpy()[0].astype(np.float64)
    want = O.fp8_e4m3_decode(np.arange(256, dtype=np.uint8)) * scale.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(y), nan)
    assert np.array_equal(y[~nan], want[~nan])


@pytest.mark.parametrize("d,k,m,T,nf,wx", [(1024, 64, 520, 12, 4, 0), (4096, 256, 1024, 10, 3, 0), (2048, 128, 528, 9, 3, 1),
                                           (512, 16, 264, 6, 2, 0)])
def test_fp8_image_single_token_stack(gsi, pu, d, k, m, T, nf, wx):
    """Single-token calls with the image stored in E4M3.

    Bars.  (a) Against the oracle fed the device's own codes and scales only kernel arithmetic differs
    (fp32 accumulation of exactly widened operands): 2e-5 as for the other stage comparisons.  (b) Against
    the oracle's own pipeline (fp64 image, rounded once to bf16, quantised by the oracle) a code differs where
    the two bf16 images differ at a rounding boundary; such a flip moves one of k terms of a row by a code
    step (2^-3 relative), so rows stay within 2^-3 / sqrt k of each other and the bar is 5e-3 on the whole
    output block.  (c) Against the exact image the E4M3 rounding itself shows: at most 2^-4 per element,
    about 2^-4 / sqrt 3 in the root mean square; bar 6e-2 per output vector.
    """
    w = wl.tiny(d, k, m, T, nf, seed=9100 + d + k, wdtype="bf16")
    say(f"case fp8 image stack: d={d} k={k} m={m} T={T} nf={nf} wx={wx}")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    ref = og.run()
    M8, scale = gsi.quantize_image_fp8(dg.M["w"])
    maps = [{"W": dg.W["w"], "M": M8, "M_scale": scale, "input_id": 0}]
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X, "flags": gsi.INPUT_SLOW_PATH_WX if wx else 0}], maps, T, w.eps)
    for t0 in range(T):
        st.refresh(token_offset=t0, B=1)
        st.run()
    torch.cuda.synchronize()
    mask = st.inputs_t[0]["mask"].cpu().numpy()
    assert np.array_equal(mask.astype(bool), g.fired_design)
    Y = st.maps_t[0]["Y"].cpu().numpy().astype(np.float64)

    def out(M):
        return (O.gated_linear_alg1(og.W["w"], M, ref["C"], og.X, mask) if wx
                else O.gated_linear(og.W["w"], M, ref["C"], ref["R"], mask))

    e_stage = pu.rel_l2_rows(Y, out(O.dequantize_image_fp8(M8.cpu().numpy(), scale.cpu().numpy())))
    assert e_stage.max() <= 2e-5, e_stage.max()
    M_bf16 = O.widen(wl.f32_to_bf16_bits(og.M["w"].astype(np.float32)), "bf16")
    codes_o, scale_o = O.quantize_image_fp8(M_bf16)
    Yo = out(O.dequantize_image_fp8(codes_o, scale_o))
    e_pipe = np.linalg.norm(Y - Yo) / np.linalg.norm(Yo)
    flips = int(np.count_nonzero(M8.cpu().numpy() != codes_o))
    assert e_pipe <= 5e-3, e_pipe
    assert np.array_equal(scale.cpu().numpy().astype(np.float64), scale_o) or flips > 0
    e_exact = pu.rel_l2_rows(Y, out(og.M["w"]))
    assert e_exact.max() <= 6e-2, e_exact.max()
    say(f"  vs device codes {e_stage.max():.3e}; vs oracle pipeline {e_pipe:.3e} ({flips} of {m * k} codes differ); "
        f"vs exact image {e_exact.max():.3e} (E4M3 rounding)")


@pytest.mark.parametrize("d,k,m,T,nf,B", [(1024, 64, 520, 24, 5, 8), (2048, 128, 528, 300, 60, 300), (776, 72, 100, 9, 3, 9),
                                          (1000, 40, 30, 3, 1, 1)])
def test_fp8_image_expanded_for_other_calls(gsi, pu, d, k, m, T, nf, B):
    """Calls whose kernels do not read codes (several tokens: the matrix-core decode and GEMM kernels; shapes the
    single-token vector kernels do not take) expand the image exactly and give the results of the same stack run
    with that expanded image stored as an ordinary one -- bit for bit."""
    w = wl.tiny(d, k, m, T, nf, seed=9400 + d + k + T, wdtype="bf16")
    say(f"case fp8 image, expanded: d={d} k={k} m={m} T={T} nf={nf} B={B}")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    M8, scale = gsi.quantize_image_fp8(dg.M["w"])
    Mdeq = O.dequantize_image_fp8(M8.cpu().numpy(), scale.cpu().numpy())
    bits = wl.f32_to_bf16_bits(Mdeq.astype(np.float32))
    assert np.array_equal(O.widen(bits, "bf16"), Mdeq)          # the expansion is exact in bf16
    outs = []
    for mp in ({"W": dg.W["w"], "M": M8, "M_scale": scale, "input_id": 0},
               {"W": dg.W["w"], "M": gsi.to_device(bits, "bf16"), "input_id": 0}):
        st = gsi.LayerStack([{"U": dg.U, "X": dg.X}], [mp], T, w.eps)
        for t0 in range(0, T, B):
            st.refresh(token_offset=t0, B=min(B, T - t0))
            st.run()
        torch.cuda.synchronize()
        outs.append((st.maps_t[0]["Y"].clone(), st.inputs_t[0]["mask"].cpu().numpy()))
    assert torch.equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1].astype(bool), g.fired_design)
    # and that common result is the oracle's, with the expanded image, to the stage bar of the call size
    ref = og.run()
    mask = outs[0][1]
    Y = outs[0][0].cpu().numpy().astype(np.float64)
    Yo = O.gated_linear(og.W["w"], Mdeq, ref["C"], ref["R"], mask)
    err = pu.rel_l2_rows(Y, Yo)
    bar = np.full(T, 2e-5)
    fired = mask.astype(bool)
    if B > pu.PREFILL_TOKENS and fired.any():   # r enters the W term rounded once to bf16 in calls of this size
        wr = np.linalg.norm(O.dense_linear(og.W["w"], ref["R"][fired]), axis=1)
        bar[fired] += 2.0 ** -8 * wr / np.maximum(np.linalg.norm(Yo[fired], axis=1), 1e-300)
    assert np.all(err <= bar), float((err / bar).max())
    say(f"  identical to the ordinary-image run; vs oracle with the expanded image {err.max():.3e}")


def test_fp8_image_beside_a_map_on_the_generic_kernels(gsi, pu):
    """Two maps of one input, one of them with a weight matrix that is not 16-byte aligned: the input then takes
    the separate norm + gate launch and the aligned map's E4M3 codes are read by the stand-alone image kernel."""
    w = wl.tiny(1024, 64, 264, 5, 2, seed=9600, wdtype="bf16")
    say("case fp8 image beside a generic map")
    g = w.groups[0]
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    ref = og.run()
    M8, scale = gsi.quantize_image_fp8(dg.M["w"])
    flat = torch.empty(dg.W["w"].numel() + 1, dtype=torch.bfloat16, device="cuda")
    W_odd = flat[1:].view_as(dg.W["w"])                      # same values, 2 bytes off a 16-byte boundary
    W_odd.copy_(dg.W["w"])
    maps = [{"W": dg.W["w"], "M": M8, "M_scale": scale, "input_id": 0}, {"W": W_odd, "M": dg.M["w"], "input_id": 0}]
    T = 5
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X}], maps, T, w.eps)
    for t0 in range(T):
        st.refresh(token_offset=t0, B=1)
        st.run()
    torch.cuda.synchronize()
    mask = st.inputs_t[0]["mask"].cpu().numpy()
    assert np.array_equal(mask.astype(bool), g.fired_design)
    Mdeq = O.dequantize_image_fp8(M8.cpu().numpy(), scale.cpu().numpy())
    Mdev = O.widen(gsi.bits_of(dg.M["w"]), "bf16")
    for j, Mj in enumerate((Mdeq, Mdev)):
        Y = st.maps_t[j]["Y"].cpu().numpy().astype(np.float64)
        err = pu.rel_l2_rows(Y, O.gated_linear(og.W["w"], Mj, ref["C"], ref["R"], mask))
        assert err.max() <= 2e-5, (j, err.max())


# ------------------------------------------------------------------------------------------------
# HIP-graph replay (the launch mode bench.py times): a captured stack must give, on every replay, the bits of
# the same calls issued eagerly -- with eager work and synchronisations between the replays, for one token per
# call, a decode batch and a prefill-sized batch (the library records no memset nodes and allocates nothing).
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,m,T,nf,B,fp8", [(1024, 64, 520, 6, 2, 1, False), (1024, 64, 520, 6, 2, 1, True),
                                              (2048, 128, 528, 24, 5, 8, False), (1024, 64, 512, 300, 60, 300, False)])
def test_graph_replay_equals_eager(gsi, pu, d, k, m, T, nf, B, fp8):
    w = wl.tiny(d, k, m, T, nf, seed=9700 + d + k + T, wdtype="bf16")
    say(f"case graph replay: d={d} k={k} m={m} T={T} nf={nf} B={B} fp8={fp8}")
    g = w.groups[0]
    dg = pu.DeviceGroup(w, g)
    mp = {"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}
    if fp8:
        mp["M"], mp["M_scale"] = gsi.quantize_image_fp8(dg.M["w"])
    st = gsi.LayerStack([{"U": dg.U, "X": dg.X}], [mp], T, w.eps)
    outs = ("C", "R", "rnorm", "xnorm", "mask")

    def snapshot():
        torch.cuda.synchronize()
        return [st.maps_t[0]["Y"].clone()] + [st.inputs_t[0][n].clone() for n in outs]

    def clear():
        st.maps_t[0]["Y"].fill_(float("nan"))
        for n in outs:
            st.inputs_t[0][n].zero_()

    # descriptor tables of every call, kept alive for the graph
    tabs = []
    for t0 in range(0, T, B):
        st.refresh(token_offset=t0, B=min(B, T - t0))
        mpd, ind = (gsi.MapDesc * 1)(), (gsi.InputDesc * 1)()
        ctypes.memmove(mpd, st._mp, ctypes.sizeof(mpd))
        ctypes.memmove(ind, st._in, ctypes.sizeof(ind))
        tabs.append((mpd, ind, min(B, T - t0)))
    ws = st.ws

    def issue(stream):
        for mpd, ind, b in tabs:
            rc = gsi.lib.gsi_layer_stack(mpd, 1, ind, 1, b, ctypes.c_float(w.eps), ws.data_ptr(), ws.numel(), stream)
            assert rc == 0, gsi.last_error()

    clear()
    issue(torch.cuda.current_stream().cuda_stream)
    eager = snapshot()
    assert np.array_equal(eager[-1].cpu().numpy().astype(bool), g.fired_design)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        issue(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        issue(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager):
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"
        issue(torch.cuda.current_stream().cuda_stream)   # eager work between the replays
        torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------
# tokens placed next to the gate threshold (Eq. (gate); Definition "Activation basis and residual ratio"):
# inside the 1e-4 band either decision is admissible and y is checked against the oracle on the device's own
# decision; just outside the band the decision must be the oracle's
# ------------------------------------------------------------------------------------------------
def _tokens_at_ratio(U64, targets, eps32, seed):
    """fp32 tokens x = U a + sigma n whose residual ratio w.r.t. the STORED basis (as the oracle computes it from
    the fp32-rounded token) is the given target, found by bisection on sigma."""
    rng = np.random.default_rng(seed)
    d, k = U64.shape
    lam = np.arange(1, k + 1, dtype=np.float64) ** -1.5
    X = np.empty((len(targets), d), dtype=np.float32)
    got = np.empty(len(targets))
    for t, target in enumerate(targets):
        a = rng.standard_normal(k) * np.sqrt(lam)
        n = rng.standard_normal(d)
        for _ in range(2):
            n = n - U64 @ (U64.T @ n)
        n /= np.linalg.norm(n)
        base = U64 @ a

        def rho(sig):
            x = (base + sig * n).astype(np.float32)
            _, _, rn, xn = O.project(U64, x[None, :].astype(np.float64))
            return float(rn[0] / xn[0]), x

        lo, hi = 0.0, 10.0 * np.linalg.norm(a)
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            if rho(mid)[0] < target:
                lo = mid
            else:
                hi = mid
        got[t], X[t] = rho(hi)
    return X, got


@pytest.mark.parametrize("d,k,m,B", [(2048, 128, 520, 1), (2048, 128, 520, 16), (1024, 64, 512, 300)])
def test_tokens_next_to_the_gate_threshold(gsi, pu, d, k, m, B):
    offsets = np.array([1e-6, -1e-6, 5e-5, -5e-5, 1.2e-4, -1.2e-4, 3e-4, -3e-4, 2e-3, -2e-3])
    w = wl.tiny(d, k, m, len(offsets), 0, seed=7000 + d + B, wdtype="bf16")
    g = w.groups[0]
    eps32 = float(np.float32(w.eps))
    U64 = O.widen(g.U, w.wdtype)
    X, got = _tokens_at_ratio(U64, eps32 + offsets, eps32, seed=7100 + B)
    assert np.all(np.abs(got - (eps32 + offsets)) < 2e-7), "calibration missed its targets"
    reps = -(-B // len(offsets))
    g.X = np.ascontiguousarray(np.tile(X, (reps, 1))[:B] if B > 1 else X)
    T = g.X.shape[0]
    say(f"case threshold d={d} k={k} m={m} B={B}: ratios eps + {offsets.tolist()}")
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    blocks = [(t, t + 1) for t in range(T)] if B == 1 else [(0, T)]
    pu.check_group(w, g, blocks, dg, og)
    # what the band rule was given to decide: the device's decisions on the tokens inside and outside the band
    res = pu.run_separate_calls(dg, w.eps)
    ref = og.run()
    mask = res["mask"].cpu().numpy()
    inside = np.abs(ref["rho"] - eps32) < pu.BAND
    assert inside.sum() >= 4 * (T // len(offsets)) and (~inside).sum() >= 6 * (T // len(offsets))
    assert np.array_equal(mask[~inside], ref["mask"][~inside])
    say(f"  in-band tokens: device {mask[inside].tolist()[:8]} oracle {ref['mask'][inside].tolist()[:8]}")
