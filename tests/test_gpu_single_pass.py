"""GPU parity of the single-pass gate (GSI_INPUT_GATE_SINGLE_PASS): the residual ratio of Eq. (rho) evaluated as
|x|^2 - |c|^2 + c^T E c with the cached E = U^T U - I, against the fp64 oracle that forms the residual explicitly."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle.gsi_oracle as O  # noqa: E402
from paper_2605_03109_amd import workload as wl  # noqa: E402

SENTINEL = 7.25  # R rows the library must not touch keep this value


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


@pytest.mark.parametrize("d,k,dt", [(33, 7, "bf16"), (768, 64, "f32"), (4096, 256, "bf16"), (16384, 512, "bf16"),
                                    (1000, 24, "f32")])
def test_build_gram(gsi, d, k, dt):
    say(f"case gram d={d} k={k} {dt}")
    U = wl.store(wl.make_basis64(d, k, seed=900 + d), dt)
    E = gsi.build_gram(gsi.to_device(U, dt)).cpu().numpy().astype(np.float64)
    ref = O.gram_defect(O.widen(U, dt))
    # fp64 accumulation, one rounding to fp32
    assert np.all(np.abs(E - ref) <= 2.0 ** -24 * np.abs(ref) + 1e-13), np.abs(E - ref).max()
    if dt == "bf16":  # storage rounding leaves a defect of the size the design notes quote
        assert 1e-5 < np.abs(ref).max() < 1e-2


def _run_tokens(st, T):
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()


def _stack(gsi, pu, w, flags):
    dgs = [pu.DeviceGroup(w, g) for g in w.groups]
    inputs, maps, names = [], [], []
    for gi, dg in enumerate(dgs):
        inputs.append({"U": dg.U, "X": dg.X, "flags": flags, "gram": gsi.build_gram(dg.U)})
        for name in dg.W:
            maps.append({"W": dg.W[name], "M": dg.M[name], "input_id": gi})
            names.append((gi, name))
    return dgs, inputs, maps, names


def _check_input(gsi, pu, w, g, dg, ti, wx):
    """Projection outputs of one input over all tokens; returns (oracle group, reference, device mask)."""
    og = pu.OracleGroup(w, g)
    ref = og.run()
    mask_dev = ti["mask"].cpu().numpy()
    fired = mask_dev.astype(bool)
    R = ti["R"].cpu().numpy()
    # r is formed only for tokens whose gate fired, and not at all with the W x form of the slow path
    untouched = np.ones(len(fired), dtype=bool) if wx else ~fired
    assert np.all(R[untouched] == SENTINEL), "R of a token that needs no residual was written"
    Rchk = ti["R"].clone()
    Rchk[torch.from_numpy(untouched)] = torch.from_numpy(ref["R"][untouched].astype(np.float32)).to(Rchk.device)
    res = dict(C=ti["C"], R=Rchk, rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
               n_fired=torch.tensor([int(mask_dev.sum())], dtype=torch.int32),
               fired_idx=torch.from_numpy(np.nonzero(mask_dev)[0].astype(np.int32)))
    mask = pu.check_projection(res, ref, w.eps)
    # the single-pass oracle (same formula in fp64) agrees with the device at least as well
    E64 = O.gram_defect(og.U)
    _, rn1, xn1 = O.project_single_pass(og.U, E64, og.X)
    rho_dev = ti["rnorm"].cpu().numpy().astype(np.float64) / np.maximum(ti["xnorm"].cpu().numpy().astype(np.float64), 1e-300)
    assert np.abs(rho_dev - rn1 / xn1).max() <= pu.TOL_RHO
    return og, ref, mask


@pytest.mark.parametrize("wx", [False, True])
@pytest.mark.parametrize("wdtype", ["bf16", "f32"])
def test_single_pass_block(gsi, pu, wdtype, wx):
    """One block (four inputs, six maps), one call per token: three launches of the staged kernel + weights."""
    w = wl.transformer_block("sp", d=512, ffn=2048, k=64, T=12, fire_rate=0.25, p=1.5, seed=4100, wdtype=wdtype)
    flags = gsi.INPUT_GATE_SINGLE_PASS | (gsi.INPUT_SLOW_PATH_WX if wx else 0)
    say(f"case single-pass block {wdtype} wx={wx}")
    dgs, inputs, maps, names = _stack(gsi, pu, w, flags)
    st = gsi.LayerStack(inputs, maps, w.T, w.eps)
    for ti in st.inputs_t:
        ti["R"].fill_(SENTINEL)
    _run_tokens(st, w.T)
    for gi, (g, dg) in enumerate(zip(w.groups, dgs)):
        og, ref, mask = _check_input(gsi, pu, w, g, dg, st.inputs_t[gi], wx)
        assert np.array_equal(mask.astype(bool), g.fired_design)
        for j, (g2, name) in enumerate(names):
            if g2 != gi:
                continue
            Y = st.maps_t[j]["Y"]
            if wx:  # Algorithm 1 as printed: fired rows are W x, the others M c with the stored image
                Mdev = O.widen(gsi.bits_of(dg.M[name]), w.wdtype)
                e = pu.rel_l2_rows(Y.cpu().numpy().astype(np.float64), O.gated_linear_alg1(og.W[name], Mdev, ref["C"], og.X, mask))
                assert e.max() <= pu.TOL_Y_STAGE[w.wdtype], e.max()
            else:
                pu.check_outputs(Y, og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype, ref, mask)


def test_single_pass_many_inputs_equal_explicit_path(gsi, pu):
    """Five blocks in one call per token (more inputs than one launch's arguments describe, so every stage runs once
    over a descriptor table in the workspace): decisions equal the explicit path's, everything else agrees with it to
    rounding, and the first and last block are checked against the oracle."""
    L, T = 5, 6
    blocks = [wl.transformer_block(f"b{l}", d=512, ffn=2048, k=64, T=T, fire_rate=0.34, p=1.5, seed=4200 + l) for l in range(L)]
    eps = blocks[0].eps
    inputs, maps = [], []
    for w in blocks:
        _, bi, bm, _ = _stack(gsi, pu, w, gsi.INPUT_GATE_SINGLE_PASS)
        base = len(inputs)
        inputs += bi
        maps += [dict(m, input_id=m["input_id"] + base) for m in bm]
    say(f"case single-pass {len(inputs)} inputs / {len(maps)} maps per call")
    sp = gsi.LayerStack(inputs, maps, T, eps)
    sp.refresh(token_offset=0, B=1)
    sp.ws.fill_(0xFF)
    for rep in range(2):
        _run_tokens(sp, T)
    ex = gsi.LayerStack([dict(i, flags=0) for i in inputs], maps, T, eps)
    _run_tokens(ex, T)
    n_fired, worst = 0, 0.0
    for a, b in zip(sp.inputs_t, ex.inputs_t):
        assert torch.equal(a["mask"], b["mask"])
        # (the table launches add the partials in another order than the 16-input launches)
        assert torch.allclose(a["C"], b["C"], rtol=0, atol=2e-6 * float(b["xnorm"].max()))
        assert torch.allclose(a["xnorm"], b["xnorm"], rtol=1e-6, atol=0)
        drho = ((a["rnorm"] - b["rnorm"]).abs() / b["xnorm"]).max().item()
        worst = max(worst, drho)
        assert drho <= 1e-5, drho
        f = b["mask"].bool()
        n_fired += int(f.sum())
        assert torch.allclose(a["R"][f], b["R"][f], rtol=0, atol=2e-6 * float(b["xnorm"].max()))
    assert n_fired > 0
    say(f"  largest |rho_single_pass - rho_explicit| over {len(inputs) * T} gate evaluations: {worst:.2e}")
    for a, b in zip(sp.maps_t, ex.maps_t):
        assert torch.allclose(a["Y"], b["Y"], rtol=0, atol=1e-5 * float(b["Y"].abs().max()))
    # and the first and last block against the oracle
    for l in (0, L - 1):
        w = blocks[l]
        for gi, g in enumerate(w.groups):
            ti = dict(sp.inputs_t[4 * l + gi])
            og = pu.OracleGroup(w, g)
            ref = og.run()
            Rchk = ti["R"].clone()
            un = ~ti["mask"].bool()
            Rchk[un] = torch.from_numpy(ref["R"].astype(np.float32)).to(Rchk.device)[un]
            m = ti["mask"].cpu().numpy()
            res = dict(C=ti["C"], R=Rchk, rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                       n_fired=torch.tensor([int(m.sum())], dtype=torch.int32),
                       fired_idx=torch.from_numpy(np.nonzero(m)[0].astype(np.int32)))
            pu.check_projection(res, ref, eps)


def test_single_pass_next_to_the_threshold(gsi, pu):
    """Tokens placed at eps + offset through the stack with the single-pass gate: outside the 1e-4 band the decision
    is the oracle's, inside it either is admissible; reports how the single-pass and the explicit decisions compare,
    and what dropping the E term (assuming U^T U = I) would have decided."""
    from test_gpu_parity import _tokens_at_ratio

    d, k, m = 2048, 128, 520
    offsets = np.array([1e-6, -1e-6, 2e-6, -2e-6, 5e-6, -5e-6, 2e-5, -2e-5, 5e-5, -5e-5, 1.2e-4, -1.2e-4, 3e-4, -3e-4, 2e-3, -2e-3])
    w = wl.tiny(d, k, m, len(offsets), 0, seed=7300, wdtype="bf16")
    g = w.groups[0]
    eps32 = float(np.float32(w.eps))
    U64 = O.widen(g.U, w.wdtype)
    X, got = _tokens_at_ratio(U64, eps32 + offsets, eps32, seed=7301)
    g.X = X
    T = len(offsets)
    dg, og = pu.DeviceGroup(w, g), pu.OracleGroup(w, g)
    maps = [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}]
    E = gsi.build_gram(dg.U)
    sp = gsi.LayerStack([{"U": dg.U, "X": dg.X, "flags": gsi.INPUT_GATE_SINGLE_PASS, "gram": E}], maps, T, w.eps)
    ex = gsi.LayerStack([{"U": dg.U, "X": dg.X}], maps, T, w.eps)
    _run_tokens(sp, T)
    _run_tokens(ex, T)
    ref = og.run()
    ti = sp.inputs_t[0]
    m_sp, m_ex = ti["mask"].cpu().numpy(), ex.inputs_t[0]["mask"].cpu().numpy()
    outside = np.abs(ref["rho"] - eps32) >= pu.BAND
    assert np.array_equal(m_sp[outside], ref["mask"][outside])
    rho_sp = (ti["rnorm"] / ti["xnorm"]).cpu().numpy().astype(np.float64)
    rho_ex = (ex.inputs_t[0]["rnorm"] / ex.inputs_t[0]["xnorm"]).cpu().numpy().astype(np.float64)
    assert np.abs(rho_sp - ref["rho"]).max() <= pu.TOL_RHO
    # outputs on the device's own decision
    Mdev = O.widen(gsi.bits_of(dg.M["w"]), w.wdtype)
    Y = sp.maps_t[0]["Y"].cpu().numpy().astype(np.float64)
    e = pu.rel_l2_rows(Y, O.gated_linear(og.W["w"], Mdev, ref["C"], ref["R"], m_sp))
    assert e.max() <= pu.TOL_Y_STAGE[w.wdtype], e.max()
    # what |x|^2 - |c|^2 alone would give (fp64): the stored bf16 basis is not orthonormal enough for it
    naive = np.sqrt(np.maximum(np.sum(og.X ** 2, axis=1) - np.sum(ref["C"] ** 2, axis=1), 0.0)) / ref["xnorm"]
    say(f"  |rho_single_pass - rho_oracle| max {np.abs(rho_sp - ref['rho']).max():.2e}; explicit kernel {np.abs(rho_ex - ref['rho']).max():.2e}")
    say(f"  decisions differing from the oracle: single pass {int((m_sp != ref['mask']).sum())}, explicit {int((m_ex != ref['mask']).sum())} "
        f"(all inside the band: {bool(np.all(~outside[(m_sp != ref['mask']) | (m_ex != ref['mask'])]))})")
    say(f"  without the E term: |rho - rho_oracle| max {np.abs(naive - ref['rho']).max():.2e}, "
        f"{int(((naive >= eps32) != ref['mask'].astype(bool)).sum())} of {T} decisions flip")


@pytest.mark.parametrize("k", [64, 256, 512])
def test_single_pass_gptj_block_full_size(gsi, pu, k):
    T = 3
    w = wl.gptj_block(T=T, k=k, fire_rate=0.34)
    say(f"case single-pass {w.name}: k={k}, full shapes")
    dgs, inputs, maps, names = _stack(gsi, pu, w, gsi.INPUT_GATE_SINGLE_PASS)
    st = gsi.LayerStack(inputs, maps, T, w.eps)
    for ti in st.inputs_t:
        ti["R"].fill_(SENTINEL)
    _run_tokens(st, T)
    for gi, (g, dg) in enumerate(zip(w.groups, dgs)):
        say(f"  input {g.name}: d={g.d}")
        og, ref, mask = _check_input(gsi, pu, w, g, dg, st.inputs_t[gi], False)
        assert np.array_equal(mask.astype(bool), g.fired_design)
        for j, (g2, name) in enumerate(names):
            if g2 == gi:
                e, es = pu.check_outputs(st.maps_t[j]["Y"], og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype, ref, mask)
                say(f"    map {name}: rel-L2 vs exact-image oracle {e:.3e}, vs stored-image oracle {es:.3e}")
        del og


@pytest.mark.parametrize("wx", [False, True])
def test_stack_plan_equals_layer_stack(gsi, pu, wx):
    """gsi_stack_plan_build + gsi_stack_plan_run give the bits of gsi_layer_stack on the same descriptors: five blocks
    (table launches either way) and a single block (which gsi_layer_stack runs through the 16-input launches, so only
    decisions are equal and the rest agrees to rounding); a call that cannot be planned is refused."""
    T = 5
    flags = gsi.INPUT_GATE_SINGLE_PASS | (gsi.INPUT_SLOW_PATH_WX if wx else 0)
    for L in (5, 1):
        blocks = [wl.transformer_block(f"p{l}", d=512, ffn=2048, k=64, T=T, fire_rate=0.4, p=1.5, seed=4400 + l) for l in range(L)]
        eps = blocks[0].eps
        inputs, maps = [], []
        for w in blocks:
            _, bi, bm, _ = _stack(gsi, pu, w, flags)
            base = len(inputs)
            inputs += bi
            maps += [dict(m, input_id=m["input_id"] + base) for m in bm]
        say(f"case plan: {len(inputs)} inputs / {len(maps)} maps, wx={wx}")
        ref = gsi.LayerStack(inputs, maps, T, eps)
        _run_tokens(ref, T)
        st = gsi.LayerStack(inputs, maps, T, eps)
        st.refresh(token_offset=0, B=1)
        st.ws.fill_(0xFF)
        plans = []
        for t in range(T):
            st.refresh(token_offset=t, B=1)
            plans.append(st.build_plan())
        torch.cuda.synchronize()
        for rep in range(2):
            for t in range(T):
                st.run_plan(plans[t][0])
        torch.cuda.synchronize()
        exact = L > 4
        nf = 0
        for a, b in zip(st.inputs_t, ref.inputs_t):
            assert torch.equal(a["mask"], b["mask"])
            nf += int(b["mask"].sum())
            for key in ("C", "rnorm", "xnorm", "R"):
                if exact:
                    assert torch.equal(a[key], b[key]), key
                else:
                    assert torch.allclose(a[key], b[key], rtol=0, atol=3e-6 * float(b["xnorm"].max())), key
        assert nf > 0
        for a, b in zip(st.maps_t, ref.maps_t):
            if exact:
                assert torch.equal(a["Y"], b["Y"])
            else:
                assert torch.allclose(a["Y"], b["Y"], rtol=0, atol=1e-5 * float(b["Y"].abs().max()))
    # an input without the single-pass gate cannot be planned
    bad = gsi.LayerStack([dict(inputs[0], flags=0)] + inputs[1:], maps, T, eps)
    bad.refresh(token_offset=0, B=1)
    with pytest.raises(gsi.GsiError) as ei:
        bad.build_plan()
    assert ei.value.code == gsi.GSI_ERR_SHAPE and "planned" in str(ei.value)


def test_single_pass_with_fp8_images_chain_and_static_entry(gsi, pu):
    """The single-pass gate beside the other options of a stack: E4M3 images (codes read as they are by the image
    workgroups), an input that is another map's output (two waves of launches), gsi_layer_stack_static (scratch and
    tables in the library's static array), and a call of 20 inputs with E4M3 images through the table launches.
    Each must agree with the same stack run with the explicit residual: equal decisions, the rest to rounding."""
    sp = gsi.INPUT_GATE_SINGLE_PASS

    def close(a, b, what):
        for x, y in zip(a.inputs_t, b.inputs_t):
            assert torch.equal(x["mask"], y["mask"]), what
            assert torch.allclose(x["C"], y["C"], rtol=0, atol=3e-6 * float(y["xnorm"].max())), what
            assert ((x["rnorm"] - y["rnorm"]).abs() / y["xnorm"].clamp_min(1e-30)).max().item() <= 1e-5, what
        for x, y in zip(a.maps_t, b.maps_t):
            assert torch.allclose(x["Y"], y["Y"], rtol=0, atol=1e-5 * float(y["Y"].abs().max())), what

    # (a) E4M3 images, one block and five blocks
    for L in (1, 5):
        T = 5
        blocks = [wl.transformer_block(f"q{l}", d=512, ffn=2048, k=64, T=T, fire_rate=0.4, p=1.5, seed=4500 + l) for l in range(L)]
        inputs, maps = [], []
        for w in blocks:
            _, bi, bm, _ = _stack(gsi, pu, w, sp)
            base = len(inputs)
            inputs += bi
            for m in bm:
                M8, scale = gsi.quantize_image_fp8(m["M"])
                maps.append({"W": m["W"], "M": M8, "M_scale": scale, "input_id": m["input_id"] + base})
        say(f"case single-pass with E4M3 images: {len(inputs)} inputs")
        a = gsi.LayerStack(inputs, maps, T, blocks[0].eps)
        b = gsi.LayerStack([dict(i, flags=0) for i in inputs], maps, T, blocks[0].eps)
        _run_tokens(a, T)
        _run_tokens(b, T)
        close(a, b, f"fp8 L={L}")
        assert sum(int(i["mask"].sum()) for i in b.inputs_t) > 0
    # (b) a chain: the second input is the first map's output
    w = wl.tiny(256, 32, 384, 6, 2, seed=4600, wdtype="bf16")
    dg = pu.DeviceGroup(w, w.groups[0])
    U1d = gsi.to_device(wl.store(wl.make_basis64(384, 64, 4601), "bf16"), "bf16")
    W1d = gsi.to_device(wl.make_weight(200, 384, 4602, "bf16"), "bf16")
    M1d = gsi.build_image(W1d, U1d)
    maps = [{"W": dg.W["w"], "M": dg.M["w"], "input_id": 0}, {"W": W1d, "M": M1d, "input_id": 1}]

    def chain(flags):
        ins = [{"U": dg.U, "X": dg.X, "flags": flags, "gram": gsi.build_gram(dg.U)},
               {"U": U1d, "src_map": 0, "flags": flags, "gram": gsi.build_gram(U1d)}]
        st = gsi.LayerStack(ins, [dict(m) for m in maps], 6, w.eps)
        _run_tokens(st, 6)
        return st

    say("case single-pass chain")
    close(chain(sp), chain(0), "chain")
    # (c) the entry point without a workspace
    wb = wl.transformer_block("s", d=512, ffn=2048, k=64, T=4, fire_rate=0.5, p=1.5, seed=4700)
    _, bi, bm, _ = _stack(gsi, pu, wb, sp)
    a = gsi.LayerStack(bi, bm, 4, wb.eps)
    b = gsi.LayerStack(bi, bm, 4, wb.eps)
    for t in range(4):
        a.refresh(token_offset=t, B=1)
        a.run_static()
        b.refresh(token_offset=t, B=1)
        b.run()
    torch.cuda.synchronize()
    say("case single-pass through gsi_layer_stack_static")
    for x, y in zip(a.inputs_t, b.inputs_t):
        for key in ("C", "rnorm", "xnorm", "mask"):
            assert torch.equal(x[key], y[key]), key
    for x, y in zip(a.maps_t, b.maps_t):
        assert torch.equal(x["Y"], y["Y"])


def test_table_launches_full_size_in_the_bench_configuration(gsi, pu):
    """Five full-size GPT-J-shaped blocks (20 inputs, 30 maps, 2 GB of W, k = 256) in ONE call per token, the way
    bench.py times its 32 layers: single-pass gate, plans built once per token, the plans' launches captured in a HIP
    graph and replayed.  Every gate decision is checked against the design; the first and the last block are checked
    against the oracle in full (projection, ratio, image, outputs)."""
    L, T, k = 5, 3, 256
    blocks = [wl.gptj_block(T=T, k=k, fire_rate=0.34, seed=wl.BASE_SEED + 1000 + 17 * l) for l in range(L)]
    eps = blocks[0].eps
    inputs, maps, names, dgs_all = [], [], [], []
    for l, w in enumerate(blocks):
        dgs, bi, bm, nm = _stack(gsi, pu, w, gsi.INPUT_GATE_SINGLE_PASS)
        base = len(inputs)
        inputs += bi
        maps += [dict(m, input_id=m["input_id"] + base) for m in bm]
        names += [(base + gi, l, name) for gi, name in nm]
        dgs_all.append(dgs)
    say(f"case table launches at full size: {len(inputs)} inputs / {len(maps)} maps, k={k}")
    st = gsi.LayerStack(inputs, maps, T, eps)
    for ti in st.inputs_t:
        ti["R"].fill_(SENTINEL)
    plans = []
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        plans.append(st.build_plan())
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.run_plan(plans[0][0], stream=side)  # (kernels loaded before the capture)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for t in range(T):
            st.run_plan(plans[t][0])
    for _ in range(2):
        g.replay()
    torch.cuda.synchronize()
    for l, w in enumerate(blocks):
        for gi, grp in enumerate(w.groups):
            ti = st.inputs_t[4 * l + gi]
            assert np.array_equal(ti["mask"].cpu().numpy().astype(bool), grp.fired_design), (l, gi)
    for l in (0, L - 1):
        w = blocks[l]
        for gi, (grp, dg) in enumerate(zip(w.groups, dgs_all[l])):
            say(f"  block {l} input {grp.name}: d={grp.d}")
            og, ref, mask = _check_input(gsi, pu, w, grp, dg, st.inputs_t[4 * l + gi], False)
            for j, (ii, ll, name) in enumerate(names):
                if ii == 4 * l + gi:
                    pu.check_image(gsi.bits_of(dg.M[name]), og.M[name], og.W[name], og.U, w.wdtype)
                    e, es = pu.check_outputs(st.maps_t[j]["Y"], og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype, ref, mask)
                    say(f"    map {name}: rel-L2 vs exact-image oracle {e:.3e}, vs stored-image oracle {es:.3e}")
            del og


@pytest.mark.parametrize("reps,every_input_single_pass", [(3, False), (5, True)])  # 30 and 50 inputs
def test_mixed_shapes_dtypes_and_gates_in_one_single_token_call(gsi, pu, reps, every_input_single_pass):
    """One call per token over 30 (50) inputs of unlike shapes, storage types and options (single-pass and explicit
    gate, both forms of the slow path, shapes that only the generic kernels take): the call sorts them into its
    launches by itself, and every input and map is checked against the oracle on its own.  With the single-pass gate
    on every input the bf16 ones are more than one launch's arguments describe and run over the descriptor table."""
    T = 6
    shapes = [  # d, k, m, wdtype, xdtype
        (512, 64, 520, "bf16", "f32"), (1024, 128, 264, "bf16", "bf16"), (776, 72, 100, "f32", "f32"),
        (33, 7, 10, "f32", "f32"), (2048, 256, 512, "bf16", "f32"), (4096, 64, 1032, "bf16", "f32"),
        (768, 64, 3072, "f32", "f32"), (256, 8, 64, "bf16", "f32"), (1536, 192, 384, "bf16", "f32"),
        (32768, 64, 136, "bf16", "f32"),  # longer than the weight kernel's LDS vector: streamed in blocks of columns
    ]
    cases = []
    for rep in range(reps):
        for si, (d, k, m, wdt, xdt) in enumerate(shapes):
            n = len(cases)
            flags = [gsi.INPUT_GATE_SINGLE_PASS, 0, gsi.INPUT_GATE_SINGLE_PASS | gsi.INPUT_SLOW_PATH_WX,
                     gsi.INPUT_SLOW_PATH_WX][(rep + si) % 4]
            if every_input_single_pass:
                flags |= gsi.INPUT_GATE_SINGLE_PASS
            w = wl.tiny(d, k, m, T, n_fired=(n % 3) + 1, seed=4700 + n, wdtype=wdt, xdtype=xdt)
            cases.append((w, flags))
    eps = cases[0][0].eps
    inputs, maps, dgs = [], [], []
    for gi, (w, flags) in enumerate(cases):
        dg = pu.DeviceGroup(w, w.groups[0])
        dgs.append(dg)
        inputs.append({"U": dg.U, "X": dg.X, "flags": flags,
                       "gram": gsi.build_gram(dg.U) if flags & gsi.INPUT_GATE_SINGLE_PASS else None})
        maps.append({"W": dg.W["w"], "M": dg.M["w"], "input_id": gi})
    say(f"case mixed call: {len(inputs)} inputs")
    st = gsi.LayerStack(inputs, maps, T, eps)
    st.refresh(token_offset=0, B=1)
    st.ws.fill_(0xFF)
    for ti in st.inputs_t:
        ti["R"].fill_(SENTINEL)
    for rep in range(2):
        _run_tokens(st, T)
    skipped = 0
    for gi, (w, flags) in enumerate(cases):
        g = w.groups[0]
        say(f"  input {gi}: d={g.d} k={g.k} {w.wdtype}/{w.xdtype} flags={flags}")
        og = pu.OracleGroup(w, g)
        ref = og.run()
        ti = st.inputs_t[gi]
        mask_dev = ti["mask"].cpu().numpy()
        fired = mask_dev.astype(bool)
        wx = bool(flags & gsi.INPUT_SLOW_PATH_WX)
        R = ti["R"].cpu().numpy()
        # rows of R the call left alone: allowed for tokens that need no residual under the single-pass gate
        untouched = np.all(R == SENTINEL, axis=1)
        if flags & gsi.INPUT_GATE_SINGLE_PASS:
            assert not np.any(untouched & fired & (not wx)), "a fired token has no residual"
            skipped += int(untouched.sum())
        else:
            assert not untouched.any(), "the explicit gate forms every residual"
        Rchk = ti["R"].clone()
        Rchk[torch.from_numpy(untouched)] = torch.from_numpy(ref["R"][untouched].astype(np.float32)).to(Rchk.device)
        res = dict(C=ti["C"], R=Rchk, rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                   n_fired=torch.tensor([int(mask_dev.sum())], dtype=torch.int32),
                   fired_idx=torch.from_numpy(np.nonzero(mask_dev)[0].astype(np.int32)))
        mask = pu.check_projection(res, ref, eps)
        assert np.array_equal(mask.astype(bool), g.fired_design)
        Y = st.maps_t[gi]["Y"]
        if wx:
            Mdev = O.widen(gsi.bits_of(dgs[gi].M["w"]), w.wdtype)
            e = pu.rel_l2_rows(Y.cpu().numpy().astype(np.float64), O.gated_linear_alg1(og.W["w"], Mdev, ref["C"], og.X, mask))
            assert e.max() <= pu.TOL_Y_STAGE[w.wdtype], e.max()
        else:
            pu.check_outputs(Y, og.W["w"], og.M["w"], gsi.bits_of(dgs[gi].M["w"]), w.wdtype, ref, mask)
    assert skipped > 0, "no input took the single-pass gate"
