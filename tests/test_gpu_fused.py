"""GPU parity of the fused single-token kernel (GSI_INPUT_FUSED_KERNEL) against the fp64 CPU oracle, through the
C ABI: one launch per call computes projection, residual, gate, image rows and, for fired tokens, the W rows
(Algorithm 1; Section 7.3 "Kernel-level implementation")."""
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


def _run_block(gsi, pu, w, flags, fused=True):
    """Every token of a transformer-block workload through gsi_layer_stack, one call per token."""
    dgs = [pu.DeviceGroup(w, g) for g in w.groups]
    inputs, maps, names = [], [], []
    fl = flags | (gsi.INPUT_FUSED_KERNEL if fused else 0)
    for gi, dg in enumerate(dgs):
        inputs.append({"U": dg.U, "X": dg.X, "flags": fl})
        for name in dg.W:
            maps.append({"W": dg.W[name], "M": dg.M[name], "input_id": gi})
            names.append((gi, name))
    st = gsi.LayerStack(inputs, maps, w.T, w.eps)
    for t in range(w.T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()
    return dgs, st, names


def _check_block(gsi, pu, w, dgs, st, names, wx=False):
    worst = 0.0
    for gi, (g, dg) in enumerate(zip(w.groups, dgs)):
        og = pu.OracleGroup(w, g)
        ref = og.run()
        ti = st.inputs_t[gi]
        n = int(ref["mask"].sum())
        res = dict(C=ti["C"], R=ti["R"], rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                   n_fired=torch.tensor([int(ti["mask"].sum().item())], dtype=torch.int32),
                   fired_idx=torch.nonzero(ti["mask"]).flatten().to(torch.int32))
        mask = pu.check_projection(res, ref, w.eps)
        assert int(mask.sum()) == n
        for j, (g2, name) in enumerate(names):
            if g2 != gi:
                continue
            Y = st.maps_t[j]["Y"]
            if wx:  # fired tokens: the dense product; the others: the image term
                Yo = O.gated_linear_alg1(og.W[name], O.widen(gsi.bits_of(dg.M[name]), w.wdtype), ref["C"], ref["X"], mask)
                e = pu.rel_l2_rows(Y.cpu().numpy().astype(np.float64), Yo)
                assert np.all(e <= pu.TOL_Y_STAGE[w.wdtype]), e.max()
            else:
                e, _ = pu.check_outputs(Y, og.W[name], og.M[name], gsi.bits_of(dg.M[name]), w.wdtype, ref, mask)
                worst = max(worst, e)
    return worst


@pytest.mark.parametrize("d,ffn,k,T,fire", [(512, 2048, 64, 10, 0.3), (1024, 4096, 128, 6, 0.5), (768, 3072, 256, 5, 0.2)])
def test_fused_block_decode(gsi, pu, d, ffn, k, T, fire):
    w = wl.transformer_block("blk", d=d, ffn=ffn, k=k, T=T, fire_rate=fire, p=1.5, seed=300 + k)
    say(f"case fused block d={d} ffn={ffn} k={k} T={T} fire={fire}")
    before = gsi.fused_timeouts()
    dgs, st, names = _run_block(gsi, pu, w, 0)
    worst = _check_block(gsi, pu, w, dgs, st, names)
    assert gsi.fused_timeouts() == before, "a bounded wait inside the fused kernel expired"
    say(f"  worst rel-L2 {worst:.3e}")
    # the default path (separate kernels) on the same tokens: same masks, outputs equal up to summation order
    dgs2, st2, _ = _run_block(gsi, pu, w, 0, fused=False)
    for a, b in zip(st.inputs_t, st2.inputs_t):
        assert torch.equal(a["mask"], b["mask"])
        assert torch.allclose(a["C"], b["C"], rtol=1e-5, atol=1e-6)
    for a, b in zip(st.maps_t, st2.maps_t):
        na = torch.linalg.norm(a["Y"] - b["Y"], dim=1) / torch.linalg.norm(b["Y"], dim=1)
        assert float(na.max()) <= 2e-5


def test_fused_block_fp32_and_wx(gsi, pu):
    w = wl.transformer_block("blk32", d=256, ffn=1024, k=64, T=6, fire_rate=0.34, p=1.5, seed=311, wdtype="f32")
    say("case fused block fp32 storage")
    dgs, st, names = _run_block(gsi, pu, w, 0)
    _check_block(gsi, pu, w, dgs, st, names)
    w2 = wl.transformer_block("blkwx", d=512, ffn=2048, k=64, T=8, fire_rate=0.5, p=1.5, seed=312)
    say("case fused block, fired tokens get W x")
    dgs, st, names = _run_block(gsi, pu, w2, gsi.INPUT_SLOW_PATH_WX)
    _check_block(gsi, pu, w2, dgs, st, names, wx=True)
    # all-fire with the W x form equals the dense stack bit for bit
    w3 = wl.transformer_block("blkall", d=512, ffn=2048, k=64, T=3, fire_rate=1.0, p=1.5, seed=313)
    dgs, st, names = _run_block(gsi, pu, w3, gsi.INPUT_SLOW_PATH_WX)
    ys = [m["Y"].clone() for m in st.maps_t]
    for t in range(w3.T):
        st.refresh(token_offset=t, B=1)
        st.run_dense()
    torch.cuda.synchronize()
    for a, m in zip(ys, st.maps_t):
        assert torch.equal(a, m["Y"])


def test_fused_several_layers_in_one_call_full_size(gsi, pu):
    """Three GPT-J-shaped layers (k = 256) in ONE call per token: several chunks per launch, chunks that hold
    inputs of two layers, gates that fire in some chunks and not in others; sampled against the oracle."""
    from paper_2605_03109_amd import workload_device as wd

    L, T, k, eps = 3, 4, 256, 0.05
    block = [(4096, [4096, 4096, 4096]), (4096, [4096]), (4096, [16384]), (16384, [4096])]
    say(f"case fused {L} full-size layers in one call, k={k}, T={T}")
    inputs, maps, keep = [], [], []
    fired_design = []
    for l in range(L):
        gen = wd.generator(4242 + l)
        for gi, (d, ms) in enumerate(block):
            U64 = wd.make_basis64(d, k, gen)
            f = torch.zeros(T, dtype=torch.bool, device="cuda")
            if (l + gi) % 3 == 0:
                f[(l + gi) % T] = True
            X, _ = wd.make_tokens(U64, f, eps, 1.2, gen)
            U = U64.to(torch.bfloat16).contiguous()
            inputs.append({"U": U, "X": X, "flags": gsi.INPUT_FUSED_KERNEL})
            fired_design.append(f)
            for m in ms:
                W = wd.make_weight(m, d, gen)
                maps.append({"W": W, "M": gsi.build_image(W, U), "input_id": len(inputs) - 1})
    before = gsi.fused_timeouts()
    st = gsi.LayerStack(inputs, maps, T, eps)
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        st.run()
    torch.cuda.synchronize()
    assert gsi.fused_timeouts() == before
    rng = np.random.default_rng(5)
    for i, ti in enumerate(st.inputs_t):
        assert torch.equal(ti["mask"].bool(), fired_design[i]), f"input {i}: mask differs from the design"
        U64 = O.widen(gsi.bits_of(ti["U"]), "bf16")
        X64 = ti["X"].cpu().numpy().astype(np.float64)
        C, R, rn, xn = O.project(U64, X64)
        ref = dict(C=C, R=R, rnorm=rn, xnorm=xn, rho=O.residual_ratio(rn, xn), X=X64)
        ref["mask"], ref["idx"], ref["n"] = O.gate(rn, xn, eps)
        res = dict(C=ti["C"], R=ti["R"], rnorm=ti["rnorm"], xnorm=ti["xnorm"], mask=ti["mask"],
                   n_fired=torch.tensor([int(ti["mask"].sum().item())], dtype=torch.int32),
                   fired_idx=torch.nonzero(ti["mask"]).flatten().to(torch.int32))
        mask = pu.check_projection(res, ref, eps)
        for j, mp in enumerate(st.maps_t):
            if mp["input_id"] != i:
                continue
            # sampled output rows: the oracle one row at a time (the device's stored image: kernel arithmetic only)
            rows = rng.choice(mp["W"].shape[0], size=48, replace=False)
            W64 = O.widen(gsi.bits_of(mp["W"][rows].contiguous()), "bf16")
            M64 = O.widen(gsi.bits_of(mp["M"][rows].contiguous()), "bf16")
            Yo = O.gated_linear(W64, M64, C, R, mask)
            Yg = mp["Y"][:, rows].cpu().numpy().astype(np.float64)
            scale = np.linalg.norm(Yo, axis=1) + 1e-30
            assert np.all(np.linalg.norm(Yg - Yo, axis=1) <= 2e-5 * scale * 4), (i, j)


def test_fused_graph_replay_equals_eager(gsi, pu):
    w = wl.transformer_block("blkg", d=512, ffn=2048, k=64, T=6, fire_rate=0.34, p=1.5, seed=320)
    dgs, st, names = _run_block(gsi, pu, w, 0)
    eager = [m["Y"].clone() for m in st.maps_t] + [i["R"].clone() for i in st.inputs_t] + [i["mask"].clone() for i in st.inputs_t]
    tabs = []
    for t in range(w.T):
        st.refresh(token_offset=t, B=1)
        mp = (gsi.MapDesc * len(st.maps_t))()
        inp = (gsi.InputDesc * len(st.inputs_t))()
        ctypes.memmove(mp, st._mp, ctypes.sizeof(mp))
        ctypes.memmove(inp, st._in, ctypes.sizeof(inp))
        tabs.append((mp, inp))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        s = torch.cuda.current_stream().cuda_stream
        for mp, inp in tabs:
            rc = gsi.lib.gsi_layer_stack(mp, len(mp), inp, len(inp), 1, ctypes.c_float(w.eps), st.ws.data_ptr(), st.ws.numel(), s)
            assert rc == 0, gsi.last_error()
    for rep in range(3):
        for m in st.maps_t:
            m["Y"].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        now = [m["Y"] for m in st.maps_t] + [i["R"] for i in st.inputs_t] + [i["mask"] for i in st.inputs_t]
        for a, b in zip(eager, now):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"
        st.refresh(token_offset=rep % w.T, B=1)
        st.run()  # eager work between the replays
        torch.cuda.synchronize()
