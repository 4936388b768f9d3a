"""The entry point that takes no workspace (gsi_layer_stack_static) against gsi_layer_stack, through the C ABI:
same outputs bit for bit, on two calls in a row of which the second is the smaller; oversize calls are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2605_03109_amd import workload as wl  # noqa: E402


def _stack(gsi, pu, w, B, flags=0):
    dgs = [pu.DeviceGroup(w, g) for g in w.groups]
    inputs, maps = [], []
    for gi, dg in enumerate(dgs):
        inputs.append({"U": dg.U, "X": dg.X[:B].contiguous(), "flags": flags})
        for name in dg.W:
            maps.append({"W": dg.W[name], "M": dg.M[name], "input_id": gi})
    return gsi.LayerStack(inputs, maps, B, w.eps)


def _outputs(st):
    out = [m["Y"].clone() for m in st.maps_t]
    for i in st.inputs_t:
        out += [i[key].clone() for key in ("C", "R", "rnorm", "xnorm", "mask", "n_fired")]
    return out


def _wipe(st):
    for m in st.maps_t:
        m["Y"].fill_(float("nan"))
    for i in st.inputs_t:
        for key in ("C", "R", "rnorm", "xnorm"):
            i[key].fill_(float("nan"))
        i["mask"].fill_(7)
        i["n_fired"].fill_(-1)


@pytest.mark.parametrize("flags", [0, 2], ids=["separate-kernels", "fused-kernel"])
def test_static_scratch_equals_workspace_call(flags):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import parity_util as pu
    from paper_2605_03109_amd import gsi

    print("case no-alloc: block d=1024 ffn=4096 k=128, then the smaller d=256 ffn=1024 k=64", flush=True)
    big = wl.transformer_block("big", d=1024, ffn=4096, k=128, T=5, fire_rate=0.4, p=1.5, seed=901)
    small = wl.transformer_block("small", d=256, ffn=1024, k=64, T=3, fire_rate=0.34, p=1.5, seed=902)
    for w, Bs in ((big, (5, 1)), (small, (3, 1))):  # first call: the larger input; then smaller ones
        for B in Bs:
            st = _stack(gsi, pu, w, B, flags)
            st.run()
            torch.cuda.synchronize()
            want = _outputs(st)
            _wipe(st)
            st.run_static()
            torch.cuda.synchronize()
            got = _outputs(st)
            for a, b in zip(want, got):
                assert torch.equal(a, b), "static-scratch call differs from the workspace call"
            assert any(int(i["n_fired"].item()) > 0 for i in st.inputs_t) or B == 1


def test_static_scratch_refuses_oversize_calls():
    import parity_util as pu
    from paper_2605_03109_amd import gsi

    # 64 tokens through a 16384-row map: the partial products of the decode-batch kernel alone exceed 8 MiB
    d, k, m, B = 4096, 64, 16384, 64
    U = torch.zeros((d, k), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((m, d), dtype=torch.bfloat16, device="cuda")
    M = torch.zeros((m, k), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((B, d), device="cuda")
    st = gsi.LayerStack([{"U": U, "X": X}], [{"W": W, "M": M, "input_id": 0}], B, 0.05)
    need = int(gsi.lib.gsi_layer_stack_workspace_bytes(st._mp, 1, st._in, 1, B))
    assert need > (8 << 20)
    with pytest.raises(gsi.GsiError) as ei:
        st.run_static()
    assert ei.value.code == gsi.GSI_ERR_WORKSPACE and "static array" in str(ei.value)
