#!/usr/bin/env python3
"""Benchmark of the gated subspace linear layer stack on one MI355X.

Workload: the OPT-6.7B-shaped 32-layer linear stack at batch-1 decode (d = 4096, FFN 16384, bf16 weights,
12.9 GB of W), rank k = 256, 5 % of the gate evaluations fired (one cell of the k x fire-rate sweep; the other
cells the run also measures are reported beside it, and `paper_2605_03109_amd.report` has the full sweep).

A *step* is one pass of the whole hot path over one decode token: for each of the 128 inputs (four per layer)
projection + residual + norms + gate; then the 192 gated linear maps (q, k, v, o, fc_in, fc_out per layer), all
through ONE ``gsi_layer_stack`` call.  Inputs, weights, bases and images are resident in HBM before the timed
region starts.

Prints ONE JSON line.  ``value`` is the effective weight-read rate: the bytes a dense bf16 GEMV pass over the
same weights would read, per second of gated execution (it may exceed the HBM peak -- that is the point of the
method).  The same line carries tokens/s, the dense-GEMV baseline timed on the same GPU, the prediction of the
paper's Eq. (speedup) and the all-bytes bound, the roofline of the dominant kernel and the CPU oracle timed on
the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

# one layer: (input name, d, [(map name, m), ...])
BLOCK = [("attn_in", 4096, [("q", 4096), ("k", 4096), ("v", 4096)]),
         ("attn_out", 4096, [("o", 4096)]),
         ("mlp_in", 4096, [("fc_in", 16384)]),
         ("mlp_hidden", 16384, [("fc_out", 4096)])]
MAPS_PER_LAYER = sum(len(m) for _, _, m in BLOCK)

KERNELS = {
    0: "gsi::proj_stage<BF16> (one launch carries consecutive stages of consecutive sets of 16 independent inputs: "
       "partial c = U^T x; sums of the partials (+ shares of c^T E c with the single-pass gate); image rows y = M c "
       "and residuals; gates)",
    1: "gsi::stream_fired<BF16> (one launch: W r of every fired map of the call)",
}
TABLE_KERNELS = [
    ("table_partial", "gsi::table_partial<BF16> (one launch: partial c = U^T x and shares of |x|^2 of every input of the call)"),
    ("table_gram", "gsi::table_gram (one launch: shares of c^T E c of every input; the sums of the partials are a launch "
                   "before it that is not timed here)"),
    ("table_rows", "gsi::table_rows<BF16> (one launch: image rows y = M c of every map of the call; the gates; r = x - U c of "
                   "the fired inputs)"),
]


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


class HipEvents:
    """Raw HIP timing events (plumbing: the library records them, the runtime reads them)."""

    def __init__(self, n: int):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.ev.append(e)

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[a], self.ev[b])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def close(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)
        self.ev = []


def counter_traffic(which: str, workload_tag: str):
    """HBM-side bytes per launch of a kernel as measured offline with the hardware counters FETCH_SIZE and
    WRITE_SIZE on this same workload (a counter run serialises the kernels and cannot be part of a timed run).
    The committed summary holds the figures and the commands; any other workload reports null."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload_tag}.md")
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch[{which}]:"):
                return int(line.split(":")[1].split()[0])
    except OSError:
        pass
    return None


class Stack:
    """The resident operands of an L-layer stack at one rank, and per-token descriptor tables."""

    def __init__(self, torch, gsi, wd, W, U64, k, T, eps, p, fire, seed, flags=0, plan=False, image="bf16"):
        self.torch, self.gsi, self.T, self.k, self.eps = torch, gsi, T, k, eps
        self.image = image
        L = len(W)
        inputs, maps = [], []
        self.designed = []
        for l in range(L):
            gen = wd.generator(seed + 7919 * l + 13 * k + int(fire * 1000) + 1)
            for gi, (_, d, mp) in enumerate(BLOCK):
                U = U64[l][gi][:, :k].to(torch.bfloat16).contiguous()
                f = wd.choose_fired(T, int(round(fire * T)), gen)
                X, _ = wd.make_tokens(U64[l][gi][:, :k], f, eps, p, gen)
                self.designed.append(f)
                inputs.append({"U": U, "X": X, "flags": flags,
                               "gram": gsi.build_gram(U) if flags & gsi.INPUT_GATE_SINGLE_PASS else None})
                for j, _ in enumerate(mp):
                    maps.append({"W": W[l][gi][j], "M": None, "input_id": len(inputs) - 1})
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for mp in maps:
            mp["M"] = gsi.build_image(mp["W"], inputs[mp["input_id"]]["U"])
            if image == "fp8":  # E4M3 codes + one power-of-two scale per row (Section 7 "Combination with quantization")
                mp["M"], mp["M_scale"] = gsi.quantize_image_fp8(mp["M"])
        torch.cuda.synchronize()
        self.image_build_s = time.perf_counter() - t0
        self.st = gsi.LayerStack(inputs, maps, T, eps)
        self.n_in, self.n_mp = len(inputs), len(maps)
        self.tabs = []
        for t in range(T):
            self.st.refresh(token_offset=t, B=1)
            mp = (gsi.MapDesc * self.n_mp)()
            inp = (gsi.InputDesc * self.n_in)()
            ctypes.memmove(mp, self.st._mp, ctypes.sizeof(mp))
            ctypes.memmove(inp, self.st._in, ctypes.sizeof(inp))
            self.tabs.append((mp, inp))
        self.ws_ptr, self.ws_n = self.st.ws.data_ptr(), self.st.ws.numel()
        self.ceps = ctypes.c_float(eps)
        # the same calls marshalled once (gsi_stack_plan_build): device tables per token, built before anything is timed
        self.plans = None
        if plan:
            self.plans = []
            for t in range(T):
                mp, inp = self.tabs[t]
                nbytes = int(gsi.lib.gsi_stack_plan_bytes(self.n_mp, self.n_in))
                mem = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
                pl = gsi.StackPlan()
                rc = gsi.lib.gsi_stack_plan_build(mp, self.n_mp, inp, self.n_in, self.ws_ptr, self.ws_n, mem.data_ptr(),
                                                  nbytes, ctypes.byref(pl), torch.cuda.current_stream().cuda_stream)
                if rc:
                    raise gsi.GsiError(rc, gsi.last_error())
                self.plans.append((pl, mem))
            torch.cuda.synchronize()

    def gated_step(self, t, s):
        if self.plans is not None:
            rc = self.gsi.lib.gsi_stack_plan_run(ctypes.byref(self.plans[t % self.T][0]), self.ceps, s)
            if rc:
                raise self.gsi.GsiError(rc, self.gsi.last_error())
            return
        mp, inp = self.tabs[t % self.T]
        rc = self.gsi.lib.gsi_layer_stack(mp, self.n_mp, inp, self.n_in, 1, self.ceps, self.ws_ptr, self.ws_n, s)
        if rc:
            raise self.gsi.GsiError(rc, self.gsi.last_error())

    def dense_step(self, t, s):
        mp, inp = self.tabs[t % self.T]
        rc = self.gsi.lib.gsi_dense_stack(mp, self.n_mp, inp, self.n_in, 1, self.ws_ptr, self.ws_n, s)
        if rc:
            raise self.gsi.GsiError(rc, self.gsi.last_error())

    def fired(self):
        """bool[n_inputs, T]: the device's gate decisions of the last pass over the trace."""
        return self.torch.stack([ti["mask"].bool() for ti in self.st.inputs_t])

    def image_row_bytes(self, m):
        """bytes of the image of a map with m rows: bf16 elements, or E4M3 codes and an fp32 scale per row"""
        return m * self.k * 2 if self.image == "bf16" else m * self.k + m * 4

    def bytes(self, fired_frac_by_input):
        """(dense bytes, image bytes, basis bytes, expected W bytes of fired inputs) per step."""
        k, bw = self.k, 2
        L = self.n_in // len(BLOCK)
        dense = L * sum(m * d * bw for _, d, mp in BLOCK for _, m in mp)
        img = L * sum(self.image_row_bytes(m) for _, d, mp in BLOCK for _, m in mp)
        bas = L * sum(d * k * bw for _, d, _ in BLOCK)
        wf = 0.0
        for i in range(self.n_in):
            _, d, mp = BLOCK[i % len(BLOCK)]
            wf += fired_frac_by_input[i] * sum(m * d * bw for _, m in mp)
        return dense, img, bas, wf


def timed_run(torch, step_fn, T, steps, warmup, mode, chunk=128):
    """Seconds for exactly `steps` steps after at least `warmup` untimed ones.  graph: the steps of the trace
    (the first min(T, steps) tokens) are captured into HIP graphs of up to `chunk` steps and replayed in order;
    a remainder that is no whole pass over the trace gets a graph of its own."""
    if mode == "graph":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for t in range(min(T, 2)):
                step_fn(t, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        Tp = min(T, steps)

        def capture(t0, t1):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream().cuda_stream
                for t in range(t0, t1):
                    step_fn(t, cs)
            return g

        full = [capture(c0, min(Tp, c0 + chunk)) for c0 in range(0, Tp, chunk)]
        reps, rem = divmod(steps, Tp)
        tail = [capture(c0, min(rem, c0 + chunk)) for c0 in range(0, rem, chunk)]
        done = 0
        while done < max(warmup, 1):
            for g in full:
                g.replay()
            done += Tp
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            for g in full:
                g.replay()
        for g in tail:
            g.replay()
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    s0 = torch.cuda.current_stream().cuda_stream
    for t in range(warmup):
        step_fn(t, s0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        step_fn(t, s0)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="graph: the decode steps are captured into HIP graphs and replayed")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--tokens", type=int, default=512, help="decode tokens in the synthetic trace")
    ap.add_argument("--k", type=int, default=256)
    ap.add_argument("--fire", type=float, default=0.05, help="fraction of gate evaluations that fire")
    ap.add_argument("--cells", default="256:0,256:0.25,256:1,64:0,128:0,512:0",
                    help="further k:fire cells measured on a shorter trace and reported beside the headline cell "
                         "('' = none)")
    ap.add_argument("--cell-tokens", type=int, default=128)
    ap.add_argument("--fused", action="store_true",
                    help="ask for the fused single-token kernel (GSI_INPUT_FUSED_KERNEL) instead of the separate kernels")
    ap.add_argument("--gate", choices=["single-pass", "explicit"], default="single-pass",
                    help="single-pass: residual ratio from |x|^2 - |c|^2 + c^T E c with the cached E = U^T U - I "
                         "(GSI_INPUT_GATE_SINGLE_PASS: the basis is read once, r is formed for fired tokens only); "
                         "explicit: r = x - U c formed for every token")
    ap.add_argument("--slow-path", choices=["mc+wr", "wx"], default="mc+wr",
                    help="wx: fired tokens get y = W x as Algorithm 1 prints it (GSI_INPUT_SLOW_PATH_WX); with the "
                         "single-pass gate a fired input's image rows are then skipped")
    ap.add_argument("--image", choices=["bf16", "fp8"], default="bf16",
                    help="storage of the cached images: the weights' bf16, or E4M3 codes with a scale per row "
                         "(Section 7 \"Combination with quantization\": half the fast-path bytes, 3e-2 output error)")
    ap.add_argument("--no-plan", action="store_true",
                    help="call gsi_layer_stack with host descriptors every step instead of running plans that "
                         "gsi_stack_plan_build marshalled once (single-pass gate only)")
    ap.add_argument("--host-qr", action="store_true", help="factor the seeded Gaussians on the host (for runs under a "
                                                          "profiler that the device QR does not survive)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the CPU-oracle leg (0 = skip)")
    ap.add_argument("--no-roofline", action="store_true")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus {args.gpus} is not "
              "supported. Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2605_03109_amd import gsi
    from paper_2605_03109_amd import workload_device as wd

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    L, T, eps, p = args.layers, args.tokens, 0.05, 1.2
    cells = [(int(c.split(":")[0]), float(c.split(":")[1])) for c in args.cells.split(",") if c]
    kmax = max([args.k] + [k for k, _ in cells])
    seed = wd.BASE_SEED + 2000
    t0 = time.perf_counter()
    W, U64 = [], []
    for l in range(L):
        gen = wd.generator(seed + 7919 * l)
        Wl, Ul = [], []
        for gi, (_, d, maps) in enumerate(BLOCK):
            Ul.append(wd.make_basis64(d, kmax, gen, args.host_qr))  # nested bases: rank k uses the first k columns
            Wl.append([wd.make_weight(m, d, gen) for _, m in maps])
        W.append(Wl)
        U64.append(Ul)
    torch.cuda.synchronize()
    log(f"[bench] {L} layers generated in {time.perf_counter()-t0:.1f}s")
    flags = gsi.INPUT_FUSED_KERNEL if args.fused else 0
    single_pass = args.gate == "single-pass" and not args.fused
    if single_pass:
        flags |= gsi.INPUT_GATE_SINGLE_PASS
    if args.slow_path == "wx":
        flags |= gsi.INPUT_SLOW_PATH_WX

    # ---- the headline cell ------------------------------------------------------------------------------
    t0 = time.perf_counter()
    use_plan = single_pass and not args.no_plan
    S = Stack(torch, gsi, wd, W, U64, args.k, T, eps, p, args.fire, seed, flags, use_plan, args.image)
    log(f"[bench] cell k={args.k} fire={args.fire}: {S.n_in} inputs, {S.n_mp} maps, {T} tokens resident in "
        f"{time.perf_counter()-t0:.1f}s (images built in {S.image_build_s*1e3:.0f} ms)")
    mode = args.mode
    try:
        sec_gated = timed_run(torch, S.gated_step, T, args.steps, args.warmup, mode)
    except Exception as exc:  # graph capture unavailable: say so and time eagerly
        if mode != "graph":
            raise
        log(f"[bench] HIP graph capture failed ({exc!r}); timing eagerly instead")
        mode = "eager"
        sec_gated = timed_run(torch, S.gated_step, T, args.steps, args.warmup, mode)
    log(f"[bench] gated stack: {sec_gated*1e6/args.steps:.1f} us/step ({mode})")
    sec_dense = timed_run(torch, S.dense_step, T, args.steps, args.warmup, mode)
    dense_us = sec_dense * 1e6 / args.steps
    log(f"[bench] dense stack: {dense_us:.1f} us/step ({mode})")

    def gate_stats(Sx, n_timed):
        s0 = torch.cuda.current_stream().cuda_stream
        for t in range(Sx.T):
            Sx.gated_step(t, s0)
        torch.cuda.synchronize()
        fired = Sx.fired()
        designed = torch.stack(Sx.designed)
        timed = torch.arange(n_timed, device=fired.device) % Sx.T  # the tokens the timed steps walked
        frac = [float(v) for v in fired[:, timed].double().mean(dim=1).cpu()]
        return fired, bool(torch.equal(fired, designed)), frac

    def cell_numbers(Sx, us, n_timed):
        fired, match, frac = gate_stats(Sx, n_timed)
        dense, img, bas, wf = Sx.bytes(frac)
        alg = img + bas + wf
        f_eff = wf / dense
        return {
            "us_per_step": round(us, 2), "tokens_per_s": round(1e6 / us, 1),
            "effective_weight_GBs": round(dense / us / 1e3, 1),
            "speedup_vs_dense_gemv": round(dense_us / us, 3),
            # Eq. (speedup) with the volume-weighted d/k of the block (weights only: the fast path costs the
            # images, a fired input its W), and the bound that also counts the bases
            "eq_speedup_weights_only": round(1.0 / ((1.0 - f_eff) * img / dense + f_eff), 2),
            "all_bytes_speedup_bound": round(dense / alg, 2),
            "algorithmic_bytes_per_step": round(alg), "algorithmic_GBs": round(alg / us / 1e3, 1),
            "measured_fire_rate": round(sum(frac) / len(frac), 4), "masks_match_design": match,
        }, fired

    head, fired = cell_numbers(S, sec_gated * 1e6 / args.steps, args.steps)
    dense_bytes = S.bytes([0.0] * S.n_in)[0]

    # ---- roofline of the dominant kernel: every launch of a step timed by its own dispatch timestamps (HIP events
    #      given to that launch), one launch per call of the whole step
    roofline, kernels = None, None
    if not args.no_roofline and not args.fused:
        SET = 16                                  # inputs per launch of the staged kernel
        nsets = (S.n_in + SET - 1) // SET
        table_mode = single_pass and nsets > 1    # every stage once for all inputs: three launches
        sum_stage = 1 if (single_pass or nsets > 1) else 0
        inline_gate = (not single_pass) and nsets == 1 and S.n_mp <= 24 and S.n_in <= 16  # the weight kernel gates
        n_launch = {0: 3 if table_mode else nsets + 2 + sum_stage - (1 if single_pass or inline_gate else 0), 1: 1}
        K = min(T, 24)
        evs = HipEvents(2)
        s0 = torch.cuda.current_stream().cuda_stream
        fired_np = fired.cpu().numpy()
        k = args.k

        def set_inputs(g):
            if table_mode:
                return range(S.n_in) if g == 0 else range(0)
            return range(g * SET, min(S.n_in, (g + 1) * SET)) if 0 <= g < nsets else range(0)

        def stage_bytes(idx, t):  # launch idx: partial projections of set idx, residuals + image rows of set idx - 2
            b = 0
            for i in set_inputs(idx):       # the basis once, x
                d = BLOCK[i % len(BLOCK)][1]
                b += d * k * 2 + d * 4
            if single_pass:
                for i in set_inputs(idx - 1):   # E and c
                    b += k * k * 4 + k * 4
            for i in set_inputs(idx - 2):   # the images, c read, y written; explicit gate: x again, r written;
                _, d, mpl = BLOCK[i % len(BLOCK)]  # single-pass gate: the basis again, x, r for a fired input only
                b += sum(S.image_row_bytes(m) + m * 4 for _, m in mpl) + k * 4
                if not single_pass:
                    b += d * 4 + d * 4
                elif fired_np[i, t]:
                    b += d * k * 2 + d * 4 + d * 4
            return b

        def stream_bytes(idx, t):  # W of a fired input's maps, r, y read and written
            b = 0
            for i in range(S.n_in):
                _, d, mpl = BLOCK[i % len(BLOCK)]
                if fired_np[i, t]:
                    b += sum(m * d * 2 + 2 * m * 4 for _, m in mpl) + d * 4
            return b

        dur = {w: np.zeros((n_launch[w], K)) for w in (0, 1)}
        nbytes = {w: np.zeros((n_launch[w], K)) for w in (0, 1)}
        for which in (0, 1):
            for t in range(K):
                mp, inp = S.tabs[t]
                for idx in range(n_launch[which]):
                    rc = gsi.lib.gsi_layer_stack_timed(mp, S.n_mp, inp, S.n_in, 1, S.ceps, S.ws_ptr, S.ws_n, s0, which,
                                                       idx, evs.ev[0], evs.ev[1])
                    if rc:
                        raise gsi.GsiError(rc, gsi.last_error())
                    torch.cuda.synchronize()
                    dur[which][idx, t] = evs.elapsed_ms(0, 1) * 1e-3
                    nbytes[which][idx, t] = stage_bytes(idx, t) if which == 0 else stream_bytes(idx, t)
        evs.close()
        def entry_of(name, text, d_all, b_all, extra):
            live = b_all > 0  # (a weight launch in which no gate fired moves no weight byte)
            d_use, b_use = (d_all[live], b_all[live]) if live.any() else (d_all, b_all)
            ach = float(b_use.sum() / d_use.sum() / 1e9) if d_use.size else 0.0
            e = {"kernel": text, "launches": int(d_use.size), "avg_launch_us": round(float(d_use.mean() * 1e6), 2),
                 "avg_algorithmic_bytes": round(float(b_use.mean())), "achieved_GBs": round(ach, 1),
                 "frac_of_hbm_peak": round(ach / HBM_PEAK_GBS, 4),
                 "us_per_step_total": round(float(d_all.sum() / K * 1e6), 1)}
            e.update(extra)
            kernels[name] = e

        kernels = {}
        if table_mode:  # one entry per kernel of the three table launches
            for idx, (name, text) in enumerate(TABLE_KERNELS):
                entry_of(name, text, dur[0][idx], nbytes[0][idx], {})
        else:
            entry_of("proj_stage", KERNELS[0], dur[0].ravel(), nbytes[0].ravel(),
                     {"launches_per_step": n_launch[0],
                      "per_launch_us": [round(float(v.mean() * 1e6), 2) for v in dur[0]],
                      "per_launch_algorithmic_MB": [round(float(v.mean() / 1e6), 2) for v in nbytes[0]]})
        d1, b1 = dur[1].ravel(), nbytes[1].ravel()
        entry_of("stream_fired", KERNELS[1], d1, b1,
                 {"launches_without_fired_gate": int((b1 == 0).sum()),
                  "unfired_launch_us": round(float(d1[b1 == 0].mean() * 1e6), 2) if (b1 == 0).any() else None})
        dom = max(kernels, key=lambda n: kernels[n]["us_per_step_total"])
        e = kernels[dom]
        tag = f"opt_stack_{L}layers_k{args.k}_fire{int(round(args.fire * 100))}_decode" + ("" if args.image == "bf16" else "_fp8")
        roofline = {"bound": "hbm", "kernel": e["kernel"], "achieved": e["achieved_GBs"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": e["frac_of_hbm_peak"], "traffic": counter_traffic(dom, tag),
                    "avg_launch_us": e["avg_launch_us"], "avg_algorithmic_bytes": e["avg_algorithmic_bytes"],
                    "launches": e["launches"], "share_of_step": round(e["us_per_step_total"] / head["us_per_step"], 3)}

    # ---- CPU oracle on a bounded sample of the same workload: layer 0, token by token ---------------------
    cpu = None
    if args.cpu_seconds > 0:
        import oracle.gsi_oracle as O

        try:
            from threadpoolctl import threadpool_info

            cores = max([q.get("num_threads", 1) for q in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        t0 = time.perf_counter()
        ng = len(BLOCK)
        groups_np = []
        for gi in range(ng):
            ti = S.st.inputs_t[gi]
            mps = [(f"m{j}", gsi.bits_of(mt["W"]), "bf16") for j, mt in enumerate(S.st.maps_t) if mt["input_id"] == gi]
            groups_np.append({"U": gsi.bits_of(ti["U"]), "udtype": "bf16", "maps": mps})
        prep = O.prepare_stack(groups_np)
        X64 = [S.st.inputs_t[gi]["X"].cpu().numpy().astype(np.float64) for gi in range(ng)]
        log(f"[bench] oracle set-up for layer 0 (widen + fp64 images, untimed): {time.perf_counter()-t0:.1f}s")
        done, spent, n_fired_sample = 0, 0.0, 0
        while spent < args.cpu_seconds:
            t_idx = done % T
            t1 = time.perf_counter()
            res = O.run_stack(prep, [x[t_idx:t_idx + 1] for x in X64], eps)
            spent += time.perf_counter() - t1
            n_fired_sample += sum(r["n_fired"] for r in res)
            done += 1
        layer_steps_s = done / spent
        cpu = {"value": round(dense_bytes / L * layer_steps_s / 1e9, 3), "unit": "GB/s", "cores": int(cores),
               "kind": "oracle", "layer_steps_per_s": round(layer_steps_s, 2),
               "tokens_per_s": round(layer_steps_s / L, 3),
               "sample": f"layer 0 of the stack, {done} decode tokens one at a time ({n_fired_sample} of {done * ng} "
                         f"gate evaluations fired), fp64 NumPy, {spent:.1f} s; tokens/s of the {L}-layer stack = "
                         f"layer-steps/s / {L}; operands widened and images built beforehand"}
        del prep, X64

    # ---- further cells of the sweep on a shorter trace ------------------------------------------------------
    others = []
    Tc = min(args.cell_tokens, T)
    del S
    torch.cuda.empty_cache()
    for k, fire in cells:
        Sx = Stack(torch, gsi, wd, W, U64, k, Tc, eps, p, fire, seed, flags, use_plan, args.image)
        n = max(Tc, min(args.steps, 2 * Tc))
        sec = timed_run(torch, Sx.gated_step, Tc, n, min(args.warmup, Tc), mode)
        c, _ = cell_numbers(Sx, sec * 1e6 / n, n)
        c.update({"k": k, "designed_fire_rate": fire, "decode_tokens": Tc, "steps": n})
        others.append(c)
        log(f"[bench] cell k={k} fire={fire}: {c['us_per_step']} us/step, {c['speedup_vs_dense_gemv']}x")
        del Sx
        torch.cuda.empty_cache()

    tokens_per_s = args.steps / sec_gated
    out = {
        "metric": "effective weight-read GB/s and tokens/s per gated layer stack vs dense GEMV",
        "value": round(dense_bytes * tokens_per_s / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_gated * 1e3 / args.steps, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"OPT-6.7B-shaped {L}-layer linear stack, batch-1 decode: per layer q,k,v,o 4096x4096, fc1 "
                        "16384x4096, fc2 4096x16384 over four inputs; bf16 weights/bases, images in "
                        + ("bf16" if args.image == "bf16" else "E4M3 with a scale per row") + ", fp32 accumulate; one "
                        "gsi_layer_stack call per decode token",
            "layers": L, "k": args.k, "eps": eps, "decode_tokens": T, "designed_fire_rate": args.fire,
            "measured_fire_rate": head["measured_fire_rate"], "masks_match_design": head["masks_match_design"],
            "launch_mode": mode, "slow_path": "W x (a fired input skips its image)" if args.slow_path == "wx" else "M c + W r",
            "call": "gsi_stack_plan_run on a plan built once per trace token (gsi_stack_plan_build)" if use_plan
                    else "gsi_layer_stack with host descriptors every step",
            "single_token_kernels": "fused" if args.fused else "separate",
            "gate": "single pass over the basis: |r|^2 = |x|^2 - |c|^2 + c^T (U^T U - I) c, r formed for fired tokens only"
                    if single_pass else "explicit residual r = x - U c for every token",
        },
        "tokens_per_s": round(tokens_per_s, 1),
        "dense_gemv_tokens_per_s": round(args.steps / sec_dense, 1),
        "dense_gemv_GBs": round(dense_bytes * args.steps / sec_dense / 1e9, 1),
        "speedup_vs_dense_gemv": head["speedup_vs_dense_gemv"],
        "eq_speedup_weights_only": head["eq_speedup_weights_only"],
        "all_bytes_speedup_bound": head["all_bytes_speedup_bound"],
        "algorithmic_GBs": head["algorithmic_GBs"],
        "algorithmic_frac_of_hbm_peak": round(head["algorithmic_GBs"] / HBM_PEAK_GBS, 4),
        "dense_weight_bytes_per_step": dense_bytes,
        "algorithmic_bytes_per_step": head["algorithmic_bytes_per_step"],
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
        "other_cells": others,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
