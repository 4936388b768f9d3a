#!/usr/bin/env python3
"""Benchmark of the gated subspace linear layer stack on one MI355X.

A *step* is one pass of the whole hot path over one decode token (batch 1): for each of the four
inputs of a GPT-J-6B-shaped transformer block, projection + residual + norms + gate; then the six
gated linear maps (q, k, v, o, fc_in, fc_out), all through ``gsi_layer_stack``.  Inputs, weights,
bases and images are resident in HBM before the timed region starts.

Prints ONE JSON line.  ``value`` is the effective weight-read rate: the bytes a dense bf16 GEMV pass
over the same six weights would read, per second of gated execution (it may exceed the HBM peak --
that is the point of the method).  The same line carries tokens/s, the dense-GEMV baseline timed on
the same GPU with the same kernels, the roofline of the dominant kernel and the CPU oracle timed on
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


def counter_traffic(args):
    """HBM-side bytes per fired launch of the weight-streaming kernel, as measured offline with the
    hardware counters FETCH_SIZE and WRITE_SIZE on this same workload (a counter run serialises the
    kernels and cannot be part of a timed run).  The committed summary holds the figure and the commands;
    it applies to the default workload only, so any other setting reports null."""
    if (args.tokens, args.k, args.fire) != (256, 256, 0.1):
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        "hbm_traffic_stream_rows_gptj_block_k256_decode.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_fired_launch:"):
                return int(line.split(":")[1].split()[0])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=512)
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="graph: the decode steps are captured once into a HIP graph and replayed")
    ap.add_argument("--tokens", type=int, default=256, help="decode tokens in the synthetic trace")
    ap.add_argument("--k", type=int, default=256)
    ap.add_argument("--fire", type=float, default=0.10, help="fraction of gate evaluations that fire")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the CPU-oracle leg (0 = skip)")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--slow-path", choices=["mc_wr", "wx"], default="mc_wr",
                    help="what a fired token gets: M c + W r (the form the metric is quoted on) or W x as "
                         "Algorithm 1 prints it")
    ap.add_argument("--image", choices=["bf16", "fp8"], default="bf16",
                    help="storage of the cached images: the weights' dtype (the form the metric is quoted on) or "
                         "8-bit E4M3 with row scales (Section 7, combination with quantization)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="copies of every basis and image, used in turn by consecutive tokens: with 8 the un-fired "
                         "working set (33.6 MB a copy) no longer stays in the 256 MB Infinity Cache (the weights, "
                         "403 MB, never do)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three device copies of 512 MiB first (a kernel of known traffic, used to "
                         "scale hardware-counter readings of a rocprofv3 --pmc run)")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus {args.gpus} is not "
              "supported. Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2605_03109_amd import gsi
    from paper_2605_03109_amd import workload as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    if args.pmc_calibration:
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    T = args.tokens
    t_gen = time.perf_counter()
    w = wl.gptj_block(T=T, k=args.k, fire_rate=args.fire)
    log(f"[bench] workload {w.name}: T={T} k={args.k} fire={args.fire} generated in {time.perf_counter()-t_gen:.1f}s")

    # ---- resident operands ----------------------------------------------------------------------
    inputs, maps, meta = [], [], []
    for gi, g in enumerate(w.groups):
        U = gsi.to_device(g.U, w.wdtype)
        inputs.append({"U": U, "X": gsi.to_device(g.X, w.xdtype),
                       "flags": gsi.INPUT_SLOW_PATH_WX if args.slow_path == "wx" else 0})
        for name, m, W in g.maps:
            Wd = gsi.to_device(W, w.wdtype)
            mp = {"W": Wd, "M": gsi.build_image(Wd, U), "input_id": gi}
            if args.image == "fp8":
                mp["M"], mp["M_scale"] = gsi.quantize_image_fp8(mp["M"])
            maps.append(mp)
            meta.append((gi, name, m, g.d, g.k))
    torch.cuda.synchronize()
    st = gsi.LayerStack(inputs, maps, T, w.eps)
    n_in, n_mp = len(st.inputs_t), len(st.maps_t)
    # further copies of the fast-path operands (bases, images, scales), same values at other addresses
    copies = [({}, {})]
    for _ in range(1, max(1, args.rotate)):
        cu = {i: t["U"].clone() for i, t in enumerate(st.inputs_t)}
        cm = {j: (t["M"].clone(), None if t["M_scale"] is None else t["M_scale"].clone()) for j, t in enumerate(st.maps_t)}
        copies.append((cu, cm))

    # one descriptor table per decode token (host structs; built once, outside the timed region)
    tabs = []
    for t in range(T):
        st.refresh(token_offset=t, B=1)
        mp = (gsi.MapDesc * n_mp)()
        inp = (gsi.InputDesc * n_in)()
        ctypes.memmove(mp, st._mp, ctypes.sizeof(mp))
        ctypes.memmove(inp, st._in, ctypes.sizeof(inp))
        cu, cm = copies[t % len(copies)]
        for i, u in cu.items():
            inp[i].U = u.data_ptr()
        for j, (mm, sc) in cm.items():
            mp[j].M = mm.data_ptr()
            if sc is not None:
                mp[j].M_scale = sc.data_ptr()
        tabs.append((mp, inp))
    ws_ptr, ws_n = st.ws.data_ptr(), st.ws.numel()
    stream = torch.cuda.current_stream()
    lib = gsi.lib
    eps = ctypes.c_float(w.eps)

    def gated_step(t, s):
        mp, inp = tabs[t % T]
        rc = lib.gsi_layer_stack(mp, n_mp, inp, n_in, 1, eps, ws_ptr, ws_n, s)
        if rc:
            raise gsi.GsiError(rc, gsi.last_error())

    def dense_step(t, s):
        mp, inp = tabs[t % T]
        rc = lib.gsi_dense_stack(mp, n_mp, inp, n_in, 1, ws_ptr, ws_n, s)
        if rc:
            raise gsi.GsiError(rc, gsi.last_error())

    def timed_run(step_fn, steps, warmup, mode):
        """Return seconds for exactly `steps` steps (after `warmup` untimed ones)."""
        if mode == "graph":
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for t in range(min(T, 8)):
                    step_fn(t, side.cuda_stream)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                cs = torch.cuda.current_stream().cuda_stream
                for t in range(T):
                    step_fn(t, cs)
            reps_w = max(1, -(-warmup // T))
            for _ in range(reps_w):
                graph.replay()
            torch.cuda.synchronize()
            reps, rem = divmod(steps, T)
            s0 = torch.cuda.current_stream().cuda_stream
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                graph.replay()
            for t in range(rem):
                step_fn(t, s0)
            torch.cuda.synchronize()
            return time.perf_counter() - t0
        s0 = stream.cuda_stream
        for t in range(warmup):
            step_fn(t, s0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(steps):
            step_fn(t, s0)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    mode = args.mode
    try:
        sec_gated = timed_run(gated_step, args.steps, args.warmup, mode)
    except Exception as exc:  # graph capture unavailable: say so and time eagerly
        if mode != "graph":
            raise
        log(f"[bench] HIP graph capture failed ({exc!r}); timing eagerly instead")
        mode = "eager"
        sec_gated = timed_run(gated_step, args.steps, args.warmup, mode)
    log(f"[bench] gated stack: {sec_gated*1e6/args.steps:.2f} us/step ({mode})")
    sec_dense = timed_run(dense_step, args.steps, args.warmup, mode)
    log(f"[bench] dense stack: {sec_dense*1e6/args.steps:.2f} us/step ({mode})")

    # gate statistics of the trace (read back once, after timing)
    for t in range(T):
        gated_step(t, stream.cuda_stream)
    torch.cuda.synchronize()
    fired = np.stack([ti["mask"].cpu().numpy().astype(bool) for ti in st.inputs_t])  # [groups, T]
    designed = np.stack([g.fired_design for g in w.groups])
    masks_match_design = bool(np.array_equal(fired, designed))

    dense_bytes = w.dense_weight_bytes
    bw = 2
    # Algorithmic bytes per step.  The weight-streaming launch (the dominant kernel) reads the partial
    # norms of every input and, for each fired input, r and the W rows of its maps, and updates y.
    # The projection launches read U and x once, write c and r, read every image M and write y.
    lin_bytes = np.zeros(T)
    proj_bytes = 0.0
    for gi, g in enumerate(w.groups):
        proj_bytes += g.d * g.k * bw + g.d * 4 + g.k * 4 + g.d * 4
        for _, m, _ in g.maps:
            proj_bytes += m * g.k * (1 if args.image == "fp8" else bw) + m * 4 + (m * 4 if args.image == "fp8" else 0)
            lin_bytes += fired[gi] * (m * g.d * bw + 2 * m * 4)
        lin_bytes += fired[gi] * (g.d * 4)
    order = np.arange(args.steps) % T
    alg_bytes_step = float(np.mean(lin_bytes[order]) + proj_bytes)

    tokens_per_s = args.steps / sec_gated
    dense_tokens_per_s = args.steps / sec_dense
    value = dense_bytes * tokens_per_s / 1e9

    # ---- roofline of the dominant kernel (the batched linear-map launch), HIP events around it -----
    roofline = None
    if not args.no_roofline:
        K = min(args.steps, 1024)
        evs = HipEvents(2 * K)
        s0 = stream.cuda_stream
        # Ballast: enough queued dense passes that the host finishes enqueueing the K instrumented steps
        # while the device is still busy, so that every event pair brackets device execution of the
        # kernel rather than host launch latency.
        for t in range(max(256, K // 2)):
            dense_step(t, s0)
        for i in range(K):
            mp, inp = tabs[i % T]
            rc = lib.gsi_layer_stack_timed(mp, n_mp, inp, n_in, 1, eps, ws_ptr, ws_n, s0, evs.ev[2 * i],
                                           evs.ev[2 * i + 1])
            if rc:
                raise gsi.GsiError(rc, gsi.last_error())
        torch.cuda.synchronize()
        dur = np.array([evs.elapsed_ms(2 * i, 2 * i + 1) for i in range(K)]) * 1e-3
        evs.close()
        idx = np.arange(K) % T
        fired_any = fired.any(axis=0)[idx]
        # Roofline of the weight-streaming launches: those of steps in which at least one gate fired.  A
        # launch of a step in which nothing fired ends after the gate and moves no weight byte; its
        # duration is reported beside it.
        if fired_any.any():
            avg_dur = float(dur[fired_any].mean())
            avg_bytes = float(np.mean(lin_bytes[idx][fired_any]))
        else:
            avg_dur, avg_bytes = float(dur.mean()), 0.0
        achieved = avg_bytes / avg_dur / 1e9
        roofline = {
            "bound": "hbm", "kernel": "gsi::stream_rows<BF16, dense=false> (W r of every fired map of a step, one launch)",
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": counter_traffic(args),
            "avg_launch_us": round(avg_dur * 1e6, 3), "avg_algorithmic_bytes": round(avg_bytes),
            "launches": int(fired_any.sum()),
            "launches_without_fired_gate": int((~fired_any).sum()),
            "unfired_launch_us": round(float(dur[~fired_any].mean() * 1e6), 3) if (~fired_any).any() else None,
        }

    # ---- CPU oracle on a bounded sample of the same workload -------------------------------------------
    cpu = None
    if args.cpu_seconds > 0:
        import oracle.gsi_oracle as O

        try:
            from threadpoolctl import threadpool_info

            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        t0 = time.perf_counter()
        prep = O.prepare_stack(
            [{"U": g.U, "udtype": w.wdtype, "maps": [(n, W, w.wdtype) for n, _, W in g.maps]} for g in w.groups])
        X64 = [O.widen(g.X, w.xdtype) for g in w.groups]
        log(f"[bench] oracle set-up (widen + fp64 images, untimed): {time.perf_counter()-t0:.1f}s")
        done, spent = 0, 0.0
        n_fired_sample = 0
        while spent < args.cpu_seconds:  # the trace is walked again if the budget allows
            t_idx = done % T
            t1 = time.perf_counter()
            res = O.run_stack(prep, [x[t_idx:t_idx + 1] for x in X64], w.eps)
            spent += time.perf_counter() - t1
            n_fired_sample += sum(r["n_fired"] for r in res)
            done += 1
        cpu_tok_s = done / spent

        def short_leg(fn, budget):
            n, used = 0, 0.0
            while used < budget:
                t1 = time.perf_counter()
                fn(n % T)
                used += time.perf_counter() - t1
                n += 1
            return n / used

        # the dense stack y = W x through the oracle, and the gated stack on one core (short samples)
        side = min(4.0, args.cpu_seconds / 3)
        dense_tok_s = short_leg(lambda t: O.run_dense_stack(prep, [x[t:t + 1] for x in X64]), side)
        one_core_tok_s = None
        try:
            from threadpoolctl import threadpool_limits

            with threadpool_limits(limits=1):
                one_core_tok_s = short_leg(lambda t: O.run_stack(prep, [x[t:t + 1] for x in X64], w.eps), side)
        except Exception as exc:
            log(f"[bench] one-core oracle leg skipped: {exc!r}")
        cpu = {
            "value": round(dense_bytes * cpu_tok_s / 1e9, 3), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "tokens_per_s": round(cpu_tok_s, 3),
            "dense_oracle_tokens_per_s": round(dense_tok_s, 3),
            "one_core_tokens_per_s": None if one_core_tok_s is None else round(one_core_tok_s, 3),
            "sample": f"{done} decode tokens of the same block (the {T}-token trace, walked in order and "
                      f"repeated), one at a time ({n_fired_sample} of {done * len(w.groups)} gate evaluations "
                      f"fired), fp64 NumPy, {spent:.1f} s; operands widened and images built beforehand",
        }

    out = {
        "metric": "effective weight-read GB/s and tokens/s per gated layer stack vs dense GEMV",
        "value": round(value, 1),
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
            "workload": "GPT-J-6B-shaped transformer block, batch-1 decode: q,k,v,o 4096x4096, fc_in 16384x4096, "
                        "fc_out 4096x16384, bf16 weights/images/bases, fp32 accumulate",
            "k": args.k, "eps": w.eps, "decode_tokens": T, "designed_fire_rate": args.fire,
            "measured_fire_rate": round(float(fired.mean()), 4), "masks_match_design": masks_match_design,
            "launch_mode": mode, "slow_path": "M c + W r" if args.slow_path == "mc_wr" else "W x (Algorithm 1, line 7)",
            "image_storage": "bf16" if args.image == "bf16" else "fp8 e4m3 + power-of-two row scales",
            "fast_path_operand_copies": max(1, args.rotate),
        },
        "tokens_per_s": round(tokens_per_s, 1),
        "dense_gemv_tokens_per_s": round(dense_tokens_per_s, 1),
        "dense_gemv_GBs": round(dense_bytes * dense_tokens_per_s / 1e9, 1),
        "speedup_vs_dense_gemv": round(sec_dense / sec_gated, 3),
        "algorithmic_GBs": round(alg_bytes_step * tokens_per_s / 1e9, 1),
        "algorithmic_frac_of_hbm_peak": round(alg_bytes_step * tokens_per_s / 1e9 / HBM_PEAK_GBS, 4),
        "dense_weight_bytes_per_step": dense_bytes,
        "algorithmic_bytes_per_step": round(alg_bytes_step),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
