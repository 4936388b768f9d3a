"""Measurements of the gated subspace layer stack beyond the headline bench line (bench.py covers the GPT-J
block at batch-1 decode):

  --config 2   32 OPT-6.7B-shaped layers, batch-1 decode, rank k x designed fire rate sweep: tokens/s,
               effective weight-read GB/s, speedup over the dense 32-layer GEMV stack, beside the
               prediction of the paper's Eq. (speedup) and the all-bytes model; here with one
               gsi_layer_stack call per LAYER and token (explicit residual, three launches per call);
               bench.py --cells runs the same sweep with one planned call per token over all layers
  --config 3   fc_in / fc_out at k = 256 with ragged decode batches B in {1, 4, 16, 64}, per-token
               Bernoulli(0.15) gate: time per step by B, compaction checked against the design
  --config 4   prefill-sized batch (T = 2048, k = 512, 20 % of the tokens fired) over the six maps of a
               block, and the six one-time image builds: time, TFLOP/s on the matrix cores, speedup over
               the dense product with the same kernels
  --config 5   online basis maintenance: gsi_extend_basis on the inputs of a block (a basis array with spare
               columns, its maps' images and E kept up to date): time per call for tokens that extend the
               basis and for tokens that do not

One JSON object per run on stdout, progress on stderr.  Inputs are seeded and synthetic (workload_device.py);
they stand in for the paper's models and its 512-token text.  Every step of the path runs in libgsi; torch
is device memory, streams and the random number source.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import sys
import time

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def copy_tables(gsi, st):
    mp = (gsi.MapDesc * len(st.maps_t))()
    inp = (gsi.InputDesc * len(st.inputs_t))()
    ctypes.memmove(mp, st._mp, ctypes.sizeof(mp))
    ctypes.memmove(inp, st._in, ctypes.sizeof(inp))
    return mp, inp


def time_steps(torch, step_fn, n_steps: int, warmup: int, mode: str, chunk: int = 64) -> float:
    """Seconds for exactly n_steps calls of step_fn(t, stream) after `warmup` untimed ones.  graph: the
    steps are captured in chunks into HIP graphs (one trace = all chunks in order) and replayed."""
    if mode == "graph":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for t in range(min(n_steps, 2)):
                step_fn(t, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for c0 in range(0, n_steps, chunk):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream().cuda_stream
                for t in range(c0, min(n_steps, c0 + chunk)):
                    step_fn(t, cs)
            graphs.append(g)
        done = 0
        while done < warmup:
            for g in graphs:
                g.replay()
            done += n_steps
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    s0 = torch.cuda.current_stream().cuda_stream
    for t in range(warmup):
        step_fn(t % n_steps, s0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(n_steps):
        step_fn(t, s0)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


BLOCK = [("attn_in", 4096, [("q", 4096), ("k", 4096), ("v", 4096)]),
         ("attn_out", 4096, [("o", 4096)]),
         ("mlp_in", 4096, [("fc_in", 16384)]),
         ("mlp_hidden", 16384, [("fc_out", 4096)])]


# ------------------------------------------------------------------------------------------------------
# config 2: 32-layer stack, k x fire sweep
# ------------------------------------------------------------------------------------------------------
def run_opt_stack(args, torch, gsi, wd):
    L, T, eps, p = args.layers, args.steps, 0.05, 1.2
    ks = [int(x) for x in args.ks.split(",")]
    fires = [float(x) for x in args.fires.split(",")]
    kmax = max(ks)
    seed = wd.BASE_SEED + 2000
    t0 = time.perf_counter()
    W, U64 = [], []
    for l in range(L):
        gen = wd.generator(seed + 7919 * l)
        Wl, Ul = [], []
        for gi, (_, d, maps) in enumerate(BLOCK):
            Ul.append(wd.make_basis64(d, kmax, gen))
            Wl.append([wd.make_weight(m, d, gen) for _, m in maps])
        W.append(Wl)
        U64.append(Ul)
    torch.cuda.synchronize()
    dense_bytes_layer = sum(m * d * 2 for _, d, maps in BLOCK for _, m in maps)
    log(f"[report] {L} layers generated in {time.perf_counter()-t0:.1f}s: {L*dense_bytes_layer/1e9:.2f} GB of W")

    lib = gsi.lib
    ceps = ctypes.c_float(eps)
    cells = []
    dense_us = None
    for k in ks:
        # stored bases, images (one-time build, timed), stacks and per-token descriptor tables for this rank
        tb = time.perf_counter()
        stacks, Xs = [], []
        for l in range(L):
            inputs, maps = [], []
            for gi, (_, d, mp) in enumerate(BLOCK):
                U = U64[l][gi][:, :k].to(torch.bfloat16).contiguous()
                X = torch.zeros((T, d), device="cuda", dtype=torch.float32)
                inputs.append({"U": U, "X": X})
                for j, _ in enumerate(mp):
                    maps.append({"W": W[l][gi][j], "M": None, "input_id": gi})
            Xs.append([i["X"] for i in inputs])
            stacks.append((inputs, maps))
        torch.cuda.synchronize()
        tb0 = time.perf_counter()
        for inputs, maps in stacks:
            for mp in maps:
                mp["M"] = gsi.build_image(mp["W"], inputs[mp["input_id"]]["U"])
        torch.cuda.synchronize()
        build_s = time.perf_counter() - tb0
        sts = [gsi.LayerStack(inputs, maps, T, eps) for inputs, maps in stacks]
        tabs = []
        for t in range(T):
            row = []
            for st in sts:
                st.refresh(token_offset=t, B=1)
                row.append(copy_tables(gsi, st) + (st.ws.data_ptr(), st.ws.numel()))
            tabs.append(row)
        n_mp, n_in = len(sts[0].maps_t), len(sts[0].inputs_t)
        log(f"[report] k={k}: images built in {build_s*1e3:.1f} ms ({L*6} maps), tables in "
            f"{time.perf_counter()-tb:.1f}s")

        def gated_step(t, s):
            for mp, inp, wsp, wsn in tabs[t]:
                rc = lib.gsi_layer_stack(mp, n_mp, inp, n_in, 1, ceps, wsp, wsn, s)
                if rc:
                    raise gsi.GsiError(rc, gsi.last_error())

        def dense_step(t, s):
            for mp, inp, wsp, wsn in tabs[t]:
                rc = lib.gsi_dense_stack(mp, n_mp, inp, n_in, 1, wsp, wsn, s)
                if rc:
                    raise gsi.GsiError(rc, gsi.last_error())

        for fire in fires:
            designed = []
            for l in range(L):
                gen = wd.generator(seed + 7919 * l + 13 * k + int(fire * 1000) + 1)
                dl = []
                for gi, (_, d, _) in enumerate(BLOCK):
                    f = wd.choose_fired(T, int(round(fire * T)), gen)
                    X, _ = wd.make_tokens(U64[l][gi][:, :k], f, eps, p, gen)
                    Xs[l][gi].copy_(X)
                    dl.append(f)
                designed.append(dl)
            torch.cuda.synchronize()
            sec = time_steps(torch, gated_step, T, args.warmup, args.mode)
            if dense_us is None:
                dense_us = time_steps(torch, dense_step, T, args.warmup, args.mode) / T * 1e6
                log(f"[report] dense 32-layer GEMV stack: {dense_us:.1f} us/step = "
                    f"{L*dense_bytes_layer/dense_us/1e3:.0f} GB/s")
            # one more pass, then compare the device masks with the design
            for t in range(T):
                gated_step(t, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            match = all(bool(torch.equal(sts[l].inputs_t[gi]["mask"].bool(), designed[l][gi]))
                        for l in range(L) for gi in range(len(BLOCK)))
            n_fired_total = sum(int(designed[l][gi].sum()) for l in range(L) for gi in range(len(BLOCK)))
            us = sec / T * 1e6
            # bytes: images + bases always; W of every fired (layer, input)'s maps
            img = sum(m * k * 2 for _, d, maps in BLOCK for _, m in maps)
            bas = sum(d * k * 2 for _, d, _ in BLOCK)
            wf = sum(float(designed[l][gi].sum()) / T * sum(m * d * 2 for _, m in maps)
                     for l in range(L) for gi, (_, d, maps) in enumerate(BLOCK))
            alg = L * (img + bas) + wf
            f_eff = wf / (L * dense_bytes_layer)
            # Eq. (speedup) with a volume-weighted d/k (weights only; the fired path costs W alone)
            fast_cost = img / dense_bytes_layer
            s_eq = 1.0 / ((1.0 - f_eff) * fast_cost + f_eff)
            s_bytes = L * dense_bytes_layer / alg
            cell = {"k": k, "designed_fire_rate": fire, "fired_gate_evaluations": n_fired_total,
                    "us_per_step": round(us, 2), "tokens_per_s": round(1e6 / us, 1),
                    "effective_weight_GBs": round(L * dense_bytes_layer / us / 1e3, 1),
                    "algorithmic_GBs": round(alg / us / 1e3, 1),
                    "algorithmic_frac_of_hbm_peak": round(alg / us / 1e3 / HBM_PEAK_GBS, 4),
                    "speedup_vs_dense_stack": round(dense_us / us, 3),
                    "eq_speedup_weights_only": round(s_eq, 2), "all_bytes_speedup_bound": round(s_bytes, 2),
                    "masks_match_design": match}
            log(f"[report] {cell}")
            cells.append(cell)
        del sts, stacks, tabs, Xs
        torch.cuda.empty_cache()
    return {"config": 2, "workload": f"{L} OPT-6.7B-shaped layers (q,k,v,o 4096x4096, fc1 16384x4096, fc2 4096x16384), "
            "bf16, batch-1 decode, one gsi_layer_stack call per layer and token",
            "steps": T, "launch_mode": args.mode, "eps": eps,
            "dense_weight_bytes_per_step": L * dense_bytes_layer,
            "dense_stack_us_per_step": round(dense_us, 2),
            "dense_stack_GBs": round(L * dense_bytes_layer / dense_us / 1e3, 1), "cells": cells}


# ------------------------------------------------------------------------------------------------------
# config 3: ragged decode batches over fc_in / fc_out
# ------------------------------------------------------------------------------------------------------
def run_ragged(args, torch, gsi, wd):
    k, eps, p, pf = 256, 0.05, 1.5, 0.15
    steps = args.steps
    seed = wd.BASE_SEED + 3000
    shapes = [("fc_in", 4096, 16384), ("fc_out", 16384, 4096)]
    gen = wd.generator(seed)
    ops = []
    for name, d, m in shapes:
        U64 = wd.make_basis64(d, k, gen)
        Wt = wd.make_weight(m, d, gen)
        U = U64.to(torch.bfloat16).contiguous()
        ops.append((name, d, m, U64, U, Wt, gsi.build_image(Wt, U)))
    lib = gsi.lib
    ceps = ctypes.c_float(eps)
    rows = []
    for B in [int(b) for b in args.batches.split(",")]:
        T = steps * B
        inputs, maps, designed = [], [], []
        for gi, (name, d, m, U64, U, Wt, M) in enumerate(ops):
            g2 = wd.generator(seed + 100 * (gi + 1) + B)
            f = wd.bernoulli_fired(T, pf, g2)
            X, _ = wd.make_tokens(U64, f, eps, p, g2)
            inputs.append({"U": U, "X": X})
            maps.append({"W": Wt, "M": M, "input_id": gi})
            designed.append(f)
        st = gsi.LayerStack(inputs, maps, T, eps)
        # --rotate N: N copies of every weight, basis and image, used in turn by consecutive steps, so that
        # nothing a step reads is left in the 256 MB Infinity Cache from the step before
        copies = [[(t["W"], t["M"]) for t in st.maps_t]]
        ucopies = [[t["U"] for t in st.inputs_t]]
        for _ in range(1, max(1, args.rotate)):
            copies.append([(t["W"].clone(), t["M"].clone()) for t in st.maps_t])
            ucopies.append([t["U"].clone() for t in st.inputs_t])
        tabs = []
        for s_ in range(steps):
            st.refresh(token_offset=s_ * B, B=B)
            mp, inp = copy_tables(gsi, st)
            for j, (Wc, Mc) in enumerate(copies[s_ % len(copies)]):
                mp[j].W, mp[j].M = Wc.data_ptr(), Mc.data_ptr()
            for i, Uc in enumerate(ucopies[s_ % len(ucopies)]):
                inp[i].U = Uc.data_ptr()
            tabs.append((mp, inp))
        wsp, wsn = st.ws.data_ptr(), st.ws.numel()

        def gated_step(t, s):
            mp, inp = tabs[t]
            rc = lib.gsi_layer_stack(mp, 2, inp, 2, B, ceps, wsp, wsn, s)
            if rc:
                raise gsi.GsiError(rc, gsi.last_error())

        def dense_step(t, s):
            mp, inp = tabs[t]
            rc = lib.gsi_dense_stack(mp, 2, inp, 2, B, wsp, wsn, s)
            if rc:
                raise gsi.GsiError(rc, gsi.last_error())

        sec = time_steps(torch, gated_step, steps, args.warmup, args.mode)
        sec_d = time_steps(torch, dense_step, steps, args.warmup, args.mode)
        # compaction check on every step: mask == design, list ascending, count right
        ok = True
        cs = torch.cuda.current_stream().cuda_stream
        w_reads = 0
        for t in range(steps):
            gated_step(t, cs)
            torch.cuda.synchronize()
            for gi in range(2):
                want = designed[gi][t * B:(t + 1) * B]
                n = int(st.inputs_t[gi]["n_fired"].item())
                idx = st.inputs_t[gi]["fired_idx"][:n]
                ok &= bool(torch.equal(st.inputs_t[gi]["mask"][t * B:(t + 1) * B].bool(), want))
                ok &= n == int(want.sum()) and bool(torch.equal(idx.long(), torch.nonzero(want).flatten()))
                w_reads += int(n > 0)
        dense_bytes = sum(m * d * 2 for _, d, m, *_ in ops)
        us, usd = sec / steps * 1e6, sec_d / steps * 1e6
        row = {"B": B, "steps": steps, "us_per_step": round(us, 2), "dense_us_per_step": round(usd, 2),
               "tokens_per_s": round(B * 1e6 / us, 1), "speedup_vs_dense": round(usd / us, 3),
               "effective_weight_GBs": round(dense_bytes / us / 1e3, 1),
               "weight_matrix_reads": w_reads, "of_possible": 2 * steps,
               "fired_tokens": int(sum(int(f.sum()) for f in designed)), "tokens": 2 * T,
               "compaction_matches_design": ok, "operand_copies": max(1, args.rotate)}
        log(f"[report] {row}")
        rows.append(row)
        del st, inputs, maps, tabs, copies, ucopies
        torch.cuda.empty_cache()
    return {"config": 3, "workload": "fc_in 16384x4096 and fc_out 4096x16384, bf16, k=256, eps=0.05, per-token "
            "Bernoulli(0.15) gate design, one gsi_layer_stack call per step", "launch_mode": args.mode, "rows": rows}


# ------------------------------------------------------------------------------------------------------
# config 4: prefill-sized batch + image builds
# ------------------------------------------------------------------------------------------------------
def run_prefill(args, torch, gsi, wd):
    T, k, eps, p, fire = args.tokens, 512, 0.05, 1.5, 0.20
    seed = wd.BASE_SEED + 4000
    gen = wd.generator(seed)
    inputs, maps, designed = [], [], []
    build_ms, build_flops = [], 0.0
    for gi, (_, d, mp) in enumerate(BLOCK):
        U64 = wd.make_basis64(d, k, gen)
        U = U64.to(torch.bfloat16).contiguous()
        f = wd.choose_fired(T, int(round(fire * T)), gen)
        X, _ = wd.make_tokens(U64, f, eps, p, gen)
        inputs.append({"U": U, "X": X.to(torch.bfloat16) if args.xdtype == "bf16" else X})
        designed.append(f)
        for name, m in mp:
            Wt = wd.make_weight(m, d, gen)
            M = gsi.build_image(Wt, U)  # warm
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                gsi.build_image(Wt, U, M)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            build_ms.append({"map": name, "m": m, "d": d, "k": k, "ms": round(ms, 4),
                             "TFLOPs": round(2.0 * m * d * k / ms / 1e9, 1)})
            build_flops += 2.0 * m * d * k
            maps.append({"W": Wt, "M": M, "input_id": gi})
    st = gsi.LayerStack(inputs, maps, T, eps)
    reps = args.steps

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    sec = timed(st.run)
    sec_d = timed(st.run_dense)
    st.run()
    torch.cuda.synchronize()
    match = all(bool(torch.equal(st.inputs_t[gi]["mask"].bool(), designed[gi])) for gi in range(len(BLOCK)))
    nf = [int(f.sum()) for f in designed]
    fl_proj = sum(4.0 * T * d * k for _, d, _ in BLOCK)
    fl_img = sum(2.0 * T * m * k for _, _, mp in BLOCK for _, m in mp)
    fl_w = sum(2.0 * nf[gi] * m * d for gi, (_, d, mp) in enumerate(BLOCK) for _, m in mp)
    fl_dense = sum(2.0 * T * m * d for _, d, mp in BLOCK for _, m in mp)
    total_build_ms = sum(b["ms"] for b in build_ms)
    return {"config": 4, "workload": f"T={T} tokens through the six maps of a GPT-J-shaped block, k={k}, eps={eps}, "
            f"{fire:.0%} of the tokens of every input fired, bf16 weights, x {args.xdtype}",
            "gated_ms": round(sec * 1e3, 4), "dense_ms": round(sec_d * 1e3, 4),
            "speedup_vs_dense_same_kernels": round(sec_d / sec, 3),
            "gated_useful_TFLOPs": round((fl_proj + fl_img + fl_w) / sec / 1e12, 1),
            "gated_useful_frac_of_mfma_peak": round((fl_proj + fl_img + fl_w) / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "dense_TFLOPs": round(fl_dense / sec_d / 1e12, 1),
            "flops": {"project": fl_proj, "image_term": fl_img, "weight_term_fired": fl_w, "dense": fl_dense},
            "masks_match_design": match, "fired_per_input": nf,
            "image_builds": build_ms, "image_build_total_ms": round(total_build_ms, 3),
            "image_build_TFLOPs": round(build_flops / total_build_ms / 1e9, 1)}



# ------------------------------------------------------------------------------------------------------
# config 5: online basis maintenance (one rank-1 extension per call)
# ------------------------------------------------------------------------------------------------------
def run_extend(args, torch, gsi, wd):
    """gsi_extend_basis at the shapes of a GPT-J block: a basis array of capacity 2k holding k columns, the maps that
    read it, E kept up to date; time per call for tokens that extend the basis and for tokens that do not."""
    dev = torch.device("cuda:0")
    gen = wd.generator(2605_03109 + 5000)
    steps = args.steps
    k0 = 256
    K = k0 + 2 * steps
    K += (-K) % 64
    rows = []
    for name, d, ms in (("q,k,v input", 4096, (4096, 4096, 4096)), ("fc_in input", 4096, (16384,)),
                        ("fc_out input", 16384, (4096,))):
        U64 = wd.make_basis64(d, k0, gen)
        U = torch.zeros((d, K), dtype=torch.bfloat16, device=dev)
        U[:, :k0] = U64.to(torch.bfloat16)
        U0 = U.clone()
        Ws = [wd.make_weight(m, d, gen) for m in ms]
        Ms = [gsi.build_image(W, U) for W in Ws]
        E = gsi.build_gram(U)
        R = torch.randn((steps, d), generator=gen, device=dev, dtype=torch.float32)
        R /= R.norm(dim=1, keepdim=True)
        rnorm = torch.full((1,), 0.3, device=dev)
        xnorm = torch.ones((1,), device=dev)
        k_cur = torch.full((1,), k0, dtype=torch.int32, device=dev)
        ext = torch.zeros((1,), dtype=torch.int32, device=dev)
        ws = torch.empty(int(gsi.lib.gsi_extend_basis_workspace_bytes(d, K)) + 256, dtype=torch.uint8, device=dev)
        pairs = list(zip(Ws, Ms))
        w_bytes = sum(m * d * 2 for m in ms)
        # what one extension must move: U for s = U^T r, for r2 = r - U s and for E's new row, W once per map
        alg_bytes = 3 * d * K * 2 + w_bytes
        res = {"input": name, "d": d, "capacity_K": K, "columns_at_start": k0, "maps_m": list(ms), "calls": steps,
               "algorithmic_MB_per_extension": round(alg_bytes / 1e6, 1)}
        for label, tau in (("extending", 0.2), ("not_extending", 0.5)):
            def call(t, stream):
                gsi.extend_basis(U, k_cur, R[t], rnorm, xnorm, tau, pairs, gram=E, extended=ext, ws=ws, stream=stream)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                call(0, side)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream()
                for t in range(steps):
                    call(t, cs)
            best = None
            for rep in range(3):
                U.copy_(U0)
                k_cur.fill_(k0)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                g.replay()
                torch.cuda.synchronize()
                sec = time.perf_counter() - t0
                best = sec if best is None else min(best, sec)
            grown = int(k_cur.item()) - k0
            us = best / steps * 1e6
            res[label] = {"us_per_call": round(us, 2), "columns_added": grown}
            if label == "extending":
                res[label]["achieved_GBs"] = round(alg_bytes / us / 1e3, 1)
                res[label]["frac_of_hbm_peak"] = round(alg_bytes / us / 1e3 / HBM_PEAK_GBS, 3)
            log(f"[report] {name} {label}: {res[label]}")
        rows.append(res)
        del U, U0, Ws, Ms, E, R, ws
        torch.cuda.empty_cache()
    # ---- every basis of a stack of blocks in one call per token (gsi_extend_many)
    L = 8
    bases, resets = [], []
    for layer in range(L):
        for name, d, ms in (("qkv", 4096, (4096, 4096, 4096)), ("o", 4096, (4096,)), ("fc_in", 4096, (16384,)),
                            ("fc_out", 16384, (4096,))):
            U = torch.zeros((d, K), dtype=torch.bfloat16, device=dev)
            U[:, :k0] = wd.make_basis64(d, k0, gen).to(torch.bfloat16)
            Ws = [wd.make_weight(m, d, gen) for m in ms]
            Ms = [gsi.build_image(W, U) for W in Ws]
            R = torch.randn((d,), generator=gen, device=dev, dtype=torch.float32)
            R /= R.norm()
            b = {"U": U, "k_cur": torch.full((1,), k0, dtype=torch.int32, device=dev), "R": R,
                 "rnorm": torch.full((1,), 0.3, device=dev), "xnorm": torch.ones((1,), device=dev),
                 "maps": list(zip(Ws, Ms)), "gram": gsi.build_gram(U)}
            bases.append(b)
            resets.append(U.clone())
    es = gsi.ExtendSet(bases)
    set_rows = {"blocks": L, "bases": len(bases), "maps": sum(len(b["maps"]) for b in bases), "calls": steps}

    def reset():
        for b, U0 in zip(bases, resets):
            b["U"].copy_(U0)
            b["k_cur"].fill_(k0)

    for label, tau, who in (("no_basis_extends", 0.5, None), ("one_basis_extends", 0.2, 1), ("every_basis_extends", 0.2, None)):
        # one_basis_extends: only the first basis sees a token above the threshold
        for i, b in enumerate(bases):
            b["rnorm"].fill_(0.3 if who is None or i < who else 0.01)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            es.step(tau, side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream()
            for t in range(steps):
                es.step(tau, cs)
        best = None
        for rep in range(3):
            reset()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.replay()
            torch.cuda.synchronize()
            sec = time.perf_counter() - t0
            best = sec if best is None else min(best, sec)
        grown = sum(int(b["k_cur"].item()) - k0 for b in bases)
        set_rows[label] = {"us_per_call": round(best / steps * 1e6, 2), "columns_added": grown}
        log(f"[report] {len(bases)} bases per call, {label}: {set_rows[label]}")
    return {"config": 5, "workload": "gsi_extend_basis on GPT-J-block shapes, bf16, basis array of capacity K holding 256 "
            "columns at the start, E kept; HIP-graph replay of `calls` consecutive calls, best of 3; then "
            "gsi_extend_many over the bases of eight blocks", "rows": rows, "many": set_rows}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, choices=[2, 3, 4, 5], required=True)
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--steps", type=int, default=None, help="decode steps (config 2: 512, config 3: 200) / repeats (config 4: 10) / calls (config 5: 64)")
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--ks", default="64,128,256,512")
    ap.add_argument("--fires", default="0,0.05,0.25,1.0")
    ap.add_argument("--batches", default="1,4,16,64")
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--rotate", type=int, default=1,
                    help="config 3: copies of every weight, basis and image used in turn by consecutive steps")
    ap.add_argument("--xdtype", choices=["f32", "bf16"], default="bf16")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = {2: 512, 3: 200, 4: 10, 5: 64}[args.config]

    import torch

    from paper_2605_03109_amd import gsi
    from paper_2605_03109_amd import workload_device as wd

    if not torch.cuda.is_available():
        print("report.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    fn = {2: run_opt_stack, 3: run_ragged, 4: run_prefill, 5: run_extend}[args.config]
    print(json.dumps(fn(args, torch, gsi, wd)), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
