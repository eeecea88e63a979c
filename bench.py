#!/usr/bin/env python3
"""Benchmark of the CLADA sparse-FFN decode path on one MI355X.

A "step" is one decode step of the whole hot path over the FFN stack of the
configuration: cognitive signals from the previous step's logits -> per-layer
token-aware thresholds -> L x thresholded sparse SwiGLU FFN (one call per layer),
with all inputs resident in HBM.  The once-per-sequence prefill (prefix statistics
on MFMA + base-threshold calibration) runs before the timed region and is reported
separately.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debug)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--option", action="append", default=[], help="library option name=value")
    ap.add_argument("--q", type=float, default=0.0, help="override the configuration's target sparsity")
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's decode batch")
    ap.add_argument("--shared-frac", type=float, default=0.0,
                    help="c in [0,1]: decode tokens of a batch share a component, x_b = sqrt(c) x_shared + sqrt(1-c) x_b'")
    ap.add_argument("--temperature", type=float, default=1.0, help="divide the Zipf logits by this (peaked < 1 < flat)")
    ap.add_argument("--tau-s", type=float, default=None, help="fix the surprisal threshold (default: median of the run's own stream)")
    ap.add_argument("--tau-h", type=float, default=None, help="fix the entropy threshold (default: median of the run's own stream)")
    ap.add_argument("--per-layer", action="store_true",
                    help="B = 1: time the step through L per-layer calls on one stream instead of the whole-stack call")
    ap.add_argument("--regimes", default="natural,off,on,neg,stack",
                    help="which measurements to run besides the natural regime and the dense twin (comma list of off, on, "
                         "neg, stack); a profiler run restricts them so that a kernel's average covers one regime")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run only a short fixed call sequence (for rocprofv3 --pmc counter runs) and exit")
    ap.add_argument("--prefill-probe", action="store_true",
                    help="run only the prefill of one layer, on the synthetic operands and on all-zero ones, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the path would shard along d_ff, not built)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2502_19078_amd as clada
    import synth
    from paper_2502_19078_amd import binding

    clada.load_library()           # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    if args.q or args.batch:
        import dataclasses
        cfg = dataclasses.replace(cfg, q=args.q or cfg.q, B=args.batch or cfg.B)
    if args.pmc_probe:
        return pmc_probe(cfg, args, clada, binding, synth, torch, dev)
    if args.prefill_probe:
        return prefill_probe(cfg, args, clada, synth, torch, dev)
    L = args.layers or cfg.L
    d, F, B, T, V = cfg.d, cfg.d_ff, cfg.B, cfg.T, cfg.V
    K, W = args.steps, args.warmup
    nsteps = K + W
    es = 2 if cfg.dtype == "bf16" else 4
    relu = cfg.name.startswith("opt")           # non-gated ReLU FFN family: two matrices + biases
    geglu = cfg.name.startswith("gemma")        # gated family with sigma = tanh-form GELU
    nmat = 2 if relu else 3                     # matrices a dense call reads
    tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    t_setup = time.time()

    def to_dev(a):
        if cfg.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    # ---------------------------------------------------------------- inputs (seeded, synthetic)
    n_host = 0 if args.no_cpu_baseline else min(4, L)   # layers whose host copy the oracle leg keeps
    host_w = {}

    def make_layer(l):
        if relu:
            w_in, b_in, w_out, b_out = synth.relu_layer(cfg, args.seed, l)
            if l < n_host:
                host_w[l] = (w_in, b_in, w_out, b_out)
            w, biases = (w_in, w_out), (b_in, b_out)
        else:
            w, biases = synth.layer_weights(cfg, args.seed, l), None
            if l < n_host:
                host_w[l] = w
        return l, [synth.bf16_bits(a).view(np.int16) if cfg.dtype == "bf16" else a for a in w], biases

    layers = [None] * L
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        for l, arrs, biases in ex.map(make_layer, range(L)):
            ts = [torch.from_numpy(a).to(dev) for a in arrs]
            if cfg.dtype == "bf16":
                ts = [t.view(torch.bfloat16) for t in ts]
            if relu:
                layers[l] = clada.Layer(ts[0], None, ts[1], kind=binding.RELU,
                                        b_in=torch.from_numpy(biases[0]).to(dev), b_out=torch.from_numpy(biases[1]).to(dev))
            else:
                layers[l] = clada.Layer(*ts, kind=binding.GEGLU if geglu else binding.SWIGLU)
    x_host = np.stack([np.stack([synth.decode_hidden(cfg, args.seed, l, s, shared_frac=args.shared_frac)
                                 for l in range(L)]) for s in range(nsteps)])
    x_all = to_dev(x_host.reshape(nsteps, L, B, d))                       # [step][layer][B][d]
    z_host = np.stack([synth.logits(cfg, args.seed, s, temperature=args.temperature)[0]
                       for s in range(nsteps)])                              # [step][B][V]
    tok_host = np.stack([synth.draw_tokens(cfg, args.seed, s, z_host[s]) for s in range(nsteps)])
    z_all = torch.from_numpy(z_host).to(dev)
    tok_all = torch.from_numpy(tok_host).to(dev)

    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, T, V))
    for opt in args.option:
        k, v = opt.split("=")
        ctx.set_option(k, int(v))

    # ---------------------------------------------------------------- prefill: stats + calibration
    tau_base = torch.empty(L, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t0 = time.time()
    for l in range(L):
        Xp = to_dev(synth.prefix_hidden(cfg, args.seed, l))
        st = clada.prefix_stats(ctx, layers[l], Xp, want_y=False, want_pool=True)
        clada.threshold_calibrate(ctx, st.abs_act_pool, cfg.q, out=tau_base[l:l + 1])
    torch.cuda.synchronize()
    prefill_wall_ms = (time.time() - t0) * 1e3
    # GPU-only prefill time of one layer (inputs resident)
    def prefill_ms(want_y, reps=3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for r in range(reps + 1):                       # first round untimed: torch's allocator warms up
            if r == 1:
                e0.record()
            st = clada.prefix_stats(ctx, layers[L - 1], Xp, want_y=want_y, want_pool=True)
            clada.threshold_calibrate(ctx, st.abs_act_pool, cfg.q, out=tau_base[L - 1:L])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps, st
    prefill_layer_ms, st = prefill_ms(True)             # gate/up + down GEMMs, aggregates, calibration
    prefill_stats_ms, _ = prefill_ms(False)             # what the decode path needs: no y, no down GEMM
    del _
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # the paper's own calibration (error-bounded search, bound 0.2) on the same prefix, for comparison
    cett_info = None
    if True:
        clada.threshold_search_cett(ctx, layers[L - 1], Xp, 0.2)
        e0.record()
        tau_cett, mean_cett = clada.threshold_search_cett(ctx, layers[L - 1], Xp, 0.2)
        e1.record()
        torch.cuda.synchronize()
        cett_ms = e0.elapsed_time(e1)
        cett_info = {"layer_ms_gpu": round(cett_ms, 3), "bound": 0.2, "tau_base": round(float(tau_cett.item()), 5),
                     "mean_cett": round(float(mean_cett.item()), 5),
                     "sparsity_on_prefix": round(float((st.abs_act_pool < tau_cett).float().mean().item()), 4),
                     "percentile_tau_base": round(float(tau_base[L - 1].item()), 5)}
    del st, Xp

    lam = torch.full((L,), 0.80, dtype=torch.float32, device=dev)     # printed coefficients
    gam = torch.full((L,), 0.12, dtype=torch.float32, device=dev)
    # universal signal thresholds (not given in the paper): medians of this run's own signal
    # streams, computed by the library over all steps before timing
    s_all, h_all = [], []
    for s in range(nsteps):
        a, b = clada.cognitive_signals(ctx, z_all[s], tok_all[s])
        s_all.append(a)
        h_all.append(b)
    tau_s = float(torch.stack(s_all).median().item()) if args.tau_s is None else args.tau_s
    tau_H = float(torch.stack(h_all).median().item()) if args.tau_h is None else args.tau_h
    mean_s, mean_H = float(torch.stack(s_all).mean().item()), float(torch.stack(h_all).mean().item())

    # ---------------------------------------------------------------- one decode step
    x_cur = torch.empty(L, B, d, dtype=tdtype, device=dev)
    z_cur = torch.empty(B, V, dtype=torch.float32, device=dev)
    tok_cur = torch.empty(B, dtype=torch.int32, device=dev)
    sur = torch.empty(B, dtype=torch.float32, device=dev)
    ent = torch.empty(B, dtype=torch.float32, device=dev)
    tau_final = torch.empty(L, B, dtype=torch.float32, device=dev)
    y_out = torch.empty(L, B, d, dtype=tdtype, device=dev)
    lib, h = ctx._lib, ctx._h
    import ctypes as C
    cl = [l.c_struct() for l in layers]

    def stream_ptr():
        return C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)

    INF = float("inf")
    lam_neg, gam_neg = -lam, -gam                     # the regression table's signs (reading R5)

    def signals_and_thresholds(ts, th, lam_t, gam_t, sp):
        # one launch: surprisal, entropy and the L thresholds of this step's token(s)
        ctx.check(lib.clada_signals_threshold(h, z_cur.data_ptr(), binding.F32, B, V, tok_cur.data_ptr(),
                                              tau_base.data_ptr(), lam_t.data_ptr(), gam_t.data_ptr(), L, ts, th,
                                              sur.data_ptr(), ent.data_ptr(), tau_final.data_ptr(), sp))

    # B = 1: the FFN stack of a step goes through the whole-stack call (the layers of the workload are
    # independent problems; by default the library sends the layers round two or three streams); the per-layer
    # calls are measured beside it.  B >= 2: per-layer calls.
    use_stack = not args.per_layer
    arr = binding.layer_array(layers)
    x_flat, y_flat, tau_flat = x_cur.view(L * B, d), y_out.view(L * B, d), tau_final.view(L * B)

    def step_body(dense, ts, th, lam_t, gam_t, counts=None, per_layer=False):
        sp = stream_ptr()
        signals_and_thresholds(ts, th, lam_t, gam_t, sp)
        if use_stack and not per_layer and counts is None:
            if dense:
                ctx.check(lib.clada_dense_ffn_stack_decode(h, arr, L, x_flat.data_ptr(), B, y_flat.data_ptr(), sp))
            else:
                ctx.check(lib.clada_sparse_ffn_stack_decode(h, arr, L, x_flat.data_ptr(), B, tau_flat.data_ptr(),
                                                            y_flat.data_ptr(), None, sp))
            return
        for l in range(L):
            if dense:
                ctx.check(lib.clada_dense_ffn_decode(h, C.byref(cl[l]), x_cur[l].data_ptr(), B,
                                                     y_out[l].data_ptr(), sp))
            else:
                ctx.check(lib.clada_sparse_ffn_decode(h, C.byref(cl[l]), x_cur[l].data_ptr(), B,
                                                      tau_final[l].data_ptr(), y_out[l].data_ptr(), None,
                                                      counts[l].data_ptr() if counts is not None else None, None, sp))

    def load_inputs(s):
        x_cur.copy_(x_all[s], non_blocking=True)
        z_cur.copy_(z_all[s], non_blocking=True)
        tok_cur.copy_(tok_all[s], non_blocking=True)

    side = torch.cuda.Stream()

    def make_runner(dense, ts, th, lam_t, gam_t, per_layer=False):
        """One decode step as a replayable HIP graph (or an eager call sequence with --no-graph)."""
        if args.no_graph:
            return lambda: step_body(dense, ts, th, lam_t, gam_t, per_layer=per_layer)
        load_inputs(0)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            step_body(dense, ts, th, lam_t, gam_t, per_layer=per_layer)      # eager once: first calls set kernel attributes
            side.synchronize()
            clada.graph_begin(ctx)                      # the library's own capture (clada_graph_*)
            step_body(dense, ts, th, lam_t, gam_t, per_layer=per_layer)
            g = clada.graph_end(ctx)
        torch.cuda.synchronize()
        return g.launch                                 # replays on the current stream; the bound method keeps g alive

    def timed(run):
        for s in range(W):
            load_inputs(s)
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(W, W + K):
            load_inputs(s)
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / K

    REPLAYS = 50

    def replay_stats(run):
        """10 warm-ups, then REPLAYS replays of the step, each bracketed by HIP events on the launch stream (the
        inputs cycle through the run's steps and are refreshed outside the bracket): median and min in ms."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(REPLAYS)]
        for i in range(10 + REPLAYS):
            load_inputs(i % nsteps)
            if i >= 10:
                evs[i - 10][0].record()
            run()
            if i >= 10:
                evs[i - 10][1].record()
        torch.cuda.synchronize()
        t = np.array([a.elapsed_time(b) for a, b in evs])
        return float(np.median(t)), float(t.min())

    def check_outputs(what):
        """The timed steps must have produced valid output: a balanced call that gave up its bounded wait turns
        every later y of the context into NaN."""
        torch.cuda.synchronize()
        if ctx.device_fault() or not bool(torch.isfinite(y_out.float()).all()):
            print(f"bench.py: invalid output after {what} (device fault flag or non-finite y)", file=sys.stderr)
            sys.exit(3)

    def measure_regime(ts, th, lam_t=lam, gam_t=gam, detail=True, per_layer=False):
        """Step time (mean over K different-input replays by the host clock; median and min over REPLAYS replays
        by HIP events), measured sparsity and, with detail, per-call and per-kernel durations."""
        run = make_runner(False, ts, th, lam_t, gam_t, per_layer=per_layer)
        ms = timed(run)
        med, mn = replay_stats(run)
        check_outputs("the timed sparse steps")
        cnt = torch.empty(K, L, 1 + B, dtype=torch.int32, device=dev)
        for i, s in enumerate(range(W, W + K)):                     # untimed pass: kept counts
            load_inputs(s)
            step_body(False, ts, th, lam_t, gam_t, counts=cnt[i])
        torch.cuda.synchronize()
        cnt_np = cnt.cpu().numpy()
        n_union = cnt_np[:, :, 0].astype(np.float64).mean()
        res = {"ms": ms, "ms_median": med, "ms_min": mn, "rho_union": 1.0 - n_union / F,
               "rho_token": 1.0 - cnt_np[:, :, 1:].mean() / F,
               "bytes_layer": (F + (nmat - 1.0) * n_union) * d * es}
        if not detail:
            return res
        nprobe = min(K, 8)                                           # events around every per-layer call
        evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
               for _ in range(nprobe)]
        for i in range(nprobe):
            load_inputs(W + i)
            sp = stream_ptr()
            signals_and_thresholds(ts, th, lam_t, gam_t, sp)
            for l in range(L):
                evs[i][l][0].record()
                ctx.check(lib.clada_sparse_ffn_decode(h, C.byref(cl[l]), x_cur[l].data_ptr(), B,
                                                      tau_final[l].data_ptr(), y_out[l].data_ptr(),
                                                      None, None, None, sp))
                evs[i][l][1].record()
        torch.cuda.synchronize()
        res["call_us"] = float(np.mean([[a.elapsed_time(b) for a, b in row] for row in evs])) * 1e3
        # the dominant kernel alone: HIP events recorded by the library on the launch stream, directly
        # before and after the main decode kernel of every call
        ctx.set_option("diag.kernel_events", 1)
        main_us, fin_us = [], []
        for i in range(nprobe):
            load_inputs(W + i)
            sp = stream_ptr()
            signals_and_thresholds(ts, th, lam_t, gam_t, sp)
            for l in range(L):
                ctx.check(lib.clada_sparse_ffn_decode(h, C.byref(cl[l]), x_cur[l].data_ptr(), B,
                                                      tau_final[l].data_ptr(), y_out[l].data_ptr(),
                                                      None, None, None, sp))
                a, b = binding.diag_kernel_times(ctx)
                main_us.append(a)
                fin_us.append(b)
        ctx.set_option("diag.kernel_events", 0)
        res["main_us"], res["finalize_us"] = float(np.mean(main_us)), float(np.mean(fin_us))
        # algorithmic bytes of exactly the probed calls (the first nprobe timed steps)
        res["bytes_probe"] = (F + (nmat - 1.0) * cnt_np[:nprobe, :, 0].astype(np.float64).mean()) * d * es
        return res

    want = set(args.regimes.split(","))
    nat = measure_regime(tau_s, tau_H)            # the method as defined: thresholds follow the signals
    off = measure_regime(INF, INF) if "off" in want else None          # indicators off: tau_final = tau_base (target sparsity)
    on = measure_regime(-INF, -INF, detail=False) if "on" in want else None                       # both indicators always on: factor 1.92
    neg = measure_regime(tau_s, tau_H, lam_neg, gam_neg, detail=False) if "neg" in want else None  # natural, coefficients -0.80 / -0.12
    # ---- B = 1: the same step through the per-layer calls (what a model whose layers depend on each other
    # would issue), and through the other modes of the whole-stack call, for the record
    per_layer, stack = None, None
    if use_stack and "stack" in want and off is not None:
        b1_opt = int(dict(o.split("=") for o in args.option).get("decode.b1", 1))
        pl_nat = measure_regime(tau_s, tau_H, detail=False, per_layer=True)
        pl_off = measure_regime(INF, INF, detail=False, per_layer=True)
        ms_pl_dense = timed(make_runner(True, tau_s, tau_H, lam, gam, per_layer=True))
        check_outputs("the dense per-layer steps")
        per_layer = {"what": "the same step as signals+thresholds and L calls of clada_sparse_ffn_decode on one stream",
                     "natural": _light(pl_nat, ms_pl_dense, lambda rho: nmat / (nmat - (nmat - 1.0) * rho), B, L),
                     "indicators_off": _light(pl_off, ms_pl_dense, lambda rho: nmat / (nmat - (nmat - 1.0) * rho), B, L),
                     "dense_ms_per_step": round(ms_pl_dense, 4)}
        stack = {}
        for mode, mode_name in ((3, "lanes"), (2, "chained_launches"), (1, "persistent_kernel")) if B == 1 else ((3, "lanes"),):
            ctx.set_option("decode.stack", mode)
            m = {}
            for name, (ts, th), reg in (("natural", (tau_s, tau_H), nat), ("indicators_off", (INF, INF), off)):
                load_inputs(W)
                if mode == 3:
                    ctx.set_option("decode.b1", 2)          # the lanes run the unbalanced instances: those are their bits
                step_body(False, ts, th, lam, gam, per_layer=True)       # per-layer calls on the same inputs: the reference bits
                torch.cuda.synchronize()
                ctx.set_option("decode.b1", b1_opt)
                y_want = y_out.clone()
                run = make_runner(False, ts, th, lam, gam)
                load_inputs(W)
                run()
                torch.cuda.synchronize()
                same = bool(torch.equal(y_out, y_want))
                if mode == 3:                               # timed above: the headline numbers
                    m[name] = {"ms_per_step": round(reg["ms"], 4), "bit_identical_to_per_layer_calls": same}
                    continue
                ms = timed(run)
                med, mn = replay_stats(run)
                check_outputs("the whole-stack steps")
                m[name] = {"ms_per_step": round(ms, 4), "ms_median": round(med, 4), "ms_min": round(mn, 4),
                           "tokens_per_s": round(1e3 / ms, 2), "sparsity_union": round(float(reg["rho_union"]), 4),
                           "step_frac_of_hbm_peak": round(reg["bytes_layer"] * L / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                           "bit_identical_to_per_layer_calls": same}
            if mode != 3:
                ms_dense_stack = timed(make_runner(True, tau_s, tau_H, lam, gam))
                check_outputs("the dense whole-stack steps")
                m["dense_ms_per_step"] = round(ms_dense_stack, 4)
            stack[mode_name] = m
        ctx.set_option("decode.stack", 3)
        stack["what"] = ("modes of clada_sparse_ffn_stack_decode (option decode.stack).  lanes (default; value and "
                         "ms_per_step of this line): the layers go round two or three streams, so that the compute units "
                         "one layer has released run the next already.  chained_launches: one stream, the kernel of "
                         "layer l also sums the partial outputs of layer l-1.  persistent_kernel: one launch walks "
                         "the L layers; slower for sparse stacks, kept for the record")
    run_dense = make_runner(True, tau_s, tau_H, lam, gam)
    ms_dense = timed(run_dense)
    dense_med, dense_min = replay_stats(run_dense)
    check_outputs("the dense-twin steps")
    ms_sparse, rho_union, rho_token = nat["ms"], nat["rho_union"], nat["rho_token"]
    bytes_layer, call_us = nat["bytes_layer"], nat["call_us"]
    bytes_probe, main_us = nat["bytes_probe"], nat["main_us"]
    bytes_dense = float(nmat) * F * d * es
    ideal = lambda rho: nmat / (nmat - (nmat - 1.0) * rho)      # dense bytes / sparse bytes
    step_us_per_layer = ms_sparse * 1e3 / L

    # stream-read ceiling on the same weights
    def ceiling():
        for l in range(min(L, 8)):
            binding.diag_stream_read(ctx, layers[l].w_gate, 1)
    ceiling()
    torch.cuda.synchronize()
    e0.record()
    ceiling()
    e1.record()
    torch.cuda.synchronize()
    ceil_gbs = min(L, 8) * F * d * es / (e0.elapsed_time(e1) * 1e-3) / 1e9

    nch = d * es // 1024
    occ2 = es == 2 and d * es % 1024 == 0 and (nch == 5 if relu else nch in (4, 8)) and (F + 255) // 256 <= 64
    n_lanes = 1 if (not use_stack or L < 4) else 3 if (B >= 2 or occ2) else 2      # what the library chooses for sparse stacks
    main_kernel = ("k_ffn_decode_b1 (input rows dense + output rows of kept neurons)" if B == 1 and relu
                   else "k_ffn_decode_b1 (gate rows dense + up/down rows of kept neurons)" if B == 1
                   else "k_bat_gateup + k_bat_down (batched decode, timed as one)")
    achieved = bytes_probe / (main_us * 1e-6) / 1e9          # dominant kernel alone
    achieved_call = bytes_probe / (call_us * 1e-6) / 1e9     # whole call: main kernel + final reduction + launch gap
    out = {
        "metric": "sparse-FFN decode tokens/s (7B shape, bs=1), HBM GB/s on bytes touched, speedup vs dense",
        "value": round(B * 1e3 / ms_sparse, 2),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_sparse, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{args.config}: {cfg.name} FFN stack, L={L}, d={d}, d_ff={F}, {cfg.dtype}, "
                               f"decode batch {B}, prefix {T}, V={V}, target sparsity {cfg.q}",
                   "weights": f"N(0, std {cfg.w_std:g})", "hidden": "N(0,1)",
                   "lambda": 0.80, "gamma": 0.12, "tau_s": round(tau_s, 4), "tau_H": round(tau_H, 4),
                   "shared_frac": args.shared_frac, "temperature": args.temperature,
                   "mean_surprisal": round(mean_s, 4), "mean_entropy": round(mean_H, 4),
                   "graph": not args.no_graph, "options": args.option},
        "sparsity_per_token": round(float(rho_token), 4),
        "sparsity_union": round(float(rho_union), 4),
        "dense_ms_per_step": round(ms_dense, 4),
        "speedup_vs_dense": round(ms_dense / ms_sparse, 4),
        "ideal_speedup": round(ideal(rho_union), 4),
        "regime": "natural: tau_s, tau_H = medians of the run's own surprisal/entropy streams",
        # ms_per_step is the host-clock mean over K steps on K different inputs; these are HIP-event times of
        # single graph replays (inputs refreshed outside the bracket)
        "replays": {"n": REPLAYS, "ms_median": round(nat["ms_median"], 4), "ms_min": round(nat["ms_min"], 4),
                    "dense_ms_median": round(dense_med, 4), "dense_ms_min": round(dense_min, 4)},
        "value_at_target_sparsity": round(B * 1e3 / off["ms"], 2) if off else None,   # indicators off: rho = the configuration's target
        "device_fault": False,
        "regime_indicators_off": None if off is None else {
            "ms_per_step": round(off["ms"], 4), "tokens_per_s": round(B * 1e3 / off["ms"], 2),
            "ms_median": round(off["ms_median"], 4), "ms_min": round(off["ms_min"], 4),
            "step_frac_of_hbm_peak": round(off["bytes_layer"] * L / (off["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "sparsity_union": round(float(off["rho_union"]), 4),
            "speedup_vs_dense": round(ms_dense / off["ms"], 4),
            "ideal_speedup": round(ideal(off["rho_union"]), 4),
            "bytes_per_launch": round(off["bytes_probe"]),
            "kernel_us": round(off["main_us"], 2), "finalize_us": round(off["finalize_us"], 2),
            "call_us": round(off["call_us"], 2),
            "kernel_gbs": round(off["bytes_probe"] / (off["main_us"] * 1e-6) / 1e9, 1),
            "kernel_frac": round(off["bytes_probe"] / (off["main_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "call_gbs": round(off["bytes_probe"] / (off["call_us"] * 1e-6) / 1e9, 1),
            "call_frac": round(off["bytes_probe"] / (off["call_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
        "regime_indicators_on": _light(on, ms_dense, ideal, B, L) if on else None,
        "regime_negative_coefficients": dict(_light(neg, ms_dense, ideal, B, L), **{"lambda": -0.80, "gamma": -0.12}) if neg else None,
        "step_path": (f"clada_signals_threshold, then clada_sparse_ffn_stack_decode (lanes on two or three streams) on the "
                      "L independent layers" if use_stack else "clada_signals_threshold, then L calls of clada_sparse_ffn_decode"),
        "per_layer_calls": per_layer,
        "stack_modes": stack,
        "step_gbs_on_bytes_touched": round(bytes_layer * L / (ms_sparse * 1e-3) / 1e9, 1),
        "dense_step_gbs": round(bytes_dense * L / (ms_dense * 1e-3) / 1e9, 1),
        "stream_read_ceiling_gbs": round(ceil_gbs, 1),   # whole-row streaming of one 90 MB matrix per launch, launch gaps included
        "prefill": {"layer_ms_gpu": round(prefill_layer_ms, 3), "stack_wall_ms_incl_h2d": round(prefill_wall_ms, 1),
                    "tflops_layer": round(2.0 * nmat * T * d * F / (prefill_layer_ms * 1e-3) / 1e12, 1),
                    "layer_ms_gpu_without_y": round(prefill_stats_ms, 3),
                    "tflops_layer_without_y": round(2.0 * (nmat - 1) * T * d * F / (prefill_stats_ms * 1e-3) / 1e12, 1),
                    "cett_search": cett_info},
        "roofline": {"bound": "hbm", "kernel": main_kernel,
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": round(bytes_probe), "us_per_launch": round(main_us, 2),
                     **_traffic(args.config, B, bytes_probe),
                     # the whole C-ABI call = that kernel + the fixed-order final reduction (k_ffn_finalize)
                     # + the launch gap between them, timed with HIP events around the call
                     "call": {"us": round(call_us, 2), "finalize_us": round(nat["finalize_us"], 2),
                              "achieved": round(achieved_call, 1), "frac": round(achieved_call / HBM_PEAK_GBS, 4)},
                     "us_per_layer_in_step": round(step_us_per_layer, 2),
                     "note": ("achieved/frac: the kernel of a per-layer call with the chip to itself, timed by kernel-own HIP "
                              "events on the timed steps' inputs (rocprofv3 row of the balanced instance at B = 1).  The "
                              "launches of the timed step run in lanes and overlap, so the duration of a single one of them "
                              "(rocprofv3 rows of the lane instance) is not the time it costs: in_step divides the same bytes "
                              "by the interval at which launches complete, step time / L"),
                     # the timed step itself: in lanes several launches share the chip at any time, so the
                     # duration of one launch says little; what counts is the rate at which launches complete
                     # (step time / L, the signals launch included)
                     "in_step": {"lanes": n_lanes,
                                 "us_per_launch_completed": round(step_us_per_layer, 2),
                                 "achieved": round(bytes_layer / (step_us_per_layer * 1e-6) / 1e9, 1),
                                 "frac": round(bytes_layer / (step_us_per_layer * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}},
        "setup_s": round(time.time() - t_setup, 1),
    }

    # ---------------------------------------------------------------- CPU baseline: the oracle itself
    if not args.no_cpu_baseline:
        import oracle
        budget, t_used, n_done = 12.0, 0.0, 0
        tf = tau_final.cpu().numpy().astype(np.float64)       # thresholds of the last step run
        for s in range(W, W + K):
            for l in range(n_host):
                t0 = time.perf_counter()
                if relu:
                    oracle.relu_decode(*host_w[l], x_host[s, l], tau=tf[l])
                else:
                    oracle.sparse_decode(*host_w[l], x_host[s, l], tf[l], sigma="gelu_tanh" if geglu else "silu")
                t_used += time.perf_counter() - t0
                n_done += 1
            if t_used > budget:
                break
        per_layer = t_used / n_done
        out["cpu_baseline"] = {"value": round(B / (per_layer * L), 3), "unit": "tokens/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"{n_done} layer-steps (layers 0..{n_host - 1}) of the same workload, "
                                         f"{per_layer * 1e3:.1f} ms each, extrapolated linearly to L={L}"}
    print(json.dumps(out))


def pmc_probe(cfg, args, clada, binding, synth, torch, dev):
    """Short fixed workload for hardware-counter runs: 4 seeded layers of the configuration, 3 rounds of
    sparse calls at three sparsities (0.45, 0.62 and 0.66), 4 dense-twin calls, 3 copies of a 256 MiB buffer
    (the known-size transfer the FETCH_SIZE / WRITE_SIZE counters are scaled by).  Batch 1 unless --batch
    is given (then --shared-frac applies to the tokens of the batch)."""
    d, F = cfg.d, cfg.d_ff
    B = args.batch or 1
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, cfg.T, 0))
    for opt in args.option:
        k, v = opt.split("=")
        ctx.set_option(k, int(v))

    def to_dev(a):
        if cfg.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    layers = [clada.Layer(*[to_dev(a) for a in synth.layer_weights(cfg, args.seed, l)]) for l in range(4)]
    x = to_dev(synth.decode_hidden(cfg, args.seed, 0, 0, B=B, shared_frac=args.shared_frac))
    # thresholds at the two sparsities from the library's own prefill statistics of layer 0
    st = clada.prefix_stats(ctx, layers[0], to_dev(synth.prefix_hidden(cfg, args.seed, 0)), want_y=False)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for q in (0.45, 0.62, 0.66):
        tau = clada.threshold_calibrate(ctx, st.abs_act_pool, q).expand(B).contiguous()
        kept = []
        for _ in range(3):
            for layer in layers:
                _, _, cnt, _ = clada.sparse_ffn_decode(ctx, layer, x, tau, want_lists=True)
                kept.append(int(cnt[0]))
        print(f"pmc-probe q={q}: kept per call {kept}")
    for layer in layers:
        clada.dense_ffn_decode(ctx, layer, x)
    for _ in range(3):
        binding.diag_copy(ctx, src, dst)
    torch.cuda.synchronize()
    print(f"pmc-probe copy bytes {src.numel()}")


def prefill_probe(cfg, args, clada, synth, torch, dev):
    """Prefill of one layer of the configuration (gate/up and down GEMMs, aggregates, no calibration), three
    timed repetitions on the seeded synthetic operands and three on all-zero operands of the same shape.
    The zero run does the same instructions on operands that toggle no bits: the difference is what the
    power limit costs the matrix-core kernels.  Prints one JSON line."""
    d, F, T = cfg.d, cfg.d_ff, cfg.T
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    for opt in args.option:
        k, v = opt.split("=")
        ctx.set_option(k, int(v))

    def to_dev(a):
        if cfg.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    w = [to_dev(a) for a in synth.layer_weights(cfg, args.seed, 0)]
    X = to_dev(synth.prefix_hidden(cfg, args.seed, 0))
    out = {"workload": f"{args.config}: prefill of one layer, T={T}, d={d}, d_ff={F}, {cfg.dtype}", "reps": 3}
    for name, ws, x in (("synthetic", w, X), ("zeros", [torch.zeros_like(a) for a in w], torch.zeros_like(X))):
        layer = clada.Layer(*ws)
        for want_y in (False, True):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for r in range(4):
                if r == 1:
                    e0.record()
                clada.prefix_stats(ctx, layer, x, want_y=want_y, want_pool=True)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 3
            flop = (6.0 if want_y else 4.0) * T * d * F
            out[f"{name}_{'with_y' if want_y else 'without_y'}"] = {"ms": round(ms, 3), "tflops": round(flop / ms / 1e9, 1)}
    print(json.dumps(out))


def _light(r, ms_dense, ideal, B, L):
    """JSON entry of a regime measured without the per-call probes."""
    return {"ms_per_step": round(r["ms"], 4), "ms_median": round(r["ms_median"], 4), "ms_min": round(r["ms_min"], 4),
            "tokens_per_s": round(B * 1e3 / r["ms"], 2), "sparsity_union": round(float(r["rho_union"]), 4),
            "speedup_vs_dense": round(ms_dense / r["ms"], 4), "ideal_speedup": round(ideal(r["rho_union"]), 4),
            "step_frac_of_hbm_peak": round(r["bytes_layer"] * L / (r["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def _traffic(config, B, bytes_per_launch):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary: the entry
    whose algorithmic bytes are within 3 % of this run's (counters cannot be read inside the run), else null."""
    p = os.path.join(ROOT, "profiles", f"traffic_sparse_ffn_decode_{config}.json")
    try:
        with open(p) as f:
            entries = json.load(f)["entries"]
    except Exception:
        return {"traffic": None, "traffic_note": "no committed counter summary for this workload"}
    entries = [e for e in entries if e.get("B", 1) == B]
    if entries:
        e = min(entries, key=lambda e: abs(e["algorithmic_bytes_per_launch"] - bytes_per_launch))
        if abs(e["algorithmic_bytes_per_launch"] - bytes_per_launch) <= 0.03 * bytes_per_launch:
            return {"traffic": e["hbm_bytes_per_launch"],
                    "traffic_source": f"profiles/{os.path.basename(p)}: rocprofv3 FETCH_SIZE + WRITE_SIZE of a committed "
                                      f"run at sparsity {e['rho']:.3f} ({e['algorithmic_bytes_per_launch']} algorithmic bytes)"}
    return {"traffic": None, "traffic_note": "the committed counter runs are at other sparsities than this run"}


if __name__ == "__main__":
    main()
