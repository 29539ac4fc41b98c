#!/usr/bin/env python3
"""Benchmark of the partially-linear FFN decode path on one MI355X.

Workload (the 7B-class decode layer): d=4096, ffn=16384, bf16 weights
~N(0, 0.02^2) with heavy-tail columns, ranges calibrated on 4096 seeded tokens
for a ~5% fallback rate, batch 1.  One *step* = 1024 distinct tokens, each sent
through tardis_ffn_forward (folded product + predictor + result fixing) on one
stream.  Consecutive tokens rotate over `--layers` independently seeded copies
of the layer so that every weight byte comes from HBM rather than from the
last-level cache ("cold", the reported value); the same loop on a single copy
("hot") and the dense FFN are reported beside it.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

D, H = 4096, 16384
TOKENS_PER_STEP = 1024
HBM_PEAK_GBS = 8000.0
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(kernel: str, sketch_bits: int, hint: bool):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter runs recorded in
    profiles/traffic.json (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size), or None if
    no record matches - never a number typed into this file."""
    try:
        with open(TRAFFIC_JSON) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    for r in rec.get("records", []):
        if r.get("kernel") == kernel and r.get("sketch_bits") == sketch_bits and bool(r.get("next_layer_hint")) == hint:
            return r.get("hbm_bytes_per_launch")
    return None


def algorithmic_bytes(d: int, h: int, p: float, sketch_bits: int = 8, wp_bytes: float = 2.0) -> float:
    """Bytes the method itself must move per token at batch 1: folded matrix (bf16) + sketch (one
    byte per weight, or 4 bits per weight plus one multiplier byte per 32) + the W1 and W2 rows
    of the flagged neurons (bf16)."""
    sketch = 1.0 * d * h if sketch_bits == 8 else 0.5 * d * h + d * h / 32.0
    return wp_bytes * d * d + sketch + 4.0 * p * d * h


def _time_us(torch, fn, reps, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(reps):
        fn()
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def prefill_run(T, synth, torch, np, to_dev):
    """2048 (and 256) tokens x d=4096 through one layer - the prompt path: predictor sums,
    pre-activations, folded product and masked-delta down projection as four matrix-core products -
    against the dense FFN as two vendor-BLAS GEMMs; also the offline calibration and fold times."""
    n = 2048
    w = synth.decode(layer=0, n_cal=4096, n_test=n, coverage=0.95, config=3)
    ffn = T.FFN(to_dev(w.layer.W1), to_dev(w.layer.W2))
    Xc = to_dev(w.X_cal)
    lo, hi, a, c = T.tardis_calibrate(ffn, Xc, w.coverage)
    cal_us = _time_us(torch, lambda: T.tardis_calibrate(ffn, Xc, w.coverage), 3, 1)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=n)
    t0 = time.time()
    L2 = T.tardis_fold(ffn, lo, hi, a, c, max_batch=1)
    torch.cuda.synchronize()
    fold_ms = (time.time() - t0) * 1e3
    L2.close()
    X = to_dev(w.X_test)
    Y = torch.empty_like(X)
    us = _time_us(torch, lambda: T.tardis_ffn_forward_batched(L, X, Y), 5, 1)
    _, counts, _ = T.tardis_get_last_outliers(L, n, want_list=False)
    p = float(counts.float().mean().item()) / H
    X256, Y256 = X[:256].contiguous(), torch.empty_like(X[:256])
    us256 = _time_us(torch, lambda: T.tardis_ffn_forward_batched(L, X256, Y256), 5, 1)
    W1, W2 = ffn.W1, ffn.W2
    dus = _time_us(torch, lambda: torch.nn.functional.linear(
        torch.nn.functional.gelu(torch.nn.functional.linear(X, W1)), W2), 5, 1)
    dus_own = _time_us(torch, lambda: T.tardis_dense_forward(L, X, Y), 5, 1)
    L.close()
    gemm_flop = 2.0 * D * D * H          # one of the two accumulating fold GEMMs, or the calibration GEMM
    work = 2.0 * n * D * D + 3 * 2.0 * n * D * H      # folded + int8 predictor + pre-activations + down projection
    return {"tokens": n, "fallback_rate": p, "us": us, "tokens_per_s": n / (us * 1e-6),
            "matrix_core_Tops": work / us / 1e6, "us_256_tokens": us256,
            "dense_torch_us": dus, "dense_torch_TFLOPs": (2.0 * 2 * n * D * H) / dus / 1e6,
            "speedup_vs_dense_torch": dus / us,
            "dense_own_us": dus_own, "dense_own_TFLOPs": (2.0 * 2 * n * D * H) / dus_own / 1e6,
            "calibrate_us": cal_us, "fold_ms_incl_alloc": fold_ms,
            "note": "fold = 2 bf16 MFMA GEMMs of %.0f GFLOP each (head + remainder of diag(a)W1); "
                    "calibrate = 1 such GEMM + per-neuron sort/fit" % (gemm_flop / 1e9)}


def sketch_study(T, torch, ffn, cal, X64):
    """Predictor width study on the decode layer (the paper's Sec. "Predictor Size" sweep, here for
    round-to-nearest codes): per code width and margin the flags of 64 tokens against the exact
    pre-activations (harness-side torch product, fp32) - flag rate, precision, recall - and the bytes
    a token would stream with codes packed at that width (3- and 2-bit codes sit in 4-bit slots in
    this build, so their measured bytes are the 4-bit sketch's)."""
    lo, hi, a, c = cal
    z = X64.float() @ ffn.W1.float().t()
    truth = ~((z >= lo[None, :]) & (z < hi[None, :]))
    rows = []
    for bits in (8, 4, 3, 2):
        for margin in (0.0, 0.1):
            L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=64, sketch_bits=bits, margin=margin)
            T.tardis_ffn_forward_batched(L, X64)
            mask, _, _ = T.tardis_get_last_outliers(L, 64, want_list=False)
            sh = torch.arange(32, device=mask.device, dtype=torch.int32)
            flags = ((mask[:, :, None] >> sh[None, None, :]) & 1).bool().reshape(64, -1)[:, :H]
            tp = float((flags & truth).sum().item())
            p = float(flags.float().mean().item())
            sketch_bytes = D * H * bits / 8.0 + (D * H / 32.0 if bits < 8 else 0.0)
            rows.append({"sketch_bits": bits, "margin": margin, "flag_rate": p,
                         "precision": tp / max(1.0, float(flags.sum().item())),
                         "recall": tp / max(1.0, float(truth.sum().item())),
                         "bytes_per_token_if_packed": 2.0 * D * D + sketch_bytes + 4.0 * p * D * H})
            L.close()
    return {"true_out_of_range_rate": float(truth.float().mean().item()), "rows": rows}


def stack_run(T, synth, torch, np, to_dev, n_layers, batches=(1, 32)):
    """n_layers independent layers chained with RMS-norm glue (config 4): per batch size the time
    of one pass through the whole stack, the per-layer measured fallback rates and the algorithmic
    bytes one pass must move (every layer's folded matrix and sketch once, the W1/W2 rows of the
    union of each layer's flagged neurons, the tokens) against the HBM peak."""
    layers = []
    for li in range(n_layers):
        w = synth.decode(layer=li, n_cal=2048, n_test=32, coverage=0.95, config=4)
        ffn = T.FFN(to_dev(w.layer.W1), to_dev(w.layer.W2))
        lo, hi, a, c = T.tardis_calibrate(ffn, to_dev(w.X_cal), w.coverage)
        layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=32))
        if li == 0:
            X = to_dev(w.X_test)
        if (li + 1) % 8 == 0:
            print(f"bench.py: stack layer {li + 1}/{n_layers} folded", file=sys.stderr, flush=True)
    out = {"layers": n_layers}
    for B in batches:
        xb = X[:B].contiguous()
        yb = torch.empty_like(xb)
        us = _time_us(torch, lambda: T.tardis_stack_forward(layers, xb, yb), 10, 2)
        rates, unions = [], []
        for L in layers:
            _, cnt, _ = T.tardis_get_last_outliers(L, B, want_list=False)
            ucnt, _ = T.tardis_get_last_union(L, B)
            rates.append(float(cnt.float().mean().item()) / H)
            unions.append(int(ucnt.item()))
        def dense_stack():
            h_ = xb
            for L in layers:
                h_ = torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(h_, L.ffn.W1)), L.ffn.W2)
                h_ = torch.nn.functional.rms_norm(h_, (D,), eps=1e-6)
            return h_
        dus = _time_us(torch, dense_stack, 10, 2)
        alg = sum(2.0 * D * D + 1.0 * D * H + u * 4.0 * D + B * 6.0 * D for u in unions)
        out[f"batch{B}"] = {"us_per_step": us, "us_per_layer": us / n_layers, "tokens_per_s": B / (us * 1e-6),
                            "dense_torch_us_per_step": dus, "speedup_vs_dense_torch": dus / us,
                            "per_layer_fallback_rate": [round(r, 4) for r in rates],
                            "per_layer_union_neurons": unions,
                            "roofline_stack": {"bound": "hbm", "algorithmic_bytes_per_step": alg,
                                               "achieved": alg / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                               "frac": alg / us / 1e3 / HBM_PEAK_GBS}}
    for L in layers:
        L.close()
    return out


def batched_sweep(T, synth, torch, np, to_dev, pre, X, coverages, chain=True):
    """Batched decode: tokens/s, algorithmic GB/s and union size per (batch, coverage), cold over
    the given layer copies (`pre`: FFN and device calibration tokens of each), against the
    vendor-BLAS dense FFN at the same batch."""
    rows = []
    ffns = [f for f, _ in pre]
    Xc = [x for _, x in pre]
    stream = torch.cuda.current_stream()
    for cov in coverages:
        layers = []
        for ffn, xc in zip(ffns, Xc):
            lo, hi, a, c = T.tardis_calibrate(ffn, xc, cov)
            layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=64))
        if chain:
            for i, L in enumerate(layers):      # the timed loop walks the copies in this order
                T.tardis_set_next_layer(L, layers[(i + 1) % len(layers)])
        for B in (2, 4, 8, 16, 64):
            xb = X[:B].contiguous()
            yb = torch.empty_like(xb)
            T.tardis_ffn_forward_batched(layers[0], xb, yb)
            _, counts, _ = T.tardis_get_last_outliers(layers[0], B, want_list=False)
            ucnt, _ = T.tardis_get_last_union(layers[0], B)
            union = int(ucnt.item())                  # computed on the device from the call's mask words
            p = float(counts.float().mean().item()) / H
            reps = 60
            for L in layers:
                T.tardis_ffn_forward_batched(L, xb, yb)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for r in range(reps):
                T.tardis_ffn_forward_batched(layers[r % len(layers)], xb, yb)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            W1s, W2s = [f.W1 for f in ffns], [f.W2 for f in ffns]
            for i in range(len(ffns)):      # untimed: the vendor library picks its kernels on the first call
                torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(xb, W1s[i])), W2s[i])
            torch.cuda.synchronize()
            e0.record(stream)
            for r in range(reps):
                i = r % len(ffns)
                torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(xb, W1s[i])), W2s[i])
            e1.record(stream)
            torch.cuda.synchronize()
            dus = e0.elapsed_time(e1) * 1e3 / reps
            alg = 2.0 * D * D + D * H + union * 4.0 * D + B * 6.0 * D
            rows.append({"batch": B, "coverage_t": cov, "fallback_rate": p, "union_neurons": union,
                         "us_per_batch": us, "tokens_per_s": B / (us * 1e-6), "algorithmic_GBs": alg / us / 1e3,
                         "frac": alg / us / 1e3 / HBM_PEAK_GBS,
                         "dense_torch_us_per_batch": dus, "speedup_vs_dense_torch": dus / us})
        for L in layers:
            L.close()
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=6, help="independently seeded layer copies for the cold loop")
    ap.add_argument("--coverage", type=float, default=0.95)
    ap.add_argument("--sketch-bits", type=int, default=8, choices=(8, 4),
                    help="predictor code width of the timed layers (8 = the headline configuration)")
    ap.add_argument("--folded-fp8", action="store_true",
                    help="time the headline layers with W' stored as 8-bit floats (an option outside the 1e-2 bar)")
    ap.add_argument("--search-step", type=float, default=0.0,
                    help="also time the greedy range search with this increment on the first layer (offline figure)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the figures beside the headline one (batched decode at the headline coverage, 4-bit sketch, prompt shape)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the headline loop (for profiler runs whose kernel average should be that loop's)")
    ap.add_argument("--no-chain", action="store_true",
                    help="do not tell each layer copy which copy runs next (no cache-warming hint)")
    ap.add_argument("--no-graph", action="store_true", help="time plain stream launches instead of a replayed HIP graph")
    ap.add_argument("--no-sweep", action="store_true",
                    help="batched decode at the headline coverage only (default: batch {2,4,8,16,64} x coverage {0.99,0.95,0.85})")
    ap.add_argument("--prefill", action="store_true", help="run the 2048-token prompt shape even with --no-extras")
    ap.add_argument("--stack", type=int, default=None,
                    help="layers of the FFN stack run at batch 1 and 32 (32 = the full configuration; 0 = skip)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a 1 GiB device copy (known HBM traffic) so that profiler counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2501_10054_amd import synth
    from paper_2501_10054_amd import tardis as T

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    to_dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(dev).contiguous()

    # ------------------------------------------------------------ set-up (untimed)
    t_setup = time.time()
    layers, works, pre, cals = [], [], [], []
    offline = {}
    for li in range(args.layers):
        w = synth.decode(layer=li, n_cal=4096, n_test=TOKENS_PER_STEP if li == 0 else 8, coverage=args.coverage)
        ffn = T.FFN(to_dev(w.layer.W1), to_dev(w.layer.W2))
        Xc = to_dev(w.X_cal)
        torch.cuda.synchronize()
        t0 = time.time()
        lo, hi, a, c = T.tardis_calibrate(ffn, Xc, w.coverage)
        torch.cuda.synchronize()
        t1 = time.time()
        L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=1, sketch_bits=args.sketch_bits, folded_fp8=args.folded_fp8)
        torch.cuda.synchronize()
        t2 = time.time()
        if li == 0:
            offline = {"calibrate_ms": (t1 - t0) * 1e3, "fold_ms": (t2 - t1) * 1e3}
            if args.search_step > 0:   # the greedy range search over the same calibration tokens (ranges not used below)
                t3 = time.time()
                T.tardis_calibrate_search(ffn, Xc, w.coverage, args.search_step)
                torch.cuda.synchronize()
                offline["calibrate_search_ms"] = (time.time() - t3) * 1e3
                offline["search_step"] = args.search_step
            works.append((w, (lo, hi, a, c)))
        layers.append(L)
        cals.append((lo, hi, a, c))
        if li < 4 and not args.no_extras:
            pre.append((ffn, Xc))            # kept for the batched figures below
        del Xc
    w0, cal0 = works[0]
    X = to_dev(w0.X_test)                      # 1024 x d, resident in HBM before timing starts
    Y = torch.empty_like(X)
    stream = torch.cuda.current_stream()
    sptr = T._stream(stream)
    lib = T.lib()
    fwd = lib.tardis_ffn_forward
    dense = lib.tardis_dense_forward
    xp = [X[t].data_ptr() for t in range(TOKENS_PER_STEP)]
    yp = [Y[t].data_ptr() for t in range(TOKENS_PER_STEP)]
    handles = [L.handle for L in layers]

    def step(hs, fn=fwd, dense_call=False):
        nl = len(hs)
        for t in range(TOKENS_PER_STEP):
            if dense_call:
                st = fn(hs[t % nl], xp[t], 1, yp[t], sptr)
            else:
                st = fn(hs[t % nl], xp[t], yp[t], sptr)
            if st != 0:
                raise RuntimeError(f"forward failed with status {st}")

    def timed(hs, steps, warmup, graph=False, **kw):
        """ms per step from HIP events on the launch stream, and host wall ms per step.  With
        graph=True one step (1024 launches) is captured once and replayed."""
        run = lambda: step(hs, **kw)
        if graph:
            step(hs, **kw)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = T._stream(torch.cuda.current_stream())     # the capture stream
                nl = len(hs)
                for t in range(TOKENS_PER_STEP):
                    st = fwd(hs[t % nl], xp[t], yp[t], cs)
                    if st != 0:
                        raise RuntimeError(f"forward failed with status {st}")
            run = g.replay
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        s_ = torch.cuda.current_stream()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.time()
        e0.record(s_)
        for _ in range(steps):
            run()
        e1.record(s_)
        torch.cuda.synchronize()
        wall = time.time() - t0
        return e0.elapsed_time(e1) / steps, wall / steps * 1e3

    # measured fallback rate of the timed tokens on layer 0
    step(handles[:1])
    torch.cuda.synchronize()
    rates = []
    for t in range(0, TOKENS_PER_STEP, 64):
        lib.tardis_ffn_forward(handles[0], xp[t], yp[t], sptr)
        _, cnt, _ = T.tardis_get_last_outliers(layers[0], 1, want_list=False)
        rates.append(int(cnt.item()) / H)
    p = float(np.mean(rates))

    use_graph = not args.no_graph
    # The timed loop walks the layer copies in a fixed order, as a model walks its layers: each
    # copy names the one that follows (tardis_set_next_layer), so a launch spends its idle tail
    # requesting the next copy's first predictor rows.  The figure without the hint is kept beside it.
    plain_ms = None
    chained = False
    if args.headline_only:
        args.no_dense = args.no_extras = args.no_cpu_baseline = True
    if args.stack is None:
        args.stack = 0 if args.no_extras else 32
    if not args.no_chain and len(layers) > 1:
        if not args.headline_only:
            plain_ms, _ = timed(handles, max(2, args.steps // 2), 1, graph=use_graph)
        chained = True
        for i, L in enumerate(layers):
            T.tardis_set_next_layer(L, layers[(i + 1) % len(layers)])
    cold_ms, cold_wall = timed(handles, args.steps, args.warmup, graph=use_graph)
    hot_ms = None
    if not args.headline_only:
        if chained:
            T.tardis_set_next_layer(layers[0], layers[0])        # one layer over and over: it follows itself
        hot_ms, _ = timed(handles[:1], max(2, args.steps // 2), 1, graph=use_graph)
        if chained:
            T.tardis_set_next_layer(layers[0], layers[1 % len(layers)])
    stream_ms = None
    if use_graph and not args.headline_only:
        stream_ms, _ = timed(handles, max(2, args.steps // 4), 1)
    # Context for the roofline figure, not part of it: the same 1024 single-token launches issued
    # alternately on TWO streams (independent request streams, each at batch 1, each walking its
    # own half of the layer copies).  The blocks of one launch start as the blocks of the other
    # finish, so a launch's ramp and tail overlap the neighbour's stream; every token still
    # streams its own 114 MB.  Wall clock over whole steps, both streams drained.
    two = None
    if not args.headline_only and len(handles) >= 4:
        sA, sB = torch.cuda.Stream(), torch.cuda.Stream()
        pa, pb = T._stream(sA), T._stream(sB)
        la, lb = layers[0::2], layers[1::2]
        if chained:
            for grp in (la, lb):
                for i, L in enumerate(grp):
                    T.tardis_set_next_layer(L, grp[(i + 1) % len(grp)])
        ha, hb = [L.handle for L in la], [L.handle for L in lb]

        def two_step():
            for t in range(0, TOKENS_PER_STEP, 2):
                k = t // 2
                if fwd(ha[k % len(ha)], xp[t], yp[t], pa) != 0 or fwd(hb[k % len(hb)], xp[t + 1], yp[t + 1], pb) != 0:
                    raise RuntimeError("forward failed")
        torch.cuda.synchronize()
        sA.wait_stream(stream)
        sB.wait_stream(stream)
        two_step()
        torch.cuda.synchronize()
        reps = max(2, args.steps // 2)
        t0 = time.time()
        for _ in range(reps):
            two_step()
        torch.cuda.synchronize()
        two_ms = (time.time() - t0) / reps * 1e3
        two = {"tokens_per_s": TOKENS_PER_STEP / (two_ms * 1e-3), "us_per_token": two_ms * 1e3 / TOKENS_PER_STEP,
               "note": "two independent batch-1 streams interleaved on two HIP streams (host wall clock); "
                       "context for where the single-stream time goes, not the headline"}
        if chained:
            for i, L in enumerate(layers):
                T.tardis_set_next_layer(L, layers[(i + 1) % len(layers)])
    res_dense = {}
    if not args.no_dense:
        dms, _ = timed(handles, max(2, args.steps // 4), 1, fn=dense, dense_call=True)
        W1, W2 = layers[0].ffn.W1, layers[0].ffn.W2
        xs = [X[t:t + 1] for t in range(TOKENS_PER_STEP)]
        def torch_step():
            for t in range(TOKENS_PER_STEP):
                torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(xs[t], W1)), W2)
        torch_step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(2):
            torch_step()
        e1.record(stream)
        torch.cuda.synchronize()
        tms = e0.elapsed_time(e1) / 2
        res_dense = {
            "dense_own_tokens_per_s": TOKENS_PER_STEP / (dms * 1e-3),
            "dense_own_GBs": 4.0 * D * H / (dms * 1e-3 / TOKENS_PER_STEP) / 1e9,
            "dense_torch_hot_tokens_per_s": TOKENS_PER_STEP / (tms * 1e-3),
        }

    tok_s = TOKENS_PER_STEP / (cold_ms * 1e-3)
    bytes_tok = algorithmic_bytes(D, H, p, args.sketch_bits, 1.0 if args.folded_fp8 else 2.0)
    launch_s = cold_ms * 1e-3 / TOKENS_PER_STEP          # one kernel launch per token
    achieved = bytes_tok / launch_s / 1e9

    # ------------------------------------------------------------ CPU baseline (the checker)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import tardis_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        lay = w0.layer
        F = O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in cal0), sketch_bits=args.sketch_bits)
        ns = 160
        t0 = time.time()
        O.forward(F, w0.X_test[:ns])
        dt = time.time() - t0
        cpu = {"value": ns / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{ns} of the 1024 timed tokens through oracle forward (fp64 numpy; folding and sketch built beforehand, untimed)"}

    out = {
        "metric": "FFN tokens/s + achieved HBM GB/s (folded+fallback vs dense), d=4096 ffn=16384",
        "value": tok_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": cold_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "decode single layer d=4096 ffn=16384 bf16, batch 1, 1024 tokens/step, "
                               f"cold over {args.layers} seeded layer copies"
                               + (", each copy naming the next (cache-warming hint)" if chained else ""),
                   "coverage_t": args.coverage,
                   "measured_fallback_rate": p, "tokens_per_step": TOKENS_PER_STEP,
                   "sketch_bits": args.sketch_bits, "folded_dtype": "e4m3" if args.folded_fp8 else "bf16"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("decode_fused_kernel", args.sketch_bits, chained),
                     "kernel": "decode_fused_kernel", "algorithmic_bytes_per_launch": bytes_tok,
                     "avg_launch_us": launch_s * 1e6},
        "cpu_baseline": cpu,
        "hot": ({"tokens_per_s": TOKENS_PER_STEP / (hot_ms * 1e-3),
                 "GBs": bytes_tok / (hot_ms * 1e-3 / TOKENS_PER_STEP) / 1e9} if hot_ms else None),
        "without_next_layer_hint": ({"tokens_per_s": TOKENS_PER_STEP / (plain_ms * 1e-3),
                                     "us_per_token": plain_ms * 1e3 / TOKENS_PER_STEP,
                                     "GBs": bytes_tok / (plain_ms * 1e-3 / TOKENS_PER_STEP) / 1e9} if plain_ms else None),
        "launch_mode": "hip graph replay (one graph = one 1024-token step)" if use_graph else "stream",
        "stream_launch_tokens_per_s": (TOKENS_PER_STEP / (stream_ms * 1e-3)) if stream_ms else None,
        "host_wall_ms_per_step": cold_wall,
        "two_streams": (dict(two, algorithmic_GBs=bytes_tok / (two["us_per_token"] * 1e-6) / 1e9) if two else None),
        "offline": offline,
        "setup_s": time.time() - t_setup,
    }
    out.update(res_dense)
    if res_dense:
        out["speedup_vs_dense_own"] = tok_s / res_dense["dense_own_tokens_per_s"]
    if not args.no_extras:
        # the same decode loop with the 4-bit sketch (same layers, same ranges and lines)
        l4 = [T.tardis_fold(L.ffn, *cal, max_batch=1, sketch_bits=4) for L, cal in zip(layers, cals)]
        h4 = [L.handle for L in l4]
        if chained:
            for i, L in enumerate(l4):
                T.tardis_set_next_layer(L, l4[(i + 1) % len(l4)])
        step(h4[:1])
        torch.cuda.synchronize()
        r4 = []
        for t in range(0, TOKENS_PER_STEP, 64):
            lib.tardis_ffn_forward(h4[0], xp[t], yp[t], sptr)
            _, cnt, _ = T.tardis_get_last_outliers(l4[0], 1, want_list=False)
            r4.append(int(cnt.item()) / H)
        p4 = float(np.mean(r4))
        ms4, _ = timed(h4, max(2, args.steps // 2), 1, graph=use_graph)
        b4 = algorithmic_bytes(D, H, p4, 4)
        out["sketch4"] = {"tokens_per_s": TOKENS_PER_STEP / (ms4 * 1e-3), "us_per_token": ms4 * 1e3 / TOKENS_PER_STEP,
                          "measured_fallback_rate": p4, "algorithmic_bytes_per_token": b4,
                          "algorithmic_GBs": b4 / (ms4 * 1e-3 / TOKENS_PER_STEP) / 1e9}
        for L in l4:
            L.close()
        out["sketch_study"] = sketch_study(T, torch, layers[0].ffn, cals[0], X[:64].contiguous())
        covs = (args.coverage,) if args.no_sweep else (0.99, 0.95, 0.85)
        out["batched_sweep"] = batched_sweep(T, synth, torch, np, to_dev, pre, X, covs, chain=not args.no_chain)
    if args.prefill or not args.no_extras:
        print("bench.py: prompt shape (2048 tokens)", file=sys.stderr, flush=True)
        out["prefill"] = prefill_run(T, synth, torch, np, to_dev)
    if args.stack > 0:
        for L in layers:                    # the headline copies are no longer needed: make room
            L.close()
        layers = []
        out["stack"] = stack_run(T, synth, torch, np, to_dev, args.stack)
    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_probe"] = "3 x torch copy_ of 1 GiB (reads 1 GiB, writes 1 GiB each)"
    print(json.dumps(out))
    for L in layers:
        L.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
