#!/usr/bin/env python3
"""Benchmark of the GRIFFIN feed-forward hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: prompt-phase
selection (FF activations, row normalisation, statistic s, top-k), compaction of the
selected neurons, and T generated tokens through the pruned FF block, for every layer of the
workload.  Inputs are resident in HBM before the timed region.  Decode cycles through enough
copies of the compact weights (>= 1 GiB) that the 256 MB Infinity Cache cannot serve them.

Prints ONE JSON line: whole-job generated tokens/s (`value`), the roofline of the dominant
kernel (the weight-streaming decode kernel, HBM-bound) and the CPU oracle timed on a bounded
sample of the same workload.  The default workload is config 3 (the Llama-2-13B-shaped stack of 40
layers, the model of the paper's latency table); configs 1 and 2 ride along as short extra runs (five steps each).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload: 3 Llama-2-13B-shaped stack of 40 layers (default: the largest single-sequence "
                         "workload, the model of the paper's latency table), 1 Llama-2-7B-shaped layer, 2 Gemma-7B-shaped layer, "
                         "4 Mistral-7B-shaped stack of 8 with 16 sequences that keep their own sets")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of configs 1 and 2 that the default run reports as extra keys")
    ap.add_argument("--k", type=int, default=0, help="kept neurons (default: the config's 50%% point)")
    ap.add_argument("--layers", type=int, default=0, help="layers to run (default: all of the config)")
    ap.add_argument("--probe-every", type=int, default=8, help="decode steps between kernel-duration probes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-full-width", action="store_true",
                    help="do not time the full-width block after the timed region (keeps a profile's per-kernel "
                         "averages to the pruned launches only)")
    ap.add_argument("--warm", action="store_true", help="single copy of the compact weights (cache-warm)")
    ap.add_argument("--layout", choices=("rows", "transposed"), default="rows",
                    help="compact block: W2 neuron-major (one stream plus a kernel that adds 256 partial rows, default) or "
                         "output-feature-major (two pure streams per token, no partial rows)")
    return ap.parse_args()


class Hip:
    """The few HIP runtime calls the benchmark needs for per-kernel event timing."""

    def __init__(self, torch):
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        self.lib = ctypes.CDLL(path)
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]

    def record(self, ev: int, stream) -> None:
        rc = self.lib.hipEventRecord(ev, stream)
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def event(self) -> int:
        e = ctypes.c_void_p()
        rc = self.lib.hipEventCreate(ctypes.byref(e))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return e.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)


def cpu_baseline(cfg, k, Wg, W1, W2, seconds_target=12.0):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the workload: the prompt
    phase (FF activations, statistic, top-k) of ONE layer and ONE prompt, and decode tokens through that
    layer's compact block."""
    import numpy as np
    import oracle
    import synth
    lens = synth.seq_lengths(cfg)
    b_sel = int(np.argmin(lens))                      # the shortest prompt of a batched workload; the only one otherwise
    X = synth.prompt(cfg, 0, b_sel, lens[b_sel])
    t0 = time.perf_counter()
    idx, _ = oracle.prefill_select(X, Wg, W1, cfg.act, k)
    sel_s = time.perf_counter() - t0
    cw = [oracle.compact(w, idx) for w in (Wg, W1, W2)]
    xt = synth.decode_inputs(cfg, 0, steps=8).astype(np.float64)
    oracle.ff_decode(xt[0], *cw, cfg.act)
    n, t0 = 0, time.perf_counter()
    while True:
        oracle.ff_decode(xt[n % 8], *cw, cfg.act)
        n += 1
        el = time.perf_counter() - t0
        if el >= seconds_target or n >= 512:
            break
    per_layer_token_s = el / n
    return {
        "value": 1.0 / (per_layer_token_s * cfg.n_layers), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "%d decode tokens through ONE layer's k=%d compact block in fp64 (%.1f ms per layer-token; value = 1 / (that x %d layers)); "
                  "prompt phase of one layer on one prompt of %d tokens: %.2f s"
                  % (n, k, per_layer_token_s * 1e3, cfg.n_layers, lens[b_sel], sel_s),
        "decode_ms_per_layer_token": per_layer_token_s * 1e3,
        "select_s_per_layer": sel_s, "select_sample_tokens": lens[b_sel],
    }


def run_batched(args, cfg, torch, np, G, synth, hip):
    """Config 4: B sequences with their own expert sets share every layer's weights.  One step =
    selection for all layers (packed variable-length prompts, one set per sequence) + T decode
    steps of B rows through every layer, each row through its own set, in ONE masked pass over the
    full block per layer-step (the per-sequence sets cover almost the whole block between them, so
    compact copies would stream B x the bytes; that variant is timed beside it, outside the region)."""
    k = args.k or cfg.k
    n_layers = args.layers or cfg.n_layers
    T, d, F, B = cfg.decode_steps, cfg.d, cfg.d_ff, cfg.n_seqs
    w = 2
    up = lambda a: torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream
    layers, host_w0 = [], None
    for l in range(n_layers):
        Wg, W1, W2 = synth.layer_weights(cfg, l)
        if l == 0:
            host_w0 = (Wg, W1, W2)
        X, cu = synth.packed_prompts(cfg, l)
        xt = np.stack([synth.decode_inputs(cfg, l, b) for b in range(B)], axis=1)      # [T][B][d]
        t = dict(Wg=up(Wg), W1=up(W1), W2=up(W2), X=up(X), xt=up(xt), cu=[int(v) for v in cu])
        t["L"] = G.layer(t["W1"], t["W2"], t["Wg"], act=cfg.act)
        t["idx"] = torch.empty((B, k), dtype=torch.int32, device="cuda")
        t["sets"] = torch.empty((G.griffin_index_sets_bytes(F, B) // 4,), dtype=torch.int32, device="cuda")
        t["y"] = torch.empty((T, B, d), dtype=torch.bfloat16, device="cuda")
        layers.append(t)
        del Wg, W1, W2
    total = layers[0]["cu"][-1]
    ws_pre = torch.empty(G.griffin_prefill_workspace_bytes(layers[0]["L"], total, B, False), dtype=torch.uint8, device="cuda")
    ws_dec = torch.empty(G.griffin_decode_workspace_bytes(d, F, B), dtype=torch.uint8, device="cuda")   # sized for the whole block
    esz = B * d * w
    for t in layers:
        t["xp"], t["yp"] = t["xt"].data_ptr(), t["y"].data_ptr()

    per_step = (T * n_layers + args.probe_every - 1) // args.probe_every
    pool = [(hip.event(), hip.event(), hip.event()) for _ in range(per_step * args.steps)]
    probes, stage_ev = [], []

    def step(record):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if record else None
        if record:
            ev[0].record()
        for t in layers:
            G.griffin_prefill_select(t["L"], t["X"], t["cu"], k, t["idx"], workspace=ws_pre, stream=stream)
            # which rows hold which neuron: once per prompt, the sets stay fixed while generating
            G.griffin_index_sets_build(t["idx"], k, B, F, t["sets"], stream=stream)
        if record:
            ev[1].record()
        for tok in range(T):
            for li, t in enumerate(layers):
                if record and (tok * n_layers + li) % args.probe_every == 0:
                    pe = pool[len(probes)]
                    probes.append(pe)
                    G.griffin_trace_next_decode(*pe)
                G.griffin_ff_decode_indexed_sets(t["L"], t["idx"], k, t["sets"], B, t["xp"] + tok * esz, t["yp"] + tok * esz,
                                                 workspace=ws_dec, stream=stream)
        if record:
            ev[2].record()
            stage_ev.append(ev)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # beside it, outside the timed region: every sequence through its own compact block (one layer)
    multi_us = None
    if not args.skip_full_width:
        t0l = layers[0]
        Cs, keep = [], []
        for b in range(B):
            blk = torch.empty((k, 3, d), dtype=torch.bfloat16, device="cuda")
            C = G.layer(blk[:, 1], blk[:, 2], blk[:, 0], act=cfg.act)
            G.griffin_compact(t0l["L"], t0l["idx"][b], k, C, stream=stream)
            Cs.append(C); keep.append(blk)
        ws_m = torch.empty(G.griffin_decode_workspace_bytes(d, k, B), dtype=torch.uint8, device="cuda")
        me = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for rep in range(11):
            if rep == 1:
                me[0].record()
            G.griffin_ff_decode_multi(Cs, t0l["xp"] + (rep % T) * esz, t0l["yp"] + (rep % T) * esz, workspace=ws_m, stream=stream)
        me[1].record()
        torch.cuda.synchronize()
        multi_us = me[0].elapsed_time(me[1]) * 1e3 / 10
        del Cs, keep, ws_m

    sel_ms = sum(e[0].elapsed_time(e[1]) for e in stage_ev) / len(stage_ev)
    dec_ms = sum(e[1].elapsed_time(e[2]) for e in stage_ev) / len(stage_ev)
    raw_main = [hip.elapsed_ms(a, m) * 1e3 for a, m, e in probes]
    raw_tok = [hip.elapsed_ms(a, e) * 1e3 for a, m, e in probes]
    n_tok = args.steps * T * n_layers
    span_us = sum(e[1].elapsed_time(e[2]) for e in stage_ev) * 1e3
    Bp = sum(raw_tok) / len(raw_tok)
    u = (span_us - len(probes) * Bp) / max(n_tok - len(probes), 1)
    event_overhead_us = max((Bp - u) / 2.0, 0.0)
    kern_us = sorted(max(v - event_overhead_us, 0.0) for v in raw_main)
    avg_us = sum(kern_us) / len(kern_us)
    # the masked pass reads the whole block once per layer-step, the B rows of x, and writes B rows of y
    alg_bytes = 3 * F * d * w + 2 * B * d * w
    achieved = alg_bytes / (avg_us * 1e-6) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh).get("config%d_k%d" % (cfg.cid, k))
    out = {
        "metric": "pruned-FF decode tokens/s + achieved HBM GB/s; select \u00b5s/layer (prefill)",
        "value": args.steps * T * B / wall,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "config %d: %s, d=%d D_ff=%d, %d prompts of %d..%d tokens (%d in all), keep k=%d per sequence, "
                        "batch %d, %d decode steps, %d layer(s)" % (cfg.cid, cfg.name, d, F, B, cfg.len_range[0], cfg.len_range[1],
                                                                    total, k, B, T, n_layers),
            "decode": "one masked pass over the full block per layer-step (griffin_ff_decode_indexed_sets, membership words built once per prompt)",
            "cache": "cold (%.1f GB of weights per step)" % (n_layers * 3 * F * d * w / 1e9),
        },
        "roofline": {
            "bound": "hbm", "kernel": "masked pass: ff_batch_gu_kernel + ff_batch_down_kernel",
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": None if traffic is None else "profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command on "
                              "two layers, both kernels of the pass, scaled by the same counters on a copy kernel of known size (stored, not re-measured in this run)",
            "algorithmic_bytes_per_launch": alg_bytes,
            "avg_kernel_us": avg_us, "median_kernel_us": kern_us[len(kern_us) // 2], "launches_timed": len(kern_us),
            "event_cost_us": event_overhead_us, "unprobed_us_per_layer_step": u,
        },
        "decode": {
            "tokens_per_s_decode_only": T * B / (dec_ms * 1e-3),
            "us_per_layer_step": dec_ms * 1e3 / (T * n_layers),
            "per_sequence_compact_blocks_us_per_layer_step": multi_us,
            "per_sequence_compact_blocks_GBps": None if multi_us is None else B * 3 * k * d * w / (multi_us * 1e-6) / 1e9,
        },
        "select_us_per_layer": sel_ms * 1e3 / n_layers,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, k, *host_w0)
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus %d is not supported (the path shards by "
              "layer or by sequence with no communication)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2404_01365_amd as G
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    hip = Hip(torch)

    cfg = synth.CONFIGS[args.config]
    if cfg.n_seqs != 1:
        if cfg.dtype != synth.DT_BF16:
            print("bench.py: config %d is a parity case, not a bench line" % args.config, file=sys.stderr)
            sys.exit(2)
        return run_batched(args, cfg, torch, np, G, synth, hip)
    if cfg.dtype != synth.DT_BF16:
        print("bench.py: config %d is a parity case, not a bench line" % args.config, file=sys.stderr)
        sys.exit(2)
    out = run_single(args, cfg, torch, np, G, synth, hip, brief=False)
    if args.config == 3 and not args.no_other_configs and not args.k and not args.layers:
        # the two single-layer workloads, a few steps each, as extra keys beside the headline line
        import copy
        for cid in (1, 2):
            a = copy.copy(args)
            a.steps, a.warmup, a.config = 5, 2, cid
            torch.cuda.empty_cache()
            o = run_single(a, synth.CONFIGS[cid], torch, np, G, synth, hip, brief=True)
            out["config%d" % cid] = {
                "workload": o["config"]["workload"], "tokens_per_s": o["value"], "ms_per_step": o["ms_per_step"],
                "roofline_frac": o["roofline"]["frac"], "avg_kernel_us": o["roofline"]["avg_kernel_us"],
                "us_per_layer_token": o["decode"]["us_per_layer_token"],
                "frac_per_layer_token": o["decode"]["GBps_per_layer_token"] / HBM_PEAK_GBS,
                "pruned_over_full_latency": o["decode"]["pruned_over_full_latency"],
                "select_us_per_layer": o["select_us_per_layer"], "select": o["select"],
            }
    print(json.dumps(out))


def run_single(args, cfg, torch, np, G, synth, hip, brief):
    """One sequence, n_layers independent FF blocks: one step = selection + compaction of every layer, then T
    tokens through every layer's compact block.  `brief` leaves out what is measured beside the timed region
    except the full-width comparison."""
    k = args.k or cfg.k
    n_layers = args.layers or cfg.n_layers
    T, d, F, S = cfg.decode_steps, cfg.d, cfg.d_ff, cfg.prompt_len
    w = 2 if cfg.dtype == synth.DT_BF16 else 4
    tdt = torch.bfloat16 if cfg.dtype == synth.DT_BF16 else torch.float32

    def up(a):
        if cfg.dtype == synth.DT_BF16:
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()

    # ---------------- inputs resident in HBM
    from concurrent.futures import ThreadPoolExecutor
    layers, host_w0 = [], None
    with ThreadPoolExecutor(synth.n_threads()) as pool:
        for l in range(n_layers):
            Wg, W1, W2 = synth.layer_weights(cfg, l, pool=pool)
            if l == 0:
                host_w0 = (Wg, W1, W2)
            t = dict(Wg=up(Wg), W1=up(W1), W2=up(W2), X=up(synth.prompt(cfg, l)), xt=up(synth.decode_inputs(cfg, l)))
            t["L"] = G.layer(t["W1"], t["W2"], t["Wg"], act=cfg.act)
            layers.append(t)
            del Wg, W1, W2

    compact_bytes = 3 * k * d * w
    if args.warm or n_layers * compact_bytes >= (1 << 30):
        n_rep = 1
    else:
        n_rep = -(-(1 << 30) // (n_layers * compact_bytes))
    transposed = args.layout == "transposed" and cfg.dtype == synth.DT_BF16 and d % 512 == 0
    ldt = -(-k // 512) * 512
    ldt_full = -(-F // 512) * 512
    for t in layers:
        t["C"], t["Ct"] = [], []
        for r in range(n_rep):
            if transposed:
                # Wg and W1 rows of a kept neuron side by side ([k][2][d]); W2 output-feature-major [d][ldt]
                blk = torch.empty((k, 2, d), dtype=tdt, device="cuda")
                w2t = torch.empty((d, ldt), dtype=tdt, device="cuda")
                t["Ct"].append((blk, w2t))
                t["C"].append(G.layer(blk[:, 1], None, blk[:, 0], act=cfg.act, W2t=w2t, n=k, d=d))
            else:
                # the three rows of a kept neuron side by side: [k][3][d], row stride 3d
                blk = torch.empty((k, 3, d), dtype=tdt, device="cuda")
                t["Ct"].append(blk)
                t["C"].append(G.layer(blk[:, 1], blk[:, 2], blk[:, 0], act=cfg.act))
        t["idx"] = torch.empty((1, k), dtype=torch.int32, device="cuda")
        t["y"] = torch.empty((T, d), dtype=tdt, device="cuda")
    ws_pre = torch.empty(G.griffin_prefill_workspace_bytes(layers[0]["L"], S, 1, False), dtype=torch.uint8, device="cuda")
    ws_dec = torch.empty(G.griffin_decode_workspace_bytes(d, k, 1), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    cu = [0, S]

    def select_and_compact(t, rep):
        G.griffin_prefill_select(t["L"], t["X"], cu, k, t["idx"], workspace=ws_pre, stream=stream)
        G.griffin_compact(t["L"], t["idx"], k, t["C"][rep], stream=stream)

    # copies 1.. of the compact weights are made once, outside the timed region (same contents)
    for t in layers:
        for r in range(1, n_rep):
            select_and_compact(t, r)
    torch.cuda.synchronize()

    # (begin, end) hipEvent pairs around the streaming decode kernel, created before timing
    per_step = (T * n_layers + args.probe_every - 1) // args.probe_every
    pool = [(hip.event(), hip.event(), hip.event()) for _ in range(per_step * args.steps)]
    probes = []
    stage_ev = []     # (e0, e1, e2) torch events: select+compact | decode
    esz = d * w
    for t in layers:
        t["xp"], t["yp"] = t["xt"].data_ptr(), t["y"].data_ptr()

    def step(record):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if record else None
        if record:
            ev[0].record()
        for t in layers:
            select_and_compact(t, 0)
        if record:
            ev[1].record()
        for tok in range(T):
            for li, t in enumerate(layers):
                if record and (tok * n_layers + li) % args.probe_every == 0:
                    pe = pool[len(probes)]
                    probes.append(pe)
                    G.griffin_trace_next_decode(*pe)
                G.griffin_ff_decode(t["C"][tok % n_rep], t["xp"] + tok * esz, t["yp"] + tok * esz, 1,
                                    workspace=ws_dec, stream=stream)
        if record:
            ev[2].record()
            stage_ev.append(ev)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # the same block at full width (k = D_ff, Eq. 1) through the same entry point, outside the
    # timed region: decode latency of the pruned block relative to the full one.  Like the compact
    # block, the full block is cycled through enough copies (>= 1 GiB in all) to stay cache-cold.
    ws_full = torch.empty(G.griffin_decode_workspace_bytes(d, F, 1), dtype=torch.uint8, device="cuda")
    fe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    full_bytes = 3 * F * d * w
    n_full = 1 if (args.warm or args.skip_full_width or n_layers * full_bytes >= (1 << 30)) else -(-(1 << 30) // (n_layers * full_bytes))
    def full_w2t(W2):
        out = torch.zeros((d, ldt_full), dtype=tdt, device="cuda")     # the paper's W_2, zero-padded (plumbing, untimed)
        out[:, :F] = W2.t()
        return out
    for t in layers:
        t["Lf"], t["Lft"] = [], []
        for r in range(0 if args.skip_full_width else n_full):
            cp = (t["Wg"], t["W1"], t["W2"]) if r == 0 else (t["Wg"].clone(), t["W1"].clone(), t["W2"].clone())
            w2t = full_w2t(cp[2]) if transposed else None
            t["Lft"].append((cp, w2t))
            t["Lf"].append(G.layer(cp[1], cp[2], cp[0], act=cfg.act, W2t=w2t))
    for rep in range(0 if args.skip_full_width else 2):
        if rep == 1:
            fe[0].record()
        for tok in range(T):
            for t in layers:
                G.griffin_ff_decode(t["Lf"][tok % n_full], t["xp"] + tok * esz, t["yp"] + tok * esz, 1, workspace=ws_full, stream=stream)
    full_us = None
    if not args.skip_full_width:
        fe[1].record()
        torch.cuda.synchronize()
        full_us = fe[0].elapsed_time(fe[1]) * 1e3 / (T * n_layers)
        for t in layers:
            t["Lf"], t["Lft"] = [], []

    # selection (FF activations, statistic, top-k) and compaction timed apart, outside the timed region
    se = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    reps_s = max(1, 8 // n_layers)
    for rep in range(2):
        if rep == 1:
            se[0].record()
        for r in range(reps_s):
            for t in layers:
                G.griffin_prefill_select(t["L"], t["X"], cu, k, t["idx"], workspace=ws_pre, stream=stream)
    se[1].record()
    for r in range(reps_s):
        for t in layers:
            G.griffin_compact(t["L"], t["idx"], k, t["C"][0], stream=stream)
    se[2].record()
    torch.cuda.synchronize()
    presel_us = se[0].elapsed_time(se[1]) * 1e3 / (reps_s * n_layers)
    comp_us = se[1].elapsed_time(se[2]) * 1e3 / (reps_s * n_layers)
    comp_bytes = 2 * 3 * k * d * w

    # the prompt's own full-width output Y = Z W_2^T (Section 5.1), outside the timed region
    prompt_out_us = prompt_phase_us = None
    if not args.skip_full_width and not brief:
        t0l = layers[0]
        Zbuf = torch.empty((S, F), dtype=torch.float32, device="cuda")
        G.griffin_prefill_select(t0l["L"], t0l["X"], cu, k, t0l["idx"], Z_out=Zbuf, workspace=ws_pre, stream=stream)
        W2p = t0l["W2"].t().contiguous()        # the paper's W_2 layout [d][D_ff] (plumbing, untimed)
        Yp = torch.empty((S, d), dtype=tdt, device="cuda")
        ws_po = torch.empty(max(G.griffin_prompt_out_workspace_bytes(S, F, d), 256), dtype=torch.uint8, device="cuda")
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for rep in range(6):
            if rep == 1:
                pe[0].record()
            G.griffin_ff_prompt_out(Zbuf, W2p, Yp, workspace=ws_po, stream=stream)
        pe[1].record()
        torch.cuda.synchronize()
        prompt_out_us = pe[0].elapsed_time(pe[1]) * 1e3 / 5
        # ... and the whole prompt phase in one call (selection + output from one Z, Section 4.2 + 5.1)
        ws_pp = torch.empty(G.griffin_prompt_phase_workspace_bytes(t0l["L"], S, 1), dtype=torch.uint8, device="cuda")
        idx_pp = torch.empty_like(t0l["idx"])
        for rep in range(6):
            if rep == 1:
                pe[0].record()
            G.griffin_prompt_phase(t0l["L"], W2p, t0l["X"], cu, k, idx_pp, Yp, workspace=ws_pp, stream=stream)
        pe[1].record()
        torch.cuda.synchronize()
        prompt_phase_us = pe[0].elapsed_time(pe[1]) * 1e3 / 5
        assert bool((idx_pp == t0l["idx"]).all()), "prompt phase and prefill_select disagree on the expert set"
        del Zbuf, W2p, Yp, ws_pp

    # further rows measured outside the timed region: the static weight-norm selector (Section 5.1
    # setup) and one shared set decoded for a batch of 16 rows (Section 5.3, Eq. 7)
    extras = None
    if not args.skip_full_width and not brief:
        t0l = layers[0]
        sc = torch.empty((F,), dtype=torch.float32, device="cuda")
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for rep in range(6):
            if rep == 1:
                ev[0].record()
            G.griffin_weight_norm_score(t0l["L"], sc, stream=stream)
        ev[1].record()
        Bsh = 16
        if transposed:
            # the batch path streams W2 neuron-major: blocks [k][3][d] of the same selection, made outside the timing
            rows_keep, rows_C = [], []
            for r in range(n_rep):
                blk = torch.empty((k, 3, d), dtype=tdt, device="cuda")
                Cr = G.layer(blk[:, 1], blk[:, 2], blk[:, 0], act=cfg.act)
                G.griffin_compact(t0l["L"], t0l["idx"], k, Cr, stream=stream)
                rows_keep.append(blk); rows_C.append(Cr)
        else:
            rows_C = t0l["C"]
        xb = t0l["xt"][:Bsh].contiguous()
        yb = torch.empty_like(xb)
        ws_b = torch.empty(G.griffin_decode_workspace_bytes(d, k, Bsh), dtype=torch.uint8, device="cuda")
        reps_b = 4 * n_rep
        for rep in range(2):
            if rep == 1:
                ev[2].record()
            for r in range(reps_b):
                G.griffin_ff_decode(rows_C[r % n_rep], xb, yb, Bsh, workspace=ws_b, stream=stream)
        ev[3].record()
        torch.cuda.synchronize()
        wn_us = ev[0].elapsed_time(ev[1]) * 1e3 / 5
        b_us = ev[2].elapsed_time(ev[3]) * 1e3 / reps_b
        extras = {
            "weight_norm_score": {"us_per_layer": wn_us, "GBps": 2 * F * d * w / (wn_us * 1e-6) / 1e9},
            "shared_set_decode_batch16": {"us_per_call": b_us, "rows": Bsh,
                                          "GBps_weights_once": (3 * k * d * w + 2 * Bsh * d * w) / (b_us * 1e-6) / 1e9},
        }

    # the box's own copy bandwidth, for scale: a plain device-to-device copy of 1 GiB (read + write
    # counted), larger than the 256 MB Infinity Cache
    cp_src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
    cp_dst = torch.empty_like(cp_src)
    cp_src.zero_()
    cp_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for rep in range(6):
        if rep == 1:
            cp_ev[0].record()
        cp_dst.copy_(cp_src)
    cp_ev[1].record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * (1 << 30) / (cp_ev[0].elapsed_time(cp_ev[1]) * 1e-3 / 5) / 1e9
    del cp_src, cp_dst

    ms_per_step = wall * 1e3 / args.steps
    sel_ms = sum(e[0].elapsed_time(e[1]) for e in stage_ev) / len(stage_ev)
    dec_ms = sum(e[1].elapsed_time(e[2]) for e in stage_ev) / len(stage_ev)
    # Probed tokens carry three events: before the streaming kernel, between it and the small
    # partial-sum kernel, after the latter.  Every recorded event costs GPU time of its own;
    # that cost is measured in the same run: a probed token takes B = end - begin, an unprobed
    # one takes u (from the whole decode span), the two extra events cost (B - u) / 2 each.
    raw_main = [hip.elapsed_ms(a, m) * 1e3 for a, m, e in probes]
    raw_tok = [hip.elapsed_ms(a, e) * 1e3 for a, m, e in probes]
    n_tok = args.steps * T * n_layers
    span_us = sum(e[1].elapsed_time(e[2]) for e in stage_ev) * 1e3
    B = sum(raw_tok) / len(raw_tok)
    u = (span_us - len(probes) * B) / (n_tok - len(probes))
    event_overhead_us = max((B - u) / 2.0, 0.0)
    kern_us = sorted(max(v - event_overhead_us, 0.0) for v in raw_main)
    avg_us = sum(kern_us) / len(kern_us)
    raw_us = raw_main
    alg_bytes = 3 * k * d * w + 2 * d * w           # one layer-token: compact weights once + x in + y out
    if transposed:
        # the timed kernel streams Wg and W1 of the kept neurons, reads x, writes z (fp32, padded)
        kern_name, kern_bytes = "ff_decode_gu_kernel", 2 * k * d * w + d * w + ldt * 4
    else:
        kern_name, kern_bytes = "ff_decode_kernel", alg_bytes
    achieved = kern_bytes / (avg_us * 1e-6) / 1e9
    # the second kernel of a token: the W2 stream (transposed layout) or the sum of the partial rows
    raw_second = [hip.elapsed_ms(m, e) * 1e3 for a, m, e in probes]
    second_us = max(sum(raw_second) / len(raw_second) - event_overhead_us, 0.0)
    second_bytes = (ldt * d * w + ldt * 4 + d * w) if transposed else None

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh).get("config%d_k%d%s" % (cfg.cid, k, "_gu" if transposed else ""))

    out = {
        "metric": "pruned-FF decode tokens/s + achieved HBM GB/s; select \u00b5s/layer (prefill)",
        "value": args.steps * T / wall,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == synth.DT_BF16 else "f32",
        "data": "synthetic",
        "config": {
            "workload": "config %d: %s, d=%d D_ff=%d, prompt %d tokens, keep k=%d, batch 1, %d decode steps, %d layer(s)"
                        % (cfg.cid, cfg.name, d, F, S, k, T, n_layers),
            "compact_weight_copies_cycled": n_rep,
            "compact_layout": "Wg,W1 [k][2][d] + W2 output-feature-major [d][%d]" % ldt if transposed else "Wg,W1,W2 [k][3][d]",
            "cache": "warm (one copy)" if n_rep == 1 and n_layers * compact_bytes < (1 << 30) else "cold (>= 1 GiB cycled)",
        },
        "roofline": {
            "bound": "hbm", "kernel": kern_name,
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": None if traffic is None else "profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command, "
                              "scaled by the same counters on a copy kernel of known size (stored, not re-measured in this run)",
            "algorithmic_bytes_per_launch": kern_bytes,
            "avg_kernel_us": avg_us, "median_kernel_us": kern_us[len(kern_us) // 2], "launches_timed": len(kern_us),
            "raw_event_span_us": sum(raw_us) / len(raw_us), "event_cost_us": event_overhead_us,
            "unprobed_us_per_layer_token": u,
            "measured_copy_GBps": copy_gbs, "frac_of_measured_copy": achieved / copy_gbs,
        },
        "decode": {
            "tokens_per_s_decode_only": T / (dec_ms * 1e-3),
            "us_per_layer_token": dec_ms * 1e3 / (T * n_layers),
            "GBps_per_layer_token": alg_bytes / (dec_ms * 1e-3 / (T * n_layers)) / 1e9,
            "second_kernel": {"name": "ff_decode_down_kernel" if transposed else "ff_decode_reduce_kernel", "avg_us": second_us,
                              "GBps": None if second_bytes is None else second_bytes / (second_us * 1e-6) / 1e9},
            "full_width_us_per_layer_token": full_us, "full_width_copies_cycled": n_full,
            "pruned_over_full_latency": (u / full_us) if full_us else None,
        },
        "select_us_per_layer": sel_ms * 1e3 / n_layers,
        "select": {
            "prefill_select_us_per_layer": presel_us, "prefill_select_TFLOPs_whole_call": 4.0 * S * F * d / (presel_us * 1e-6) / 1e12,
            "compact_us_per_layer": comp_us, "compact_GBps": comp_bytes / (comp_us * 1e-6) / 1e9,
            "compact_frac_of_peak": comp_bytes / (comp_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        },
        "prompt_out": None if prompt_out_us is None else {
            "us_per_layer": prompt_out_us, "TFLOPs": 2.0 * S * F * d / (prompt_out_us * 1e-6) / 1e12},
        "prompt_phase_one_call": None if prompt_phase_us is None else {
            "us_per_layer": prompt_phase_us, "TFLOPs": (4.0 + 2.0) * S * F * d / (prompt_phase_us * 1e-6) / 1e12},
    }
    if extras:
        out.update(extras)
    if not args.no_cpu_baseline and not brief:
        out["cpu_baseline"] = cpu_baseline(cfg, k, *host_w0)
    return out


if __name__ == "__main__":
    main()
