#!/usr/bin/env python3
"""Writes tests/golden/config<N>.json: expected results for the full-size configs.

Calls ONLY the CPU oracle (oracle/), the seeded input generator (synth/) and the test-side
margin helper; nothing here touches the HIP library.  For every (layer, sequence, k) it stores
what a GPU test needs to assert bit-exact selection and in-tolerance outputs without running
the oracle's prompt phase again (minutes to hours of fp64 loops at these sizes):

  nudges      (row, factor) pairs applied to W1 so that every top-k boundary has a relative
              gap > 2e-3 (see tests/margin.py); replayed by synth.layer_weights(nudges=...)
  idx_sha256  SHA-256 of the oracle's ascending int32 index array (little endian)
  margin      relative gap at the boundary, s_k the k-th largest s
  s_samples   s_j of 64 fixed sample positions; sum_s2 = sum_j s_j^2 (= prompt length)
  decode      for the first steps: y at 32 fixed columns and max|y| through the oracle's
              compact block, and the same for the full-width block (k = D_ff)

usage: python tests/golden/make_golden.py --config 1 [--layers 0,1,...]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import oracle  # noqa: E402
import synth  # noqa: E402
from margin import boundary_report, open_margin  # noqa: E402

N_S_SAMPLES = 64
N_Y_SAMPLES = 32
DECODE_STEPS = 2


def sample_positions(n: int, count: int, salt: int) -> np.ndarray:
    rng = np.random.default_rng([synth.ROOT_SEED, salt, n])
    return np.sort(rng.choice(n, size=min(count, n), replace=False))


def sha_idx(idx: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(idx, dtype="<i4").tobytes()).hexdigest()


def layer_record(cfg: synth.Config, layer: int, verbose: bool = True) -> dict:
    t0 = time.time()
    Wg, W1, W2 = synth.layer_weights(cfg, layer)
    lens = synth.seq_lengths(cfg)
    Xs = [synth.prompt(cfg, layer, b, lens[b]) for b in range(cfg.n_seqs)]
    if verbose:
        print("config %d layer %d: inputs in %.1fs, oracle prompt phase over %d tokens ..."
              % (cfg.cid, layer, time.time() - t0, sum(lens)), flush=True)
    nudges, s_list = open_margin(Xs, Wg, W1, cfg.act, cfg.dtype, list(cfg.ks), verbose=verbose)
    s_pos = sample_positions(cfg.d_ff, N_S_SAMPLES, 1)
    y_pos = sample_positions(cfg.d, N_Y_SAMPLES, 2)
    rec = {"layer": layer, "nudges": [[int(r), float(f)] for r, f in nudges],
           "s_positions": s_pos.tolist(), "y_positions": y_pos.tolist(), "seqs": []}
    for b in range(cfg.n_seqs):
        s = s_list[b]
        srec = {"seq": b, "length": lens[b], "sum_s2": float(np.sum(s ** 2)),
                "s_samples": [float(v) for v in s[s_pos]], "k": {}}
        xt = synth.decode_inputs(cfg, layer, b, steps=DECODE_STEPS)
        for k in cfg.ks:
            idx = oracle.topk(s, k)
            gap, sk = boundary_report(s, k)
            cw = [oracle.compact(w, idx) for w in (Wg, W1, W2)]
            dec = []
            for t in range(DECODE_STEPS):
                y = oracle.ff_decode(xt[t], *cw, cfg.act)
                dec.append({"y_samples": [float(v) for v in y[y_pos]], "y_absmax": float(np.max(np.abs(y)))})
            srec["k"][str(k)] = {"idx_sha256": sha_idx(idx), "margin": gap, "s_k": sk,
                                 "idx_head": idx[:8].tolist(), "decode": dec}
            del cw
        if b == 0:   # the full-width block (Eq. 1), once per layer
            full = []
            for t in range(DECODE_STEPS):
                y = oracle.ff_decode(xt[t], Wg, W1, W2, cfg.act)
                full.append({"y_samples": [float(v) for v in y[y_pos]], "y_absmax": float(np.max(np.abs(y)))})
            srec["full_decode"] = full
        rec["seqs"].append(srec)
    if verbose:
        worst = min(v["margin"] for sr in rec["seqs"] for v in sr["k"].values())
        print("config %d layer %d done in %.1fs: %d rows nudged, worst margin %.2e"
              % (cfg.cid, layer, time.time() - t0, len(nudges), worst), flush=True)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--layers", type=str, default="")
    args = ap.parse_args()
    cfg = synth.CONFIGS[args.config]
    layers = [int(v) for v in args.layers.split(",")] if args.layers else list(range(cfg.n_layers))
    path = os.path.join(HERE, "config%d.json" % cfg.cid)
    doc = {"config": cfg.cid, "name": cfg.name, "d": cfg.d, "d_ff": cfg.d_ff, "ks": list(cfg.ks),
           "citation": "selection per Section 4.2 / Eq. 6 and pruned output per Eq. 4-5, computed by oracle/ in fp64",
           "layers": {}}
    if os.path.exists(path):
        with open(path) as fh:
            doc = json.load(fh)
    for layer in layers:
        doc["layers"][str(layer)] = layer_record(cfg, layer)
        tmp = path + ".tmp"
        with open(tmp, "w") as fh:
            json.dump(doc, fh, indent=0, separators=(",", ":"))
        os.replace(tmp, path)
    print("wrote", path)


if __name__ == "__main__":
    main()
