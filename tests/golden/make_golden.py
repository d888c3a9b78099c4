#!/usr/bin/env python3
"""Writes tests/golden/config<N>.json and config<N>_s.npz: expected results for the full-size configs.

Calls ONLY the CPU oracle (oracle/), the seeded input generator (synth/) and the test-side
margin helper; nothing here touches the HIP library.  The oracle's prompt phase takes minutes to
hours of fp64 loops at these sizes, so what it yields is stored once:

  config<N>.json, per layer
    nudges      (row, factor) pairs applied to W1 so that every top-k boundary has a relative
                gap > 2e-3 (see tests/margin.py); replayed by synth.layer_weights(nudges=...)
    per sequence: length, sum_s2 = sum_j s_j^2 (= prompt length), and per k
      idx_sha256  SHA-256 of the oracle's ascending int32 index array (little endian)
      margin      relative gap at the boundary, s_k the k-th largest s, idx_head the first 8 indices
  config<N>_s.npz
    l<layer>_b<seq>  the whole statistic s (Eq. 6) of that prompt, float64 [D_ff]

The decode outputs are not stored: the GPU test recomputes the oracle's expert set from the stored
s (oracle.topk) and runs the oracle's decode on it live, whole vectors.

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

def sha_idx(idx: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(idx, dtype="<i4").tobytes()).hexdigest()


def layer_record(cfg: synth.Config, layer: int, verbose: bool = True):
    t0 = time.time()
    Wg, W1, W2 = synth.layer_weights(cfg, layer)
    lens = synth.seq_lengths(cfg)
    Xs = [synth.prompt(cfg, layer, b, lens[b]) for b in range(cfg.n_seqs)]
    if verbose:
        print("config %d layer %d: inputs in %.1fs, oracle prompt phase over %d tokens ..."
              % (cfg.cid, layer, time.time() - t0, sum(lens)), flush=True)
    nudges, s_list = open_margin(Xs, Wg, W1, cfg.act, cfg.dtype, list(cfg.ks), verbose=verbose)
    rec = {"layer": layer, "nudges": [[int(r), float(f)] for r, f in nudges], "seqs": []}
    for b in range(cfg.n_seqs):
        s = s_list[b]
        srec = {"seq": b, "length": lens[b], "sum_s2": float(np.sum(s ** 2)), "k": {}}
        for k in cfg.ks:
            idx = oracle.topk(s, k)
            gap, sk = boundary_report(s, k)
            srec["k"][str(k)] = {"idx_sha256": sha_idx(idx), "margin": gap, "s_k": sk, "idx_head": idx[:8].tolist()}
        rec["seqs"].append(srec)
    if verbose:
        worst = min(v["margin"] for sr in rec["seqs"] for v in sr["k"].values())
        print("config %d layer %d done in %.1fs: %d nudges on %d rows (%.2f %% of D_ff), worst margin %.2e"
              % (cfg.cid, layer, time.time() - t0, len(nudges), len({r for r, _ in nudges}),
                 100.0 * len({r for r, _ in nudges}) / cfg.d_ff, worst), flush=True)
    return rec, {"l%d_b%d" % (layer, b): np.asarray(s_list[b], dtype=np.float64) for b in range(cfg.n_seqs)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--layers", type=str, default="")
    ap.add_argument("--fresh", action="store_true", help="start from empty files instead of adding layers to the stored ones")
    args = ap.parse_args()
    cfg = synth.CONFIGS[args.config]
    layers = [int(v) for v in args.layers.split(",")] if args.layers else list(range(cfg.n_layers))
    path = os.path.join(HERE, "config%d.json" % cfg.cid)
    path_s = os.path.join(HERE, "config%d_s.npz" % cfg.cid)
    doc = {"config": cfg.cid, "name": cfg.name, "d": cfg.d, "d_ff": cfg.d_ff, "ks": list(cfg.ks),
           "citation": "statistic per Section 4.1 / Eq. 6 and expert sets per Section 4.2, computed by oracle/ in fp64",
           "layers": {}}
    stats = {}
    if not args.fresh and os.path.exists(path) and os.path.exists(path_s):
        with open(path) as fh:
            doc = json.load(fh)
        with np.load(path_s) as z:
            stats = {name: z[name] for name in z.files}
    for layer in layers:
        rec, s_arrays = layer_record(cfg, layer)
        doc["layers"][str(layer)] = rec
        stats.update(s_arrays)
        tmp = path + ".tmp"
        with open(tmp, "w") as fh:
            json.dump(doc, fh, indent=0, separators=(",", ":"))
        os.replace(tmp, path)
        tmp = path_s + ".tmp.npz"
        np.savez_compressed(tmp, **stats)
        os.replace(tmp, path_s)
    print("wrote", path, "and", path_s)


if __name__ == "__main__":
    main()
