"""The stored oracle results are well-formed and were made on inputs with a real top-k margin."""
import hashlib
import json
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_stored_results_cover_the_config(cid):
    path = os.path.join(GOLDEN, "config%d.json" % cid)
    path_s = os.path.join(GOLDEN, "config%d_s.npz" % cid)
    if not (os.path.exists(path) and os.path.exists(path_s)):
        pytest.skip("config %d not stored yet" % cid)
    doc = json.load(open(path))
    stats = np.load(path_s)
    cfg = synth.CONFIGS[cid]
    assert doc["d"] == cfg.d and doc["d_ff"] == cfg.d_ff and tuple(doc["ks"]) == cfg.ks
    assert len(doc["layers"]) == cfg.n_layers
    lens = synth.seq_lengths(cfg)
    for key, rec in doc["layers"].items():
        assert rec["layer"] == int(key) and 0 <= rec["layer"] < cfg.n_layers
        assert all(0 <= r < cfg.d_ff and 0.9 < f < 1.1 for r, f in rec["nudges"])
        # the inputs stay the recipe's: only a few rows of W1 carry a nudge
        assert len({r for r, _ in rec["nudges"]}) < 0.02 * cfg.d_ff, (cid, key)
        assert len(rec["seqs"]) == cfg.n_seqs
        for b, sr in enumerate(rec["seqs"]):
            s = stats["l%s_b%d" % (key, b)]
            assert s.dtype == np.float64 and s.shape == (cfg.d_ff,) and np.all(s >= 0.0)
            assert sr["length"] == lens[b]
            assert sr["sum_s2"] == pytest.approx(lens[b], rel=1e-9)     # unit rows: sum_j s_j^2 = S
            assert float(np.sum(s ** 2)) == pytest.approx(lens[b], rel=1e-9)
            for k in cfg.ks:
                g = sr["k"][str(k)]
                assert g["margin"] > 2e-3, (cid, key, b, k)
                assert len(g["idx_sha256"]) == 64
                assert g["idx_head"] == sorted(g["idx_head"])


def test_stored_index_hash_is_the_oracle_topk_of_the_stored_statistic():
    doc = json.load(open(os.path.join(GOLDEN, "config1.json")))
    stats = np.load(os.path.join(GOLDEN, "config1_s.npz"))
    cfg = synth.CONFIGS[1]
    g = doc["layers"]["0"]["seqs"][0]["k"][str(cfg.k)]
    idx = oracle.topk(stats["l0_b0"], cfg.k)
    assert hashlib.sha256(np.ascontiguousarray(idx, dtype="<i4").tobytes()).hexdigest() == g["idx_sha256"]
    assert oracle.topk_margin(stats["l0_b0"], cfg.k) == pytest.approx(g["margin"], rel=1e-9)
