"""The stored oracle results are well-formed and were made on inputs with a real top-k margin."""
import json
import os

import pytest

import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_stored_results_cover_the_config(cid):
    path = os.path.join(GOLDEN, "config%d.json" % cid)
    if not os.path.exists(path):
        pytest.skip("config %d not stored yet" % cid)
    doc = json.load(open(path))
    cfg = synth.CONFIGS[cid]
    assert doc["d"] == cfg.d and doc["d_ff"] == cfg.d_ff and tuple(doc["ks"]) == cfg.ks
    assert len(doc["layers"]) >= 1
    lens = synth.seq_lengths(cfg)
    for key, rec in doc["layers"].items():
        assert rec["layer"] == int(key) and 0 <= rec["layer"] < cfg.n_layers
        assert all(0 <= r < cfg.d_ff and 0.5 < f < 1.0 for r, f in rec["nudges"])
        assert len(rec["seqs"]) == cfg.n_seqs
        for b, sr in enumerate(rec["seqs"]):
            assert sr["length"] == lens[b]
            assert sr["sum_s2"] == pytest.approx(lens[b], rel=1e-9)     # unit rows: sum_j s_j^2 = S
            assert len(sr["s_samples"]) == len(rec["s_positions"])
            for k in cfg.ks:
                g = sr["k"][str(k)]
                assert g["margin"] > 1e-3, (cid, key, b, k)
                assert len(g["idx_sha256"]) == 64 and len(g["decode"]) >= 1
                assert g["idx_head"] == sorted(g["idx_head"])
