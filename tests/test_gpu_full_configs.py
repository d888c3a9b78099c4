"""Parity at the full sizes of the named configs, in the launch configuration bench.py times.

The oracle's prompt phase at these sizes takes minutes to hours of fp64 loops, so what it yields is
stored under tests/golden/ by tests/golden/make_golden.py (which calls only oracle/ and the input
generator): the whole statistic s of every prompt (config<N>_s.npz, float64) and, per (layer,
sequence, k), the SHA-256 of the oracle's index array and the boundary gap (config<N>.json).
Here the HIP path runs on the same regenerated inputs and is compared element by element:
  * s over all of D_ff against the stored statistic (Eq. 6);
  * the selected indices against oracle.topk of the stored statistic, bit for bit (and that array
    against the stored SHA-256);
  * whole rows of Z, at token positions that straddle the tile boundaries, against oracle.ff1 (Eq. 3);
  * every decode output, the whole vector over D, against oracle.ff_decode run live on the oracle's
    own compact weights (Eq. 4-5), and the full-width block the same way (Eq. 1).
Every stored layer of configs 3 and 4 is run.
"""
import hashlib
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2404_01365_amd as G
import synth
from devio import dev_layer, empty_compact, max_rel, to_dev, to_host, workspace
from margin import boundary_report

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL_S = 2e-5
TOL_Z = 2e-5
TOL_OUT = 2e-2      # bf16 outputs: max error over the oracle's max |y|
DECODE_STEPS = 2


def load_golden(cid):
    path = os.path.join(GOLDEN, "config%d.json" % cid)
    path_s = os.path.join(GOLDEN, "config%d_s.npz" % cid)
    if not (os.path.exists(path) and os.path.exists(path_s)):
        pytest.skip("no stored oracle results for config %d" % cid)
    with open(path) as fh:
        return json.load(fh), np.load(path_s)


def sha_idx(a):
    return hashlib.sha256(np.ascontiguousarray(a, dtype="<i4").tobytes()).hexdigest()


def z_sample_rows(cu, total):
    """Token rows whose whole row of Z is compared: both ends of the packed prompt, both sides of the first
    tile boundaries, of one in the middle and of the last one, and each sequence's first and last token."""
    rows = {0, total - 1}
    for edge in (128, 256, 512, (total // 2) // 256 * 256, (total - 1) // 256 * 256):
        rows.update(r for r in (edge - 1, edge) if 0 <= r < total)
    for b in range(len(cu) - 1):
        if cu[b + 1] > cu[b]:
            rows.update((int(cu[b]), int(cu[b + 1]) - 1))
    return np.array(sorted(rows))


def check_layer(cfg, rec, stats):
    layer = rec["layer"]
    nudges = [(int(r), float(f)) for r, f in rec["nudges"]]
    Wg, W1, W2 = synth.layer_weights(cfg, layer, nudges=nudges)
    L, t = dev_layer(Wg, W1, W2, cfg.act, cfg.dtype)
    W64 = [np.ascontiguousarray(w, dtype=np.float64) for w in (Wg, W1, W2)]     # the oracle's inputs, widened once
    X, cu = synth.packed_prompts(cfg, layer)
    n_seqs, total = cfg.n_seqs, int(cu[-1])
    Xd = to_dev(X, cfg.dtype)
    Z = torch.empty((total, cfg.d_ff), dtype=torch.float32, device="cuda")
    ws = workspace(G.griffin_prefill_workspace_bytes(L, total, n_seqs, True))
    s = torch.empty((n_seqs, cfg.d_ff), dtype=torch.float32, device="cuda")
    xh = [synth.decode_inputs(cfg, layer, b, steps=DECODE_STEPS) for b in range(n_seqs)]
    xt = [to_dev(x, cfg.dtype) for x in xh]
    s_ref = [np.asarray(stats["l%d_b%d" % (layer, b)], dtype=np.float64) for b in range(n_seqs)]
    for ki, k in enumerate(cfg.ks):
        idx = torch.full((n_seqs, k), -1, dtype=torch.int32, device="cuda")
        G.griffin_prefill_select(L, Xd, [int(v) for v in cu], k, idx, s_out=s, Z_out=Z, workspace=ws)
        torch.cuda.synchronize()
        idx_h, s_h = idx.cpu().numpy(), s.cpu().numpy().astype(np.float64)
        if ki == 0:
            rows = z_sample_rows(cu, total)
            Z_ref = oracle.ff1(X[rows], Wg, W1, cfg.act)
            assert max_rel(Z[torch.from_numpy(rows).cuda()].cpu().numpy(), Z_ref) <= TOL_Z, (layer, "Z rows")
        idx_ref = []
        for b in range(n_seqs):
            g = rec["seqs"][b]
            gk = g["k"][str(k)]
            assert g["length"] == int(cu[b + 1] - cu[b])
            assert boundary_report(s_ref[b], k)[0] > 1e-3
            ir = oracle.topk(s_ref[b], k)
            assert sha_idx(ir) == gk["idx_sha256"] and ir[:8].tolist() == gk["idx_head"]
            idx_ref.append(ir)
            # the statistic, every entry (Eq. 6)
            assert np.max(np.abs(s_h[b] - s_ref[b])) <= TOL_S * np.max(s_ref[b]), (layer, b, k)
            assert np.sum(s_h[b] ** 2) == pytest.approx(g["length"], rel=1e-4)
            np.testing.assert_array_equal(idx_h[b], ir, err_msg="selected set differs: config %d layer %d seq %d k %d" % (cfg.cid, layer, b, k))
        Cs, keep = [], []
        for b in range(n_seqs):
            C, ct = empty_compact(L, k, t, interleaved=True)
            G.griffin_compact(L, idx[b], k, C)
            Cs.append(C); keep.append(ct)
        # the oracle's outputs through its own compact weights
        y_ref = np.empty((DECODE_STEPS, n_seqs, cfg.d))
        for b in range(n_seqs):
            cw = [oracle.compact(w, idx_ref[b]) for w in W64]
            for step in range(DECODE_STEPS):
                y_ref[step, b] = oracle.ff_decode(xh[b][step], *cw, cfg.act)
            del cw
        # decode through the compact blocks, one token at a time as in generation
        # (workspace sized for the whole block: with several sequences the index lists then take one masked pass over it)
        wsd = workspace(max(G.griffin_decode_workspace_bytes(cfg.d, k, max(n_seqs, 1)),
                            G.griffin_decode_workspace_bytes(cfg.d, cfg.d_ff, max(n_seqs, 1))))
        for step in range(DECODE_STEPS):
            ys = {}
            y1 = torch.empty((n_seqs, cfg.d), dtype=xt[0].dtype, device="cuda")
            for b in range(n_seqs):
                G.griffin_ff_decode(Cs[b], xt[b][step], y1[b], 1, workspace=wsd)
            ys["compact"] = to_host(y1)
            if n_seqs > 1:
                xb = torch.stack([xt[b][step] for b in range(n_seqs)])
                y2 = torch.empty_like(xb)
                G.griffin_ff_decode_multi(Cs, xb, y2, workspace=wsd)
                ys["multi"] = to_host(y2)
                y3 = torch.empty_like(xb)
                G.griffin_ff_decode_indexed(L, idx, k, n_seqs, xb, y3, workspace=wsd)
                ys["indexed"] = to_host(y3)
            torch.cuda.synchronize()
            for name, y in ys.items():
                for b in range(n_seqs):
                    err = max_rel(y[b], y_ref[step, b])          # all of D (Eq. 4-5)
                    assert err <= TOL_OUT, (name, layer, b, k, step, err)
        del Cs, keep
    # the full-width block (k = D_ff, Eq. 1) through the same decode entry point
    wsd = workspace(G.griffin_decode_workspace_bytes(cfg.d, cfg.d_ff, 1))
    for step in range(DECODE_STEPS):
        y = torch.empty((cfg.d,), dtype=xt[0].dtype, device="cuda")
        G.griffin_ff_decode(L, xt[0][step], y, 1, workspace=wsd)
        torch.cuda.synchronize()
        assert max_rel(to_host(y), oracle.ff_decode(xh[0][step], *W64, cfg.act)) <= TOL_OUT, (layer, "full width", step)


def test_config1_llama2_7b_shape():
    doc, stats = load_golden(1)
    check_layer(synth.CONFIGS[1], doc["layers"]["0"], stats)


def test_config2_gemma_7b_shape_three_keep_fractions():
    doc, stats = load_golden(2)
    check_layer(synth.CONFIGS[2], doc["layers"]["0"], stats)


def test_config3_llama2_13b_stack():
    doc, stats = load_golden(3)
    for layer in sorted(int(v) for v in doc["layers"]):
        print("config 3 layer %d" % layer, flush=True)
        check_layer(synth.CONFIGS[3], doc["layers"][str(layer)], stats)
        torch.cuda.empty_cache()


def test_config4_mistral_batched_per_sequence_sets():
    doc, stats = load_golden(4)
    for layer in sorted(int(v) for v in doc["layers"]):
        print("config 4 layer %d" % layer, flush=True)
        check_layer(synth.CONFIGS[4], doc["layers"][str(layer)], stats)
        torch.cuda.empty_cache()
