"""Seeded sweep of shapes through the HIP path against the oracle: ragged sizes around the tile,
chunk and wave boundaries of the kernels (multiples of 8 in d, anything in D_ff, k, lengths and
batch), gated and Eq. 2 blocks, with and without biases, all activations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_01365_amd as G
import synth
from devio import dev_layer, empty_compact, max_rel, to_dev, to_host, workspace
from margin import boundary_report

pytestmark = pytest.mark.gpu

TOL_OUT = {synth.DT_F32: 1e-5, synth.DT_BF16: 2e-2}
ACTS = (synth.ACT_SILU, synth.ACT_GELU_TANH, synth.ACT_RELU)


def _cases(seed, count, d_choices):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        out.append(dict(
            dtype=synth.DT_BF16 if rng.random() < 0.7 else synth.DT_F32,
            d=int(rng.choice(d_choices)),
            n=int(rng.integers(1, 700)),
            act=ACTS[int(rng.integers(0, 3))],
            gated=bool(rng.random() < 0.75),
            bias=bool(rng.random() < 0.4),
            batch=int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 33])),
            seed=int(rng.integers(1, 1 << 30)),
        ))
    return out


@pytest.mark.parametrize("c", _cases(101, 36, [8, 24, 64, 136, 256, 512, 520, 1024, 1536, 2048, 3072, 4096]),
                         ids=lambda c: "%s-d%d-n%d-b%d-%s%s" % ("bf16" if c["dtype"] == synth.DT_BF16 else "f32", c["d"], c["n"],
                                                                 c["batch"], "g" if c["gated"] else "u", "b" if c["bias"] else ""))
def test_decode_sweep(c):
    dtype, d, n, batch = c["dtype"], c["d"], c["n"], c["batch"]
    s = synth.small_case(c["seed"], d, n, 2, dtype, T=batch, with_bias=c["bias"])
    Wg = s["Wg"] if c["gated"] else None
    bg = s.get("bg") if c["gated"] else None
    L, t = dev_layer(Wg, s["W1"], s["W2"], c["act"], dtype, bg, s.get("b1"), s.get("b2"))
    x = to_dev(s["xt"], dtype)
    y = torch.empty_like(x)
    G.griffin_ff_decode(L, x, y, batch, workspace=workspace(G.griffin_decode_workspace_bytes(d, n, batch)))
    torch.cuda.synchronize()
    got = to_host(y)
    for b in range(batch):
        ref = oracle.ff_decode(s["xt"][b], Wg, s["W1"], s["W2"], c["act"], bg, s.get("b1"), s.get("b2"))
        assert max_rel(got[b], ref) <= TOL_OUT[dtype], (c, b)
    # the same rows through a compact block of a random subset
    k = max(1, n // 2)
    idx_h = np.sort(np.random.default_rng(c["seed"]).choice(n, k, replace=False)).astype(np.int32)
    C, keep = empty_compact(L, k, t, interleaved=bool(c["seed"] & 1))
    G.griffin_compact(L, torch.from_numpy(idx_h).cuda(), k, C)
    y2 = torch.empty_like(x)
    G.griffin_ff_decode(C, x, y2, batch, workspace=workspace(G.griffin_decode_workspace_bytes(d, k, batch)))
    torch.cuda.synchronize()
    got2 = to_host(y2)
    sub = lambda a: None if a is None else a[idx_h]
    for b in range(0, batch, 3):
        ref = oracle.ff_decode(s["xt"][b], sub(Wg), s["W1"][idx_h], s["W2"][idx_h], c["act"], sub(bg), sub(s.get("b1")), s.get("b2"))
        assert max_rel(got2[b], ref) <= TOL_OUT[dtype], (c, b)


def _prefill_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        n_seqs = int(rng.choice([1, 1, 2, 3, 5]))
        out.append(dict(
            dtype=synth.DT_BF16 if rng.random() < 0.75 else synth.DT_F32,
            d=int(rng.choice([8, 40, 64, 72, 128, 192, 256, 320, 512, 1024])),
            F=int(rng.integers(1, 600)),
            lens=[int(v) for v in rng.integers(0, 300, size=n_seqs)],
            act=ACTS[int(rng.integers(0, 3))],
            gated=bool(rng.random() < 0.75),
            bias=bool(rng.random() < 0.4),
            seed=int(rng.integers(1, 1 << 30)),
        ))
    return out


@pytest.mark.parametrize("c", _prefill_cases(202, 30),
                         ids=lambda c: "%s-d%d-F%d-%s-%s%s" % ("bf16" if c["dtype"] == synth.DT_BF16 else "f32", c["d"], c["F"],
                                                                "+".join(map(str, c["lens"])), "g" if c["gated"] else "u", "b" if c["bias"] else ""))
def test_prefill_sweep(c):
    dtype, d, F, lens = c["dtype"], c["d"], c["F"], c["lens"]
    total = sum(lens)
    s = synth.small_case(c["seed"], d, F, max(total, 1), dtype, with_bias=c["bias"])
    Wg = s["Wg"] if c["gated"] else None
    bg = s.get("bg") if c["gated"] else None
    b1 = s.get("b1")
    L, _ = dev_layer(Wg, s["W1"], s["W2"], c["act"], dtype, bg, b1)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    k = max(1, F // 3)
    n_seqs = len(lens)
    idx = torch.full((n_seqs, k), -1, dtype=torch.int32, device="cuda")
    sd = torch.empty((n_seqs, F), dtype=torch.float32, device="cuda")
    Z = torch.full((max(total, 1), F), float("nan"), dtype=torch.float32, device="cuda")
    G.griffin_prefill_select(L, to_dev(s["X"], dtype), [int(v) for v in cu], k, idx, s_out=sd, Z_out=Z,
                             workspace=workspace(G.griffin_prefill_workspace_bytes(L, total, n_seqs, True)))
    torch.cuda.synchronize()
    idx_h, s_h, Z_h = idx.cpu().numpy(), sd.cpu().numpy().astype(np.float64), Z.cpu().numpy().astype(np.float64)
    for b in range(n_seqs):
        if lens[b] == 0:
            assert np.all(s_h[b] == 0.0) and idx_h[b].tolist() == list(range(k))
            continue
        Xb = s["X"][cu[b]:cu[b + 1]]
        Z_ref = oracle.ff1(Xb, Wg, s["W1"], c["act"], bg, b1)
        assert max_rel(Z_h[cu[b]:cu[b + 1]], Z_ref) <= 2e-5, c
        s_ref = oracle.stat(Z_ref)
        if np.max(s_ref) > 0:
            assert np.max(np.abs(s_h[b] - s_ref)) <= 2e-5 * np.max(s_ref), c
        # selected set: exact where the oracle's boundary gap is open, else a valid top-k of the device's own s
        assert np.all(np.diff(idx_h[b]) > 0) and idx_h[b][0] >= 0 and idx_h[b][-1] < F
        if boundary_report(s_ref, k)[0] > 1e-3:
            np.testing.assert_array_equal(idx_h[b], oracle.topk(s_ref, k))
        elif k < F:
            assert np.min(s_h[b][idx_h[b]]) >= np.max(np.delete(s_h[b], idx_h[b]))


def _set_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        n = int(rng.integers(64, 1500))
        out.append(dict(
            d=int(rng.choice([512, 1024, 1536, 2560, 4096, 5120])),
            n=n,
            k=int(rng.integers(1, n + 1)),
            act=ACTS[int(rng.integers(0, 3))],
            gated=bool(rng.random() < 0.75),
            bias=bool(rng.random() < 0.4),
            batch=int(rng.choice([1, 2, 4, 5, 6, 16, 17, 40])),
            mode=str(rng.choice(["transposed", "masked", "indexed", "multi"])),
            seed=int(rng.integers(1, 1 << 30)),
        ))
    return out


@pytest.mark.parametrize("c", _set_cases(303, 28),
                         ids=lambda c: "%s-d%d-n%d-k%d-b%d-%s%s" % (c["mode"], c["d"], c["n"], c["k"], c["batch"],
                                                                     "g" if c["gated"] else "u", "b" if c["bias"] else ""))
def test_selected_set_decode_sweep(c):
    """Rows through their selected sets (Eq. 4-5) by every route the library has: a compact block that
    carries W2 in the paper's orientation (one row), index lists into the full block with the workspace
    of the masked pass or the smaller one, and one compact block per row."""
    dtype, d, n, k, B, act = synth.DT_BF16, c["d"], c["n"], c["k"], c["batch"], c["act"]
    s = synth.small_case(c["seed"], d, n, 2, dtype, T=B, with_bias=c["bias"])
    Wg = s["Wg"] if c["gated"] else None
    bg = s.get("bg") if c["gated"] else None
    b1, b2 = s.get("b1"), s.get("b2")
    L, t = dev_layer(Wg, s["W1"], s["W2"], act, dtype, bg, b1, b2)
    rng = np.random.default_rng(c["seed"])
    shared = c["mode"] == "transposed"
    sets = [np.sort(rng.choice(n, k, replace=False)).astype(np.int32) for _ in range(1 if shared else B)]
    x = to_dev(s["xt"], dtype)
    y = torch.full_like(x, float("nan"))
    keep = []
    if c["mode"] == "transposed":
        C, ct = empty_compact(L, k, t, interleaved=bool(c["seed"] & 1), transposed="only")
        G.griffin_compact(L, torch.from_numpy(sets[0]).cuda(), k, C)
        ws = workspace(G.griffin_decode_workspace_bytes(d, k, 1))
        for b in range(B):          # one row per call: the route that reads W2 in the paper's orientation
            G.griffin_ff_decode(C, x[b], y[b], 1, workspace=ws)
    elif c["mode"] == "multi":
        Cs = []
        for b in range(B):
            Cb, kb = empty_compact(L, k, t, interleaved=bool(c["seed"] & 1))
            G.griffin_compact(L, torch.from_numpy(sets[b]).cuda(), k, Cb)
            Cs.append(Cb); keep.append(kb)
        G.griffin_ff_decode_multi(Cs, x, y, workspace=workspace(G.griffin_decode_workspace_bytes(d, k, B)))
    else:
        idx = torch.from_numpy(np.stack(sets)).cuda()
        nbytes = G.griffin_decode_workspace_bytes(d, n if c["mode"] == "masked" else k, B)
        G.griffin_ff_decode_indexed(L, idx, k, B, x, y, workspace=workspace(nbytes))
    torch.cuda.synchronize()
    got = to_host(y)
    for b in range(B):
        e = sets[0] if shared else sets[b]
        sub = lambda a: None if a is None else a[e]
        ref = oracle.ff_decode(s["xt"][b], sub(Wg), s["W1"][e], s["W2"][e], act, sub(bg), sub(b1), b2)
        assert max_rel(got[b], ref) <= TOL_OUT[dtype], (c, b)


def _phase_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        n_seqs = int(rng.choice([1, 1, 2, 3]))
        F = int(rng.integers(1, 12)) * 64 if rng.random() < 0.6 else int(rng.integers(1, 700))
        out.append(dict(
            dtype=synth.DT_BF16 if rng.random() < 0.8 else synth.DT_F32,
            d=int(rng.choice([8, 64, 128, 192, 256, 384, 512, 1024])),
            F=F,
            lens=[int(v) for v in rng.integers(0, 400, size=n_seqs)],
            act=ACTS[int(rng.integers(0, 3))],
            gated=bool(rng.random() < 0.75),
            bias=bool(rng.random() < 0.3),
            seed=int(rng.integers(1, 1 << 30)),
        ))
    return out


@pytest.mark.parametrize("c", _phase_cases(404, 20),
                         ids=lambda c: "%s-d%d-F%d-%s-%s%s" % ("bf16" if c["dtype"] == synth.DT_BF16 else "f32", c["d"], c["F"],
                                                                "+".join(map(str, c["lens"])), "g" if c["gated"] else "u", "b" if c["bias"] else ""))
def test_prompt_phase_sweep(c):
    """Selection and the prompt's own output from one Z (Section 4.2 + Section 5.1), random shapes."""
    dtype, d, F, lens, act = c["dtype"], c["d"], c["F"], c["lens"], c["act"]
    total = sum(lens)
    s = synth.small_case(c["seed"], d, F, max(total, 1), dtype, with_bias=c["bias"])
    Wg = s["Wg"] if c["gated"] else None
    bg = s.get("bg") if c["gated"] else None
    b1, b2 = s.get("b1"), s.get("b2")
    L, _ = dev_layer(Wg, s["W1"], s["W2"], act, dtype, bg, b1, b2)
    W2p = to_dev(np.ascontiguousarray(s["W2"].T), dtype)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    k = max(1, F // 2)
    n_seqs = len(lens)
    idx = torch.full((n_seqs, k), -1, dtype=torch.int32, device="cuda")
    sd = torch.empty((n_seqs, F), dtype=torch.float32, device="cuda")
    Y = torch.full((max(total, 1), d), float("nan"), dtype=W2p.dtype, device="cuda")
    G.griffin_prompt_phase(L, W2p, to_dev(s["X"][:max(total, 1)], dtype), [int(v) for v in cu], k, idx, Y, s_out=sd,
                           workspace=workspace(G.griffin_prompt_phase_workspace_bytes(L, total, n_seqs)))
    torch.cuda.synchronize()
    idx_h, s_h = idx.cpu().numpy(), sd.cpu().numpy().astype(np.float64)
    if total > 0:
        Z_ref = oracle.ff1(s["X"][:total], Wg, s["W1"], act, bg, b1)
        assert max_rel(to_host(Y)[:total], oracle.ff2(Z_ref, s["W2"], b2)) <= TOL_OUT[dtype], c
    for b in range(n_seqs):
        if lens[b] == 0:
            assert np.all(s_h[b] == 0.0) and idx_h[b].tolist() == list(range(k))
            continue
        s_ref = oracle.stat(Z_ref[cu[b]:cu[b + 1]])
        if np.max(s_ref) > 0:
            assert np.max(np.abs(s_h[b] - s_ref)) <= 2e-5 * np.max(s_ref), c
        assert np.all(np.diff(idx_h[b]) > 0) and idx_h[b][0] >= 0 and idx_h[b][-1] < F
        if boundary_report(s_ref, k)[0] > 1e-3:
            np.testing.assert_array_equal(idx_h[b], oracle.topk(s_ref, k))
        elif k < F:
            assert np.min(s_h[b][idx_h[b]]) >= np.max(np.delete(s_h[b], idx_h[b]))
