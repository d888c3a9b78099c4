"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on
seeded inputs small enough for the oracle to finish in seconds but spanning several tiles
and ragged tails.  Tolerances (max error over the oracle's inf-norm): outputs 1e-5 for fp32
and 2e-2 for bf16; indices bit-exact on inputs whose top-k margin was opened to > 1e-3.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_01365_amd as G
import synth
from devio import dev_layer, empty_compact, max_rel, round_like, to_dev, to_host, workspace
from margin import boundary_report, open_margin

pytestmark = pytest.mark.gpu

TOL_OUT = {synth.DT_F32: 1e-5, synth.DT_BF16: 2e-2}
# Z and s are fp32 on the device whatever the storage type; products of bf16 inputs are exact
# in fp32, so only the accumulation order and the fast exp differ from the oracle.
TOL_Z = 2e-5
TOL_S = 2e-5


def sync():
    torch.cuda.synchronize()


def run_prefill(L, X_dev, cu, k, want_z=True):
    n_seqs = len(cu) - 1
    total = int(cu[-1])
    idx = torch.full((n_seqs, k), -1, dtype=torch.int32, device="cuda")
    s = torch.full((n_seqs, L.n), -1.0, dtype=torch.float32, device="cuda")
    Z = torch.full((max(total, 1), L.n), float("nan"), dtype=torch.float32, device="cuda") if want_z else None
    ws = workspace(G.griffin_prefill_workspace_bytes(L, total, n_seqs, want_z))
    G.griffin_prefill_select(L, X_dev, [int(v) for v in cu], k, idx, s_out=s, Z_out=Z, workspace=ws)
    sync()
    return idx.cpu().numpy(), s.cpu().numpy().astype(np.float64), (None if Z is None else Z.cpu().numpy().astype(np.float64))


def run_decode(C, x_dev, batch=1):
    y = torch.empty_like(x_dev)
    ws = workspace(G.griffin_decode_workspace_bytes(C.d, C.n, batch))
    G.griffin_ff_decode(C, x_dev, y, batch, workspace=ws)
    sync()
    return to_host(y)


# ------------------------------------------------------------------ decode (full block = Eq. 1)
@pytest.mark.parametrize("dtype,d,n,act,gated,bias", [
    (synth.DT_F32, 256, 688, synth.ACT_SILU, True, False),        # config-0 shape
    (synth.DT_F32, 264, 77, synth.ACT_GELU_TANH, True, True),     # ragged chunks, few neurons
    (synth.DT_F32, 40, 9, synth.ACT_RELU, False, True),           # Eq. 2, fewer neurons than waves
    (synth.DT_BF16, 512, 1000, synth.ACT_SILU, True, False),
    (synth.DT_BF16, 520, 333, synth.ACT_GELU_TANH, True, True),   # ragged lanes
    (synth.DT_BF16, 3072, 257, synth.ACT_RELU, True, False),
    (synth.DT_BF16, 5120, 130, synth.ACT_SILU, False, True),      # widest register tiling in use
    (synth.DT_BF16, 6144, 64, synth.ACT_SILU, True, False),
    (synth.DT_BF16, 8192, 40, synth.ACT_GELU_TANH, True, True),   # widest row this build covers
    (synth.DT_BF16, 8, 5, synth.ACT_SILU, True, False),           # one 16-byte chunk per row
    (synth.DT_F32, 4096, 33, synth.ACT_SILU, True, False),        # 16 waves per team
])
def test_ff_decode_matches_oracle(dtype, d, n, act, gated, bias):
    c = synth.small_case(d * 7 + n, d, n, 4, dtype, T=3, with_bias=bias)
    Wg = c["Wg"] if gated else None
    bg = c.get("bg") if gated else None
    L, _ = dev_layer(Wg, c["W1"], c["W2"], act, dtype, bg, c.get("b1"), c.get("b2"))
    for t in range(3):
        ref = oracle.ff_decode(c["xt"][t], Wg, c["W1"], c["W2"], act, bg, c.get("b1"), c.get("b2"))
        got = run_decode(L, to_dev(c["xt"][t], dtype))
        assert max_rel(got, ref) <= TOL_OUT[dtype], (dtype, d, n, t)


@pytest.mark.parametrize("dtype,d,n,batch,bias", [
    (synth.DT_BF16, 1024, 300, 5, False),     # 4 rows per pass + a ragged group
    (synth.DT_BF16, 4096, 96, 2, True),       # 2 rows per pass
    (synth.DT_BF16, 3072, 130, 16, False),
    (synth.DT_F32, 264, 77, 7, True),
    (synth.DT_BF16, 4096, 1001, 16, True),    # matrix-core path: odd neuron count, biases
    (synth.DT_BF16, 2048, 777, 9, False),     # matrix-core path: 9 of 16 rows used
    (synth.DT_BF16, 512, 64, 40, False),      # matrix-core path: three groups of rows (16 + 16 + 8)
    (synth.DT_BF16, 5120, 200, 16, False),    # matrix-core path: 10 slices per row
    (synth.DT_BF16, 8192, 100, 8, False),     # 16 slices per row: stays on the four-rows-per-pass path
])
def test_ff_decode_batch_shares_one_block(dtype, d, n, batch, bias):
    c = synth.small_case(5 + batch, d, n, 4, dtype, T=batch, with_bias=bias)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, dtype, c.get("bg"), c.get("b1"), c.get("b2"))
    x = to_dev(c["xt"], dtype)
    got = run_decode(L, x, batch=batch)
    for t in range(batch):
        ref = oracle.ff_decode(c["xt"][t], c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, c.get("bg"), c.get("b1"), c.get("b2"))
        assert max_rel(got[t], ref) <= TOL_OUT[dtype], t
        # a row alone gives the same result up to the order of the fp32 partial sums (the
        # number of partial rows depends on the batch size)
        assert max_rel(got[t], run_decode(L, x[t:t + 1].contiguous(), batch=1)[0]) <= (2.0 ** -7 if dtype == synth.DT_BF16 else 1e-6)
    # deterministic: a second run gives the same bits
    assert np.array_equal(got, run_decode(L, x, batch=batch))


@pytest.mark.parametrize("gated,interleaved", [(True, True), (False, False), (False, True)])
def test_ff_decode_batch_matrix_core_path_layouts(gated, interleaved):
    """16 rows through one block on the matrix-core path: Eq. 2 blocks and the interleaved compact layout."""
    d, n, batch = 1024, 500, 16
    c = synth.small_case(91, d, n, 4, synth.DT_BF16, T=batch)
    Wg = c["Wg"] if gated else None
    L, t = dev_layer(Wg, c["W1"], c["W2"], synth.ACT_GELU_TANH, synth.DT_BF16)
    k = 300
    idx_h = np.sort(np.random.default_rng(4).choice(n, k, replace=False)).astype(np.int32)
    idx = torch.from_numpy(idx_h).cuda()
    C, keep = empty_compact(L, k, t, interleaved=interleaved)
    G.griffin_compact(L, idx, k, C)
    x = to_dev(c["xt"], synth.DT_BF16)
    got = run_decode(C, x, batch=batch)
    for b in range(batch):
        ref = oracle.ff_decode(c["xt"][b], None if Wg is None else Wg[idx_h], c["W1"][idx_h], c["W2"][idx_h], synth.ACT_GELU_TANH)
        assert max_rel(got[b], ref) <= TOL_OUT[synth.DT_BF16], b


# ------------------------------------------------------------------ blocks that carry W2 in the paper's orientation
@pytest.mark.parametrize("d,n,k,gated,bias,mode,interleaved", [
    (1024, 700, 333, True, False, "only", True),      # k not a multiple of anything, two teams... of two waves
    (4096, 600, 600, True, True, "both", False),      # keep all, biases, eight waves per team
    (512, 2000, 1025, False, True, "only", False),    # Eq. 2 block, one wave per team, padding of 511 columns
    (5120, 300, 64, True, False, "only", True),       # ten waves per team
    (3072, 1000, 512, True, False, "both", True),     # k exactly one slice
])
def test_decode_through_transposed_w2_matches_oracle(d, n, k, gated, bias, mode, interleaved):
    dtype, act = synth.DT_BF16, synth.ACT_SILU
    c = synth.small_case(d + n + k, d, n, 4, dtype, T=3, with_bias=bias)
    Wg = c["Wg"] if gated else None
    bg = c.get("bg") if gated else None
    L, t = dev_layer(Wg, c["W1"], c["W2"], act, dtype, bg, c.get("b1"), c.get("b2"))
    idx_h = np.sort(np.random.default_rng(k).choice(n, k, replace=False)).astype(np.int32)
    idx = torch.from_numpy(idx_h).cuda()
    C, ct = empty_compact(L, k, t, interleaved=interleaved, transposed=mode)
    G.griffin_compact(L, idx, k, C)
    sync()
    # the transposed copy is the gathered W2 turned round, bit for bit, zero-padded
    W2t = ct["W2t"].view(torch.int16).cpu().numpy().view(np.uint16)
    ref_bits = synth.bf16_bits(c["W2"][idx_h]).T
    assert np.array_equal(W2t[:, :k], ref_bits) and not W2t[:, k:].any()
    sub = lambda a: None if a is None else a[idx_h]
    for step in range(3):
        got = run_decode(C, to_dev(c["xt"][step], dtype))
        ref = oracle.ff_decode(c["xt"][step], sub(Wg), c["W1"][idx_h], c["W2"][idx_h], act, sub(bg), sub(c.get("b1")), c.get("b2"))
        assert max_rel(got, ref) <= TOL_OUT[dtype], step
    if mode == "both":
        # a batch of rows through the same block takes the neuron-major copy
        xb = to_dev(c["xt"], dtype)
        gotb = run_decode(C, xb, batch=3)
        for b in range(3):
            ref = oracle.ff_decode(c["xt"][b], sub(Wg), c["W1"][idx_h], c["W2"][idx_h], act, sub(bg), sub(c.get("b1")), c.get("b2"))
            assert max_rel(gotb[b], ref) <= TOL_OUT[dtype]


def test_decode_through_transposed_w2_reuses_a_workspace_with_anything_in_it():
    """The workspace (z between the two streams) may hold anything at first use, and the same workspace
    serves call after call on one stream with no synchronisation in between (Eq. 4-5, one row)."""
    dtype, act, d, n, k = synth.DT_BF16, synth.ACT_SILU, 2048, 900, 450
    c = synth.small_case(77, d, n, 4, dtype, T=6)
    L, t = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype)
    idx_h = np.sort(np.random.default_rng(8).choice(n, k, replace=False)).astype(np.int32)
    C, ct = empty_compact(L, k, t, interleaved=True, transposed="only")
    G.griffin_compact(L, torch.from_numpy(idx_h).cuda(), k, C)
    nbytes = G.griffin_decode_workspace_bytes(C.d, C.n, 1)
    for fill in (0xFF, 0x00, 0x5A):
        ws = workspace(nbytes)
        ws.view(torch.uint8).fill_(fill)
        ys = [torch.empty(d, dtype=torch.bfloat16, device="cuda") for _ in range(6)]
        for step in range(6):           # back to back on one stream, no synchronisation in between
            G.griffin_ff_decode(C, to_dev(c["xt"][step], dtype), ys[step], 1, workspace=ws)
        sync()
        for step in range(6):
            ref = oracle.ff_decode(c["xt"][step], c["Wg"][idx_h], c["W1"][idx_h], c["W2"][idx_h], act)
            assert max_rel(to_host(ys[step]), ref) <= TOL_OUT[dtype], (fill, step)


@pytest.mark.parametrize("d,n,k,B", [(1024, 700, 300, 19), (512, 9000, 150, 6), (1024, 300, 100, 3)])
def test_indexed_decode_with_sets_built_once(d, n, k, B):
    """The membership words built once per prompt (the sets stay fixed during generation, Section 4.2)
    give, token after token, bit for bit what griffin_ff_decode_indexed gives, and the oracle's result;
    with fewer than five rows the index lists are used and the words are not read."""
    dtype, act = synth.DT_BF16, synth.ACT_SILU
    T = 3
    c = synth.small_case(d + n + B, d, n, 4, dtype, T=B * T)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype)
    rng = np.random.default_rng(B)
    idx = np.stack([np.sort(rng.choice(n, k, replace=False)) for _ in range(B)]).astype(np.int32)
    idx_dev = torch.from_numpy(idx).cuda()
    sets = torch.full((G.griffin_index_sets_bytes(n, B) // 4,), -1, dtype=torch.int32, device="cuda")
    G.griffin_index_sets_build(idx_dev, k, B, n, sets)
    sync()
    # the words themselves: bit b of word j of group g <=> neuron j in the set of row 16 g + b
    words = sets.cpu().numpy().view(np.uint32).reshape(-1, n)
    want = np.zeros_like(words)
    for b in range(B):
        want[b // 16, idx[b]] |= np.uint32(1 << (b % 16))
    assert np.array_equal(words, want)
    ws = workspace(G.griffin_decode_workspace_bytes(d, n, B))
    for t in range(T):
        x = to_dev(c["xt"][t * B:(t + 1) * B], dtype)
        y1, y2 = torch.empty_like(x), torch.empty_like(x)
        G.griffin_ff_decode_indexed_sets(L, idx_dev, k, sets, B, x, y1, workspace=ws)
        G.griffin_ff_decode_indexed(L, idx_dev, k, B, x, y2, workspace=ws)
        sync()
        assert np.array_equal(to_host(y1), to_host(y2)), t
        for b in range(0, B, 4):
            ref = oracle.ff_decode(c["xt"][t * B + b], c["Wg"][idx[b]], c["W1"][idx[b]], c["W2"][idx[b]], act)
            assert max_rel(to_host(y1)[b], ref) <= TOL_OUT[dtype], (t, b)


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
def test_compact_is_a_bit_exact_row_gather(dtype, interleaved):
    d, n, k = 264, 301, 97
    c = synth.small_case(11, d, n, 4, dtype, with_bias=True)
    L, t = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, dtype, c["bg"], c["b1"], c["b2"])
    idx = np.sort(np.random.default_rng(3).choice(n, k, replace=False)).astype(np.int32)
    C, ct = empty_compact(L, k, t, interleaved)
    G.griffin_compact(L, torch.from_numpy(idx).cuda(), k, C)
    sync()
    for name in ("Wg", "W1", "W2", "bg", "b1"):
        assert np.array_equal(to_host(ct[name]), oracle.compact(c[name], idx)), name
    # pruned decode through the compact block = oracle on the oracle's compact weights
    x = c["xt"][0]
    ref = oracle.ff_decode(x, *(oracle.compact(c[m], idx) for m in ("Wg", "W1", "W2")), synth.ACT_SILU,
                           oracle.compact(c["bg"], idx), oracle.compact(c["b1"], idx), c["b2"])
    assert max_rel(run_decode(C, to_dev(x, dtype)), ref) <= TOL_OUT[dtype]


def test_keep_all_equals_full_block_bitwise_on_device():
    dtype, d, n = synth.DT_BF16, 512, 200
    c = synth.small_case(12, d, n, 4, dtype)
    L, t = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, dtype)
    C, _ = empty_compact(L, n, t)
    G.griffin_compact(L, torch.arange(n, dtype=torch.int32, device="cuda"), n, C)
    x = to_dev(c["xt"][0], dtype)
    assert np.array_equal(run_decode(L, x), run_decode(C, x))


def test_indexed_and_multi_decode_match_compact_decode():
    dtype, d, n, k, B = synth.DT_BF16, 1024, 500, 250, 3
    c = synth.small_case(13, d, n, 4, dtype, T=B, with_bias=True)
    L, t = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_GELU_TANH, dtype, c["bg"], c["b1"], c["b2"])
    rng = np.random.default_rng(4)
    idx = np.stack([np.sort(rng.choice(n, k, replace=False)) for _ in range(B)]).astype(np.int32)
    idx_dev = torch.from_numpy(idx).cuda()
    x = to_dev(c["xt"], dtype)
    refs = []
    for b in range(B):
        cw = [oracle.compact(c[m], idx[b]) for m in ("Wg", "W1", "W2")]
        refs.append(oracle.ff_decode(c["xt"][b], *cw, synth.ACT_GELU_TANH, oracle.compact(c["bg"], idx[b]),
                                     oracle.compact(c["b1"], idx[b]), c["b2"]))
    ws = workspace(G.griffin_decode_workspace_bytes(d, k, B))
    y = torch.empty_like(x)
    G.griffin_ff_decode_indexed(L, idx_dev, k, B, x, y, workspace=ws)
    sync()
    y_idx = to_host(y)
    Cs, keep = [], []
    for b in range(B):
        C, ct = empty_compact(L, k, t)
        G.griffin_compact(L, idx_dev[b], k, C)
        Cs.append(C); keep.append(ct)
    y2 = torch.empty_like(x)
    G.griffin_ff_decode_multi(Cs, x, y2, workspace=ws)
    sync()
    y_multi = to_host(y2)
    for b in range(B):
        assert max_rel(y_idx[b], refs[b]) <= TOL_OUT[dtype]
        assert max_rel(y_multi[b], refs[b]) <= TOL_OUT[dtype]
    assert np.array_equal(y_idx, y_multi)   # same rows, same order of operations


# ------------------------------------------------------------------ top-k
@pytest.mark.parametrize("n,k", [(1, 1), (7, 3), (64, 64), (688, 344), (1000, 1), (5000, 4999), (24576, 12288),
                                 (8200, 4100), (36864, 20000), (40000, 777)])   # 8 loads + tail; the largest cached row; uncached
def test_topk_matches_oracle(n, k):
    rng = np.random.default_rng(n * 31 + k)
    rows = 3
    s = rng.random((rows, n)).astype(np.float32)
    s[1] = np.round(s[1] * 8) / 8          # many exact ties, also across the boundary
    s[2, : n // 2] = 0.0                   # zeros (an empty-prompt statistic is all zero)
    out = torch.full((rows, k), -1, dtype=torch.int32, device="cuda")
    G.griffin_topk(torch.from_numpy(s).cuda(), k, out)
    sync()
    got = out.cpu().numpy()
    for r in range(rows):
        np.testing.assert_array_equal(got[r], oracle.topk(s[r], k))


def test_stat_shared_matches_oracle():
    rng = np.random.default_rng(8)
    n, B = 1000, 4
    s = rng.random((B, n)).astype(np.float32)
    cu = [0, 10, 10, 74, 300]                # one empty sequence: skipped
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    G.griffin_stat_shared(torch.from_numpy(s).cuda(), cu, out)
    sync()
    keep = [0, 2, 3]
    ref = oracle.stat_shared(s[keep], np.array([10, 64, 226]))
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-6)


# ------------------------------------------------------------------ prefill: Z, s, indices
PREFILL_CASES = [
    # dtype, d, F, lens, k, act, gated, bias
    (synth.DT_F32, 256, 688, [64], 344, synth.ACT_SILU, True, False),            # config 0 shape
    (synth.DT_F32, 72, 150, [70, 1, 33], 40, synth.ACT_GELU_TANH, True, True),   # ragged tiles, 3 seqs
    (synth.DT_F32, 64, 130, [9], 130, synth.ACT_RELU, False, True),              # Eq. 2, keep all
    (synth.DT_BF16, 512, 1000, [300], 500, synth.ACT_SILU, True, False),         # 3 x 8 tiles, ragged both
    (synth.DT_BF16, 136, 260, [129, 0, 200], 77, synth.ACT_GELU_TANH, True, True),  # k tail, empty seq
    (synth.DT_BF16, 256, 384, [256], 100, synth.ACT_RELU, False, False),         # Eq. 2 on the MFMA path
    (synth.DT_BF16, 64, 131, [1, 2, 130], 7, synth.ACT_SILU, True, False),       # one-token prompts, D_ff odd, KT = 2
    (synth.DT_BF16, 32, 40, [5], 40, synth.ACT_GELU_TANH, True, True),           # a single k-tile, keep all
    (synth.DT_BF16, 1024, 2500, [700], 1, synth.ACT_SILU, True, False),          # k = 1, three 256-token tiles
    (synth.DT_BF16, 64, 16520, [300], 8000, synth.ACT_RELU, False, True),        # Eq. 2 with biases, enough tiles for the
                                                                                 # 256-column tiles; the last tile 136 wide
    (synth.DT_BF16, 64, 33000, [100], 3000, synth.ACT_GELU_TANH, False, False),  # the same with 128-token tiles, last tile 232 wide
]


@pytest.mark.parametrize("dtype,d,F,lens,k,act,gated,bias", PREFILL_CASES)
def test_prefill_select_matches_oracle(dtype, d, F, lens, k, act, gated, bias):
    seed = d * 13 + F
    c = synth.small_case(seed, d, F, max(sum(lens), 1), dtype, with_bias=bias)
    Wg = c["Wg"] if gated else None
    bg = c.get("bg") if gated else None
    b1 = c.get("b1")
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    Xs = [c["X"][cu[b]:cu[b + 1]] for b in range(len(lens))]
    live = [b for b in range(len(lens)) if lens[b] > 0]
    W1 = c["W1"].copy()
    nudges, s_ref_live = open_margin([Xs[b] for b in live], Wg, W1, act, dtype, [k], bg, b1)
    L, _ = dev_layer(Wg, W1, c["W2"], act, dtype, bg, b1, c.get("b2"))
    idx, s, Z = run_prefill(L, to_dev(c["X"], dtype), cu, k)
    for pos, b in enumerate(live):
        s_ref = s_ref_live[pos]
        Z_ref = oracle.ff1(Xs[b], Wg, W1, act, bg, b1)
        gap, _ = boundary_report(s_ref, k)
        assert gap > 1e-3
        assert max_rel(Z[cu[b]:cu[b + 1]], Z_ref) <= TOL_Z
        assert max_rel(s[b], s_ref) <= TOL_S
        assert np.sum(s[b] ** 2) == pytest.approx(lens[b], rel=1e-4)     # unit rows: sum s^2 = S
        np.testing.assert_array_equal(idx[b], oracle.topk(s_ref, k))
    for b in range(len(lens)):
        if lens[b] == 0:
            assert np.all(s[b] == 0.0)
            np.testing.assert_array_equal(idx[b], np.arange(k))


# ------------------------------------------------------------------ prefill: workgroups that walk several tiles
# The matrix-core kernel runs one workgroup per CU; with more tiles than CUs (every full-size config) each
# workgroup walks through several tiles, sends the next tile's first loads before the epilogue of the
# current one and decides from the kind of tile it just finished (whole, or ragged in tokens or neurons)
# how many stores may still be outstanding when it starts to read.  These cases have 280 to 780 tiles at a
# small model width, so that the oracle stays cheap, two or three k-tiles, ragged last tiles in both
# directions, and a token-tile count coprime to the walking stride so that whole and ragged tiles alternate
# within one workgroup.
WALK_CASES = [
    # dtype, d, F, lens, k, act, gated, bias
    (synth.DT_BF16, 192, 11000, [1700], 5500, synth.ACT_SILU, True, False),        # 7 x 86 = 602 tiles, lean kernel
    (synth.DT_BF16, 128, 11000, [900, 800], 4000, synth.ACT_GELU_TANH, True, True),  # the same walk with biases, two prompts
    (synth.DT_BF16, 128, 16600, [1000], 8000, synth.ACT_RELU, False, True),        # Eq. 2, 128-column tiles: 4 x 130 = 520
    (synth.DT_BF16, 128, 16520, [1300], 8000, synth.ACT_GELU_TANH, False, True),   # Eq. 2, 256-column tiles: 6 x 65 = 390
    (synth.DT_BF16, 128, 33000, [100], 9000, synth.ACT_SILU, True, False),         # 128-token tiles: 258 of them, lean
    (synth.DT_BF16, 64, 40000, [128], 20000, synth.ACT_SILU, True, True),          # 128-token tiles with biases: 313
    (synth.DT_BF16, 64, 66000, [90], 30000, synth.ACT_RELU, False, False),         # Eq. 2, 128-token tiles, 516 narrow tiles
    (synth.DT_BF16, 64, 128000, [70], 50000, synth.ACT_SILU, False, True),         # Eq. 2, 128-token tiles, 500 wide tiles
    # more than eight token tiles: the tiles are walked in panels of eight token tiles, the last panel narrower
    (synth.DT_BF16, 64, 4000, [1500, 1190], 2000, synth.ACT_SILU, True, False),    # 11 x 32 = 352 tiles: one panel of 8, one of 3, ragged both ways
    (synth.DT_BF16, 64, 2100, [4100], 1000, synth.ACT_GELU_TANH, True, True),      # 17 x 17 = 289 tiles: two panels of 8, one of 1
    (synth.DT_BF16, 64, 2500, [2560], 1200, synth.ACT_RELU, False, True),          # Eq. 2, wide tiles: 10 x 10 = 100 tiles, panels of 8 and 2, no walk
    # Z of 406 MB, more than the product keeps in the caches: it leaves through the streaming stores (24 x 130 tiles)
    (synth.DT_BF16, 64, 16640, [3100, 3000], 8000, synth.ACT_SILU, True, False),
]


@pytest.mark.parametrize("dtype,d,F,lens,k,act,gated,bias", WALK_CASES)
def test_prefill_select_when_workgroups_walk_tiles(dtype, d, F, lens, k, act, gated, bias):
    test_prefill_select_matches_oracle(dtype, d, F, lens, k, act, gated, bias)


@pytest.mark.parametrize("d,F,lens,k,gated,bias", [
    (192, 11000, [1700], 5000, True, False),     # the first product leaves the bf16 copy of Z while it walks 602 tiles
    (128, 11000, [1000, 700], 5000, True, True), # the same with biases
    (64, 40000, [100], 20000, True, False),      # 128-token tiles, 313 of them
])
def test_prompt_phase_when_workgroups_walk_tiles(d, F, lens, k, gated, bias):
    test_prompt_phase_is_selection_plus_prompt_output_from_one_z(synth.DT_BF16, d, F, lens, k, gated, bias)


@pytest.mark.parametrize("d,F,S,bias", [
    (4200, 320, 6000, True),      # 24 x 17 = 408 output tiles of 256 x 256, five k-tiles, ragged in both directions
    (66000, 128, 100, False),     # a 128-token tile and 258 feature tiles
    (5000, 8192, 3300, True),     # the contraction cut into ranges AND more work items than CUs
])
def test_prompt_output_when_workgroups_walk_tiles(d, F, S, bias):
    """The second product of the prompt phase (Section 5.1) on the same kernel in its plain mode."""
    dtype = synth.DT_BF16
    g = np.random.default_rng(d + F + S)
    Z = (g.standard_normal((S, F)) * (g.random((S, F)) < 0.7)).astype(np.float32)
    W2 = synth.round_to_bf16((g.standard_normal((F, d)) * F ** -0.5).astype(np.float32))     # neuron-major
    b2 = synth.round_to_bf16((g.standard_normal(d) * 0.1).astype(np.float32)) if bias else None
    W2p = to_dev(np.ascontiguousarray(W2.T), dtype)
    Y = torch.full((S, d), float("nan"), dtype=W2p.dtype, device="cuda")
    G.griffin_ff_prompt_out(torch.from_numpy(Z).cuda(), W2p, Y, b2=to_dev(b2, dtype),
                            workspace=workspace(G.griffin_prompt_out_workspace_bytes(S, F, d)))
    sync()
    got = to_host(Y)
    assert np.all(np.isfinite(got))
    # rows of Y are independent (Eq. 1 row-wise): where the oracle's plain loops would take minutes for all
    # of them, every 11th token goes through it (some of every token tile, at all lane positions), whole rows
    rows = np.arange(S) if S * F * d < 2e10 else np.arange(0, S, 11)
    # the device rounds Z to bf16 on its way into the matrix cores: the reference does the same rounding
    # and nothing else (fp64 sums), so what is left is the rounding of Y itself
    Y_ref = oracle.ff2(synth.round_to_bf16(Z[rows]).astype(np.float64), W2, b2)
    assert max_rel(got[rows], Y_ref) <= 2.0 ** -8
    if rows.size == S:          # and against the unrounded Z, at the tolerance of the outputs
        assert max_rel(got, oracle.ff2(Z.astype(np.float64), W2, b2)) <= TOL_OUT[dtype]


def test_prefill_with_biases_at_odd_addresses():
    """Biases need no alignment beyond their element size: vectors that start 2 bytes past an 8-byte boundary
    take the element-wise store path of the first product and give the same sets and statistic."""
    dtype, d, F, S, k, act = synth.DT_BF16, 256, 512, 200, 200, synth.ACT_SILU
    c = synth.small_case(91, d, F, S, dtype, with_bias=True)
    W1 = c["W1"].copy()
    _, (s_ref,) = open_margin([c["X"]], c["Wg"], W1, act, dtype, [k], c["bg"], c["b1"])
    L, t = dev_layer(c["Wg"], W1, c["W2"], act, dtype, c["bg"], c["b1"], c["b2"])
    idx_a, s_a, Z_a = run_prefill(L, to_dev(c["X"], dtype), [0, S], k)
    # the same biases one element into a larger buffer
    shift = lambda v: torch.cat([torch.zeros(1, dtype=v.dtype, device="cuda"), v])[1:]
    bg2, b12 = shift(t["bg"]), shift(t["b1"])
    assert bg2.data_ptr() % 8 == 2 and b12.data_ptr() % 8 == 2
    L2 = G.layer(t["W1"], t["W2"], t["Wg"], act=act, bg=bg2, b1=b12, b2=t["b2"])
    idx_b, s_b, Z_b = run_prefill(L2, to_dev(c["X"], dtype), [0, S], k)
    np.testing.assert_array_equal(idx_a[0], oracle.topk(s_ref, k))
    np.testing.assert_array_equal(idx_b[0], idx_a[0])
    assert max_rel(s_b[0], s_ref) <= TOL_S and max_rel(Z_b, Z_a) <= 1e-6


def test_prefill_without_z_out_and_zero_row():
    dtype, d, F, S, k = synth.DT_F32, 64, 96, 20, 30
    c = synth.small_case(77, d, F, S, dtype)
    X = c["X"].copy()
    X[5] = 0.0                               # FF_1(0) = 0 without biases: an all-zero row of Z
    W1 = c["W1"].copy()
    _, (s_ref,) = open_margin([X], c["Wg"], W1, synth.ACT_SILU, dtype, [k])
    L, _ = dev_layer(c["Wg"], W1, c["W2"], synth.ACT_SILU, dtype)
    idx, s, Z = run_prefill(L, to_dev(X, dtype), [0, S], k, want_z=False)
    assert Z is None and np.all(np.isfinite(s))
    assert np.sum(s[0] ** 2) == pytest.approx(S - 1, rel=1e-4)
    assert max_rel(s[0], s_ref) <= TOL_S
    np.testing.assert_array_equal(idx[0], oracle.topk(s_ref, k))


# ------------------------------------------------------------------ config 0 end to end
def test_config0_end_to_end():
    cfg = synth.CONFIGS[0]
    Wg, W1, W2 = synth.layer_weights(cfg, 0)
    X = synth.prompt(cfg, 0)
    nudges, (s_ref,) = open_margin([X], Wg, W1, cfg.act, cfg.dtype, [cfg.k])
    idx_ref = oracle.topk(s_ref, cfg.k)
    L, t = dev_layer(Wg, W1, W2, cfg.act, cfg.dtype)
    idx, s, _ = run_prefill(L, to_dev(X, cfg.dtype), [0, cfg.prompt_len], cfg.k)
    np.testing.assert_array_equal(idx[0], idx_ref)
    assert max_rel(s[0], s_ref) <= TOL_S
    C, ct = empty_compact(L, cfg.k, t, interleaved=True)
    G.griffin_compact(L, torch.from_numpy(idx[0]).cuda(), cfg.k, C)
    cw = [oracle.compact(w, idx_ref) for w in (Wg, W1, W2)]
    xt = synth.decode_inputs(cfg, 0)
    for step in range(cfg.decode_steps):
        ref = oracle.ff_decode(xt[step], *cw, cfg.act)
        got = run_decode(C, to_dev(xt[step], cfg.dtype))
        assert max_rel(got, ref) <= TOL_OUT[cfg.dtype]
        full = oracle.ff_decode(xt[step], Wg, W1, W2, cfg.act)
        assert max_rel(run_decode(L, to_dev(xt[step], cfg.dtype)), full) <= TOL_OUT[cfg.dtype]


# ------------------------------------------------------------------ one shared set for a batch (Eq. 7)
def test_shared_set_for_a_batch_end_to_end():
    """Section 5.3: the samples of a batch are aggregated with s_bar = sum_b s_b / sqrt(S_b), one
    set is selected and every row decodes through the same compact block."""
    dtype, d, F, k, act = synth.DT_BF16, 512, 1200, 600, synth.ACT_SILU
    lens = [40, 170, 90, 300, 64]
    B = len(lens)
    c = synth.small_case(4242, d, F, sum(lens), dtype, T=B)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    Xs = [c["X"][cu[b]:cu[b + 1]] for b in range(B)]
    W1 = c["W1"].copy()
    shared = lambda s_list: [oracle.stat_shared(np.stack(s_list), np.array(lens))]
    _, s_list = open_margin(Xs, c["Wg"], W1, act, dtype, [k], combine=shared)
    sbar_ref = shared(s_list)[0]
    assert boundary_report(sbar_ref, k)[0] > 1e-3
    idx_ref = oracle.topk(sbar_ref, k)

    L, t = dev_layer(c["Wg"], W1, c["W2"], act, dtype)
    idx_seq = torch.empty((B, k), dtype=torch.int32, device="cuda")
    s_dev = torch.empty((B, F), dtype=torch.float32, device="cuda")
    ws = workspace(G.griffin_prefill_workspace_bytes(L, int(cu[-1]), B, False))
    G.griffin_prefill_select(L, to_dev(c["X"], dtype), [int(v) for v in cu], k, idx_seq, s_out=s_dev, workspace=ws)
    sbar = torch.empty((F,), dtype=torch.float32, device="cuda")
    G.griffin_stat_shared(s_dev, [int(v) for v in cu], sbar)
    idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
    G.griffin_topk(sbar, k, idx)
    sync()
    assert max_rel(sbar.cpu().numpy(), sbar_ref) <= TOL_S
    np.testing.assert_array_equal(idx.cpu().numpy()[0], idx_ref)

    C, _ = empty_compact(L, k, t, interleaved=True)
    G.griffin_compact(L, idx, k, C)
    got = run_decode(C, to_dev(c["xt"], dtype), batch=B)
    cw = [oracle.compact(w, idx_ref) for w in (c["Wg"], W1, c["W2"])]
    for b in range(B):
        assert max_rel(got[b], oracle.ff_decode(c["xt"][b], *cw, act)) <= TOL_OUT[dtype]


# ------------------------------------------------------------------ the prompt's own output (full block)
@pytest.mark.parametrize("dtype,d,F,S,bias", [
    (synth.DT_BF16, 512, 1000, 300, True),     # MFMA tiles, ragged in every dimension
    (synth.DT_BF16, 256, 4096, 40, True),      # direct-to-LDS GEMM, 128-token tile, contraction cut into 4 ranges
    (synth.DT_BF16, 384, 2048, 300, False),    # direct-to-LDS GEMM, two ragged 256-token tiles
    (synth.DT_BF16, 520, 1024, 130, True),     # direct-to-LDS GEMM, last feature tile 8 wide
    (synth.DT_BF16, 256, 4104, 40, True),      # D_ff not in whole 64-wide k-tiles: register-staged GEMM, ranges
    (synth.DT_BF16, 136, 264, 70, False),      # k tail (264 = 4 * 64 + 8)
    (synth.DT_BF16, 64, 131, 9, True),         # D_ff not a multiple of 8: plain path
    (synth.DT_F32, 256, 688, 64, True),        # config-0 shape, fp32
])
def test_prompt_output_uses_the_full_block(dtype, d, F, S, bias):
    act = synth.ACT_SILU
    c = synth.small_case(d + F + S, d, F, S, dtype, with_bias=bias)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype, c.get("bg"), c.get("b1"), c.get("b2"))
    idx, s, Z = run_prefill(L, to_dev(c["X"], dtype), [0, S], min(8, F))
    Zd = torch.from_numpy(Z.astype(np.float32)).cuda()
    W2p = to_dev(np.ascontiguousarray(c["W2"].T), dtype)          # the paper's W_2: [d][D_ff]
    Y = torch.empty((S, d), dtype=W2p.dtype, device="cuda")
    G.griffin_ff_prompt_out(Zd, W2p, Y, b2=to_dev(c.get("b2"), dtype),
                            workspace=workspace(G.griffin_prompt_out_workspace_bytes(S, F, d)))
    sync()
    Z_ref = oracle.ff1(c["X"], c["Wg"], c["W1"], act, c.get("bg"), c.get("b1"))
    Y_ref = oracle.ff2(Z_ref, c["W2"], c.get("b2"))
    assert max_rel(to_host(Y), Y_ref) <= TOL_OUT[dtype]
    # row by row it is the full-width decode of the same token (Eq. 1)
    y0 = oracle.ff_decode(c["X"][0], c["Wg"], c["W1"], c["W2"], act, c.get("bg"), c.get("b1"), c.get("b2"))
    assert max_rel(Y_ref[0], y0) <= 1e-12


@pytest.mark.parametrize("dtype,d,F,lens,k,gated,bias", [
    (synth.DT_BF16, 512, 1024, [300, 77], 400, True, False),    # one pass: the first product leaves the bf16 copy
    (synth.DT_BF16, 256, 4096, [40], 2048, True, False),        # 128-token tile, contraction cut into ranges
    (synth.DT_BF16, 384, 2048, [10, 0, 290], 1000, False, False),  # Eq. 2 block, an empty prompt in the middle
    (synth.DT_BF16, 384, 2048, [300], 1000, True, True),        # biases: Z is converted by its own pass
    (synth.DT_BF16, 136, 264, [70], 100, True, False),          # k tail: register-staged kernels
    (synth.DT_F32, 256, 688, [64], 344, True, True),            # config-0 shape, fp32
])
def test_prompt_phase_is_selection_plus_prompt_output_from_one_z(dtype, d, F, lens, k, gated, bias):
    """Section 4.2 + Section 5.1 in one call: the sets of griffin_prefill_select, the output of
    griffin_ff_prompt_out, both checked against the oracle and, bit for bit, against the two calls."""
    act = synth.ACT_SILU
    S = sum(lens)
    c = synth.small_case(d * 3 + F + S, d, F, S, dtype, with_bias=bias)
    Wg = c["Wg"] if gated else None
    bg = c.get("bg") if gated else None
    b1, b2 = c.get("b1"), c.get("b2")
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    live = [b for b in range(len(lens)) if lens[b] > 0]
    W1 = c["W1"].copy()
    _, s_ref_live = open_margin([c["X"][cu[b]:cu[b + 1]] for b in live], Wg, W1, act, dtype, [k], bg, b1)
    L, _ = dev_layer(Wg, W1, c["W2"], act, dtype, bg, b1, b2)
    Xd = to_dev(c["X"], dtype)
    W2p = to_dev(np.ascontiguousarray(c["W2"].T), dtype)          # the paper's W_2: [d][D_ff]
    n_seqs = len(lens)
    idx = torch.full((n_seqs, k), -1, dtype=torch.int32, device="cuda")
    sd = torch.full((n_seqs, F), -1.0, dtype=torch.float32, device="cuda")
    Y = torch.full((S, d), float("nan"), dtype=W2p.dtype, device="cuda")
    ws = workspace(G.griffin_prompt_phase_workspace_bytes(L, S, n_seqs))
    ws.fill_(0xFF)
    G.griffin_prompt_phase(L, W2p, Xd, [int(v) for v in cu], k, idx, Y, s_out=sd, workspace=ws)
    sync()
    # against the oracle
    Z_ref = oracle.ff1(c["X"], Wg, W1, act, bg, b1)
    assert max_rel(to_host(Y), oracle.ff2(Z_ref, c["W2"], b2)) <= TOL_OUT[dtype]
    s_got = sd.cpu().numpy().astype(np.float64)
    for pos, b in enumerate(live):
        assert boundary_report(s_ref_live[pos], k)[0] > 1e-3
        assert max_rel(s_got[b], s_ref_live[pos]) <= TOL_S
        np.testing.assert_array_equal(idx.cpu().numpy()[b], oracle.topk(s_ref_live[pos], k))
    # against the two calls
    idx2, s2, Z2 = run_prefill(L, Xd, cu, k)
    Zd = torch.from_numpy(Z2.astype(np.float32)).cuda()
    Y2 = torch.empty_like(Y)
    G.griffin_ff_prompt_out(Zd, W2p, Y2, b2=to_dev(b2, dtype),
                            workspace=workspace(G.griffin_prompt_out_workspace_bytes(S, F, d)))
    sync()
    np.testing.assert_array_equal(idx.cpu().numpy(), idx2)
    assert np.array_equal(s_got, s2)
    assert np.array_equal(to_host(Y), to_host(Y2))


# ------------------------------------------------------------------ static and sampled selectors, set similarity
@pytest.mark.parametrize("dtype,d,F,gated", [
    (synth.DT_BF16, 512, 1000, True), (synth.DT_BF16, 8, 5, True), (synth.DT_BF16, 4096, 700, False),
    (synth.DT_F32, 256, 688, True), (synth.DT_F32, 72, 150, False)])
def test_weight_norm_score_matches_oracle(dtype, d, F, gated):
    c = synth.small_case(d * 7 + F, d, F, 4, dtype)
    Wg = c["Wg"] if gated else None
    L, _ = dev_layer(Wg, c["W1"], c["W2"], synth.ACT_SILU, dtype)
    out = torch.empty(F, dtype=torch.float32, device="cuda")
    G.griffin_weight_norm_score(L, out)
    sync()
    ref = oracle.weight_norm_score(Wg, c["W1"])
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=2e-6)
    # the static expert set: top-k of the score (exact where the oracle's boundary gap is open)
    k = max(F // 2, 1)
    if oracle.topk_margin(ref, k) > 1e-4:
        idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
        G.griffin_topk(out, k, idx)
        sync()
        np.testing.assert_array_equal(idx.cpu().numpy()[0], oracle.topk(ref, k))


def open_sampling_margin(s, e, k, k_top, gap=1e-4, max_iter=50):
    """The device decides the draw on q = s / e in single precision, the oracle in double: the sets agree
    bit for bit where no quotient sits within `gap` (relative; a single-precision quotient is off by 6e-8)
    of the value that separates drawn from not drawn, exact ties aside (equal operands give equal quotients
    in either precision and go to the lower index on both sides).  Clocks e of neurons that sit too close
    are moved by 0.3 % until that holds.  Uses the oracle's own top-k for the part that is not drawn."""
    e = e.copy()
    m = k - k_top
    if m <= 0:
        return e
    rest = np.setdiff1d(np.arange(s.shape[0]), oracle.topk(s, k_top) if k_top > 0 else np.empty(0, dtype=np.int64))
    if m >= rest.shape[0]:
        return e
    for _ in range(max_iter):
        q = s[rest].astype(np.float64) / e[rest].astype(np.float64)
        order = np.argsort(-q, kind="stable")
        a, b = q[order[m - 1]], q[order[m]]              # last one drawn, first one left
        if a == 0.0:
            return e                                     # only zero weights left to draw from: decided by index alone
        near = np.zeros(q.shape[0], dtype=bool)
        for v in {a, b}:
            if v > 0.0:
                near |= (np.abs(q - v) < gap * v) & (q != v)
        if a != b and (a - b) < gap * a:
            near[order[m]] = True
        if not near.any():
            return e
        up = q[near] >= a                                 # drawn ones ring a little earlier, the others later
        e[rest[near]] = (e[rest[near]] * np.where(up, np.float32(0.997), np.float32(1.003))).astype(np.float32)
    raise RuntimeError("sampling margin did not open")


@pytest.mark.parametrize("n,k", [(11008, 5504), (1000, 1), (257, 256), (64, 64)])
def test_select_sampled_matches_oracle(n, k):
    """Appendix B: the oracle decides on q = s / e in double precision, the device in single; the inputs keep
    every quotient clear of the deciding value, so the sets must agree bit for bit."""
    rng = np.random.default_rng(n + k)
    s = (rng.random(n) ** 4).astype(np.float32)            # concentrated like the statistic (Appendix A)
    s[rng.choice(n, n // 10, replace=False)] = 0.0          # neurons that never fired
    e0 = rng.exponential(size=n).astype(np.float32)
    e0 = np.maximum(e0, np.float32(1e-6))
    e0[: n // 8] = np.float32(0.5)                          # equal clocks: exact ties in q wherever s ties too
    s[: n // 16] = np.float32(0.25)
    sd = torch.from_numpy(s).cuda()
    for k_top in sorted({0, k // 2, k}):
        e = open_sampling_margin(s, e0, k, k_top)
        ed = torch.from_numpy(e).cuda()
        ws = workspace(G.griffin_select_sampled_workspace_bytes(n, k_top))
        idx = torch.full((k,), -1, dtype=torch.int32, device="cuda")
        G.griffin_select_sampled(sd, ed, k, k_top, idx, workspace=ws)
        sync()
        np.testing.assert_array_equal(idx.cpu().numpy(), oracle.select_sampled(s, e, k, k_top), err_msg="k_top=%d" % k_top)


def test_jaccard_of_selected_sets_matches_oracle():
    rng = np.random.default_rng(12)
    n, k, B = 5000, 1200, 5
    s = rng.random((B, n)).astype(np.float32)
    s[1] = s[0]                                             # identical sets -> 1
    idx = torch.empty((B, k), dtype=torch.int32, device="cuda")
    G.griffin_topk(torch.from_numpy(s).cuda(), k, idx)
    out = torch.empty((B, B), dtype=torch.float32, device="cuda")
    G.griffin_jaccard(idx, out)
    sync()
    sets = idx.cpu().numpy()
    ref = np.array([[oracle.jaccard(sets[a], sets[b]) for b in range(B)] for a in range(B)])
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-6)
    assert out[0, 1].item() == 1.0 and np.allclose(np.diag(out.cpu().numpy()), 1.0)


# ------------------------------------------------------------------ the documented maxima
def test_prefill_takes_the_maximum_number_of_sequences():
    """GRIFFIN_MAX_SEQS prompts in one call: lengths 0..5, many of them empty."""
    dtype, d, F, k = synth.DT_BF16, 64, 96, 24
    rng = np.random.default_rng(21)
    lens = rng.integers(0, 6, size=G.MAX_SEQS).tolist()
    lens[0], lens[-1] = 0, 5
    c = synth.small_case(77, d, F, sum(lens), dtype)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, dtype)
    idx, s, Z = run_prefill(L, to_dev(c["X"], dtype), cu, k)
    Z_ref = oracle.ff1(c["X"], c["Wg"], c["W1"], synth.ACT_SILU)
    assert max_rel(Z, Z_ref) <= TOL_Z
    for b in range(G.MAX_SEQS):
        if lens[b] == 0:
            assert np.all(s[b] == 0.0) and idx[b].tolist() == list(range(k))
            continue
        s_ref = oracle.stat(Z_ref[cu[b]:cu[b + 1]])
        assert np.max(np.abs(s[b] - s_ref)) <= TOL_S * np.max(s_ref)
        if boundary_report(s_ref, k)[0] > 1e-3:
            np.testing.assert_array_equal(idx[b], oracle.topk(s_ref, k))
        else:       # the boundary is too tight to pin the set: what is selected must still be a top-k of the device's own s
            assert np.min(s[b][idx[b]]) >= np.max(np.delete(s[b], idx[b])) - 1e-12


def test_statistic_with_many_short_prompts_beside_a_long_one():
    """255 prompts of 8 tokens and one of 9000 in one call: few chunks are left for the long prompt, each of
    them holds more rows than a workgroup keeps weights for at a time (its second block of rows), and every
    short prompt is one partial chunk.  Z and s are compared for every sequence (Section 4.1, Eq. 6)."""
    dtype, d, F, k, act = synth.DT_BF16, 64, 7168, 3000, synth.ACT_SILU
    lens = [8] * 255 + [9000]
    c = synth.small_case(2024, d, F, sum(lens), dtype)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype)
    idx, s, Z = run_prefill(L, to_dev(c["X"], dtype), cu, k)
    Z_ref = oracle.ff1(c["X"], c["Wg"], c["W1"], act)
    assert max_rel(Z, Z_ref) <= TOL_Z
    for b in range(len(lens)):
        s_ref = oracle.stat(Z_ref[cu[b]:cu[b + 1]])
        assert np.max(np.abs(s[b] - s_ref)) <= TOL_S * np.max(s_ref), b
        assert np.sum(s[b] ** 2) == pytest.approx(lens[b], rel=1e-4)
        if boundary_report(s_ref, k)[0] > 1e-3:
            np.testing.assert_array_equal(idx[b], oracle.topk(s_ref, k))
        else:       # the boundary is too tight to pin the set: what is selected must still be a top-k of the device's own s
            assert np.all(np.diff(idx[b]) > 0)
            assert np.min(s[b][idx[b]]) >= np.max(np.delete(s[b], idx[b])) - 1e-12


def test_decode_takes_the_maximum_batch():
    """GRIFFIN_MAX_BATCH rows: per-row index lists, per-row compact blocks, one shared block."""
    dtype, d, n, k, B = synth.DT_BF16, 512, 200, 64, G.MAX_BATCH
    c = synth.small_case(31, d, n, 4, dtype, T=B)
    L, t = dev_layer(c["Wg"], c["W1"], c["W2"], synth.ACT_SILU, dtype)
    rng = np.random.default_rng(5)
    idx = np.stack([np.sort(rng.choice(n, k, replace=False)) for _ in range(B)]).astype(np.int32)
    idx_dev = torch.from_numpy(idx).cuda()
    x = to_dev(c["xt"], dtype)
    ws = workspace(max(G.griffin_decode_workspace_bytes(d, k, B), G.griffin_decode_workspace_bytes(d, n, B)))
    y = torch.empty_like(x)
    G.griffin_ff_decode_indexed(L, idx_dev, k, B, x, y, workspace=ws)
    sync()
    y_idx = to_host(y)
    Cs, keep = [], []
    for b in range(B):
        C, ct = empty_compact(L, k, t)
        G.griffin_compact(L, idx_dev[b], k, C)
        Cs.append(C); keep.append(ct)
    y2 = torch.empty_like(x)
    G.griffin_ff_decode_multi(Cs, x, y2, workspace=ws)
    sync()
    y_multi = to_host(y2)
    y3 = torch.empty_like(x)
    G.griffin_ff_decode(L, x, y3, B, workspace=ws)          # all rows through the full block (Eq. 1)
    sync()
    y_full = to_host(y3)
    for b in range(0, B, 7):
        ref = oracle.ff_decode(c["xt"][b], c["Wg"][idx[b]], c["W1"][idx[b]], c["W2"][idx[b]], synth.ACT_SILU)
        assert max_rel(y_idx[b], ref) <= TOL_OUT[dtype] and max_rel(y_multi[b], ref) <= TOL_OUT[dtype]
        assert max_rel(y_full[b], oracle.ff_decode(c["xt"][b], c["Wg"], c["W1"], c["W2"], synth.ACT_SILU)) <= TOL_OUT[dtype]
    # with a workspace sized for the whole block the index lists take one masked pass over the block
    # (other order of summation than row by row): equal up to bf16 rounding of the output
    assert np.max(np.abs(y_idx - y_multi)) <= 2.0 ** -6 * np.max(np.abs(y_multi))
    # with a workspace sized for k neurons they go row by row: the same arithmetic as the compact blocks
    y4 = torch.empty_like(x)
    G.griffin_ff_decode_indexed(L, idx_dev, k, B, x, y4, workspace=workspace(G.griffin_decode_workspace_bytes(d, k, B)))
    sync()
    assert np.array_equal(to_host(y4), y_multi)


@pytest.mark.parametrize("d,n,k,B,gated,bias", [
    (1024, 300, 100, 7, False, True),      # Eq. 2 block with biases, 7 of 16 rows
    (2048, 999, 500, 19, True, True),      # two groups of rows (16 + 3), odd block size
    (512, 64, 64, 5, True, False),         # every row keeps the whole block
    (512, 9000, 150, 6, True, False),      # a longer block, lists partly unsorted
])
def test_indexed_decode_masked_pass_matches_oracle(d, n, k, B, gated, bias):
    """Rows with their own sets inside one block, one masked pass over the block (workspace sized for it)."""
    dtype, act = synth.DT_BF16, synth.ACT_GELU_TANH
    c = synth.small_case(d + n + B, d, n, 4, dtype, T=B, with_bias=bias)
    Wg = c["Wg"] if gated else None
    bg = c.get("bg") if gated else None
    L, _ = dev_layer(Wg, c["W1"], c["W2"], act, dtype, bg, c.get("b1"), c.get("b2"))
    rng = np.random.default_rng(B)
    # the lists need not be ascending: odd rows are left in the order they were drawn
    idx = np.stack([(np.sort if b % 2 == 0 else np.asarray)(rng.choice(n, k, replace=False)) for b in range(B)]).astype(np.int32)
    x = to_dev(c["xt"], dtype)
    y = torch.empty_like(x)
    G.griffin_ff_decode_indexed(L, torch.from_numpy(idx).cuda(), k, B, x, y,
                                workspace=workspace(G.griffin_decode_workspace_bytes(d, n, B)))
    sync()
    got = to_host(y)
    sub = lambda a, b: None if a is None else a[idx[b]]
    for b in range(B):
        ref = oracle.ff_decode(c["xt"][b], sub(Wg, b), c["W1"][idx[b]], c["W2"][idx[b]], act, sub(bg, b), sub(c.get("b1"), b), c.get("b2"))
        assert max_rel(got[b], ref) <= TOL_OUT[dtype], b
