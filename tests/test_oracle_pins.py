"""Pins for the CPU oracle: each oracle function is checked against something other than
itself -- a hand-derived example, closed forms and invariants that follow from the paper's
definitions, special cases that reduce to a library routine, and brute force on tiny inputs.
A dropped term, a wrong sign/index or a transposed operand in the oracle fails one of these.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from golden_io import read_kv

ACTS = [oracle.ACT_SILU, oracle.ACT_GELU_TANH, oracle.ACT_RELU]


def np_act(act, a):
    a = np.asarray(a, dtype=np.float64)
    if act == oracle.ACT_SILU:
        return a * (1.0 / (1.0 + np.exp(-a)))
    if act == oracle.ACT_GELU_TANH:
        return 0.5 * a * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (a + 0.044715 * a ** 3)))
    return np.maximum(a, 0.0)


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------ activation: known values
def test_activation_known_values():
    # one neuron, d=1, W1 = 1 so Z = act(g): isolates sigma.
    def sigma(act, g):
        return oracle.ff1(np.array([[g]]), np.array([[1.0]]), np.array([[1.0]]), act)[0, 0] / g

    # silu(1) = 1/(1+e^-1); tanh-GELU(1) from its closed form; relu
    assert sigma(oracle.ACT_SILU, 1.0) == pytest.approx(0.7310585786300049, rel=1e-14)
    assert sigma(oracle.ACT_SILU, -2.0) == pytest.approx(-2.0 / (1.0 + math.exp(2.0)), rel=1e-14)
    g1 = 0.5 * (1.0 + math.tanh(math.sqrt(2 / math.pi) * 1.044715))
    assert sigma(oracle.ACT_GELU_TANH, 1.0) == pytest.approx(g1, rel=1e-14)
    assert g1 == pytest.approx(0.8411919906082768, rel=1e-12)   # textbook value of gelu_tanh(1)
    assert sigma(oracle.ACT_RELU, 3.0) == 3.0
    assert oracle.ff1(np.array([[-3.0]]), np.array([[1.0]]), np.array([[1.0]]), oracle.ACT_RELU)[0, 0] == 0.0
    # large a: silu(a) -> a, gelu(a) -> a; large negative a: both -> 0
    assert sigma(oracle.ACT_SILU, 40.0) == pytest.approx(40.0, rel=1e-15)
    assert sigma(oracle.ACT_GELU_TANH, 10.0) == pytest.approx(10.0, rel=1e-15)
    assert abs(sigma(oracle.ACT_SILU, -40.0)) < 1e-15 and abs(sigma(oracle.ACT_GELU_TANH, -10.0)) < 1e-15


# ------------------------------------------------------------------ ff1
@pytest.mark.parametrize("act", ACTS)
def test_ff1_reduces_to_library_matmul(act):
    S, d, n = 5, 7, 11   # all different: a transposed operand cannot pass
    X, Wg, W1 = rand((S, d), 1), rand((n, d), 2), rand((n, d), 3)
    Z = oracle.ff1(X, Wg, W1, act)
    ref = np_act(act, X @ Wg.T) * (X @ W1.T)
    np.testing.assert_allclose(Z, ref, rtol=1e-12, atol=1e-13)
    # gate and up are not interchangeable
    assert not np.allclose(Z, oracle.ff1(X, W1, Wg, act))


def test_ff1_biases_and_non_glu():
    S, d, n = 4, 6, 9
    X, Wg, W1 = rand((S, d), 4), rand((n, d), 5), rand((n, d), 6)
    bg, b1 = rand(n, 7), rand(n, 8)
    Z = oracle.ff1(X, Wg, W1, oracle.ACT_SILU, bg=bg, b1=b1)
    ref = np_act(oracle.ACT_SILU, X @ Wg.T + bg) * (X @ W1.T + b1)
    np.testing.assert_allclose(Z, ref, rtol=1e-12, atol=1e-13)
    # Eq. 2: no gate
    Z2 = oracle.ff1(X, None, W1, oracle.ACT_RELU, b1=b1)
    np.testing.assert_allclose(Z2, np.maximum(X @ W1.T + b1, 0), rtol=1e-12, atol=1e-13)


def test_ff1_integer_relu_exact():
    rng = np.random.default_rng(9)
    X = rng.integers(-3, 4, (6, 8)).astype(np.float64)
    Wg = rng.integers(-3, 4, (10, 8)).astype(np.float64)
    W1 = rng.integers(-3, 4, (10, 8)).astype(np.float64)
    Z = oracle.ff1(X, Wg, W1, oracle.ACT_RELU)
    G = np.zeros((6, 10)); U = np.zeros((6, 10))
    for c in range(8):            # independent triple loop, different loop order
        for i in range(6):
            for j in range(10):
                G[i, j] += X[i, c] * Wg[j, c]
                U[i, j] += X[i, c] * W1[j, c]
    ref = np.where(G > 0, G, 0.0) * U
    assert np.array_equal(Z, ref)


# ------------------------------------------------------------------ stat
def test_stat_sum_of_squares_equals_S_and_bounds():
    for S, F, seed in [(1, 5, 0), (7, 13, 1), (33, 64, 2)]:
        Z = rand((S, F), seed)
        s = oracle.stat(Z)
        assert s.shape == (F,)
        assert np.sum(s ** 2) == pytest.approx(S, rel=1e-12)
        assert np.all(s >= 0) and np.all(s <= math.sqrt(S) + 1e-12)


def test_stat_against_plain_definition():
    Z = rand((9, 14), 3)
    Zb = Z / np.linalg.norm(Z, axis=1, keepdims=True)       # Section 4.1
    ref = np.linalg.norm(Zb, axis=0)                          # Eq. 6
    s, r = oracle.stat(Z, return_row_norms=True)
    np.testing.assert_allclose(s, ref, rtol=1e-13)
    np.testing.assert_allclose(r, np.linalg.norm(Z, axis=1), rtol=1e-13)
    # not the un-normalised column norm
    assert not np.allclose(s, np.linalg.norm(Z, axis=0))


def test_stat_row_scaling_invariance():
    Z = rand((8, 12), 4)
    c = np.random.default_rng(5).uniform(0.1, 50.0, size=(8, 1))
    np.testing.assert_allclose(oracle.stat(Z * c), oracle.stat(Z), rtol=1e-12)


def test_stat_permutations():
    Z = rand((10, 17), 6)
    s = oracle.stat(Z)
    pt = np.random.default_rng(7).permutation(10)
    pn = np.random.default_rng(8).permutation(17)
    np.testing.assert_allclose(oracle.stat(Z[pt]), s, rtol=1e-12)       # token order is irrelevant
    np.testing.assert_allclose(oracle.stat(Z[:, pn]), s[pn], rtol=1e-12)  # neurons carry their s


def test_stat_single_token_and_identical_rows():
    z = rand((1, 9), 9)
    np.testing.assert_allclose(oracle.stat(z), np.abs(z[0]) / np.linalg.norm(z[0]), rtol=1e-13)
    S = 6
    Z = np.repeat(z, S, axis=0) * np.arange(1, S + 1)[:, None]   # same direction, different scale
    np.testing.assert_allclose(oracle.stat(Z), math.sqrt(S) * np.abs(z[0]) / np.linalg.norm(z[0]), rtol=1e-12)


def test_stat_zero_row_contributes_nothing():
    Z = rand((5, 7), 10)
    Z0 = np.vstack([Z[:2], np.zeros((1, 7)), Z[2:]])
    s0 = oracle.stat(Z0)
    assert np.all(np.isfinite(s0))
    np.testing.assert_allclose(s0, oracle.stat(Z), rtol=1e-13)
    assert np.sum(s0 ** 2) == pytest.approx(5, rel=1e-12)      # S minus the zero row


def test_stat_shared_eq7():
    sa = np.abs(rand((3, 8), 11))
    lens = np.array([4, 9, 16])
    ref = sa[0] / 2 + sa[1] / 3 + sa[2] / 4
    np.testing.assert_allclose(oracle.stat_shared(sa, lens), ref, rtol=1e-14)
    # a single sample whose rows all point the same way: s/sqrt(S) = |z|/||z||
    z = rand((1, 6), 12)
    Z = np.repeat(z, 25, axis=0)
    np.testing.assert_allclose(oracle.stat_shared(oracle.stat(Z)[None], np.array([25])),
                               np.abs(z[0]) / np.linalg.norm(z[0]), rtol=1e-12)


# ------------------------------------------------------------------ topk
def test_topk_equals_full_sort():
    rng = np.random.default_rng(13)
    for F in (1, 2, 17, 300):
        s = rng.random(F)
        order = np.argsort(-s, kind="stable")
        for k in sorted({1, F // 2 or 1, F}):
            np.testing.assert_array_equal(oracle.topk(s, k), np.sort(order[:k]).astype(np.int32))


def test_topk_brute_force_subsets():
    rng = np.random.default_rng(14)
    for F in range(1, 10):
        s = rng.random(F)
        for k in range(1, F + 1):
            best = max(itertools.combinations(range(F), k), key=lambda c: sum(s[list(c)]))
            np.testing.assert_array_equal(oracle.topk(s, k), np.array(best, dtype=np.int32))


def test_topk_ties_lowest_index_and_ascending_output():
    s = np.array([0.5, 0.9, 0.9, 0.1, 0.9, 0.5])
    np.testing.assert_array_equal(oracle.topk(s, 1), [1])
    np.testing.assert_array_equal(oracle.topk(s, 2), [1, 2])
    np.testing.assert_array_equal(oracle.topk(s, 3), [1, 2, 4])
    np.testing.assert_array_equal(oracle.topk(s, 4), [0, 1, 2, 4])
    np.testing.assert_array_equal(oracle.topk(np.zeros(5), 3), [0, 1, 2])
    np.testing.assert_array_equal(oracle.topk(s, 6), np.arange(6))
    assert oracle.topk(s, 0).shape == (0,)


def test_topk_margin():
    s = np.array([4.0, 1.0, 3.0, 2.0])
    assert oracle.topk_margin(s, 2) == pytest.approx((3.0 - 2.0) / 3.0)
    assert oracle.topk_margin(s, 4) == float("inf")


# ------------------------------------------------------------------ compact + ff_decode
def test_compact_rows_and_vectors():
    W = rand((9, 4), 15)
    idx = np.array([0, 3, 8], dtype=np.int32)
    np.testing.assert_array_equal(oracle.compact(W, idx), W[idx])
    b = rand(9, 16)
    np.testing.assert_array_equal(oracle.compact(b, idx), b[idx])
    with pytest.raises(RuntimeError):
        oracle.compact(W, np.array([9], dtype=np.int32))


@pytest.mark.parametrize("act", ACTS)
def test_ff_decode_reduces_to_library_matvec(act):
    d, n = 6, 10
    x, Wg, W1, W2 = rand(d, 17), rand((n, d), 18), rand((n, d), 19), rand((n, d), 20)
    bg, b1, b2 = rand(n, 21), rand(n, 22), rand(d, 23)
    y, z = oracle.ff_decode(x, Wg, W1, W2, act, bg, b1, b2, return_z=True)
    zr = np_act(act, Wg @ x + bg) * (W1 @ x + b1)
    np.testing.assert_allclose(z, zr, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, W2.T @ zr + b2, rtol=1e-12, atol=1e-13)
    # consistent with ff1 on a one-row sequence
    np.testing.assert_allclose(oracle.ff1(x[None], Wg, W1, act, bg, b1)[0], z, rtol=1e-13, atol=1e-14)
    # Eq. 2 form
    y2 = oracle.ff_decode(x, None, W1, W2, oracle.ACT_RELU, b1=b1)
    np.testing.assert_allclose(y2, W2.T @ np.maximum(W1 @ x + b1, 0), rtol=1e-12, atol=1e-13)


def test_keep_all_is_the_full_block_bit_for_bit():
    d, n = 8, 21
    x, Wg, W1, W2 = rand(d, 24), rand((n, d), 25), rand((n, d), 26), rand((n, d), 27)
    idx = oracle.topk(np.abs(rand(n, 28)), n)
    np.testing.assert_array_equal(idx, np.arange(n))
    full = oracle.ff_decode(x, Wg, W1, W2, oracle.ACT_SILU)
    pruned = oracle.ff_decode(x, oracle.compact(Wg, idx), oracle.compact(W1, idx),
                              oracle.compact(W2, idx), oracle.ACT_SILU)
    assert np.array_equal(full, pruned)


def test_pruned_output_is_additive_over_disjoint_sets_and_keeps_b2_whole():
    d, n = 5, 12
    x, Wg, W1, W2 = rand(d, 29), rand((n, d), 30), rand((n, d), 31), rand((n, d), 32)
    b2 = rand(d, 33)
    E1 = np.array([0, 2, 5, 7], dtype=np.int32)
    E2 = np.array([1, 3, 11], dtype=np.int32)
    E12 = np.sort(np.concatenate([E1, E2])).astype(np.int32)

    def y(E, bias=None):
        return oracle.ff_decode(x, oracle.compact(Wg, E), oracle.compact(W1, E), oracle.compact(W2, E),
                                oracle.ACT_GELU_TANH, b2=bias)

    np.testing.assert_allclose(y(E12), y(E1) + y(E2), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(y(E1, b2) - y(E1), b2, rtol=1e-12, atol=1e-14)   # b2 is not pruned


def test_one_hot_input_reads_one_weight_column():
    d, n = 6, 9
    Wg, W1, W2 = rand((n, d), 34), rand((n, d), 35), rand((n, d), 36)
    c = 4
    x = np.zeros(d); x[c] = 1.0
    _, z = oracle.ff_decode(x, Wg, W1, W2, oracle.ACT_SILU, return_z=True)
    np.testing.assert_allclose(z, np_act(oracle.ACT_SILU, Wg[:, c]) * W1[:, c], rtol=1e-13)


# ------------------------------------------------------------------ hand-derived example
def test_hand_example_end_to_end():
    g = read_kv("hand_example.txt")
    assert g["act"] == "relu"
    Wg, W1, W2, X = g["Wg"], g["W1"], g["W2"], g["X"]
    Z = oracle.ff1(X, Wg, W1, oracle.ACT_RELU)
    assert np.array_equal(Z, g["Z"])
    s, r = oracle.stat(Z, return_row_norms=True)
    np.testing.assert_allclose(r ** 2, g["r2"], rtol=1e-15)
    np.testing.assert_allclose(s ** 2, g["s2"], rtol=1e-15)
    E2 = oracle.topk(s, 2)
    np.testing.assert_array_equal(E2, g["E2"].astype(np.int32))
    np.testing.assert_array_equal(oracle.topk(s, 1), g["E1"].astype(np.int32).reshape(1))
    idx, s_chain = oracle.prefill_select(X, Wg, W1, oracle.ACT_RELU, 2)
    np.testing.assert_array_equal(idx, E2)
    np.testing.assert_array_equal(s_chain, s)
    y_full, z = oracle.ff_decode(g["x"], Wg, W1, W2, oracle.ACT_RELU, return_z=True)
    assert np.array_equal(z, g["z"]) and np.array_equal(y_full, g["y_full"])
    y_p = oracle.ff_decode(g["x"], oracle.compact(Wg, E2), oracle.compact(W1, E2),
                           oracle.compact(W2, E2), oracle.ACT_RELU)
    assert np.array_equal(y_p, g["y_E2"])


def test_ff2_prompt_output_is_library_matmul():
    Z, W2, b2 = rand((4, 9), 37), rand((9, 5), 38), rand(5, 39)
    np.testing.assert_allclose(oracle.ff2(Z, W2, b2), Z @ W2 + b2, rtol=1e-12, atol=1e-13)


def test_active_parameter_arithmetic_matches_the_paper():
    # Section 4.2: halving the FF neurons takes Llama 2 13B from 13B to 8.8B active parameters.
    import synth
    c = synth.CONFIGS[3]
    ff_params = c.n_layers * 3 * c.d * c.d_ff
    assert ff_params == pytest.approx(8.49e9, rel=2e-3)
    assert 13.0e9 - ff_params * (1 - c.k / c.d_ff) == pytest.approx(8.8e9, rel=1e-2)


# ------------------------------------------------------------------ static and sampled selectors, set similarity
def test_weight_norm_score_known_rows_and_library_norms():
    W1 = np.array([[3.0, 4.0, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0], [0.0, 0.0, 0.0, 0.0]])
    Wg = np.array([[0.0, 0.0, 12.0, 5.0], [2.0, 0.0, 0.0, 0.0], [7.0, 1.0, 1.0, 1.0]])
    np.testing.assert_allclose(oracle.weight_norm_score(Wg, W1), [65.0, 2.0, 0.0], rtol=1e-15)
    np.testing.assert_allclose(oracle.weight_norm_score(None, W1), [5.0, 1.0, 0.0], rtol=1e-15)
    A, B = rand((7, 11), 51), rand((7, 11), 52)       # non-square: a transposed operand would fail
    ref = np.linalg.norm(A, axis=1) * np.linalg.norm(B, axis=1)
    np.testing.assert_allclose(oracle.weight_norm_score(B, A), ref, rtol=1e-13)
    A2 = A.copy()
    A2[3] *= -2.5                                      # scaling one neuron's W1 row scales its score only
    out = oracle.weight_norm_score(B, A2)
    np.testing.assert_allclose(out[3], 2.5 * ref[3], rtol=1e-13)
    np.testing.assert_allclose(np.delete(out, 3), np.delete(ref, 3), rtol=1e-13)


def test_select_sampled_hand_example_and_limits():
    s = np.array([4.0, 1.0, 2.0, 0.5])
    e = np.array([2.0, 0.25, 4.0, 1.0], dtype=np.float32)      # q = s / e = 2, 4, 0.5, 0.5
    np.testing.assert_array_equal(oracle.select_sampled(s, e, 2, 0), [0, 1])
    np.testing.assert_array_equal(oracle.select_sampled(s, e, 3, 0), [0, 1, 2])    # tie 0.5 = 0.5 -> lower index
    np.testing.assert_array_equal(oracle.select_sampled(s, e, 2, 1), [0, 1])      # top-1 of s is 0, then q
    np.testing.assert_array_equal(oracle.select_sampled(s, e, 2, 2), [0, 2])      # k_top = k is plain top-k
    rng = np.random.default_rng(7)
    s = rng.random(50)
    e = rng.exponential(size=50).astype(np.float32)
    for k in (1, 10, 50):
        np.testing.assert_array_equal(oracle.select_sampled(s, e, k, k), oracle.topk(s, k))
    # equal weights: the earliest clocks (smallest e) win
    np.testing.assert_array_equal(oracle.select_sampled(np.ones(50), e, 12, 0), np.sort(np.argsort(e, kind="stable")[:12]))
    # a zero weight is never drawn while positive weights remain, whatever its clock says
    s0 = s.copy()
    s0[[3, 17, 40]] = 0.0
    e0 = e.copy()
    e0[[3, 17, 40]] = 1e-30
    got = oracle.select_sampled(s0, e0, 47, 5)
    assert not set(got) & {3, 17, 40}
    # the top-k half is always inside the result
    assert set(oracle.topk(s, 5)) <= set(oracle.select_sampled(s, e, 20, 5))


def test_select_sampled_draws_like_sequential_weighted_sampling_without_replacement():
    # P({a, b}) of drawing two of four items one after the other with probability proportional to
    # the weight of what is left, written out; the oracle's draws must follow it.
    w = np.array([5.0, 3.0, 1.5, 0.5])
    W = w.sum()
    pairs = list(itertools.combinations(range(4), 2))
    p_exact = np.array([w[a] / W * w[b] / (W - w[a]) + w[b] / W * w[a] / (W - w[b]) for a, b in pairs])
    assert p_exact.sum() == pytest.approx(1.0, abs=1e-12)
    rng = np.random.default_rng(11)
    n_draws = 40000
    E = rng.exponential(size=(n_draws, 4)).astype(np.float32)
    counts = dict.fromkeys(pairs, 0)
    for t in range(n_draws):
        a, b = oracle.select_sampled(w, E[t], 2, 0)
        counts[(int(a), int(b))] += 1
    freq = np.array([counts[p] for p in pairs]) / n_draws
    sigma = np.sqrt(p_exact * (1 - p_exact) / n_draws)
    assert np.all(np.abs(freq - p_exact) < 4.5 * sigma), (freq, p_exact)


def test_jaccard_known_sets_and_python_sets():
    assert oracle.jaccard([1, 2, 3], [2, 3, 4]) == pytest.approx(0.5)
    assert oracle.jaccard([5, 9], [5, 9]) == 1.0
    assert oracle.jaccard([0, 1], [2, 3]) == 0.0
    rng = np.random.default_rng(3)
    for _ in range(5):
        a = np.sort(rng.choice(200, 60, replace=False))
        b = np.sort(rng.choice(200, 45, replace=False))
        sa, sb = set(a.tolist()), set(b.tolist())
        assert oracle.jaccard(a, b) == pytest.approx(len(sa & sb) / len(sa | sb), abs=1e-15)
