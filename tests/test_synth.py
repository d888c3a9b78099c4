"""The seeded input generator: deterministic, independent of thread count, shaped as stated."""
import numpy as np

import synth


def test_configs_match_the_named_shapes():
    c = synth.CONFIGS
    assert (c[0].d, c[0].d_ff, c[0].prompt_len, c[0].k, c[0].decode_steps) == (256, 688, 64, 344, 16)
    assert (c[1].d, c[1].d_ff, c[1].prompt_len, c[1].k) == (4096, 11008, 512, 5504)
    assert (c[2].d, c[2].d_ff, c[2].prompt_len, c[2].ks) == (3072, 24576, 2048, (6144, 12288, 18432))
    assert (c[3].d, c[3].d_ff, c[3].n_layers, c[3].k) == (5120, 13824, 40, 6912)
    assert (c[4].d, c[4].d_ff, c[4].n_layers, c[4].n_seqs, c[4].k) == (4096, 14336, 8, 16, 7168)
    lens = synth.seq_lengths(c[4])
    assert len(lens) == 16 and all(256 <= v <= 2048 for v in lens) and lens == synth.seq_lengths(c[4])


def test_generation_is_deterministic_and_thread_independent():
    cfg = synth.CONFIGS[0]
    a = synth.layer_weights(cfg, 0)
    b = synth.layer_weights(cfg, 0, pool=None)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(1) as pool:
        c = synth.layer_weights(cfg, 0, pool=pool)
    for x, y, z in zip(a, b, c):
        assert np.array_equal(x, y) and np.array_equal(x, z)
    assert not np.array_equal(a[0], a[1])
    assert np.array_equal(synth.prompt(cfg, 0), synth.prompt(cfg, 0))
    assert not np.array_equal(synth.prompt(cfg, 0), synth.decode_inputs(cfg, 0)[:64])


def test_statistics_of_the_recipe():
    cfg = synth.CONFIGS[0]
    Wg, W1, W2 = synth.layer_weights(cfg, 0)
    assert Wg.shape == (688, 256) and W2.shape == (688, 256)
    assert abs(Wg.std() * 16 - 1) < 0.02 and abs(W2.std() * 688 ** 0.5 - 1) < 0.02
    X = synth.prompt(cfg, 0)
    assert X.shape == (64, 256)
    np.testing.assert_allclose(np.sqrt((X.astype(np.float64) ** 2).mean(axis=1)), 1.0, rtol=1e-6)
    # tokens share a mean direction: high cosine similarity between rows
    Xn = X / np.linalg.norm(X, axis=1, keepdims=True)
    cos = Xn @ Xn.T
    assert cos[np.triu_indices(64, 1)].mean() > 0.7


def test_bf16_storage_round_trip_and_nudges():
    a = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-3], dtype=np.float32)
    r = synth.round_to_bf16(a)
    assert np.array_equal(synth.from_bf16_bits(synth.bf16_bits(r)), r)
    assert r[1] == 1.0 and r[2] == np.float32(1.015625)       # ties to even, both directions
    assert np.all(np.abs(r - a) <= np.abs(a) * 2.0 ** -8)
    case = synth.small_case(1, 64, 40, 8, synth.DT_BF16)
    W1 = case["W1"].copy()
    synth.apply_nudges(W1, [(3, 0.98)], synth.DT_BF16)
    assert np.array_equal(W1[2], case["W1"][2]) and not np.array_equal(W1[3], case["W1"][3])
    synth.bf16_bits(W1)   # still bf16-representable


def test_packed_prompts():
    cfg = synth.CONFIGS[4]
    lens = synth.seq_lengths(cfg)
    small = synth.Config(4, cfg.name, 64, 96, cfg.act, cfg.dtype, 1, 3, 0, (48,), 2, len_range=(5, 9))
    X, cu = synth.packed_prompts(small, 0)
    assert cu[0] == 0 and cu[-1] == X.shape[0] and X.shape[1] == 64 and len(cu) == 4
    assert lens  # silence linters
