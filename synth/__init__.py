"""Seeded synthetic inputs shaped like the paper's models (shapes only, no trained weights).

This module serves both the CPU oracle and the HIP path with the *same* arrays and contains
none of the method's arithmetic: it draws Gaussian weights, builds prompts with a shared
mean plus per-token noise (the structure that makes neurons "flock" within a sequence,
Section 4.1 and Appendix C of the paper), RMS-normalises rows, and rounds to the storage
type.  Everything is keyed by (config, layer, sequence, tag, block) so any tensor can be
regenerated independently and in parallel with identical bits.

Values for bf16 configs are returned as float32 arrays holding exactly bf16-representable
numbers, so the oracle can widen them to float64 without loss and the HIP path can take the
upper 16 bits without rounding again.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

ROOT_SEED = 20240401

TAG_WG, TAG_W1, TAG_W2, TAG_MU, TAG_PROMPT, TAG_DECODE, TAG_LENGTHS = range(7)

ACT_SILU, ACT_GELU_TANH, ACT_RELU = 0, 1, 2
DT_F32, DT_BF16 = 0, 1

_ROW_BLOCK = 1024  # rows drawn per independent Philox stream


@dataclass(frozen=True)
class Config:
    """One workload: a stack of independent gated FF layers and a set of prompts."""

    cid: int
    name: str
    d: int
    d_ff: int
    act: int
    dtype: int
    n_layers: int
    n_seqs: int
    prompt_len: int            # fixed length; ignored when len_range is set
    ks: Tuple[int, ...]        # kept-neuron counts to run (config 2 sweeps three)
    decode_steps: int
    len_range: Optional[Tuple[int, int]] = None   # inclusive, per-sequence uniform length

    @property
    def k(self) -> int:
        return self.ks[len(self.ks) // 2] if len(self.ks) > 1 else self.ks[0]


CONFIGS: Dict[int, Config] = {
    0: Config(0, "tiny-fp32-swiglu", 256, 688, ACT_SILU, DT_F32, 1, 1, 64, (344,), 16),
    1: Config(1, "llama2-7b-ff", 4096, 11008, ACT_SILU, DT_BF16, 1, 1, 512, (5504,), 256),
    2: Config(2, "gemma-7b-ff", 3072, 24576, ACT_GELU_TANH, DT_BF16, 1, 1, 2048,
              (6144, 12288, 18432), 256),
    3: Config(3, "llama2-13b-ff-x40", 5120, 13824, ACT_SILU, DT_BF16, 40, 1, 1024, (6912,), 128),
    4: Config(4, "mistral-7b-ff-x8-b16", 4096, 14336, ACT_SILU, DT_BF16, 8, 16, 0, (7168,), 128,
              len_range=(256, 2048)),
}


def _rng(cid: int, layer: int, seq: int, tag: int, block: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([ROOT_SEED, cid, layer, seq, tag, block])
    return np.random.Generator(np.random.Philox(ss))


def n_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return min(int(env), 32)
    return min(os.cpu_count() or 1, 16)


# ----------------------------------------------------------------------------- storage types
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("array holds values that are not bf16-representable")
    return (u >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == DT_BF16 else a


# ----------------------------------------------------------------------------- weights
def _gauss_rows(cid: int, layer: int, tag: int, rows: int, cols: int, scale: float,
                dtype: int, pool: Optional[ThreadPoolExecutor]) -> np.ndarray:
    out = np.empty((rows, cols), dtype=np.float32)

    def fill(b: int) -> None:
        lo, hi = b * _ROW_BLOCK, min(rows, (b + 1) * _ROW_BLOCK)
        blk = _rng(cid, layer, 0, tag, b).standard_normal((hi - lo, cols), dtype=np.float32)
        blk *= np.float32(scale)
        out[lo:hi] = store(blk, dtype)

    blocks = range((rows + _ROW_BLOCK - 1) // _ROW_BLOCK)
    if pool is None:
        for b in blocks:
            fill(b)
    else:
        list(pool.map(fill, blocks))
    return out


Nudges = Sequence[Tuple[int, float]]


def layer_weights(cfg: Config, layer: int, nudges: Optional[Nudges] = None,
                  pool: Optional[ThreadPoolExecutor] = None):
    """Wg, W1, W2 of one layer, all neuron-major [d_ff][d] (row j = neuron j).

    Wg and W1 are the paper's W_g, W_1 (D_FF x D); W2 here is the transpose of the paper's
    W_2 (D x D_FF), so that selecting a neuron selects one contiguous row in all three.
    Entries are N(0, 1/d) for Wg, W1 and N(0, 1/d_ff) for W2, rounded to the storage type.
    `nudges` is a list of (neuron, factor): row `neuron` of W1 is multiplied by `factor`
    before rounding again; it is data produced offline to open a gap at the top-k boundary.
    """
    own = pool is None
    if own:
        pool = ThreadPoolExecutor(n_threads())
    try:
        Wg = _gauss_rows(cfg.cid, layer, TAG_WG, cfg.d_ff, cfg.d, cfg.d ** -0.5, cfg.dtype, pool)
        W1 = _gauss_rows(cfg.cid, layer, TAG_W1, cfg.d_ff, cfg.d, cfg.d ** -0.5, cfg.dtype, pool)
        W2 = _gauss_rows(cfg.cid, layer, TAG_W2, cfg.d_ff, cfg.d, cfg.d_ff ** -0.5, cfg.dtype, pool)
    finally:
        if own:
            pool.shutdown()
    if nudges:
        apply_nudges(W1, nudges, cfg.dtype)
    return Wg, W1, W2


def apply_nudges(W1: np.ndarray, nudges: Nudges, dtype: int) -> None:
    for row, factor in nudges:
        W1[row] = store(W1[row] * np.float32(factor), dtype)


# ----------------------------------------------------------------------------- activations in
def seq_lengths(cfg: Config, layer: int = 0) -> List[int]:
    """Prompt length of every sequence (the same for all layers of a config)."""
    if cfg.len_range is None:
        return [cfg.prompt_len] * cfg.n_seqs
    lo, hi = cfg.len_range
    g = _rng(cfg.cid, 0, 0, TAG_LENGTHS)
    return [int(v) for v in g.integers(lo, hi + 1, size=cfg.n_seqs)]


def _mu(cfg: Config, layer: int, seq: int) -> np.ndarray:
    return _rng(cfg.cid, layer, seq, TAG_MU).standard_normal(cfg.d, dtype=np.float32)


def _rms_rows(a: np.ndarray) -> np.ndarray:
    ms = np.mean(a.astype(np.float64) ** 2, axis=1, keepdims=True)
    return (a / np.sqrt(ms)).astype(np.float32)


def _tokens(cfg: Config, layer: int, seq: int, tag: int, n: int) -> np.ndarray:
    eps = _rng(cfg.cid, layer, seq, tag).standard_normal((n, cfg.d), dtype=np.float32)
    x = _mu(cfg, layer, seq)[None, :] + np.float32(0.5) * eps
    return store(_rms_rows(x), cfg.dtype)


def prompt(cfg: Config, layer: int, seq: int = 0, length: Optional[int] = None) -> np.ndarray:
    """X[S][d]: a shared row mu ~ N(0, I) plus 0.5 N(0, I) per token, rows RMS-normalised."""
    if length is None:
        length = seq_lengths(cfg)[seq]
    return _tokens(cfg, layer, seq, TAG_PROMPT, length)


def decode_inputs(cfg: Config, layer: int, seq: int = 0, steps: Optional[int] = None) -> np.ndarray:
    """x_t[T][d]: generated-token inputs around the same mu as the prompt, fresh noise."""
    return _tokens(cfg, layer, seq, TAG_DECODE, cfg.decode_steps if steps is None else steps)


def packed_prompts(cfg: Config, layer: int) -> Tuple[np.ndarray, np.ndarray]:
    """All sequences of a layer packed row-wise, and cu_seqlens[n_seqs+1] (int32)."""
    lens = seq_lengths(cfg)
    xs = [prompt(cfg, layer, b, lens[b]) for b in range(cfg.n_seqs)]
    cu = np.zeros(cfg.n_seqs + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return np.concatenate(xs, axis=0), cu


# ----------------------------------------------------------------------------- small ad-hoc cases
def small_case(seed: int, d: int, d_ff: int, S: int, dtype: int, T: int = 4,
               with_bias: bool = False):
    """A free-shape case with the same recipe, for parity tests off the named configs."""
    g = np.random.Generator(np.random.Philox(np.random.SeedSequence([ROOT_SEED, 99, seed])))
    Wg = store(g.standard_normal((d_ff, d), dtype=np.float32) * np.float32(d ** -0.5), dtype)
    W1 = store(g.standard_normal((d_ff, d), dtype=np.float32) * np.float32(d ** -0.5), dtype)
    W2 = store(g.standard_normal((d_ff, d), dtype=np.float32) * np.float32(d_ff ** -0.5), dtype)
    mu = g.standard_normal(d, dtype=np.float32)
    X = store(_rms_rows(mu[None] + np.float32(0.5) * g.standard_normal((S, d), dtype=np.float32)), dtype)
    xt = store(_rms_rows(mu[None] + np.float32(0.5) * g.standard_normal((T, d), dtype=np.float32)), dtype)
    out = dict(Wg=Wg, W1=W1, W2=W2, X=X, xt=xt)
    if with_bias:
        out["bg"] = store(g.standard_normal(d_ff, dtype=np.float32) * np.float32(0.1), dtype)
        out["b1"] = store(g.standard_normal(d_ff, dtype=np.float32) * np.float32(0.1), dtype)
        out["b2"] = store(g.standard_normal(d, dtype=np.float32) * np.float32(0.1), dtype)
    return out
