"""ctypes face of the C oracle (oracle/griffin_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the HIP library never does and there is no route from it to here.  Every function
converts its arguments to contiguous float64 (exact for fp32 and bf16-valued inputs) and
calls the plain-loop C routine of the same name.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Tuple

import numpy as np

from .build import build as _build

ACT_SILU, ACT_GELU_TANH, ACT_RELU = 0, 1, 2

_lib = ctypes.CDLL(_build())

_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)
_lp = ctypes.POINTER(ctypes.c_int64)

_lib.oracle_ff1.argtypes = [_i64, _i64, _i64, _dp, _dp, _dp, _dp, _dp, ctypes.c_int, _dp]
_lib.oracle_stat.argtypes = [_i64, _i64, _dp, _dp, _dp]
_lib.oracle_stat_shared.argtypes = [_i64, _i64, _dp, _lp, _dp]
_lib.oracle_topk.argtypes = [_i64, _dp, _i64, _ip]
_lib.oracle_compact.argtypes = [_i64, _i64, _dp, _i64, _ip, _dp]
_lib.oracle_ff_decode.argtypes = [_i64, _i64, _dp, _dp, _dp, _dp, _dp, _dp, _dp, ctypes.c_int, _dp, _dp]
_lib.oracle_ff2.argtypes = [_i64, _i64, _i64, _dp, _dp, _dp, _dp]
_fp = ctypes.POINTER(ctypes.c_float)
_lib.oracle_weight_norm_score.argtypes = [_i64, _i64, _dp, _dp, _dp]
_lib.oracle_select_sampled.argtypes = [_i64, _dp, _fp, _i64, _i64, _ip]
_lib.oracle_jaccard.argtypes = [_i64, _ip, _i64, _ip, _dp]
for _f in ("oracle_ff1", "oracle_stat", "oracle_stat_shared", "oracle_topk", "oracle_compact",
           "oracle_ff_decode", "oracle_ff2", "oracle_num_threads"):
    getattr(_lib, _f).restype = ctypes.c_int


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_dp)


def _opt(a) -> Optional[np.ndarray]:
    return None if a is None else _f64(a)


def _check(rc: int, name: str) -> None:
    if rc != 0:
        raise RuntimeError("%s failed with code %d" % (name, rc))


def num_threads() -> int:
    return int(_lib.oracle_num_threads())


def ff1(X, Wg, W1, act: int, bg=None, b1=None) -> np.ndarray:
    """Z = sigma(X Wg^T + bg) * (X W1^T + b1) (Eq. 3), or sigma(X W1^T + b1) if Wg is None (Eq. 2)."""
    X, W1 = _f64(X), _f64(W1)
    Wg, bg, b1 = _opt(Wg), _opt(bg), _opt(b1)
    S, d = X.shape
    n = W1.shape[0]
    assert W1.shape == (n, d) and (Wg is None or Wg.shape == (n, d))
    Z = np.empty((S, n), dtype=np.float64)
    _check(_lib.oracle_ff1(S, d, n, _p(X), _p(Wg), _p(W1), _p(bg), _p(b1), act, _p(Z)), "oracle_ff1")
    return Z


def stat(Z, return_row_norms: bool = False):
    """s_j = || column j of the row-normalised Z ||_2 (Section 4.1, Eq. 6)."""
    Z = _f64(Z)
    S, F = Z.shape
    s = np.empty(F, dtype=np.float64)
    r = np.empty(S, dtype=np.float64)
    _check(_lib.oracle_stat(S, F, _p(Z), _p(s), _p(r)), "oracle_stat")
    return (s, r) if return_row_norms else s


def stat_shared(s_all, lens) -> np.ndarray:
    """s_bar = sum_i s_i / sqrt(S_i) (Eq. 7)."""
    s_all = _f64(s_all)
    n, F = s_all.shape
    lens = np.ascontiguousarray(lens, dtype=np.int64)
    assert lens.shape == (n,)
    out = np.empty(F, dtype=np.float64)
    _check(_lib.oracle_stat_shared(n, F, _p(s_all), lens.ctypes.data_as(_lp), _p(out)), "oracle_stat_shared")
    return out


def topk(s, k: int) -> np.ndarray:
    """Indices of the k largest s_j, ties to the lowest index, ascending (Section 4.2)."""
    s = _f64(s)
    idx = np.empty(k, dtype=np.int32)
    _check(_lib.oracle_topk(s.shape[0], _p(s), k, idx.ctypes.data_as(_ip)), "oracle_topk")
    return idx


def compact(W, idx) -> np.ndarray:
    """Rows idx of a neuron-major matrix, or entries idx of a per-neuron vector (Eq. 4-5)."""
    W = _f64(W)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    vec = W.ndim == 1
    W2d = W.reshape(W.shape[0], -1)
    out = np.empty((idx.shape[0], W2d.shape[1]), dtype=np.float64)
    _check(_lib.oracle_compact(W2d.shape[0], W2d.shape[1], _p(W2d), idx.shape[0],
                               idx.ctypes.data_as(_ip), _p(out)), "oracle_compact")
    return out[:, 0].copy() if vec else out


def ff_decode(x, Wg, W1, W2, act: int, bg=None, b1=None, b2=None, return_z: bool = False):
    """y = W2^T-rows combination of z = FF1_hat(x) plus b2 (Eq. 1, Eq. 4-5)."""
    x, W1, W2 = _f64(x), _f64(W1), _f64(W2)
    Wg, bg, b1, b2 = _opt(Wg), _opt(bg), _opt(b1), _opt(b2)
    n, d = W1.shape
    assert x.shape == (d,) and W2.shape == (n, d) and (Wg is None or Wg.shape == (n, d))
    y = np.empty(d, dtype=np.float64)
    z = np.empty(n, dtype=np.float64)
    _check(_lib.oracle_ff_decode(d, n, _p(x), _p(Wg), _p(W1), _p(W2), _p(bg), _p(b1), _p(b2),
                                 act, _p(y), _p(z)), "oracle_ff_decode")
    return (y, z) if return_z else y


def ff2(Z, W2, b2=None) -> np.ndarray:
    """Y = Z W2 + b2 for every prompt row with the full block (Section 5.1)."""
    Z, W2, b2 = _f64(Z), _f64(W2), _opt(b2)
    S, n = Z.shape
    d = W2.shape[1]
    assert W2.shape == (n, d)
    Y = np.empty((S, d), dtype=np.float64)
    _check(_lib.oracle_ff2(S, d, n, _p(Z), _p(W2), _p(b2), _p(Y)), "oracle_ff2")
    return Y


def weight_norm_score(Wg, W1) -> np.ndarray:
    """Static magnitude metric: ||W1_j||_2 * ||Wg_j||_2 per neuron (Section 5.1, Setup)."""
    W1, Wg = _f64(W1), _opt(Wg)
    n, d = W1.shape
    out = np.empty(n, dtype=np.float64)
    _check(_lib.oracle_weight_norm_score(n, d, _p(Wg), _p(W1), _p(out)), "oracle_weight_norm_score")
    return out


def select_sampled(s, e, k: int, k_top: int) -> np.ndarray:
    """k_top experts by top-k of s, k - k_top by weighted sampling without replacement (Appendix B);
    e holds one unit-exponential variate per neuron (float32)."""
    s = _f64(s)
    e = np.ascontiguousarray(e, dtype=np.float32)
    assert e.shape == s.shape
    idx = np.empty(k, dtype=np.int32)
    _check(_lib.oracle_select_sampled(s.shape[0], _p(s), e.ctypes.data_as(_fp), k, k_top,
                                      idx.ctypes.data_as(_ip)), "oracle_select_sampled")
    return idx


def jaccard(a, b) -> float:
    """|A n B| / |A u B| of two index sets (Section 4.1)."""
    a = np.ascontiguousarray(a, dtype=np.int32)
    b = np.ascontiguousarray(b, dtype=np.int32)
    out = ctypes.c_double(0.0)
    _check(_lib.oracle_jaccard(a.shape[0], a.ctypes.data_as(_ip), b.shape[0], b.ctypes.data_as(_ip),
                               ctypes.byref(out)), "oracle_jaccard")
    return float(out.value)


def prefill_select(X, Wg, W1, act: int, k: int, bg=None, b1=None) -> Tuple[np.ndarray, np.ndarray]:
    """The prompt-phase chain ff1 -> stat -> topk; returns (idx, s)."""
    s = stat(ff1(X, Wg, W1, act, bg, b1))
    return topk(s, k), s


def topk_margin(s, k: int) -> float:
    """(s_(k) - s_(k+1)) / s_(k): the relative gap at the selection boundary (inf if k == F)."""
    s = np.sort(_f64(s))[::-1]
    if k >= s.shape[0]:
        return float("inf")
    return float((s[k - 1] - s[k]) / s[k - 1]) if s[k - 1] > 0 else 0.0
