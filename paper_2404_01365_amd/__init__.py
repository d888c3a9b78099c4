"""Thin Python binding of libgriffin.so (the C ABI declared in include/griffin.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the current stream; nothing here
computes, and there is no CPU or PyTorch fallback -- if the library is missing the import
fails.  Function names match the C entry points.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgriffin.so")

OK, EINVAL, ESHAPE, EWORKSPACE, EUNSUPPORTED, EHIP = range(6)
ACT_SILU, ACT_GELU_TANH, ACT_RELU = 0, 1, 2
F32, BF16 = 0, 1
MAX_SEQS, MAX_BATCH = 256, 64


class GriffinError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.griffin_status_string(status).decode()
        if status == EHIP:
            msg += " (" + lib.griffin_last_hip_error().decode() + ")"
        super().__init__("%s: %s [status %d]" % (where, msg, status))


class griffin_layer(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("n", ctypes.c_int32), ("dtype", ctypes.c_int32), ("act", ctypes.c_int32),
        ("Wg", ctypes.c_void_p), ("W1", ctypes.c_void_p), ("W2", ctypes.c_void_p),
        ("ld", ctypes.c_int64),
        ("bg", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("b2", ctypes.c_void_p),
        ("W2t", ctypes.c_void_p), ("ldt", ctypes.c_int64),
    ]


def _load() -> ctypes.CDLL:
    # libgriffin.so needs libamdhip64.so.7.  PyTorch ships its own copy of that runtime; a
    # process must not end up with two HIP runtimes (the second one sees no device), so
    # PyTorch's is loaded first and the dynamic loader hands the same object to libgriffin.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python paper_2404_01365_amd/build.py` "
            "(there is no fallback path)" % LIB_PATH)
    return ctypes.CDLL(LIB_PATH)


lib = _load()

_vp, _i32, _i64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
_LP = ctypes.POINTER(griffin_layer)
_IP = ctypes.POINTER(ctypes.c_int32)

_SIGS = {
    "griffin_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "griffin_last_hip_error": (ctypes.c_char_p, []),
    "griffin_version": (ctypes.c_char_p, []),
    "griffin_k_from_fraction": (_i32, [_i32, ctypes.c_double]),
    "griffin_prefill_workspace_bytes": (_sz, [_LP, _i64, _i32, _i32]),
    "griffin_prefill_select": (ctypes.c_int, [_LP, _vp, _i64, _IP, _i32, _i32, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "griffin_topk": (ctypes.c_int, [_vp, _i32, _i32, _i32, _vp, _vp]),
    "griffin_stat_shared": (ctypes.c_int, [_vp, _IP, _i32, _i32, _vp, _vp]),
    "griffin_compact": (ctypes.c_int, [_LP, _vp, _i32, _LP, _vp]),
    "griffin_weight_norm_score": (ctypes.c_int, [_LP, _vp, _vp]),
    "griffin_select_sampled_workspace_bytes": (_sz, [_i32, _i32]),
    "griffin_select_sampled": (ctypes.c_int, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _sz, _vp]),
    "griffin_jaccard": (ctypes.c_int, [_vp, _i32, _i32, _vp, _vp]),
    "griffin_decode_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "griffin_trace_next_decode": (ctypes.c_int, [_vp, _vp, _vp]),
    "griffin_prompt_out_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "griffin_ff_prompt_out": (ctypes.c_int, [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _i64, _vp, _vp, _i64, _vp, _sz, _vp]),
    "griffin_prompt_phase_workspace_bytes": (_sz, [_LP, _i64, _i32]),
    "griffin_prompt_phase": (ctypes.c_int, [_LP, _vp, _i64, _vp, _i64, _IP, _i32, _i32, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "griffin_ff_decode": (ctypes.c_int, [_LP, _vp, _vp, _i32, _vp, _sz, _vp]),
    "griffin_ff_decode_static_max_bytes": (_sz, []),
    "griffin_ff_decode_static": (ctypes.c_int, [_LP, _vp, _vp, _i32, _vp]),
    "griffin_ff_decode_multi": (ctypes.c_int, [_LP, _i32, _vp, _vp, _vp, _sz, _vp]),
    "griffin_ff_decode_indexed": (ctypes.c_int, [_LP, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "griffin_index_sets_bytes": (_sz, [_i32, _i32]),
    "griffin_index_sets_build": (ctypes.c_int, [_vp, _i32, _i32, _i32, _vp, _sz, _vp]),
    "griffin_ff_decode_indexed_sets": (ctypes.c_int, [_LP, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _sz, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTS = tuple(_SIGS)


# ------------------------------------------------------------------ marshalling helpers
def _ptr(t) -> Optional[int]:
    """Device (or raw integer) address of a tensor; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise GriffinError(status, where)


def layer(W1, W2, Wg=None, *, act: int, dtype: Optional[int] = None, bg=None, b1=None, b2=None,
          d: Optional[int] = None, n: Optional[int] = None, ld: Optional[int] = None, W2t=None) -> griffin_layer:
    """Describe one FF block held in torch tensors ([n][d] neuron-major, contiguous rows).
    W2t: optional [d][ldt] copy of W2 in the paper's orientation (W2 may then be None)."""
    import torch
    if dtype is None:
        dtype = BF16 if W1.dtype == torch.bfloat16 else F32
    L = griffin_layer()
    L.n = W1.shape[0] if n is None else n
    L.d = W1.shape[1] if d is None else d
    L.ld = W1.stride(0) if ld is None else ld
    L.dtype, L.act = dtype, act
    L.Wg, L.W1, L.W2 = _ptr(Wg), _ptr(W1), _ptr(W2)
    L.bg, L.b1, L.b2 = _ptr(bg), _ptr(b1), _ptr(b2)
    L.W2t = _ptr(W2t)
    L.ldt = 0 if W2t is None else W2t.stride(0)
    # keep the tensors alive as long as the descriptor
    L._keep = (W1, W2, Wg, bg, b1, b2, W2t)
    return L


def _cu_array(cu_seqlens: Sequence[int]):
    arr = (ctypes.c_int32 * len(cu_seqlens))(*[int(v) for v in cu_seqlens])
    return arr


# ------------------------------------------------------------------ entry points
def griffin_version() -> str:
    return lib.griffin_version().decode()


def griffin_status_string(status: int) -> str:
    return lib.griffin_status_string(status).decode()


def griffin_k_from_fraction(d_ff: int, keep: float) -> int:
    return int(lib.griffin_k_from_fraction(d_ff, keep))


def griffin_prefill_workspace_bytes(L: griffin_layer, total_tokens: int, n_seqs: int = 1,
                                    have_z_out: bool = False) -> int:
    return int(lib.griffin_prefill_workspace_bytes(ctypes.byref(L), total_tokens, n_seqs, int(have_z_out)))


def griffin_prefill_select(L: griffin_layer, X, cu_seqlens: Sequence[int], k: int, idx_out, *,
                           s_out=None, Z_out=None, workspace, ldx: Optional[int] = None,
                           ldz: Optional[int] = None, stream=None) -> None:
    n_seqs = len(cu_seqlens) - 1
    if ldx is None:
        ldx = X.stride(0) if X is not None and X.dim() == 2 else L.d
    if ldz is None:
        ldz = Z_out.stride(0) if Z_out is not None else 0
    st = lib.griffin_prefill_select(ctypes.byref(L), _ptr(X), ldx, _cu_array(cu_seqlens), n_seqs, k,
                                    _ptr(idx_out), _ptr(s_out), _ptr(Z_out), ldz,
                                    _ptr(workspace), _nbytes(workspace), _stream(stream))
    _check(st, "griffin_prefill_select")


def griffin_topk(scores, k: int, idx_out, *, stream=None) -> None:
    n_rows, n = (1, scores.shape[0]) if scores.dim() == 1 else scores.shape
    _check(lib.griffin_topk(_ptr(scores), n_rows, n, k, _ptr(idx_out), _stream(stream)), "griffin_topk")


def griffin_stat_shared(s, cu_seqlens: Sequence[int], sbar_out, *, stream=None) -> None:
    n_seqs = len(cu_seqlens) - 1
    _check(lib.griffin_stat_shared(_ptr(s), _cu_array(cu_seqlens), n_seqs, s.shape[-1], _ptr(sbar_out),
                                   _stream(stream)), "griffin_stat_shared")


def griffin_weight_norm_score(L: griffin_layer, score_out, *, stream=None) -> None:
    _check(lib.griffin_weight_norm_score(ctypes.byref(L), _ptr(score_out), _stream(stream)),
           "griffin_weight_norm_score")


def griffin_select_sampled_workspace_bytes(n: int, k_top: int) -> int:
    return int(lib.griffin_select_sampled_workspace_bytes(n, k_top))


def griffin_select_sampled(s, e, k: int, k_top: int, idx_out, *, workspace, stream=None) -> None:
    _check(lib.griffin_select_sampled(_ptr(s), _ptr(e), s.shape[-1], k, k_top, _ptr(idx_out),
                                      _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "griffin_select_sampled")


def griffin_jaccard(idx, out, *, stream=None) -> None:
    n_sets, k = idx.shape
    _check(lib.griffin_jaccard(_ptr(idx), n_sets, k, _ptr(out), _stream(stream)), "griffin_jaccard")


def griffin_compact(L: griffin_layer, idx, k: int, C: griffin_layer, *, stream=None) -> None:
    _check(lib.griffin_compact(ctypes.byref(L), _ptr(idx), k, ctypes.byref(C), _stream(stream)),
           "griffin_compact")


def griffin_decode_workspace_bytes(d: int, n: int, batch: int = 1) -> int:
    return int(lib.griffin_decode_workspace_bytes(d, n, batch))


def griffin_ff_decode(C: griffin_layer, x, y, batch: int = 1, *, workspace, stream=None) -> None:
    _check(lib.griffin_ff_decode(ctypes.byref(C), _ptr(x), _ptr(y), batch, _ptr(workspace),
                                 _nbytes(workspace), _stream(stream)), "griffin_ff_decode")


def griffin_ff_decode_static_max_bytes() -> int:
    return int(lib.griffin_ff_decode_static_max_bytes())


def griffin_ff_decode_static(C: griffin_layer, x, y, batch: int = 1, *, stream=None) -> None:
    """griffin_ff_decode with the partial rows in the library's own device array (no workspace)."""
    _check(lib.griffin_ff_decode_static(ctypes.byref(C), _ptr(x), _ptr(y), batch, _stream(stream)),
           "griffin_ff_decode_static")


def griffin_ff_decode_multi(Cs: Sequence[griffin_layer], x, y, *, workspace, stream=None) -> None:
    arr = (griffin_layer * len(Cs))(*Cs)
    _check(lib.griffin_ff_decode_multi(arr, len(Cs), _ptr(x), _ptr(y), _ptr(workspace),
                                       _nbytes(workspace), _stream(stream)), "griffin_ff_decode_multi")


def griffin_ff_decode_indexed(L: griffin_layer, idx, k: int, batch: int, x, y, *, workspace,
                              stream=None) -> None:
    _check(lib.griffin_ff_decode_indexed(ctypes.byref(L), _ptr(idx), k, batch, _ptr(x), _ptr(y),
                                         _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "griffin_ff_decode_indexed")


def griffin_index_sets_bytes(n: int, batch: int) -> int:
    return int(lib.griffin_index_sets_bytes(n, batch))


def griffin_index_sets_build(idx, k: int, batch: int, n: int, sets, *, stream=None) -> None:
    _check(lib.griffin_index_sets_build(_ptr(idx), k, batch, n, _ptr(sets), _nbytes(sets), _stream(stream)),
           "griffin_index_sets_build")


def griffin_ff_decode_indexed_sets(L: griffin_layer, idx, k: int, sets, batch: int, x, y, *, workspace,
                                   stream=None) -> None:
    _check(lib.griffin_ff_decode_indexed_sets(ctypes.byref(L), _ptr(idx), k, _ptr(sets), batch, _ptr(x), _ptr(y),
                                              _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "griffin_ff_decode_indexed_sets")


def griffin_prompt_phase_workspace_bytes(L: griffin_layer, total_tokens: int, n_seqs: int) -> int:
    return int(lib.griffin_prompt_phase_workspace_bytes(ctypes.byref(L), total_tokens, n_seqs))


def griffin_prompt_phase(L: griffin_layer, W2p, X, cu_seqlens: Sequence[int], k: int, idx_out, Y, *,
                         s_out=None, workspace, ldx: Optional[int] = None, stream=None) -> None:
    """Selection and the prompt's own output from one Z (W2p is the paper's W_2, [d][d_ff])."""
    n_seqs = len(cu_seqlens) - 1
    if ldx is None:
        ldx = X.stride(0) if X is not None and X.dim() == 2 else L.d
    st = lib.griffin_prompt_phase(ctypes.byref(L), _ptr(W2p), W2p.stride(0), _ptr(X), ldx, _cu_array(cu_seqlens),
                                  n_seqs, k, _ptr(idx_out), _ptr(s_out), _ptr(Y), Y.stride(0),
                                  _ptr(workspace), _nbytes(workspace), _stream(stream))
    _check(st, "griffin_prompt_phase")


def griffin_trace_next_decode(event_begin: Optional[int], event_mid: Optional[int],
                              event_end: Optional[int]) -> None:
    """Arm one-shot hipEvent_t handles before / between / after the next decode call's two kernels."""
    _check(lib.griffin_trace_next_decode(event_begin, event_mid, event_end), "griffin_trace_next_decode")


def griffin_prompt_out_workspace_bytes(total_tokens: int, d_ff: int, d: int) -> int:
    return int(lib.griffin_prompt_out_workspace_bytes(total_tokens, d_ff, d))


def griffin_ff_prompt_out(Z, W2p, Y, *, b2=None, dtype: Optional[int] = None, workspace=None, stream=None) -> None:
    """Y = Z W2p^T + b2 for the prompt rows (W2p is the paper's W_2, [d][d_ff])."""
    import torch
    if dtype is None:
        dtype = BF16 if W2p.dtype == torch.bfloat16 else F32
    _check(lib.griffin_ff_prompt_out(_ptr(Z), Z.stride(0), Z.shape[0], Z.shape[1], W2p.shape[0], dtype,
                                     _ptr(W2p), W2p.stride(0), _ptr(b2), _ptr(Y), Y.stride(0),
                                     _ptr(workspace), _nbytes(workspace), _stream(stream)), "griffin_ff_prompt_out")
