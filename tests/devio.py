"""Host <-> device plumbing for the GPU tests (torch is used for memory only)."""
import numpy as np
import torch

import paper_2404_01365_amd as G
import synth


def to_dev(a, dtype):
    """float32 host array (bf16-valued when dtype is bf16) -> device tensor of the storage type."""
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == synth.DT_BF16:
        bits = synth.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    """device tensor -> float64 host array (exact widening)."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.from_bf16_bits(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def dev_layer(Wg, W1, W2, act, dtype, bg=None, b1=None, b2=None):
    t = dict(Wg=to_dev(Wg, dtype), W1=to_dev(W1, dtype), W2=to_dev(W2, dtype),
             bg=to_dev(bg, dtype), b1=to_dev(b1, dtype), b2=to_dev(b2, dtype))
    L = G.layer(t["W1"], t["W2"], t["Wg"], act=act, dtype=G.BF16 if dtype == synth.DT_BF16 else G.F32,
                bg=t["bg"], b1=t["b1"], b2=t["b2"])
    return L, t


def empty_compact(L, k, tensors, interleaved=False, transposed=None):
    """Caller-allocated compact block for k neurons of L.  `interleaved` stores the three rows
    of a neuron side by side ([k][3][d], row stride 3d) instead of three separate matrices.
    `transposed`: "both" adds the output-feature-major copy W2t [d][ldt] next to W2, "only" keeps
    W2 in that form alone (Wg and W1 then sit side by side, [k][2][d], when interleaved)."""
    W1 = tensors["W1"]
    vec = lambda src: None if src is None else torch.empty((k,), dtype=W1.dtype, device="cuda")
    if transposed:
        ldt = -(-k // 512) * 512
        W2t = torch.full((L.d, ldt), float("nan"), dtype=W1.dtype, device="cuda")
        if transposed == "only":
            if interleaved:
                blk = torch.empty((k, 2, L.d), dtype=W1.dtype, device="cuda")
                mats = dict(Wg=None if tensors["Wg"] is None else blk[:, 0], W1=blk[:, 1], W2=None)
            else:
                mk = lambda: torch.empty((k, L.d), dtype=W1.dtype, device="cuda")
                mats = dict(Wg=None if tensors["Wg"] is None else mk(), W1=mk(), W2=None)
            c = dict(mats, bg=vec(tensors["bg"]), b1=vec(tensors["b1"]), b2=tensors["b2"], W2t=W2t)
            C = G.layer(c["W1"], None, c["Wg"], act=L.act, dtype=L.dtype, bg=c["bg"], b1=c["b1"], b2=c["b2"],
                        W2t=W2t, n=k, d=L.d)
            return C, c
    if interleaved:
        blk = torch.empty((k, 3, L.d), dtype=W1.dtype, device="cuda")
        mats = dict(Wg=None if tensors["Wg"] is None else blk[:, 0], W1=blk[:, 1], W2=blk[:, 2])
    else:
        mk = lambda: torch.empty((k, L.d), dtype=W1.dtype, device="cuda")
        mats = dict(Wg=None if tensors["Wg"] is None else mk(), W1=mk(), W2=mk())
    c = dict(mats, bg=vec(tensors["bg"]), b1=vec(tensors["b1"]), b2=tensors["b2"])
    if transposed:
        c["W2t"] = W2t
    C = G.layer(c["W1"], c["W2"], c["Wg"], act=L.act, dtype=L.dtype, bg=c["bg"], b1=c["b1"], b2=c["b2"],
                W2t=c.get("W2t"))
    return C, c


def workspace(nbytes):
    return torch.empty((max(nbytes, 256),), dtype=torch.uint8, device="cuda")


def max_rel(y, ref):
    """max_c |y_c - ref_c| / max_c |ref_c|  (error against the reference's inf-norm)."""
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(np.asarray(y, dtype=np.float64) - ref)) / (den if den > 0 else 1.0))


def round_like(y, dtype):
    """Round an fp64 reference once to the output storage type."""
    y32 = np.asarray(y, dtype=np.float64).astype(np.float32)
    return (synth.round_to_bf16(y32) if dtype == synth.DT_BF16 else y32).astype(np.float64)
