"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the HIP runtime."""
import ctypes
import os
import re

import pytest

import paper_2404_01365_amd as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # never dereferenced on these paths (16- and 256-byte aligned)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "griffin.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(griffin_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert "griffin_prefill_select" in names and "griffin_compact" in names and "griffin_ff_decode" in names
    for name in names:
        assert hasattr(G.lib, name), name
    assert set(names) == set(G.EXPORTS)


def test_struct_layout_matches_header():
    # 4 x int32, 3 pointers, int64, 3 pointers, pointer, int64
    assert ctypes.sizeof(G.griffin_layer) == 16 + 24 + 8 + 24 + 16
    assert G.griffin_layer.ld.offset == 40 and G.griffin_layer.b2.offset == 64
    assert G.griffin_layer.W2t.offset == 72 and G.griffin_layer.ldt.offset == 80


def test_status_strings_and_version():
    assert G.griffin_status_string(G.OK) == "ok"
    assert "workspace" in G.griffin_status_string(G.EWORKSPACE)
    assert G.griffin_status_string(99) == "unknown status"
    assert "gfx950" in G.griffin_version()


def test_k_from_fraction():
    assert G.griffin_k_from_fraction(11008, 0.5) == 5504
    assert G.griffin_k_from_fraction(24576, 0.25) == 6144
    assert G.griffin_k_from_fraction(24576, 0.75) == 18432
    assert G.griffin_k_from_fraction(10, 0.0) == 1
    assert G.griffin_k_from_fraction(10, 2.0) == 10
    assert G.griffin_k_from_fraction(7, 0.5) == 4     # 3.5 rounds half up


def mk(d=256, n=688, dtype=G.F32, act=G.ACT_SILU, ld=None, Wg=FAKE, W1=FAKE, W2=FAKE, bg=None):
    L = G.griffin_layer()
    L.d, L.n, L.dtype, L.act = d, n, dtype, act
    L.Wg, L.W1, L.W2, L.ld = Wg, W1, W2, d if ld is None else ld
    L.bg = bg
    return L


def prefill(L, cu, k, X=FAKE, idx=FAKE, ws=FAKE, ws_bytes=1 << 40, ldx=None, Z=None, ldz=0):
    arr = (ctypes.c_int32 * len(cu))(*cu) if cu is not None else None
    return G.lib.griffin_prefill_select(ctypes.byref(L), X, L.d if ldx is None else ldx, arr,
                                        (len(cu) - 1) if cu is not None else 1, k, idx, None, Z, ldz,
                                        ws, ws_bytes, None)


def test_prefill_rejects_bad_arguments_without_hip():
    L = mk()
    assert prefill(mk(W1=None), [0, 64], 344) == G.EINVAL
    assert prefill(mk(dtype=7), [0, 64], 344) == G.EINVAL
    assert prefill(mk(act=3), [0, 64], 344) == G.EINVAL
    assert prefill(mk(d=250), [0, 64], 344) == G.ESHAPE          # d not a multiple of 8
    assert prefill(mk(ld=128), [0, 64], 344) == G.ESHAPE         # ld < d
    assert prefill(mk(W1=FAKE + 4), [0, 64], 344) == G.ESHAPE    # misaligned rows
    assert prefill(mk(Wg=None, bg=FAKE), [0, 64], 344) == G.EINVAL
    assert prefill(L, [0, 64], 0) == G.ESHAPE
    assert prefill(L, [0, 64], 689) == G.ESHAPE
    assert prefill(L, [1, 64], 344) == G.ESHAPE                  # cu[0] != 0
    assert prefill(L, [0, 64, 32], 344) == G.ESHAPE              # decreasing
    assert prefill(L, None, 344) == G.EINVAL
    assert prefill(L, [0, 64], 344, idx=None) == G.EINVAL
    assert prefill(L, [0, 64], 344, X=None) == G.EINVAL
    assert prefill(L, [0, 64], 344, ldx=100) == G.ESHAPE
    assert prefill(L, [0, 64], 344, Z=FAKE, ldz=10) == G.ESHAPE
    assert prefill(L, [0, 64], 344, ws=None) == G.EWORKSPACE
    assert prefill(L, [0, 64], 344, ws_bytes=16) == G.EWORKSPACE
    assert prefill(L, [0, 64], 344, ws=FAKE + 16) == G.EWORKSPACE  # not 256-byte aligned
    assert prefill(L, [0] * (G.MAX_SEQS + 2), 344) == G.EUNSUPPORTED


def test_workspace_queries():
    L = mk(d=4096, n=11008, dtype=G.BF16)
    full = G.griffin_prefill_workspace_bytes(L, 512, 1, False)
    lean = G.griffin_prefill_workspace_bytes(L, 512, 1, True)
    assert full - lean == 512 * 11008 * 4          # Z lives in the workspace unless Z_out is given
    assert lean > 0 and lean % 256 == 0
    assert G.griffin_prefill_workspace_bytes(mk(d=250), 512, 1, False) == 0
    assert G.griffin_decode_workspace_bytes(4096, 5504, 1) == 256 * 4096 * 4
    assert G.griffin_decode_workspace_bytes(4096, 5504, 0) == 0
    assert G.griffin_decode_workspace_bytes(4096, 5504, G.MAX_BATCH + 1) == 0


def test_compact_and_decode_reject_bad_arguments_without_hip():
    L = mk()
    C = mk(n=344)
    lib = G.lib
    assert lib.griffin_compact(ctypes.byref(L), None, 344, ctypes.byref(C), None) == G.EINVAL
    assert lib.griffin_compact(ctypes.byref(L), FAKE, 343, ctypes.byref(C), None) == G.ESHAPE
    assert lib.griffin_compact(ctypes.byref(L), FAKE, 344, ctypes.byref(mk(n=344, d=128)), None) == G.ESHAPE
    assert lib.griffin_compact(ctypes.byref(L), FAKE, 344, ctypes.byref(mk(n=344, Wg=None)), None) == G.EINVAL
    assert lib.griffin_compact(None, FAKE, 344, ctypes.byref(C), None) == G.EINVAL

    assert lib.griffin_ff_decode(ctypes.byref(C), None, FAKE, 1, FAKE, 1 << 30, None) == G.EINVAL
    assert lib.griffin_ff_decode(ctypes.byref(C), FAKE, FAKE, 1, None, 0, None) == G.EWORKSPACE
    assert lib.griffin_ff_decode(ctypes.byref(C), FAKE, FAKE, 1, FAKE, 8, None) == G.EWORKSPACE
    assert lib.griffin_ff_decode(ctypes.byref(C), FAKE, FAKE, G.MAX_BATCH + 1, FAKE, 1 << 40, None) == G.EUNSUPPORTED
    assert lib.griffin_ff_decode(ctypes.byref(C), FAKE + 2, FAKE, 1, FAKE, 1 << 30, None) == G.ESHAPE
    assert lib.griffin_ff_decode(ctypes.byref(C), FAKE, FAKE, 0, FAKE, 1 << 30, None) == G.OK   # nothing to do
    assert lib.griffin_ff_decode_indexed(ctypes.byref(L), None, 344, 1, FAKE, FAKE, FAKE, 1 << 30, None) == G.EINVAL
    assert lib.griffin_ff_decode_indexed(ctypes.byref(L), FAKE, 689, 1, FAKE, FAKE, FAKE, 1 << 30, None) == G.ESHAPE
    two = (G.griffin_layer * 2)(mk(n=344), mk(n=300))
    assert lib.griffin_ff_decode_multi(two, 2, FAKE, FAKE, FAKE, 1 << 30, None) == G.ESHAPE
    assert lib.griffin_ff_decode_multi(None, 2, FAKE, FAKE, FAKE, 1 << 30, None) == G.EINVAL
    # per-row blocks are streamed neuron-major: a block that carries only the transposed copy of W2 is
    # refused on the host (no launch), whichever row it belongs to
    def only_w2t():
        B = mk(d=512, n=512, dtype=G.BF16, W2=None)
        B.W2t, B.ldt = FAKE, 512
        return B
    assert lib.griffin_ff_decode_multi((G.griffin_layer * 2)(only_w2t(), only_w2t()), 2, FAKE, FAKE, FAKE, 1 << 30, None) == G.EUNSUPPORTED
    assert lib.griffin_ff_decode_multi((G.griffin_layer * 2)(mk(d=512, n=512, dtype=G.BF16), only_w2t()), 2,
                                       FAKE, FAKE, FAKE, 1 << 30, None) == G.EUNSUPPORTED
    assert lib.griffin_ff_decode_multi((G.griffin_layer * 1)(only_w2t()), 1, FAKE, FAKE, FAKE, 1 << 30, None) == G.EUNSUPPORTED

    assert lib.griffin_topk(None, 1, 10, 3, FAKE, None) == G.EINVAL
    assert lib.griffin_topk(FAKE, 1, 10, 11, FAKE, None) == G.ESHAPE
    assert lib.griffin_topk(FAKE, 0, 10, 3, FAKE, None) == G.OK
    cu = (ctypes.c_int32 * 2)(0, 5)
    assert lib.griffin_stat_shared(None, cu, 1, 10, FAKE, None) == G.EINVAL


def test_selectors_and_prompt_out_reject_bad_arguments_without_hip():
    L = mk()
    lib = G.lib
    assert lib.griffin_weight_norm_score(ctypes.byref(L), None, None) == G.EINVAL
    assert lib.griffin_weight_norm_score(None, FAKE, None) == G.EINVAL
    assert G.griffin_select_sampled_workspace_bytes(1000, 10) % 256 == 0
    assert G.griffin_select_sampled_workspace_bytes(1000, 1001) == 0
    big = 1 << 30
    assert lib.griffin_select_sampled(None, FAKE, 100, 10, 5, FAKE, FAKE, big, None) == G.EINVAL
    assert lib.griffin_select_sampled(FAKE, FAKE, 100, 101, 5, FAKE, FAKE, big, None) == G.ESHAPE
    assert lib.griffin_select_sampled(FAKE, FAKE, 100, 10, 11, FAKE, FAKE, big, None) == G.ESHAPE      # k_top > k
    assert lib.griffin_select_sampled(FAKE, FAKE, 100, 10, 5, FAKE, None, 0, None) == G.EWORKSPACE
    assert lib.griffin_select_sampled(FAKE, FAKE, 100, 10, 5, FAKE, FAKE, 64, None) == G.EWORKSPACE
    assert lib.griffin_jaccard(None, 2, 10, FAKE, None) == G.EINVAL
    assert lib.griffin_jaccard(FAKE, 0, 10, FAKE, None) == G.ESHAPE
    assert lib.griffin_jaccard(FAKE, G.MAX_SEQS + 1, 10, FAKE, None) == G.ESHAPE
    # prompt output: Z, ldz, tokens, d_ff, d, dtype, W2p, ldw, b2, Y, ldy, ws, ws_bytes, stream
    po = lib.griffin_ff_prompt_out
    assert po(None, 688, 64, 688, 256, G.F32, FAKE, 688, None, FAKE, 256, None, 0, None) == G.EINVAL
    assert po(FAKE, 600, 64, 688, 256, G.F32, FAKE, 688, None, FAKE, 256, None, 0, None) == G.ESHAPE   # ldz < d_ff
    assert po(FAKE, 688, 64, 688, 256, 7, FAKE, 688, None, FAKE, 256, None, 0, None) == G.EINVAL


def test_prompt_phase_rejects_bad_arguments_without_hip():
    L = mk()
    cu = (ctypes.c_int32 * 2)(0, 64)
    big = 1 << 40
    # L, W2p, ldw, X, ldx, cu, n_seqs, k, idx_out, s_out, Y, ldy, ws, ws_bytes, stream
    pp = lambda **kw: G.lib.griffin_prompt_phase(
        ctypes.byref(kw.get("L", L)), kw.get("W2p", FAKE), kw.get("ldw", 688), kw.get("X", FAKE), kw.get("ldx", 256), cu, 1,
        kw.get("k", 344), kw.get("idx", FAKE), None, kw.get("Y", FAKE), kw.get("ldy", 256), kw.get("ws", FAKE),
        kw.get("ws_bytes", big), None)
    assert pp(W2p=None) == G.EINVAL
    assert pp(Y=None) == G.EINVAL
    assert pp(idx=None) == G.EINVAL
    assert pp(X=None) == G.EINVAL
    assert pp(L=mk(W1=None)) == G.EINVAL
    assert pp(k=0) == G.ESHAPE
    assert pp(k=689) == G.ESHAPE
    assert pp(ldw=600) == G.ESHAPE            # W_2's rows shorter than D_ff
    assert pp(ldy=100) == G.ESHAPE
    assert pp(ldx=100) == G.ESHAPE
    assert pp(ws=None) == G.EWORKSPACE
    assert pp(ws_bytes=1024) == G.EWORKSPACE
    assert pp(ws=FAKE + 16) == G.EWORKSPACE
    # the workspace holds what griffin_prefill_select needs (Z included) and what the output product needs
    Lb = mk(d=4096, n=11008, dtype=G.BF16)
    both = G.griffin_prompt_phase_workspace_bytes(Lb, 512, 1)
    assert both >= G.griffin_prefill_workspace_bytes(Lb, 512, 1, False) + G.griffin_prompt_out_workspace_bytes(512, 11008, 4096)
    assert both % 256 == 0
    assert G.griffin_prompt_phase_workspace_bytes(mk(d=250), 512, 1) == 0


def test_index_sets_reject_bad_arguments_without_hip():
    lib = G.lib
    assert G.griffin_index_sets_bytes(14336, 16) == 14336 * 4
    assert G.griffin_index_sets_bytes(14336, 17) == 2 * 14336 * 4        # one word per neuron and group of 16 rows
    assert G.griffin_index_sets_bytes(0, 16) == 0 and G.griffin_index_sets_bytes(100, G.MAX_BATCH + 1) == 0
    big = 1 << 30
    # idx, k, batch, n, sets, sets_bytes, stream
    assert lib.griffin_index_sets_build(None, 10, 4, 100, FAKE, big, None) == G.EINVAL
    assert lib.griffin_index_sets_build(FAKE, 10, 4, 100, None, big, None) == G.EINVAL
    assert lib.griffin_index_sets_build(FAKE, 101, 4, 100, FAKE, big, None) == G.ESHAPE
    assert lib.griffin_index_sets_build(FAKE, 10, 4, 100, FAKE + 2, big, None) == G.ESHAPE
    assert lib.griffin_index_sets_build(FAKE, 10, 4, 100, FAKE, 399, None) == G.EWORKSPACE
    assert lib.griffin_index_sets_build(FAKE, 10, G.MAX_BATCH + 1, 100, FAKE, big, None) == G.EUNSUPPORTED
    assert lib.griffin_index_sets_build(FAKE, 10, 0, 100, FAKE, 0, None) == G.OK
    L = mk(d=512, n=688, dtype=G.BF16)
    # L, idx, k, sets, batch, x, y, ws, ws_bytes, stream
    ds = lib.griffin_ff_decode_indexed_sets
    assert ds(ctypes.byref(L), None, 10, FAKE, 8, FAKE, FAKE, FAKE, big, None) == G.EINVAL
    assert ds(ctypes.byref(L), FAKE, 10, None, 8, FAKE, FAKE, FAKE, big, None) == G.EINVAL
    assert ds(ctypes.byref(L), FAKE, 689, FAKE, 8, FAKE, FAKE, FAKE, big, None) == G.ESHAPE
    assert ds(ctypes.byref(L), FAKE, 10, FAKE, 8, FAKE, FAKE, None, 0, None) == G.EWORKSPACE
    assert ds(ctypes.byref(L), FAKE, 10, FAKE, 0, FAKE, FAKE, FAKE, big, None) == G.OK


def test_batch_decode_workspace_covers_the_matrix_core_path():
    # 16 rows through one block: partial rows [16][ranges][d] plus the table of Z [n][16]
    d, n = 4096, 5504
    need16 = G.griffin_decode_workspace_bytes(d, n, 16)
    assert need16 >= (16 * 32 * d + n * 16) * 4
    assert G.griffin_decode_workspace_bytes(d, n, 16) <= G.griffin_decode_workspace_bytes(d, n, 64)
    # shapes the matrix-core path does not take keep the four-rows-per-pass size
    assert G.griffin_decode_workspace_bytes(8192, 500, 16) == G.griffin_decode_workspace_bytes(8192, 500, 13) // 13 * 16


def test_decode_static_judges_sizes_before_it_touches_the_runtime():
    lib = G.lib
    assert G.griffin_ff_decode_static_max_bytes() == 8 << 20
    C = mk(d=4096, n=5504, dtype=G.BF16)
    # C, x, y, batch, stream
    assert lib.griffin_ff_decode_static(None, FAKE, FAKE, 1, None) == G.EINVAL
    assert lib.griffin_ff_decode_static(ctypes.byref(C), None, FAKE, 1, None) == G.EINVAL
    assert lib.griffin_ff_decode_static(ctypes.byref(C), FAKE, FAKE, G.MAX_BATCH + 1, None) == G.EUNSUPPORTED
    assert G.griffin_decode_workspace_bytes(4096, 5504, 1) <= G.griffin_ff_decode_static_max_bytes()
    assert G.griffin_decode_workspace_bytes(4096, 5504, 16) > G.griffin_ff_decode_static_max_bytes()
    assert lib.griffin_ff_decode_static(ctypes.byref(C), FAKE, FAKE, 16, None) == G.EWORKSPACE     # more than the array holds
    assert lib.griffin_ff_decode_static(ctypes.byref(C), FAKE, FAKE, 0, None) == G.OK              # nothing to do
