"""The decode entry point that allocates nothing: partial rows in the library's own device array."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2404_01365_amd as G
import synth
from devio import dev_layer, max_rel, to_dev, to_host, workspace

pytestmark = pytest.mark.gpu


def both_ways(L, x_dev, batch):
    """y through griffin_ff_decode_static (called through the C ABI) and through griffin_ff_decode."""
    y_static = torch.full_like(x_dev, float("nan"))
    st = torch.cuda.current_stream().cuda_stream or None
    rc = G.lib.griffin_ff_decode_static(ctypes.byref(L), x_dev.data_ptr(), y_static.data_ptr(), batch, st)
    assert rc == G.OK, G.griffin_status_string(rc)
    y_ws = torch.full_like(x_dev, float("nan"))
    G.griffin_ff_decode(L, x_dev, y_ws, batch, workspace=workspace(G.griffin_decode_workspace_bytes(L.d, L.n, batch)))
    torch.cuda.synchronize()
    return to_host(y_static), to_host(y_ws)


def test_decode_static_matches_decode_on_two_calls_the_second_smaller():
    dtype, act = synth.DT_BF16, synth.ACT_SILU
    # first call: a wide block, the array filled up to 256 partial rows of 4096 floats
    c1 = synth.small_case(401, 4096, 700, 4, dtype, T=2)
    L1, _ = dev_layer(c1["Wg"], c1["W1"], c1["W2"], act, dtype)
    x1 = to_dev(c1["xt"][0], dtype)
    # second call: a narrower, shorter block with biases, which leaves most of the array as the first call left it
    c2 = synth.small_case(402, 1024, 130, 4, dtype, T=2, with_bias=True)
    L2, _ = dev_layer(c2["Wg"], c2["W1"], c2["W2"], act, dtype, c2["bg"], c2["b1"], c2["b2"])
    x2 = to_dev(c2["xt"][1], dtype)
    torch.cuda.synchronize()
    a1, b1 = both_ways(L1, x1, 1)
    a2, b2 = both_ways(L2, x2, 1)
    # same kernels, same order of additions: bit for bit, and within the output tolerance of the oracle
    assert np.array_equal(a1, b1) and np.array_equal(a2, b2)
    assert max_rel(a1, oracle.ff_decode(c1["xt"][0], c1["Wg"], c1["W1"], c1["W2"], act)) <= 2e-2
    assert max_rel(a2, oracle.ff_decode(c2["xt"][1], c2["Wg"], c2["W1"], c2["W2"], act, c2["bg"], c2["b1"], c2["b2"])) <= 2e-2
    # two rows through one block, then one row again (fp32 block)
    c3 = synth.small_case(403, 264, 77, 4, synth.DT_F32, T=2)
    L3, _ = dev_layer(c3["Wg"], c3["W1"], c3["W2"], act, synth.DT_F32)
    a3, b3 = both_ways(L3, to_dev(c3["xt"], synth.DT_F32), 2)
    assert np.array_equal(a3, b3)
    for b in range(2):
        assert max_rel(a3[b], oracle.ff_decode(c3["xt"][b], c3["Wg"], c3["W1"], c3["W2"], act)) <= 1e-5
    a4, b4 = both_ways(L1, to_dev(c1["xt"][1], dtype), 1)
    assert np.array_equal(a4, b4)


def test_decode_static_rejects_what_does_not_fit():
    dtype, act = synth.DT_BF16, synth.ACT_SILU
    c = synth.small_case(404, 4096, 64, 4, dtype, T=16)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype)
    x = to_dev(c["xt"], dtype)
    y = torch.empty_like(x)
    assert G.griffin_decode_workspace_bytes(4096, 64, 16) > G.griffin_ff_decode_static_max_bytes()
    assert G.lib.griffin_ff_decode_static(ctypes.byref(L), x.data_ptr(), y.data_ptr(), 16, None) == G.EWORKSPACE
    assert G.lib.griffin_ff_decode_static(ctypes.byref(L), None, y.data_ptr(), 1, None) == G.EINVAL
    assert G.lib.griffin_ff_decode_static(ctypes.byref(L), x.data_ptr(), y.data_ptr(), 0, None) == G.OK


def test_decode_static_replays_in_a_hip_graph():
    """What the entry point is for: three decode calls recorded into a HIP graph (after one eager call on the
    device, which looks the array's address up) and replayed with new inputs, eager work and synchronisations
    between the replays; every replay must give the eager result bit for bit."""
    dtype, act, d, n, T = synth.DT_BF16, synth.ACT_SILU, 2048, 700, 3
    c = synth.small_case(405, d, n, 4, dtype, T=3 * T)
    L, _ = dev_layer(c["Wg"], c["W1"], c["W2"], act, dtype)
    xs = to_dev(c["xt"], dtype)                               # three sets of T inputs
    x_buf = torch.empty((T, d), dtype=xs.dtype, device="cuda")
    y_buf = torch.empty((T, d), dtype=xs.dtype, device="cuda")
    x_buf.copy_(xs[:T])
    G.griffin_ff_decode_static(L, x_buf[0], y_buf[0], 1)      # the eager call before any capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for t in range(T):
                G.griffin_ff_decode_static(L, x_buf[t], y_buf[t], 1)
    torch.cuda.synchronize()
    ws = workspace(G.griffin_decode_workspace_bytes(d, n, 1))
    for rep in range(3):
        x_buf.copy_(xs[rep * T:(rep + 1) * T])
        y_buf.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = to_host(y_buf)
        want = torch.empty_like(y_buf)
        for t in range(T):                                    # eager, through the entry point with a workspace
            G.griffin_ff_decode(L, x_buf[t], want[t], 1, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(got, to_host(want)), rep
        ref = oracle.ff_decode(c["xt"][rep * T], c["Wg"], c["W1"], c["W2"], act)
        assert max_rel(got[0], ref) <= 2e-2
