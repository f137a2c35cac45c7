"""HIP graph replays of the library's calls.  No entry point allocates, synchronises or clears
memory behind the caller's back, so a captured sequence of calls must give the oracle's result
on every replay: with other work and synchronisations between the replays, and with new inputs
copied into the captured buffers each time."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from paper_2208_00763_amd.cnn import PackedCnn
    from gpu_util import conv1d_plan, dnn_plan, dev, compact, oracle_conv1d, oracle_cnn
    from oracle import direct


def _capture(fn):
    """One eager run on a side stream first (first-call set-up stays outside the capture), then the graph."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return graph


def _between_replays():
    # the program's own eager work and a synchronisation between two replays
    junk = torch.arange(1 << 16, device="cuda", dtype=torch.int32)
    junk.mul_(3).add_(1)
    torch.cuda.synchronize()


def test_graph_replay_conv1d_packed_and_unpacked():
    rows, length, taps, bits = 37, 6007, 5, 4
    plan = conv1d_plan(bits, True, True, taps)
    x0 = wl.uniform_values(wl.rng_for("gr1", 0), (rows, length), bits, True)
    g = wl.uniform_values(wl.rng_for("gr1g"), (taps,), bits, True)
    x_bd, g_d = compact(x0, bits).clone(), dev(g)
    out_len = length - taps + 1
    y_p = torch.zeros(rows * out_len, dtype=torch.int32, device="cuda")
    y_u = torch.zeros(rows * out_len, dtype=torch.int32, device="cuda")

    def calls():
        hk.hikonv_conv1d(plan, x_bd, hk.FMT_BITDENSE, rows, length, g_d, taps, hk.OUT_VALID, y_p)
        hk.hikonv_conv1d_unpacked(bits, bits, hk.signedness(True, True), x_bd, hk.FMT_BITDENSE, rows, length, g_d, taps,
                                  hk.OUT_VALID, y_u)

    graph = _capture(calls)
    for rep in range(4):
        x = wl.uniform_values(wl.rng_for("gr1", rep + 1), (rows, length), bits, True)
        x_bd.copy_(compact(x, bits))
        y_p.fill_(-5)
        y_u.fill_(-5)
        _between_replays()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle_conv1d(x, g, hk.OUT_VALID)
        assert np.array_equal(y_p.cpu().numpy().reshape(ref.shape), ref), rep
        assert np.array_equal(y_u.cpu().numpy().reshape(ref.shape), ref), rep


def test_graph_replay_layer_without_allocation():
    """hikonv_conv2d_noalloc is the layer call for callers under graph capture: captured and replayed."""
    n, c, h, w, co, k = 2, 24, 19, 23, 16, 3
    plan = dnn_plan(4, 4, True, True, k, 0)
    wt = wl.uniform_values(wl.rng_for("gr2w"), (co, c, k, k), 4, True)
    x_d = torch.zeros(n * c * h * w, dtype=torch.uint8, device="cuda")
    w_d = dev(wt)
    y = torch.zeros(n * co * h * w, dtype=torch.int32, device="cuda")
    graph = _capture(lambda: hk.hikonv_conv2d_noalloc(plan, x_d, hk.FMT_INT8, n, c, h, w, w_d, co, k, k, 1, 1, y))
    for rep in range(4):
        x = wl.uniform_values(wl.rng_for("gr2", rep), (n, c, h, w), 4, True)
        x_d.copy_(dev(x).view(-1))
        y.fill_(-5)
        _between_replays()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().reshape(n, co, h, w), direct.conv2d(x, wt, 1, 1)), rep


def test_graph_replay_cnn_chain_one_kernel_per_layer():
    h, w = 38, 70
    x0, weights, specs = wl.config5(h, w)
    _, shifts = oracle_cnn(x0, weights, specs)
    net = PackedCnn([dev(wt).view(torch.uint8).reshape(wt.shape) for wt in weights], specs, fused="layer",
                    keep_accs=False, objective=hk.OBJ_MEASURED_COST)
    x_bd = compact(x0.reshape(3 * h, w), 4).clone()
    out = {}

    def forward():
        out["last"], _ = net.forward(x_bd, 1, h, w, shifts)

    graph = _capture(forward)
    for rep in range(3):
        x = wl.uniform_values(wl.rng_for("gr3", rep), x0.shape, 4, False)
        x_bd.copy_(compact(x.reshape(3 * h, w), 4))
        out["last"].fill_(-5)
        _between_replays()
        graph.replay()
        torch.cuda.synchronize()
        ref_accs, _ = oracle_cnn(x, weights, specs, shifts=shifts)
        assert np.array_equal(out["last"].cpu().numpy().reshape(ref_accs[-1].shape), ref_accs[-1]), rep
