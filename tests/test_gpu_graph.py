"""Parity in the mode the benchmark runs: per-frame HIP graphs of the fused int8 stack, replayed over whole
sequences and across the sequence boundary; and graphs mixed with eager steps (nothing a replayed step does
may depend on host-side state)."""
import os
import sys

import numpy as np
import pytest

import oracle
import rrm_synth as S
from gpu_util import assert_matches, to_device

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

pytestmark = pytest.mark.gpu


def _oracle_stack(st, frame_one_stream):
    """every layer's projection of one stream's frame, through the oracle and its own nonlinearity"""
    ys, x = [], frame_one_stream
    for i, l in enumerate(st.cfg["layers"]):
        y = oracle.dense(l["shape"].with_n(1), S.I8, l["weights"], l["bias"], x)
        ys.append(y)
        x = oracle.relu_requant_pool(y, st.shifts[i], l["pool"])
    return ys, x


def test_benchmark_graphs_replayed_over_two_sequences_and_the_wrap():
    """bench.Stack exactly as the benchmark builds and captures it (fused f, one graph per frame of two 32-frame
    sequences), replayed 0..63 and on into the next pass (64, 65 = frames 0, 1 again): sampled streams of every
    layer's stored projection, and of the last layer's f output, against the oracle on every frame."""
    import torch
    import bench
    n, sample = 64, (0, 37, 63)
    st = bench.Stack(n, T=32, fuse=True)
    st.set_path(0)
    st.capture()
    nf = len(st.frames)
    assert nf == 64
    # the capture ran frames[0] eagerly and then captured (not ran) the graphs: start from a clean state
    for L in st.layers:
        L.reset()
    for buf in st.bufs:
        buf.fill_(-1)
    torch.cuda.synchronize()
    for k in range(nf + 2):
        st.graph[k % nf].replay()
        torch.cuda.synchronize()
        got = [L.y_snapshot() for L in st.layers]
        for s in sample:
            ys, x_last = _oracle_stack(st, np.ascontiguousarray(st.host_frames[k % nf][s:s + 1]))
            for i, l in enumerate(st.cfg["layers"]):
                assert_matches(got[i][s:s + 1].cpu().numpy(), ys[i], S.I8, f"replay {k} {l['name']} stream {s}")
            assert np.array_equal(st.bufs[-1][s:s + 1].cpu().numpy(), x_last), f"replay {k}: f of the last layer, stream {s}"
    stats = st.layers[2].stats()
    assert stats["delta_steps"] == nf + 2  # counted on the device: replays advance it
    for L in st.layers:
        L.destroy()


@pytest.mark.parametrize("fuse", [False, True])
def test_dense_and_delta_graphs_mixed_with_eager_steps(fuse):
    """A dense ("path" = 2) graph and a delta graph of a two-layer stack, replayed in mixed order with eager
    steps in between: the incremental nonlinearity (and the fused consumer) must see what the last step wrote,
    whichever way that step was issued."""
    import torch
    import paper_1802_09723_amd as rrm
    cfg = S.config1(n=2, T=6)
    l0, l1 = cfg["layers"][0], cfg["layers"][1]
    A = rrm.Layer(l0["shape"], S.I8, l0["weights"], l0["bias"])
    B = rrm.Layer(l1["shape"], S.I8, l1["weights"], l1["bias"])
    y0 = oracle.dense(l0["shape"], S.I8, l0["weights"], l0["bias"], cfg["frames"][0])
    shift = oracle.calibrate_shift(y0)
    ho, wo = A.y_shape[1], A.y_shape[2]
    po, qo = (ho - 3) // 2 + 1, (wo - 3) // 2 + 1
    buf = torch.full((2, po, qo, l0["shape"].c_out), -1, dtype=torch.int8, device="cuda")
    frames = [to_device(f, S.I8) for f in cfg["frames"]]
    xin = torch.empty_like(frames[0])  # static input of the graphs

    def step(path):
        A.set_option("path", path)
        A.step(xin)
        if fuse and path != 2:
            B.step_from_projection(A, shift, True)
        else:
            A.relu_requant_pool_changed(buf, shift, True)
            B.step(buf)

    xin.copy_(frames[0])
    step(0)  # warm-up outside capture
    torch.cuda.synchronize()
    graphs = {}
    for path in (0, 2):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(path)
        graphs[path] = g
    for L in (A, B):
        L.reset()
    buf.fill_(-1)
    # (mode, frame): eager delta, dense replay, delta replay, eager dense, delta replay, delta replay
    plan = [("e0", 0), ("g2", 1), ("g0", 2), ("e2", 3), ("g0", 4), ("g0", 5), ("g2", 0), ("e0", 1)]
    for mode, f in plan:
        xin.copy_(frames[f])
        if mode[0] == "g":
            graphs[int(mode[1])].replay()
        else:
            step(int(mode[1]))
        torch.cuda.synchronize()
        ya = oracle.dense(l0["shape"], S.I8, l0["weights"], l0["bias"], cfg["frames"][f])
        x1 = oracle.relu_requant_pool(ya, shift, True)
        yb = oracle.dense(l1["shape"], S.I8, l1["weights"], l1["bias"], x1)
        assert_matches(A.y_snapshot().cpu().numpy(), ya, S.I8, f"{mode} frame {f} conv1")
        assert_matches(B.y_snapshot().cpu().numpy(), yb, S.I8, f"{mode} frame {f} conv2")
        if not (fuse and mode[1] == "0"):
            assert np.array_equal(buf.cpu().numpy(), x1), f"{mode} frame {f}: incremental nonlinearity"
    A.destroy()
    B.destroy()


def test_many_subtiles_power_of_two_grid():
    """Sub-tile ids beyond the range where a bare reciprocal multiply is exact: 257 streams of a 256 x 256
    output (64 x 64 sub-tiles per image).  A change in the last stream's last sub-tile must land there."""
    import torch
    import paper_1802_09723_amd as rrm
    n, hw = 257, 256
    shp = S.conv_shape(hw, hw, 16, 4, 3, 1, 1, n=n)
    rng = S.rng_for(S.seed_for(0, 61))
    w = S.draw_i8_weight(rng, shp.w_shape)
    b = S.draw_i32_bias(rng, 4)
    L = rrm.Layer(shp, S.I8, w, b)
    L.set_option("path", 1)  # the sparse path also for the first (all-changed) frame
    x0 = S.draw_i8_act(rng, (1, hw, hw, 16))
    xd = torch.from_numpy(x0).cuda().expand(n, hw, hw, 16).contiguous()
    L.step(xd)
    shp1 = shp.with_n(1)
    want0 = oracle.dense(shp1, S.I8, w, b, x0)
    got = L.y_snapshot()
    for s in (0, 15, 16, 255, 256):
        assert_matches(got[s:s + 1].cpu().numpy(), want0, S.I8, f"frame 0 stream {s}")
    # second frame: the last 2 x 2 positions of streams 16 and 256 change
    x1 = x0.copy()
    x1[0, -2:, -2:, :] = S.draw_i8_act(rng, (2, 2, 16))
    xd[16, -2:, -2:, :] = torch.from_numpy(x1[0, -2:, -2:, :]).cuda()
    xd[256, -2:, -2:, :] = torch.from_numpy(x1[0, -2:, -2:, :]).cuda()
    L.step(xd)
    want1 = oracle.dense(shp1, S.I8, w, b, x1)
    got = L.y_snapshot()
    for s, want in ((0, want0), (15, want0), (16, want1), (17, want0), (255, want0), (256, want1)):
        assert_matches(got[s:s + 1].cpu().numpy(), want, S.I8, f"frame 1 stream {s}")
    L.destroy()


def _replay_case(seq, **opts):
    """A whole-sequence graph (ping-pong through the frames, so that it ends where it starts) of one layer, replayed
    three times with eager steps and a reset in between; after every replay and eager step the stored projection is the
    oracle's dense projection of the frame last stepped."""
    import torch
    from gpu_util import make_layer
    L = make_layer(seq, **opts)
    xs = [to_device(f, seq.dtype) for f in seq.frames]
    want = [oracle.dense(seq.shape, seq.dtype, seq.weights, seq.bias, f) for f in seq.frames]
    for x in xs:  # eager pass: the snapshot is at the last frame
        L.step(x)
    torch.cuda.synchronize()
    T = len(xs)
    order = list(range(T - 2, -1, -1)) + list(range(1, T))  # T-2 .. 0 .. T-1
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for k in order:
            L.step(xs[k])
    def check(k, what):
        assert_matches(L.y_snapshot().cpu().numpy(), want[k], seq.dtype, f"{seq.name} {what}", 1e-3)
    s0 = L.stats()["delta_steps"]
    g.replay(); check(T - 1, "replay 1")
    L.step(xs[0]); check(0, "eager step after replay 1")
    L.step(xs[T - 1])
    g.replay(); check(T - 1, "replay 2")
    L.reset()
    L.step(xs[T - 1]); check(T - 1, "first step after reset")
    g.replay(); check(T - 1, "replay 3")
    if seq.dtype != S.BIN:  # (a binary layer's first step after a reset is a dense one)
        assert L.stats()["delta_steps"] == len(order) + 1  # (the reset cleared the counters; replays advance them)
    L.destroy()


@pytest.mark.parametrize("case", ["scatter_bf16", "scatter_i8", "binary_one_launch", "binary_two_launches", "fc_walk",
                                  "fc_pruned", "fc_batched_i8", "fc_batched_bf16"])
def test_single_layer_graphs_of_the_newer_paths_replay_correctly(case):
    """The paths whose step keeps state on the device between launches (arrival counters that the last workgroup
    rearms, stored inputs committed by whoever finishes last, difference buffers): captured once, replayed several
    times, mixed with eager steps and a reset."""
    if case == "scatter_bf16":
        _replay_case(S.config2("r14", 0.10, T=5))
    elif case == "scatter_i8":
        _replay_case(S.config0(T=5), path=3)
    elif case == "binary_one_launch":
        _replay_case(S.config4("b14", 0.10, n=3, T=5))
    elif case == "binary_two_launches":
        _replay_case(S.config4("b14", 0.10, n=3, T=5), bin_single_launch=0)
    elif case == "fc_walk":
        _replay_case(S.config3("fc7", S.I8, 0.10, T=5))
    elif case == "fc_pruned":
        _replay_case(S.pruned(S.config3("fc7", S.BF16, 0.10, T=5), 0.1, 4242), fc_sparse_weights=1)
    elif case == "fc_batched_i8":
        _replay_case(S.random_layer(9101, S.fc_shape(1024, 512, n=40), S.I8, T=5, frac=0.1))
    else:
        _replay_case(S.random_layer(9102, S.fc_shape(512, 256, n=24), S.BF16, T=5, frac=0.1))
