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
