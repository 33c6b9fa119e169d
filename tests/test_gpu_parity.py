"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer and binary paths must be bit-exact; bf16-in / fp32-accumulate must stay within
1e-3 * max|y| of the float64 oracle after 16 frames.
"""
import numpy as np
import pytest

import oracle
import rrm_synth as S
from gpu_util import assert_matches, make_layer, run_sequence, to_device

pytestmark = pytest.mark.gpu


def test_config0_every_frame_bit_exact():
    seq = S.config0()
    st, _ = run_sequence(seq, check_dense=(0, 3), y_out_frames=(0, 2))
    assert st["steps"] == 8 and st["delta_steps"] == 8
    # frames 1..7 change about 10 % of the positions; frame 0 changes (nearly) everything
    assert 0 < st["active_tiles"] < st["total_tiles"]


def test_config0_batched_streams():
    run_sequence(S.config0(n=3, T=4))


def _pos_kernel_takes(shp, dt):
    """the position-gather kernel's conditions (stride 1, channel runs of 16-byte multiples, outputs in fours)"""
    es = 1 if dt == S.I8 else 2
    return (shp.stride == 1 and (shp.c_in // shp.groups * es) % 16 == 0 and (shp.c_out // shp.groups) % 4 == 0
            and shp.c_out % 4 == 0)


def _kernel_opts(shp, dt, kern):
    """options that select the convolution kernel under test: 1 window-tile, 2 position-gather (skipped where that
    kernel does not apply)"""
    if kern == 2 and not _pos_kernel_takes(shp, dt):
        pytest.skip("layer not eligible for the position-gather kernel")
    return {"conv_kernel": kern}


SMALL_CONV = [
    # odd sizes, strides, pads, groups, channel counts off the 16-byte chunk
    S.conv_shape(9, 11, 6, 10, 3, 1, 1, 1, n=2),
    S.conv_shape(12, 10, 8, 12, 5, 1, 2, 2),
    S.conv_shape(23, 19, 3, 7, 11, 4, 0, 1),
    S.conv_shape(17, 17, 4, 4, 3, 2, 1, 1),
    S.conv_shape(8, 9, 6, 9, 3, 2, 0, 3),
    S.LayerShape(S.CONV, 1, 7, 9, 5, 3, 2, 3, 1, 1, 1),
    S.conv_shape(7, 7, 16, 16, 1, 1, 0, 1),
    S.conv_shape(20, 20, 48, 40, 3, 1, 1, 1),
    S.conv_shape(10, 10, 160, 24, 3, 1, 1, 1),
    S.conv_shape(13, 13, 32, 96, 3, 1, 1, 2, n=2),
    S.conv_shape(9, 9, 16, 16, 3, 1, 2, 1),
]


@pytest.mark.parametrize("shp", SMALL_CONV)
@pytest.mark.parametrize("dt", [S.I8, S.BF16])
@pytest.mark.parametrize("kern", [1, 2])
def test_small_conv_shapes(shp, dt, kern):
    seq = S.random_layer(4000 + shp.h * 7 + shp.c_in, shp, dt, T=4, frac=0.2, block=2)
    run_sequence(seq, check_dense=(0, 2), **_kernel_opts(shp, dt, kern))


SMALL_FC = [S.fc_shape(67, 29, n=2), S.fc_shape(256, 128), S.fc_shape(1000, 515, n=3), S.fc_shape(48, 4100)]


@pytest.mark.parametrize("shp", SMALL_FC)
@pytest.mark.parametrize("dt", [S.I8, S.BF16])
def test_small_fc_shapes(shp, dt):
    seq = S.random_layer(5000 + shp.c_in, shp, dt, T=5, frac=0.1)
    run_sequence(seq, check_dense=(0, 2), rel=1e-4)


SMALL_BIN = [
    S.conv_shape(9, 10, 32, 8, 3, 1, 1, 1),
    S.conv_shape(12, 12, 64, 40, 3, 1, 1, 1, n=2),
    S.conv_shape(11, 9, 128, 32, 3, 2, 1, 2),
    S.conv_shape(8, 8, 96, 16, 5, 1, 2, 1),
    S.conv_shape(6, 6, 160, 24, 1, 1, 0, 1),
]


@pytest.mark.parametrize("shp", SMALL_BIN)
def test_small_binary_shapes(shp):
    seq = S.random_layer(6000 + shp.c_in, shp, S.BIN, T=4, frac=0.1, block=2)
    st, _ = run_sequence(seq, check_dense=(0, 2))
    assert st["delta_steps"] == 3  # the first frame of a binary layer is a dense recomputation


def test_zero_delta_leaves_projection_untouched():
    import torch
    for seq in (S.config0(T=2), S.config3("fc7", S.BF16, 0.05, T=2), S.config4("b14", 0.05, T=2)):
        layer = make_layer(seq)
        x = to_device(seq.frames[1], seq.dtype)
        layer.step(to_device(seq.frames[0], seq.dtype))
        layer.step(x)
        before = layer.y_snapshot().clone()
        s0 = layer.stats()
        layer.step(x)
        torch.cuda.synchronize()
        s1 = layer.stats()
        assert torch.equal(before, layer.y_snapshot())
        assert s1["changed_elems"] == s0["changed_elems"] and s1["active_tiles"] == s0["active_tiles"]
        layer.destroy()


def test_reset_restarts_from_the_bias():
    seq = S.config0(T=4)
    layer = make_layer(seq)
    for x in seq.frames[:3]:
        layer.step(to_device(x, seq.dtype))
    layer.reset()
    y0 = layer.y_snapshot().cpu().numpy()
    assert (y0 == seq.bias.reshape(1, 1, 1, -1)).all()
    layer.step(to_device(seq.frames[3], seq.dtype))
    want = oracle.dense(seq.shape, seq.dtype, seq.weights, seq.bias, seq.frames[3])
    assert np.array_equal(layer.y_snapshot().cpu().numpy(), want)
    layer.destroy()


def test_dense_every_step_option_matches():
    run_sequence(S.config0(T=3), path=2)
    run_sequence(S.config3("fc7", S.I8, 0.05, T=3), path=2)


def test_int8_difference_out_of_range_is_flagged():
    import paper_1802_09723_amd as rrm
    shp = S.conv_shape(8, 8, 16, 16, 3, 1, 1)
    rng = S.rng_for(1)
    w = S.draw_i8_weight(rng, shp.w_shape)
    layer = rrm.Layer(shp, S.I8, w, None)
    a = np.full(shp.x_shape, 100, np.int8)
    b = np.full(shp.x_shape, -100, np.int8)
    layer.step(to_device(a, S.I8))
    assert layer.stats()["range_error"] == 0
    layer.step(to_device(b, S.I8))  # difference -200 does not fit int8
    with pytest.raises(rrm.RRMError):
        layer.stats()
    assert layer.stats(allow_range_error=True)["range_error"] == 1
    layer.destroy()


def test_determinism_bf16_conv_is_bit_reproducible():
    """Every output element of the conv tile paths has one owner, so two runs give the same bits (the scatter path,
    which one stream of this map would take by default, adds with fp32 atomics in arrival order and does not)."""
    import torch
    seq = S.config2("r14", 0.25, T=4)
    outs = []
    for _ in range(2):
        layer = make_layer(seq, path=1)
        for x in seq.frames:
            layer.step(to_device(x, seq.dtype))
        outs.append(layer.y_snapshot().clone())
        layer.destroy()
    assert torch.equal(outs[0], outs[1])


def test_conv_list_longer_than_one_ranking_round():
    """So many active sub-tiles that a workgroup's share of the ranked list does not fit its LDS list at
    once (more than 64 work units per workgroup): the gather kernel ranks in several rounds."""
    n = 80000  # streams of 8x8 maps: 320000 sub-tiles
    shp = S.conv_shape(8, 8, 16, 16, 3, 1, 1, n=n)
    rng = S.rng_for(S.seed_for(0, 77))
    w = S.draw_i8_weight(rng, shp.w_shape)
    bias = S.draw_i32_bias(rng, shp.c_out)
    f0 = S.draw_i8_act(rng, shp.x_shape)
    f1 = f0.copy()
    redraw = rng.random(n) < 0.9  # most streams change completely: still several rounds
    f1[redraw] = S.draw_i8_act(rng, (int(redraw.sum()),) + shp.x_shape[1:])
    f2 = f1.copy()
    f2[::7, 2:5, 3:6, :] = S.draw_i8_act(rng, f2[::7, 2:5, 3:6, :].shape)  # a sparse step: one round
    seq = S.Sequence_(shp, S.I8, w, bias, [f0, f1, f2], "many_units")
    st, _ = run_sequence(seq, check_frames=(0, 1, 2), check_dense=(), check_x=False)
    assert st["active_tiles"] > 2 * 64 * 16 * 256


@pytest.mark.parametrize("pct", [1, 100])
def test_dense_switch_threshold_both_ways(pct):
    """A delta step above the threshold recomputes the projection instead of updating it: forced always
    (1 %) and never (100 %), both must match the oracle on every frame."""
    run_sequence(S.config0(T=5), dense_switch_pct=pct)
    run_sequence(S.config2("r14", 0.25, T=5), dense_switch_pct=pct)
    run_sequence(S.random_layer(4321, S.conv_shape(19, 23, 24, 40, 3, 1, 1, n=3), S.I8, T=4, frac=0.3), dense_switch_pct=pct)


def _perturbed_frames(seq, seed, sigma=0.02):
    """The sequence's frames plus small perturbations of half of the entries, so that many differences fall
    below a truncation threshold of a few hundredths."""
    rng = S.rng_for(seed)
    frames = [seq.frames[0]]
    for f in seq.frames[1:]:
        v = S.bf16_bits_to_f32(f) + rng.normal(0, sigma, size=f.shape).astype(np.float32) * (rng.random(f.shape) < 0.5)
        frames.append(S.f32_to_bf16_bits(np.maximum(v, 0).astype(np.float32)))
    return frames


@pytest.mark.parametrize("kind", ["conv", "conv_multi", "fc", "conv_scatter"])
@pytest.mark.parametrize("eps", [0.0, 0.03])
def test_bf16_truncation_threshold_matches_oracle(kind, eps):
    """rrm_set_threshold: stored input bit-identical to the oracle's (same fp32 decision per entry), stored
    projection within the bf16 tolerance, same number of truncated entries (Sec. 3.4, Improving sparsity)."""
    if kind == "fc":
        seq = S.config3("fc7", S.BF16, 0.10, n=2, T=5)
    elif kind in ("conv", "conv_scatter"):
        seq = S.config2("r28", 0.10, T=5)
    else:
        seq = S.random_layer(7007, S.conv_shape(21, 17, 24, 40, 3, 1, 1, n=3), S.BF16, T=5, frac=0.3, block=3)
    frames = _perturbed_frames(seq, 4242)
    layer = make_layer(seq, **({"path": 3} if kind == "conv_scatter" else {}))
    layer.set_threshold(eps)
    st = oracle.State(seq.shape, S.BF16, seq.weights, seq.bias)
    trunc = 0
    for t, x in enumerate(frames):
        layer.step(to_device(x, S.BF16))
        want_p = st.step(x, eps=eps)
        trunc += st.last_truncated
        got_x = layer.x_snapshot_bytes().cpu().numpy().view(np.uint16).reshape(x.shape)
        want_x = S.f32_to_bf16_bits(st.i_prev.astype(np.float32))
        assert np.array_equal(S.bf16_bits_to_f32(got_x), S.bf16_bits_to_f32(want_x)), f"frame {t}: stored input differs"
        assert_matches(layer.y_snapshot().cpu().numpy(), want_p, S.BF16, f"{kind} eps {eps} frame {t}")
    stats = layer.stats()
    assert stats["truncated_elems"] == trunc
    assert (trunc > 0) == (eps > 0)
    layer.destroy()


def test_threshold_is_refused_for_integer_layers():
    import paper_1802_09723_amd as rrm
    layer = make_layer(S.config0(T=1))
    with pytest.raises(rrm.RRMError):
        layer.set_threshold(0.01)
    layer.destroy()


def _random_conv_shapes(count, seed):
    """Seeded random convolution shapes: kernels 1..5 (also non-square), strides 1..3, pads 0..2, groups 1..4,
    channel counts on and off the 16-byte chunk, 1..6 streams."""
    rng = S.rng_for(seed)
    out = []
    while len(out) < count:
        groups = int(rng.choice([1, 1, 1, 2, 3, 4]))
        cg = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 20, 32, 48]))
        og = int(rng.choice([1, 3, 4, 7, 8, 16, 24, 33, 40, 64]))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        h, w = int(rng.integers(max(kh - 2 * pad, 1) + 2, 26)), int(rng.integers(max(kw - 2 * pad, 1) + 2, 26))
        n = int(rng.integers(1, 7))
        if (h + 2 * pad - kh) < 0 or (w + 2 * pad - kw) < 0:
            continue
        shp = S.LayerShape(S.CONV, n, h, w, cg * groups, og * groups, kh, kw, stride, pad, groups)
        if shp.h_out < 1 or shp.w_out < 1 or n * h * w * cg * groups * og * kh * kw > 4e8:
            continue
        out.append(shp)
    return out


@pytest.mark.parametrize("idx", range(24))
def test_random_conv_shapes(idx):
    shp = _random_conv_shapes(24, 20240)[idx]
    dt = S.I8 if idx % 2 == 0 else S.BF16
    seq = S.random_layer(8100 + idx, shp, dt, T=4, frac=0.25, block=2)
    run_sequence(seq, check_dense=(0, 3), conv_kernel=1)


# Large filter windows and many channels: the weights of one slab of chunks and the input windows no longer fit
# LDS together with slabs of whole K steps, so the layer runs with padded slabs and fewer sub-tiles per workgroup
# (down to one for the 11 x 11 windows).  (kernel, stride, channels per group, groups, streams, height)
LARGE_WINDOWS = [(5, 1, 64, 1, 2, 14), (5, 2, 96, 2, 1, 17), (7, 1, 96, 1, 1, 12), (7, 2, 64, 1, 3, 19),
                 (3, 4, 64, 1, 2, 21), (3, 3, 128, 2, 1, 20), (11, 1, 32, 1, 1, 13), (11, 2, 16, 1, 2, 23),
                 (11, 1, 64, 1, 1, 12), (7, 4, 512, 1, 1, 23)]


@pytest.mark.parametrize("case", LARGE_WINDOWS, ids=lambda c: "k%ds%dc%dg%dn%dh%d" % c)
@pytest.mark.parametrize("dt", [S.I8, S.BF16])
def test_large_windows_with_many_channels(case, dt):
    k, stride, cg, groups, n, h = case
    shp = S.LayerShape(S.CONV, n, h, h + 3, cg * groups, 40 * groups, k, k, stride, k // 2, groups)
    for frac in (0.05, 0.6):
        seq = S.random_layer(7000 + k * stride + cg, shp, dt, T=3, frac=frac, block=2)
        run_sequence(seq, check_dense=(0, 2))


@pytest.mark.parametrize("case", [(5, 4, 96, 1, 1, 31), (11, 4, 128, 1, 1, 33), (7, 4, 384, 4, 1, 24), (9, 4, 192, 2, 5, 17),
                                  (11, 3, 256, 1, 2, 30)], ids=lambda c: "k%ds%dc%dg%dn%dh%d" % c)
def test_binary_large_strided_windows(case):
    """the 8 x 8 tile's window takes more than 64 KB of LDS (both copies): the tile kernel runs with the large
    allocation, for the dense pass and, where no band fits, for the delta steps"""
    k, stride, c_in, groups, n, h = case
    shp = S.LayerShape(S.CONV, n, h, h + 5, c_in, 13 * groups, k, k, stride, k // 2, groups)
    for frac in (0.02, 0.5):
        seq = S.random_layer(7200 + k + stride, shp, S.BIN, T=3, frac=frac, block=2)
        run_sequence(seq, check_dense=(0, 2))


def test_window_too_large_for_lds_is_refused_with_a_message():
    import paper_1802_09723_amd as rrm
    shp = S.LayerShape(S.CONV, 1, 35, 38, 32, 40, 11, 11, 4, 5, 1)
    seq = S.random_layer(7100, shp, S.BF16, T=1, frac=1.0)
    with pytest.raises(rrm.binding.RRMError, match="does not fit LDS"):
        make_layer(seq)


def _random_pos_shapes(count, seed):
    """Seeded random shapes the position-gather kernel takes: stride 1, kernels 1..5 (also non-square), pads 0..2,
    groups 1..2, channel runs of 16-byte multiples (odd chunk counts too), outputs in fours, 1..40 streams."""
    rng = S.rng_for(seed)
    out = []
    while len(out) < count:
        dt = S.I8 if len(out) % 2 == 0 else S.BF16
        groups = int(rng.choice([1, 1, 2]))
        cg = (16 if dt == S.I8 else 8) * int(rng.choice([1, 2, 3, 4, 5, 8]))
        og = 4 * int(rng.choice([1, 2, 5, 8, 16, 33, 40]))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        pad = int(rng.integers(0, 3))
        h, w = int(rng.integers(max(kh - 2 * pad, 1) + 1, 30)), int(rng.integers(max(kw - 2 * pad, 1) + 1, 30))
        n = int(rng.choice([1, 2, 3, 7, 40]))
        shp = S.LayerShape(S.CONV, n, h, w, cg * groups, og * groups, kh, kw, 1, pad, groups)
        if shp.h_out < 1 or shp.w_out < 1 or n * shp.h_out * shp.w_out * cg * groups * og * kh * kw > 6e8:
            continue
        out.append((shp, dt))
    return out


@pytest.mark.parametrize("idx", range(20))
def test_random_shapes_on_the_position_kernel(idx):
    shp, dt = _random_pos_shapes(20, 20250)[idx]
    seq = S.random_layer(8300 + idx, shp, dt, T=4, frac=0.25, block=2)
    run_sequence(seq, check_dense=(0, 3), conv_kernel=2)


def _random_bin_shapes(count, seed):
    rng = S.rng_for(seed)
    out = []
    while len(out) < count:
        groups = int(rng.choice([1, 1, 2, 4]))
        cg = 32 * int(rng.integers(1, 6))
        og = int(rng.choice([1, 4, 8, 12, 16, 24, 40]))
        kh, kw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
        h, w = int(rng.integers(4, 22)), int(rng.integers(4, 22))
        shp = S.LayerShape(S.CONV, int(rng.integers(1, 5)), h, w, cg * groups, og * groups, kh, kw, stride, pad, groups)
        if (h + 2 * pad - kh) < 0 or (w + 2 * pad - kw) < 0 or shp.h_out < 1 or shp.w_out < 1:
            continue
        out.append(shp)
    return out


@pytest.mark.parametrize("idx", range(10))
def test_random_binary_shapes(idx):
    shp = _random_bin_shapes(10, 777)[idx]
    seq = S.random_layer(8300 + idx, shp, S.BIN, T=4, frac=0.1, block=2)
    st, _ = run_sequence(seq, check_dense=(0, 3))
    # the same with a difference kernel in front of the band kernel: same results, same change counts
    st2, _ = run_sequence(seq, check_dense=(), bin_single_launch=0)
    assert (st2["changed_elems"], st2["changed_units"], st2["active_tiles"]) == \
        (st["changed_elems"], st["changed_units"], st["active_tiles"])


def test_binary_band_list_longer_than_one_pass_and_wide_layer_on_the_tile_kernel():
    """The binary delta step's band kernel with several 128-entry passes over a band's list, dealt over several
    workgroups (one stream, half of the positions changing), with three streams, and a layer so wide that no
    band of it fits LDS, which takes the tile kernel."""
    big = S.conv_shape(40, 40, 64, 32, 3, 1, 1, 1)
    seq = S.random_layer(8501, big, S.BIN, T=4, frac=0.5, block=3)
    run_sequence(seq, check_dense=(0, 3))
    seq = S.random_layer(8502, S.conv_shape(30, 26, 128, 48, 3, 1, 1, 1, n=3), S.BIN, T=4, frac=0.2, block=4)
    st, _ = run_sequence(seq, check_dense=(0, 3))
    assert st["tile_positions"] == 1
    st2, _ = run_sequence(seq, check_dense=(), bin_single_launch=0)
    assert (st2["changed_elems"], st2["changed_units"], st2["active_tiles"]) == \
        (st["changed_elems"], st["changed_units"], st["active_tiles"])
    wide = S.conv_shape(6, 300, 256, 16, 3, 1, 1, 1)
    seq = S.random_layer(8503, wide, S.BIN, T=3, frac=0.05, block=4)
    st, _ = run_sequence(seq, check_dense=(0, 2))
    assert st["tile_positions"] == 64


@pytest.mark.parametrize("idx", range(8))
def test_random_fc_shapes(idx):
    rng = S.rng_for(900 + idx)
    shp = S.fc_shape(int(rng.integers(1, 3000)), int(rng.integers(1, 3000)), n=int(rng.integers(1, 5)))
    seq = S.random_layer(8400 + idx, shp, S.I8 if idx % 2 else S.BF16, T=4, frac=float(rng.choice([0.01, 0.1, 0.5])))
    run_sequence(seq, check_dense=(0, 3), rel=1e-4)


@pytest.mark.parametrize("case", [
    # (h, c_in, c_out, k, groups, streams, changed fraction): flag arrays of 320 .. 4900 sub-tiles, several work
    # units per workgroup, densities below and above the recomputation switch
    (13, 64, 128, 3, 1, 20, 0.10), (13, 64, 128, 3, 1, 64, 0.30), (13, 96, 64, 3, 2, 100, 0.05),
    (27, 32, 64, 5, 1, 100, 0.15), (13, 64, 128, 3, 1, 64, 0.90),
    # exactly 256 and 4096 sub-tiles: the borders between the ways the flag array is split over threads
    (13, 64, 64, 3, 1, 16, 0.30), (13, 64, 64, 3, 1, 256, 0.10),
])
@pytest.mark.parametrize("dt", [S.I8, S.BF16])
@pytest.mark.parametrize("kern", [1, 2])
def test_many_streams_mid_size(case, dt, kern):
    h, ci, co, k, groups, n, frac = case
    shp = S.conv_shape(h, h, ci, co, k, 1, k // 2, groups, n=n)
    rng = S.rng_for(8500 + n + h)
    draw = S.draw_i8_act if dt == S.I8 else S.draw_bf16_relu
    w = S.draw_i8_weight(rng, shp.w_shape) if dt == S.I8 else S.draw_bf16_weight(rng, shp.w_shape)
    frames = [draw(rng, shp.x_shape)]
    for t in range(3):  # per frame: a random subset of streams gets a re-drawn 6x6 block
        f = frames[-1].copy()
        for b in np.nonzero(rng.random(n) < min(1.0, 4 * frac))[0]:
            y0, x0 = int(rng.integers(0, h - 5)), int(rng.integers(0, h - 5))
            f[b, y0:y0 + 6, x0:x0 + 6, :] = draw(rng, (6, 6, ci))
        if frac > 0.5:
            f = draw(rng, shp.x_shape)
        frames.append(f)
    seq = S.Sequence_(shp, dt, w, None, frames, "mid")
    run_sequence(seq, check_dense=(1,), check_x=False, conv_kernel=kern)


# ---- the single-launch scatter path ("path" = 3) ---------------------------------------------------------------------
def _scatter_takes(shp, dt):
    es = 1 if dt == S.I8 else 2
    return (shp.c_in // shp.groups * es) % 16 == 0


def _random_scatter_shapes(count, seed):
    """Seeded random shapes the scatter path takes: any stride, kernels 1..5 (also non-square), pads 0..2, groups
    1..3, channel runs of 16-byte multiples, any output-channel count, 1..40 streams."""
    rng = S.rng_for(seed)
    out = []
    while len(out) < count:
        dt = S.I8 if len(out) % 2 == 0 else S.BF16
        groups = int(rng.choice([1, 1, 2, 3]))
        cg = (16 if dt == S.I8 else 8) * int(rng.choice([1, 2, 3, 4, 6, 8]))
        og = int(rng.choice([1, 3, 4, 8, 20, 32, 33, 64, 70]))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        h, w = int(rng.integers(max(kh - 2 * pad, 1) + 1, 28)), int(rng.integers(max(kw - 2 * pad, 1) + 1, 28))
        n = int(rng.choice([1, 2, 3, 7, 40]))
        shp = S.LayerShape(S.CONV, n, h, w, cg * groups, og * groups, kh, kw, stride, pad, groups)
        if shp.h_out < 1 or shp.w_out < 1 or n * shp.h_out * shp.w_out * cg * groups * og * kh * kw > 4e8:
            continue
        out.append((shp, dt))
    return out


@pytest.mark.parametrize("idx", range(24))
def test_scatter_path_random_shapes(idx):
    shp, dt = _random_scatter_shapes(24, 20260)[idx]
    import paper_1802_09723_amd as rrm
    seq = S.random_layer(8600 + idx, shp, dt, T=4, frac=0.2, block=2)
    try:
        st, _ = run_sequence(seq, check_dense=(0,), path=3)
    except rrm.binding.RRMError as e:
        if e.status != -2:
            raise
        pytest.skip("shape beyond the window-tile kernel's LDS limit (the handle needs that kernel for its dense path)")
    assert st["delta_steps"] == 4 and st["tile_positions"] in (1, 16)


@pytest.mark.parametrize("dt", [S.I8, S.BF16])
def test_scatter_path_many_streams_and_shared_blocks(dt):
    """64 streams of a 13 x 13 map (many position blocks, one workgroup each) and one stream of a 7 x 7 map with 512
    channels (two position blocks shared by sixteen output-channel splits: the last split to compare commits)."""
    for shp, frac in ((S.conv_shape(13, 13, 64, 128, 3, 1, 1, n=64), 0.1), (S.conv_shape(7, 7, 512, 512, 3, 1, 1), 0.3)):
        seq = S.random_layer(8700 + shp.h, shp, dt, T=5, frac=frac, block=2)
        run_sequence(seq, check_dense=(), path=3)


def test_scatter_and_tile_steps_interleave():
    """Steps of the scatter path and of the scan + tile path on one handle, in turn: each leaves the state the other
    expects (difference buffer, change bitmap, stored input), int8 bit-exact on every frame."""
    import paper_1802_09723_amd as rrm
    shp = S.conv_shape(14, 14, 32, 64, 3, 1, 1, n=3)
    seq = S.random_layer(8801, shp, S.I8, T=9, frac=0.15, block=3)
    layer = make_layer(seq)
    for t, x in enumerate(seq.frames):
        layer.set_option("path", 3 if t % 3 == 1 else (1 if t % 3 == 2 else 0))
        layer.step(to_device(x, S.I8))
        want = oracle.dense(shp, S.I8, seq.weights, seq.bias, x)
        assert_matches(layer.y_snapshot().cpu().numpy(), want, S.I8, f"frame {t}")
        assert np.array_equal(layer.x_snapshot_bytes().cpu().numpy(), x.view(np.uint8).reshape(-1))
    layer.destroy()


def test_fused_consumer_after_a_scatter_step_of_the_producer():
    """The scatter path keeps no flags of what it wrote; a consumer fed through rrm_step_from_projection, and the
    incremental nonlinearity, must then look at everything."""
    import torch
    import paper_1802_09723_amd as rrm
    cfg = S.config1(n=2, T=5)
    l1, l2 = cfg["layers"][1], cfg["layers"][2]  # conv2 (5x5, groups 2) feeds conv3 through ReLU / shift / pool
    rng = S.rng_for(8802)
    A = rrm.Layer(l1["shape"], S.I8, l1["weights"], l1["bias"])
    B = rrm.Layer(l2["shape"], S.I8, l2["weights"], l2["bias"])
    frames = [S.draw_i8_relu(rng, l1["shape"].x_shape)]
    for t in range(4):
        f = frames[-1].copy()
        f[:, 3 * t:3 * t + 4, 5:9, :] = S.draw_i8_relu(rng, (2, 4, 4, l1["shape"].c_in))
        frames.append(f)
    shift = oracle.calibrate_shift(oracle.dense(l1["shape"], S.I8, l1["weights"], l1["bias"], frames[0]))
    ho = A.y_shape[1]
    buf = torch.full((2, (ho - 3) // 2 + 1, (ho - 3) // 2 + 1, l1["shape"].c_out), -1, dtype=torch.int8, device="cuda")
    for t, f in enumerate(frames):
        A.set_option("path", 3 if t in (1, 3) else 0)
        A.step(to_device(f, S.I8))
        B.step_from_projection(A, shift, True)
        A.relu_requant_pool_changed(buf, shift, True)
        ya = oracle.dense(l1["shape"], S.I8, l1["weights"], l1["bias"], f)
        x2 = oracle.relu_requant_pool(ya, shift, True)
        assert_matches(A.y_snapshot().cpu().numpy(), ya, S.I8, f"frame {t} producer")
        assert np.array_equal(buf.cpu().numpy(), x2), f"frame {t}: incremental nonlinearity"
        assert_matches(B.y_snapshot().cpu().numpy(), oracle.dense(l2["shape"], S.I8, l2["weights"], l2["bias"], x2), S.I8,
                       f"frame {t} consumer")
    A.destroy()
    B.destroy()


@pytest.mark.parametrize("dtype", [S.I8, S.BF16])
def test_fc_pruned_weights_walk_nonzeros_only(dtype):
    """FC layers whose weights are mostly zero (pruned models, Sec. 4.3): the delta step walks the (row, value)
    lists of the changed columns.  Several streams, a ragged shape, a full-size layer, the list longer than one
    compare round (c_in above 8192), an all-zero column; and the dense-column walk forced on the same handle."""
    import paper_1802_09723_amd as rrm
    cases = [(S.fc_shape(700, 300, n=3), 0.10, 0.2), (S.fc_shape(4096, 4096), 0.10, 0.05), (S.fc_shape(9216, 1000, n=2), 0.25, 0.5),
             (S.fc_shape(33, 17), 0.3, 0.5)]
    for i, (shp, keep, frac) in enumerate(cases):
        seq = S.pruned(S.random_layer(8600 + i, shp, dtype, T=4, frac=frac), keep, 8700 + i)
        seq.weights[:, min(5, shp.c_in - 1)] = 0  # a column without any non-zero
        st, _ = run_sequence(seq, check_dense=(0, 3), rel=1e-4, fc_sparse_weights=1)
        assert st["delta_steps"] == 4
        st2, _ = run_sequence(seq, check_dense=(), rel=1e-4)
        assert st2["changed_elems"] == st["changed_elems"]
    dense_w = S.random_layer(8650, S.fc_shape(64, 64), dtype, T=2, frac=0.5)
    L = make_layer(dense_w)
    with pytest.raises(rrm.binding.RRMError):
        L.set_option("fc_sparse_weights", 1)
    L.destroy()


@pytest.mark.parametrize("dtype", [S.I8, S.BF16])
def test_fc_many_streams_as_one_product(dtype):
    """FC layers with 16 or more streams run as one product on the matrix cores (dense layer and delta step): a
    ragged stream count, one tile exactly, several tiles, the full-size fc7 at 64 streams; and the same handles on
    the per-stream column walk."""
    cases = [(S.fc_shape(192, 48, n=16), 0.3), (S.fc_shape(640, 272, n=37), 0.1), (S.fc_shape(4096, 4096, n=64), 0.05),
             (S.fc_shape(128, 16, n=200), 0.5)]
    for i, (shp, frac) in enumerate(cases):
        seq = S.random_layer(8800 + i, shp, dtype, T=4, frac=frac)
        st, _ = run_sequence(seq, check_dense=(0, 3), rel=1e-4)
        assert st["delta_steps"] == 4
        st2, _ = run_sequence(seq, check_dense=(3,), rel=1e-4, fc_batched=0)
        assert st2["changed_elems"] == st["changed_elems"]


def _batched_fc_shapes():
    """every stream-tile count the product kernel is built for (1, 2, 3, 4, 6, 8, 12, 16 tiles of 16 streams, and
    ragged counts between them), row counts that are not multiples of the 64-row group, k ranges that leave a ragged
    last chunk, one split and several"""
    rng = S.rng_for(9100)
    out = []
    for n in (16, 17, 32, 33, 48, 64, 65, 90, 96, 100, 128, 129, 190, 200, 256, 300, 512):
        for dt in (S.I8, S.BF16):
            es = 1 if dt == S.I8 else 2
            steps = int(rng.choice([1, 2, 3, 5, 7, 13, 24, 37, 50]))
            c_out = 16 * int(rng.choice([1, 2, 3, 4, 5, 9, 17]))
            out.append((S.fc_shape(steps * 64 // es, c_out, n=n), dt))
    return out


@pytest.mark.parametrize("idx", range(34))
def test_fc_product_kernel_shapes(idx):
    shp, dt = _batched_fc_shapes()[idx]
    seq = S.random_layer(9100 + idx, shp, dt, T=3, frac=0.3)
    st, _ = run_sequence(seq, check_dense=(0, 2), rel=1e-4)
    assert st["delta_steps"] == 3

