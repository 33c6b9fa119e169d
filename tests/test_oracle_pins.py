"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

The paper prints no worked numeric example of a layer, so the oracle is tied down by closed
forms, special cases that reduce to a library routine, an independent library convolution,
brute force on tiny layers and the linearity invariants of Eq. 4 (Sec. 3.1).
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import accounting
import rrm_synth as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------
# Eq. 3, dense: closed forms
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("k,stride,pad,groups", [(3, 1, 1, 1), (5, 1, 2, 2), (3, 2, 1, 1), (11, 4, 0, 1), (2, 1, 0, 1)])
def test_impulse_response_is_reversed_filter(k, stride, pad, groups):
    """A one-hot input at (iy, ix, c) produces, at output (oy, ox, o), the filter tap that
    looks at it: w[o][iy + pad - oy*stride][ix + pad - ox*stride][c'] when that tap exists and
    o is in c's group, and nothing elsewhere."""
    rng = S.rng_for(11 + k)
    h, w, ci, co = 13, 15, 4 * groups, 6 * groups
    shp = S.LayerShape(S.CONV, 1, h, w, ci, co, k, k, stride, pad, groups)
    wt = S.draw_i8_weight(rng, shp.w_shape)
    cg, og = ci // groups, co // groups
    for (iy, ix, c, v) in [(0, 0, 0, 5), (h - 1, w - 1, ci - 1, -3), (6, 7, cg % ci, 7), (3, 11, 1, 1)]:
        x = np.zeros(shp.x_shape, dtype=np.int8)
        x[0, iy, ix, c] = v
        y = oracle.dense(shp, S.I8, wt, None, x)
        exp = np.zeros(shp.y_shape, dtype=np.int64)
        g = c // cg
        for oy in range(shp.h_out):
            for ox in range(shp.w_out):
                ky, kx = iy + pad - oy * stride, ix + pad - ox * stride
                if 0 <= ky < k and 0 <= kx < k:
                    exp[0, oy, ox, g * og:(g + 1) * og] = v * wt[g * og:(g + 1) * og, ky, kx, c % cg].astype(np.int64)
        assert np.array_equal(y, exp)


def test_all_ones_counts_in_bounds_taps():
    """x = 1 and w = 1 everywhere: y = (C_in/groups) * number of taps inside the image; for a
    3x3 window with pad 1 that is 9C inside, 6C on an edge, 4C in a corner."""
    for groups in (1, 2):
        c = 8
        shp = S.conv_shape(6, 7, c, 4, 3, 1, 1, groups)
        y = oracle.dense(shp, S.I8, np.ones(shp.w_shape, np.int8), None, np.ones(shp.x_shape, np.int8))[0]
        cg = c // groups
        assert (y[1:-1, 1:-1] == 9 * cg).all()
        assert (y[0, 1:-1] == 6 * cg).all() and (y[-1, 1:-1] == 6 * cg).all()
        assert (y[1:-1, 0] == 6 * cg).all() and (y[1:-1, -1] == 6 * cg).all()
        for cy, cx in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
            assert (y[cy, cx] == 4 * cg).all()
    # 5x5 window, pad 2, stride 1 on a 5x5 map: centre sees 25 taps, corner 9
    shp = S.conv_shape(5, 5, 2, 1, 5, 1, 2, 1)
    y = oracle.dense(shp, S.I8, np.ones(shp.w_shape, np.int8), None, np.ones(shp.x_shape, np.int8))[0, :, :, 0]
    assert y[2, 2] == 50 and y[0, 0] == 18 and y[0, 2] == 30


def test_bias_is_added_once():
    shp = S.conv_shape(4, 4, 3, 5, 3, 1, 1)
    b = np.arange(5, dtype=np.int32) * 100 - 200
    y0 = oracle.dense(shp, S.I8, np.zeros(shp.w_shape, np.int8), b, np.ones(shp.x_shape, np.int8))
    assert (y0 == b.reshape(1, 1, 1, -1)).all()


def test_special_cases_reduce_to_matvec():
    """1x1 convolution on a 1x1 map is an FC layer; a window as large as the (unpadded) map is
    an FC layer on the flattened input; both equal a library matrix-vector product."""
    rng = S.rng_for(5)
    ci, co = 37, 11
    wt = S.draw_i8_weight(rng, (co, ci))
    b = S.draw_i32_bias(rng, co)
    x = S.draw_i8_act(rng, (2, ci))
    ref = x.astype(np.int64) @ wt.astype(np.int64).T + b
    fc = oracle.dense(S.fc_shape(ci, co, 2), S.I8, wt, b, x)
    assert np.array_equal(fc, ref)
    c11 = oracle.dense(S.conv_shape(1, 1, ci, co, 1, n=2), S.I8, wt.reshape(co, 1, 1, ci), b, x.reshape(2, 1, 1, ci))
    assert np.array_equal(c11.reshape(2, co), ref)
    h, w, c = 3, 4, 5
    wt2 = S.draw_i8_weight(rng, (co, h, w, c))
    x2 = S.draw_i8_act(rng, (2, h, w, c))
    shp = S.LayerShape(S.CONV, 2, h, w, c, co, h, w, 1, 0, 1)
    full = oracle.dense(shp, S.I8, wt2, b, x2)
    ref2 = x2.reshape(2, -1).astype(np.int64) @ wt2.reshape(co, -1).astype(np.int64).T + b
    assert np.array_equal(full.reshape(2, co), ref2)


def test_float_fc_matches_numpy_matvec():
    """The floating-point FC branches (Eq. 3 in FC form; Algorithm 1, FC branch) against numpy's float64
    matrix product on a non-square layer with two streams and a bias: the dense projection of every
    frame and every frame of the recurrence.  A transposed weight index, in either branch or in both
    at once, fails here (the layer is not square, so W and W^T index different entries)."""
    rng = S.rng_for(6)
    ci, co, n = 45, 13, 2
    shp = S.fc_shape(ci, co, n)
    wt = S.draw_bf16_weight(rng, (co, ci))
    b = rng.normal(size=(co,)).astype(np.float32)
    W = oracle.bf16_to_f64(wt)
    st = oracle.State(shp, S.BF16, wt, b)
    x_prev = np.zeros((n, ci))
    for t in range(4):
        x = S.draw_bf16_relu(rng, (n, ci))
        if t:  # keep most entries so that the step is a genuine sparse difference
            keep = rng.random((n, ci)) < 0.7
            x = np.where(keep, prev_bits, x).astype(np.uint16)
        prev_bits = x
        xv = oracle.bf16_to_f64(x)
        ref = xv @ W.T + b.astype(np.float64)
        d = oracle.dense(shp, S.BF16, wt, b, x)
        assert np.allclose(d, ref, rtol=1e-13, atol=1e-13)
        p = st.step(x)
        assert np.allclose(p, ref, rtol=0, atol=1e-11 * max(1.0, np.abs(ref).max()))
        assert st.last_nnz == int((xv != x_prev).sum())
        x_prev = xv


# ------------------------------------------------------------------------------------------
# Eq. 3, dense: an independent library routine (float64 is exact for these integers)
# ------------------------------------------------------------------------------------------
def _torch_conv(shp, w, b, x):
    xt = torch.from_numpy(np.asarray(x, dtype=np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.asarray(w, dtype=np.float64)).permute(0, 3, 1, 2)
    bt = None if b is None else torch.from_numpy(np.asarray(b, dtype=np.float64))
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=shp.stride, padding=shp.pad, groups=shp.groups)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


SHAPES = [
    S.conv_shape(9, 11, 6, 10, 3, 1, 1, 1, n=2),
    S.conv_shape(12, 10, 8, 12, 5, 1, 2, 2),
    S.conv_shape(23, 19, 3, 7, 11, 4, 0, 1),
    S.conv_shape(10, 10, 4, 4, 3, 2, 1, 1),
    S.conv_shape(8, 9, 6, 9, 3, 2, 0, 3),
    S.LayerShape(S.CONV, 1, 7, 9, 5, 3, 2, 3, 1, 1, 1),
    S.conv_shape(7, 7, 16, 16, 1, 1, 0, 1),
]


@pytest.mark.parametrize("shp", SHAPES)
def test_dense_i8_matches_library_conv(shp):
    rng = S.rng_for(100 + shp.h)
    w = S.draw_i8_weight(rng, shp.w_shape)
    b = S.draw_i32_bias(rng, shp.c_out)
    x = rng.integers(-128, 128, size=shp.x_shape).astype(np.int8)
    y = oracle.dense(shp, S.I8, w, b, x)
    assert np.array_equal(y.astype(np.float64), _torch_conv(shp, w, b, x))


@pytest.mark.parametrize("shp", SHAPES[:4])
def test_dense_f64_matches_library_conv(shp):
    rng = S.rng_for(200 + shp.h)
    w = S.draw_bf16_weight(rng, shp.w_shape)
    x = S.draw_bf16_relu(rng, shp.x_shape)
    b = rng.normal(size=(shp.c_out,)).astype(np.float32)
    y = oracle.dense(shp, S.BF16, w, b, x)
    ref = _torch_conv(shp, oracle.bf16_to_f64(w), b.astype(np.float64), oracle.bf16_to_f64(x))
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_brute_force_tiny_im2col():
    """A differently organised computation (explicit patch matrix, then one matrix product)."""
    rng = S.rng_for(7)
    shp = S.conv_shape(5, 4, 3, 2, 3, 1, 1)
    w = S.draw_i8_weight(rng, shp.w_shape)
    x = S.draw_i8_act(rng, shp.x_shape)
    xp = np.zeros((7, 6, 3), dtype=np.int64)
    xp[1:6, 1:5] = x[0]
    rows = []
    for oy in range(5):
        for ox in range(4):
            rows.append(xp[oy:oy + 3, ox:ox + 3, :].reshape(-1))
    ref = (np.stack(rows) @ w.reshape(2, -1).astype(np.int64).T).reshape(1, 5, 4, 2)
    assert np.array_equal(oracle.dense(shp, S.I8, w, None, x), ref)


def test_int32_overflow_is_reported():
    shp = S.fc_shape(200000, 1)
    w = np.full(shp.w_shape, 127, np.int8)
    x = np.full(shp.x_shape, 127, np.int8)
    with pytest.raises(OverflowError):
        oracle.dense(shp, S.I8, w, None, x)


# ------------------------------------------------------------------------------------------
# Algorithm 1: the linearity invariants (Eq. 4; "exactly the same as the output of a normal
# convolution layer", Sec. 3.2)
# ------------------------------------------------------------------------------------------
STEP_SHAPES = [
    (S.conv_shape(9, 8, 6, 10, 3, 1, 1, 1, n=2), S.I8),
    (S.conv_shape(12, 10, 8, 12, 5, 1, 2, 2), S.I8),
    (S.conv_shape(23, 19, 3, 7, 11, 4, 0, 1), S.I8),
    (S.conv_shape(10, 11, 4, 6, 3, 2, 1, 2), S.I8),
    (S.fc_shape(67, 29, n=2), S.I8),
    (S.conv_shape(9, 8, 6, 10, 3, 1, 1, 1), S.BF16),
    (S.fc_shape(67, 29), S.BF16),
    (S.conv_shape(6, 6, 32, 8, 3, 1, 1, 1), S.BIN),
]


@pytest.mark.parametrize("shp,dt", STEP_SHAPES)
def test_step_invariants(shp, dt):
    seq = S.random_layer(900 + shp.c_in, shp, dt, T=5, frac=0.25, block=2)
    st = oracle.State(shp, dt, seq.weights, seq.bias)
    # P_0 = b
    if seq.bias is not None:
        assert np.array_equal(st.p_prev.reshape(-1, shp.c_out)[0], seq.bias.astype(st.p_prev.dtype))
    for t, x in enumerate(seq.frames):
        p = st.step(x).copy()
        d = oracle.dense(shp, dt, seq.weights, seq.bias, x)
        if dt == S.BF16:
            # I2 / I3: accumulated result equals dense inference of this frame, up to the
            # rounding of float64 sums
            assert np.allclose(p, d, rtol=0, atol=1e-10 * max(1.0, np.abs(d).max()))
        else:
            assert np.array_equal(p, d)
        if t > 0:
            n_changed = int((oracle._as_values(dt, x) != oracle._as_values(dt, seq.frames[t - 1])).sum())
            assert st.last_nnz == n_changed
        # I1: the same frame again is a zero difference and leaves P untouched
        before = st.p_prev.copy()
        st.step(x)
        assert st.last_nnz == 0
        assert np.array_equal(before, st.p_prev)


def test_step_skips_exactly_the_zero_entries():
    """Table 1: work is proportional to the density of the difference; the oracle reports the
    number of non-zero difference entries it multiplied."""
    shp = S.fc_shape(50, 7)
    rng = S.rng_for(3)
    w = S.draw_i8_weight(rng, shp.w_shape)
    st = oracle.State(shp, S.I8, w, None)
    x0 = S.draw_i8_act(rng, shp.x_shape)
    x0[0, :10] = 0
    st.step(x0)
    assert st.last_nnz == int((x0 != 0).sum())
    x1 = x0.copy()
    x1[0, 3] = 9
    x1[0, 40] = (int(x1[0, 40]) + 1) % 128
    st.step(x1)
    assert st.last_nnz == 2


# ------------------------------------------------------------------------------------------
# binary: +1/-1 products as XNOR/popcount (Sec. 4.3, XNOR-Net paragraph)
# ------------------------------------------------------------------------------------------
def test_binary_dot_is_k_minus_twice_popcount_exhaustive():
    """For +1/-1 vectors of length k: sum w*x = k - 2*popcount(w_bits XOR x_bits).  Checked for
    every pair of bit patterns with k = 5 against the integer oracle."""
    k = 5
    pats = list(itertools.product([-1, 1], repeat=k))
    shp = S.fc_shape(k, len(pats))
    w = np.array(pats, dtype=np.int8)
    for xp in pats:
        x = np.array([xp], dtype=np.int8)
        y = oracle.dense(shp, S.BIN, w, None, x)[0]
        wb = (w > 0).astype(np.int64)
        xb = (x > 0).astype(np.int64)
        pop = (wb ^ xb).sum(axis=1)
        assert np.array_equal(y, k - 2 * pop)


def test_binary_delta_entries_are_plus_minus_two():
    """After the difference, surviving entries are all +2 or -2 (Sec. 4.3)."""
    seq = S.config4("b14", 0.05, T=3)
    for a, b in zip(seq.frames[:-1], seq.frames[1:]):
        d = b.astype(np.int16) - a.astype(np.int16)
        assert set(np.unique(d).tolist()) <= {-2, 0, 2}
    p = S.pack_pm1(seq.frames[0])
    assert np.array_equal(S.unpack_pm1(p), seq.frames[0])
    # LSB-first: channel 0 is bit 0 of word 0
    one = -np.ones((1, 64), dtype=np.int8)
    one[0, 0] = 1
    one[0, 33] = 1
    assert S.pack_pm1(one).tolist() == [[1, 2]]


# ------------------------------------------------------------------------------------------
# accounting (Table 1, Eq. 6, 9, 10) and formats
# ------------------------------------------------------------------------------------------
def test_table4_speedups_follow_from_eq9_eq10():
    rows = []
    with open(os.path.join(GOLDEN, "table4_overall_sparsity.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            m, d, s, sr, eta = line.split()
            rows.append((float(s) / 100, float(sr) / 100, float(eta) / 100))
    assert len(rows) == 4
    for s, sr, eta in rows:
        assert accounting.eta_from_overall(s, sr) == pytest.approx(eta, rel=0.01)


def test_eq10_equals_ratio_of_eq6_costs_and_eq9_closed_form():
    shapes = [sh for _, sh, _ in S.alexnet_shapes()] + [S.fc_shape(9216, 4096), S.fc_shape(4096, 4096)]
    rng = S.rng_for(1)
    rho = rng.uniform(0.3, 0.9, len(shapes))
    rho_r = rho * rng.uniform(0.1, 0.9, len(shapes))
    eta = accounting.speedup_eta(shapes, rho, rho_r)
    S0 = accounting.overall_sparsity(shapes, 1 - rho)
    S1 = accounting.overall_sparsity(shapes, 1 - rho_r)
    assert eta == pytest.approx(accounting.eta_from_overall(S0, S1), rel=1e-12)
    # Table 1: a layer's cost is its dense count scaled by the density
    assert accounting.sparse_macs(shapes[2], 0.25) == pytest.approx(0.25 * accounting.layer_macs(shapes[2]))
    # dense counts of the AlexNet-shaped stack (multiplications)
    macs = [accounting.layer_macs(s) for s in shapes]
    assert macs[0] == 55 * 55 * 96 * 3 * 11 * 11
    assert macs[1] == 27 * 27 * 256 * 48 * 25
    assert macs[2] == 13 * 13 * 384 * 256 * 9
    assert macs[5] == 9216 * 4096


def test_step_nnz_matches_table1_density():
    """The number of multiplications Algorithm 1 does for an FC layer is rho * C_in * C_out."""
    seq = S.config3("fc7", S.I8, 0.05, T=3)
    st = oracle.State(seq.shape, S.I8, seq.weights, seq.bias)
    st.step(seq.frames[0])
    st.step(seq.frames[1])
    rho = st.last_nnz / seq.shape.c_in
    assert rho == pytest.approx(0.05, abs=1e-3)
    assert accounting.sparse_macs(seq.shape, rho) == st.last_nnz * seq.shape.c_out


def test_bf16_format_matches_library():
    rng = S.rng_for(2)
    a = np.concatenate([rng.normal(size=4096).astype(np.float32) * 10,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    bits = S.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(S.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())
    assert np.array_equal(oracle.bf16_to_f64(bits), ref.to(torch.float64).numpy())


def test_relu_requant_pool_matches_library_pool():
    rng = S.rng_for(4)
    y = rng.integers(-40000, 40000, size=(2, 9, 11, 5)).astype(np.int32)
    out = oracle.relu_requant_pool(y, 7, True)
    a = np.minimum(np.maximum(y, 0) >> 7, 127).astype(np.float32)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(a).permute(0, 3, 1, 2), 3, 2).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(out.astype(np.float32), ref)
    assert np.array_equal(oracle.relu_requant_pool(y, 7, False).astype(np.float32), a)
    assert oracle.calibrate_shift(np.array([127, 0, -5])) == 0
    assert oracle.calibrate_shift(np.array([128 * 8 + 3] * 10)) == 4


# ------------------------------------------------------------------------------------------
# the generators give the stated structure
# ------------------------------------------------------------------------------------------
def test_generators_are_seeded_and_shaped():
    a, b = S.config0(), S.config0()
    assert all(np.array_equal(x, y) for x, y in zip(a.frames, b.frames))
    assert a.frames[0].shape == (1, 32, 32, 16) and len(a.frames) == 8
    for p, c in zip(a.frames[:-1], a.frames[1:]):
        d = S.density(p, c)
        assert 0.095 <= d["rho_pos"] <= 0.14
        assert c.min() >= 0
    q = S.config3("fc6", S.BF16, 0.10, T=3)
    assert S.density(q.frames[0], q.frames[1])["rho_elem"] == pytest.approx(922 / 9216)
    c1 = S.config1(T=3)
    assert c1["frames"][0].shape == (1, 227, 227, 3)
    assert 0.01 < S.density(c1["frames"][0], c1["frames"][1])["rho_pos"] < 0.12


# ---- truncation threshold (Sec. 3.4, "Improving sparsity") ----------------------------------------
def _eps_case(T=5, n=2):
    shp = S.conv_shape(9, 7, 8, 6, 3, 1, 1, n=n)
    seq = S.random_layer(991, shp, S.BF16, T=T, frac=0.4, block=2)
    rng = S.rng_for(992)
    # small perturbations on top of the block redraws, so that some differences fall below a threshold
    frames = [seq.frames[0]]
    for t in range(1, T):
        f = S.bf16_bits_to_f32(seq.frames[t]) + rng.normal(0, 0.02, size=seq.frames[t].shape).astype(np.float32) * (rng.random(seq.frames[t].shape) < 0.5)
        frames.append(S.f32_to_bf16_bits(np.maximum(f, 0).astype(np.float32)))
    return seq, frames


def test_threshold_zero_is_the_exact_method():
    seq, frames = _eps_case()
    a = oracle.State(seq.shape, S.BF16, seq.weights, seq.bias)
    b = oracle.State(seq.shape, S.BF16, seq.weights, seq.bias)
    for x in frames:
        pa = a.step(x).copy()
        pb = b.step(x, eps=0.0)
        assert np.array_equal(pa, pb) and b.last_truncated == 0


def test_threshold_keeps_projection_consistent_with_stored_input():
    """What is truncated is not committed: after every step P equals the dense projection (Eq. 3) of the
    stored input, and the stored input differs from x_t exactly where a difference was truncated."""
    seq, frames = _eps_case()
    st = oracle.State(seq.shape, S.BF16, seq.weights, seq.bias)
    eps = 0.03
    total_trunc = 0
    for x in frames:
        before = st.i_prev.copy()
        p = st.step(x, eps=eps)
        xv = oracle.bf16_to_f64(x)
        d32 = xv.astype(np.float32) - before.astype(np.float32)
        trunc = (d32 != 0) & (np.abs(d32) < np.float32(eps))
        # brute-force classification of every entry, written independently of the C loop
        assert st.last_truncated == int(trunc.sum())
        assert np.isclose(st.last_truncated_sumsq, float((d32[trunc].astype(np.float64) ** 2).sum()), rtol=1e-12, atol=0)
        assert np.array_equal(st.i_prev[trunc], before[trunc]) and np.array_equal(st.i_prev[~trunc], xv[~trunc])
        stored_bits = S.f32_to_bf16_bits(st.i_prev.astype(np.float32))
        want = oracle.dense(seq.shape, S.BF16, seq.weights, seq.bias, stored_bits)
        assert np.abs(p - want).max() <= 1e-9 * max(1.0, np.abs(want).max())
        total_trunc += st.last_truncated
    assert total_trunc > 0  # the case does exercise the threshold


def test_threshold_above_every_difference_changes_nothing():
    seq, frames = _eps_case(T=3)
    st = oracle.State(seq.shape, S.BF16, seq.weights, seq.bias)
    p0 = st.p_prev.copy()
    for x in frames:
        st.step(x, eps=1e30)
        assert np.array_equal(st.p_prev, p0) and not st.i_prev.any() and st.last_nnz == 0
