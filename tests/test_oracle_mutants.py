"""Planted mistakes in a copy of the oracle must be caught by the pins (CPU only).

Each mutant is the oracle's C source with one plausible slip (a flipped kernel, transposed
taps, a dropped group offset, a wrong sign, an ignored stride, a bias added by the recurrence);
it is compiled to a temporary library, swapped in, and the pin set must fail on it.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
import rrm_synth as S
from test_oracle_pins import SHAPES, STEP_SHAPES, _torch_conv, test_float_fc_matches_numpy_matvec

SRC = os.path.join(os.path.dirname(oracle.__file__), "rrm_oracle.c")

MUTANTS = {
    "kernel_flip": ("const int iy = oy * s->stride - s->pad + ky;", "const int iy = oy * s->stride - s->pad + (s->kh - 1 - ky);"),
    "group_offset_dropped": ("* s->c_in + (size_t)g * cg;\n                            const int8_t* wp", "* s->c_in;\n                            const int8_t* wp"),
    "step_sign": ("const int d = (int)x_t[xi] - (int)i_prev[xi];", "const int d = (int)i_prev[xi] - (int)x_t[xi];"),
    "step_stride_ignored": ("if (ty < 0 || ty % s->stride) continue;\n                        const int oy = ty / s->stride;\n                        if (oy >= ho) continue;\n                        for (int kx = 0; kx < s->kw; ++kx) {\n                            const int tx = ix + s->pad - kx;\n                            if (tx < 0 || tx % s->stride) continue;\n                            const int ox = tx / s->stride;\n                            if (ox >= wo) continue;\n                            for (int oo = 0; oo < og; ++oo) {\n                                const int o = g * og + oo;\n                                const size_t yi",
                            "if (ty < 0) continue;\n                        const int oy = ty / s->stride;\n                        if (oy >= ho) continue;\n                        for (int kx = 0; kx < s->kw; ++kx) {\n                            const int tx = ix + s->pad - kx;\n                            if (tx < 0 || tx % s->stride) continue;\n                            const int ox = tx / s->stride;\n                            if (ox >= wo) continue;\n                            for (int oo = 0; oo < og; ++oo) {\n                                const int o = g * og + oo;\n                                const size_t yi"),
    "pad_sign": ("const int ty = iy + s->pad - ky;\n                        if (ty < 0 || ty % s->stride) continue;\n                        const int oy = ty / s->stride;\n                        if (oy >= ho) continue;\n                        for (int kx = 0; kx < s->kw; ++kx) {\n                            const int tx = ix + s->pad - kx;\n                            if (tx < 0 || tx % s->stride) continue;\n                            const int ox = tx / s->stride;\n                            if (ox >= wo) continue;\n                            for (int oo = 0; oo < og; ++oo) {\n                                const int o = g * og + oo;\n                                const size_t yi",
                 "const int ty = iy - s->pad - ky;\n                        if (ty < 0 || ty % s->stride) continue;\n                        const int oy = ty / s->stride;\n                        if (oy >= ho) continue;\n                        for (int kx = 0; kx < s->kw; ++kx) {\n                            const int tx = ix + s->pad - kx;\n                            if (tx < 0 || tx % s->stride) continue;\n                            const int ox = tx / s->stride;\n                            if (ox >= wo) continue;\n                            for (int oo = 0; oo < og; ++oo) {\n                                const int o = g * og + oo;\n                                const size_t yi"),
    "fc_transposed": ("acc += (int64_t)wt[(size_t)o * s->c_in + j] * x[(size_t)b * s->c_in + j];",
                      "acc += (int64_t)wt[(size_t)j * s->c_out + o] * x[(size_t)b * s->c_in + j];"),
    "dense_bias_dropped": ("int64_t acc = bias ? bias[o] : 0;\n                    for (int ky", "int64_t acc = 0;\n                    for (int ky"),
}
MUTANTS["weight_taps_swapped"] = ("const int8_t* wp = wt + (((size_t)o * s->kh + ky) * s->kw + kx) * cg;",
                                  "const int8_t* wp = wt + (((size_t)o * s->kh + kx) * s->kw + ky) * cg;")
# floating-point FC branches (a mutant may be a list of replacements applied together)
_FC_DENSE_F64 = ("acc += wt[(size_t)o * s->c_in + j] * x[(size_t)b * s->c_in + j];",
                 "acc += wt[(size_t)j * s->c_out + o] * x[(size_t)b * s->c_in + j];")
_FC_STEP_F64 = ("p_prev[(size_t)b * s->c_out + o] += d * wt[(size_t)o * s->c_in + j];",
                "p_prev[(size_t)b * s->c_out + o] += d * wt[(size_t)j * s->c_out + o];")
MUTANTS["fc_f64_dense_transposed"] = _FC_DENSE_F64
MUTANTS["fc_f64_step_transposed"] = _FC_STEP_F64
MUTANTS["fc_f64_both_transposed"] = [_FC_DENSE_F64, _FC_STEP_F64]
MUTANTS["fc_f64_bias_dropped"] = ("double acc = bias ? bias[o] : 0.0;\n                for (int j", "double acc = 0.0;\n                for (int j")
MUTANTS["step_f64_sign"] = ("const double d = x_t[xi] - i_prev[xi];", "const double d = i_prev[xi] - x_t[xi];")


def _pin_set():
    """A condensed run of the pins: library convolution, mat-vec special case, invariants."""
    for shp in SHAPES[:5]:
        rng = S.rng_for(100 + shp.h)
        w = S.draw_i8_weight(rng, shp.w_shape)
        b = S.draw_i32_bias(rng, shp.c_out)
        x = rng.integers(-128, 128, size=shp.x_shape).astype(np.int8)
        assert np.array_equal(oracle.dense(shp, S.I8, w, b, x).astype(np.float64), _torch_conv(shp, w, b, x))
    rng = S.rng_for(5)
    wt = S.draw_i8_weight(rng, (4, 4))
    x = S.draw_i8_act(rng, (1, 4))
    assert np.array_equal(oracle.dense(S.fc_shape(4, 4), S.I8, wt, None, x), x.astype(np.int64) @ wt.astype(np.int64).T)
    for shp, dt in STEP_SHAPES:
        seq = S.random_layer(900 + shp.c_in, shp, dt, T=3, frac=0.25, block=2)
        st = oracle.State(shp, dt, seq.weights, seq.bias)
        for xx in seq.frames:
            p, d = st.step(xx), oracle.dense(shp, dt, seq.weights, seq.bias, xx)
            if dt == S.BF16:
                assert np.allclose(p, d, rtol=0, atol=1e-10 * max(1.0, np.abs(d).max()))
            else:
                assert np.array_equal(p, d)
    # floating-point dense convolution against the library routine, FC branches against numpy
    for shp in SHAPES[:2]:
        rng = S.rng_for(200 + shp.h)
        w = S.draw_bf16_weight(rng, shp.w_shape)
        x = S.draw_bf16_relu(rng, shp.x_shape)
        ref = _torch_conv(shp, oracle.bf16_to_f64(w), None, oracle.bf16_to_f64(x))
        assert np.allclose(oracle.dense(shp, S.BF16, w, None, x), ref, rtol=1e-12, atol=1e-12)
    test_float_fc_matches_numpy_matvec()


def test_pin_set_passes_on_the_real_oracle():
    _pin_set()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, tmp_path, monkeypatch):
    edits = MUTANTS[name]
    if isinstance(edits, tuple):
        edits = [edits]
    mutated = open(SRC).read()
    for old, new in edits:
        assert mutated.count(old) >= 1, f"mutation site for {name} not found"
        mutated = mutated.replace(old, new, 1)
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c)], check=True)
    real = oracle.lib()
    mut = ctypes.CDLL(str(so))
    for fn in ("orc_dense_i8", "orc_dense_f64", "orc_step_i8", "orc_step_f64"):
        getattr(mut, fn).argtypes = getattr(real, fn).argtypes
        getattr(mut, fn).restype = getattr(real, fn).restype
    monkeypatch.setattr(oracle, "_lib", mut)
    with pytest.raises(AssertionError):
        _pin_set()
