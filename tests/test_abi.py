"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
before touching the GPU (runs without a GPU: no compute calls)."""
import ctypes
import os
import re

import pytest

import paper_1802_09723_amd as rrm
from paper_1802_09723_amd.binding import Shape
import rrm_synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rrm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rrm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert {"rrm_layer_create", "rrm_step", "rrm_dense", "rrm_reset", "rrm_snapshot", "rrm_read_snapshot",
            "rrm_set_option", "rrm_get_stats", "rrm_layer_destroy", "rrm_status_string", "rrm_last_error",
            "rrm_aux_relu_requant_pool_i8", "rrm_aux_relu_requant_pool_changed_i8", "rrm_set_threshold", "rrm_step_from_projection",
            "rrm_stack_step", "rrm_dense_noalloc"} <= set(names)
    L = ctypes.CDLL(rrm.lib_path())
    for n in names:
        assert hasattr(L, n), f"{n} is declared in rrm.h but not exported"


def test_shape_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "rrm.h")).read()
    m = re.search(r"int kind;[^}]*?int ([a-z_, ]+);\s*}\s*rrm_shape;", text, flags=re.S)
    fields = ["kind"] + [f.strip() for f in m.group(1).split(",")]
    assert fields == [k for k, _ in Shape._fields_]
    assert fields == [f.name for f in __import__("dataclasses").fields(S.LayerShape)]


def _create(shape, dtype, weights=b"\0" * 64, out=True):
    L = rrm.lib()
    cs = Shape.of(shape) if shape is not None else None
    h = ctypes.c_void_p()
    buf = ctypes.create_string_buffer(weights) if weights is not None else None
    return L.rrm_layer_create(buf, None, ctypes.byref(cs) if cs is not None else None, dtype,
                              ctypes.byref(h) if out else None)


def test_stats_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "rrm.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\}\s*rrm_stats;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    decl = [(t, n) for t, n in re.findall(r"(uint64_t|int32_t|double)\s+([a-z_]+)\s*;", body)]
    ctype = {"uint64_t": ctypes.c_uint64, "int32_t": ctypes.c_int32, "double": ctypes.c_double}
    assert [(n, ctype[t]) for t, n in decl] == list(rrm.binding.Stats._fields_)


def test_argument_errors_come_back_as_status_codes():
    L = rrm.lib()
    ok = S.conv_shape(8, 8, 16, 16, 3, 1, 1)
    assert _create(ok, 0, out=False) == -1            # RRM_ERR_NULL
    assert _create(ok, 0, weights=None) == -1
    assert _create(None, 0) == -1
    assert _create(ok, 7) == -3                        # RRM_ERR_DTYPE
    assert _create(S.fc_shape(64, 64), 2) == -3        # binary FC
    assert _create(S.conv_shape(8, 8, 16, 16, 3, 0, 1), 0) == -2     # stride 0
    assert _create(S.conv_shape(8, 8, 16, 15, 3, 1, 1, groups=2), 0) == -2
    assert _create(S.conv_shape(2, 2, 16, 16, 5, 1, 0), 0) == -2     # window larger than input
    assert _create(S.conv_shape(8, 8, 48, 16, 3, 1, 1), 2) == -2     # binary c_in not multiple of 32
    assert b"multiple of 32" in L.rrm_last_error()
    assert _create(S.conv_shape(8, 8, 16, 16, 3, 1, 1, n=0), 0) == -2
    assert L.rrm_step(None, None, None, None) == -1
    assert L.rrm_dense(None, None, None, None) == -1
    assert L.rrm_reset(None, None) == -1
    assert L.rrm_stack_step(None, 0, None, None, None) == -1
    assert L.rrm_dense_noalloc(None, None, None, None) == -1
    assert L.rrm_aux_probe_copy(None, None, 0, None) == -1
    assert L.rrm_aux_probe_mfma(0, None, 1, 1, None) == -1
    assert L.rrm_set_option(None, b"path", 0) == -1
    assert L.rrm_get_stats(None, None) == -1
    assert L.rrm_status_string(-9) == b"misaligned pointer"
    assert L.rrm_status_string(0) == b"ok"
    L.rrm_layer_destroy(None)  # no-op


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_1802_09723_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(RuntimeError, match="missing"):
        binding.lib()
