"""Helpers of the GPU parity tests: boundary-format conversion and oracle comparison."""
import numpy as np

import oracle
import rrm_synth as S


def to_device(frame: np.ndarray, dtype: int):
    """numpy frame in generator format -> contiguous CUDA tensor in the library's boundary format."""
    import torch
    if dtype == S.I8:
        return torch.from_numpy(np.ascontiguousarray(frame, dtype=np.int8)).cuda()
    if dtype == S.BF16:
        return torch.from_numpy(np.ascontiguousarray(frame, dtype=np.uint16).view(np.int16)).cuda()
    return torch.from_numpy(S.pack_pm1(frame).view(np.int32)).cuda()


def boundary_weights(seq):
    """weights in the format rrm_layer_create takes"""
    if seq.dtype == S.BIN:
        return S.pack_pm1(seq.weights)
    return seq.weights


def make_layer(seq, **opts):
    """A layer handle with the given options.  "conv_kernel" = 2 (the position-gather kernel) is dropped for layers
    that kernel does not take (stride > 1, channel runs that are not 16-byte multiples, FC, binary)."""
    import paper_1802_09723_amd as rrm
    layer = rrm.Layer(seq.shape, seq.dtype, boundary_weights(seq), seq.bias)
    for k, v in opts.items():
        if k == "conv_kernel":
            try:
                layer.set_option(k, v)
            except rrm.binding.RRMError:
                pass
            continue
        layer.set_option(k, v)
    return layer


def x_bytes(frame: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == S.I8:
        return np.ascontiguousarray(frame, dtype=np.int8).view(np.uint8).reshape(-1)
    if dtype == S.BF16:
        return np.ascontiguousarray(frame, dtype=np.uint16).view(np.uint8).reshape(-1)
    return S.pack_pm1(frame).view(np.uint8).reshape(-1)


def assert_matches(got: np.ndarray, want: np.ndarray, dtype: int, what: str, rel: float = 1e-3):
    """Bit-exact for the integer paths; |err| <= rel * max|y| for bf16-in / fp32-accumulate."""
    assert got.shape == want.shape, f"{what}: shape {got.shape} != {want.shape}"
    if dtype == S.BF16:
        scale = float(np.abs(want).max())
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= rel * max(scale, 1e-30), f"{what}: max err {err:.3e} > {rel:g} * max|y| = {rel * scale:.3e}"
        return err / max(scale, 1e-30)
    bad = int((got != want).sum())
    assert bad == 0, f"{what}: {bad} of {got.size} elements differ"
    return 0.0


def run_sequence(seq, check_frames=None, check_dense=(0,), check_x=True, y_out_frames=(), rel=1e-3, **opts):
    """Drive rrm_step over a sequence and compare the stored projection with the oracle's dense
    projection (Eq. 3) of the same frame."""
    import torch
    layer = make_layer(seq, **opts)
    worst = 0.0
    T = len(seq.frames)
    for t, x in enumerate(seq.frames):
        xd = to_device(x, seq.dtype)
        y_out = None
        if t in y_out_frames:
            y_out = torch.empty(layer.y_shape, dtype=torch.float32 if seq.dtype == S.BF16 else torch.int32, device="cuda")
        layer.step(xd, y_out)
        if check_frames is None or t in check_frames or t == T - 1:
            want = oracle.dense(seq.shape, seq.dtype, seq.weights, seq.bias, x)
            got = layer.y_snapshot().cpu().numpy()
            worst = max(worst, assert_matches(got, want, seq.dtype, f"{seq.name} frame {t}", rel))
            if y_out is not None:
                assert np.array_equal(y_out.cpu().numpy(), got), f"{seq.name} frame {t}: y_out differs from snapshot"
            if t in check_dense:
                yd = torch.empty_like(layer.y_snapshot())
                layer.dense(xd, yd)
                torch.cuda.synchronize()
                assert_matches(yd.cpu().numpy(), want, seq.dtype, f"{seq.name} rrm_dense frame {t}", rel)
            if check_x:
                assert np.array_equal(layer.x_snapshot_bytes().cpu().numpy(), x_bytes(x, seq.dtype)), \
                    f"{seq.name} frame {t}: stored input differs from x_t"
    st = layer.stats()
    layer.destroy()
    return st, worst
