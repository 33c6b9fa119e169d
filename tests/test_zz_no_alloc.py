"""rrm_dense_noalloc: the dense FC layer whose partial-sum scratch is a static device array (for callers that
cannot allocate).  Two calls in a row, the second on a smaller layer, each checked against rrm_dense of the same
handle (same kernels, same summation order: bit-identical) and against the oracle."""
import numpy as np
import pytest

import oracle
import rrm_synth as S
from gpu_util import assert_matches, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", [S.I8, S.BF16])
def test_dense_noalloc_two_calls_second_smaller(dt):
    import torch
    import paper_1802_09723_amd as rrm
    shapes = [S.fc_shape(1500, 1030, n=3), S.fc_shape(300, 77, n=2)]  # the second call has the smaller input
    layers, xs, wants = [], [], []
    for k, shp in enumerate(shapes):
        seq = S.random_layer(4200 + 10 * k + dt, shp, dt, T=1)
        layers.append(rrm.Layer(shp, dt, seq.weights, seq.bias))
        xs.append(to_device(seq.frames[0], dt))
        wants.append(oracle.dense(shp, dt, seq.weights, seq.bias, seq.frames[0]))
    tdt = torch.float32 if dt == S.BF16 else torch.int32
    for rep in range(2):  # twice: the array keeps the last call's contents
        for L, x, want in zip(layers, xs, wants):
            y_ref = torch.empty(L.y_shape, dtype=tdt, device="cuda")
            y_new = torch.full(L.y_shape, 7, dtype=tdt, device="cuda")
            L.dense(x, y_ref)
            L.dense_noalloc(x, y_new)
            torch.cuda.synchronize()
            assert torch.equal(y_ref, y_new), f"rep {rep}: rrm_dense_noalloc differs from rrm_dense"
            assert_matches(y_new.cpu().numpy(), want, dt, f"rrm_dense_noalloc {L.shape}")
    for L in layers:
        L.destroy()


def test_dense_noalloc_rejects_what_does_not_fit():
    import torch
    import paper_1802_09723_amd as rrm
    from paper_1802_09723_amd.binding import RRMError
    # conv layers have no such variant
    seq = S.config0(T=1)
    L = rrm.Layer(seq.shape, S.I8, seq.weights, seq.bias)
    x = to_device(seq.frames[0], S.I8)
    y = torch.empty(L.y_shape, dtype=torch.int32, device="cuda")
    with pytest.raises(RRMError) as e:
        L.dense_noalloc(x, y)
    assert e.value.status == -2
    L.destroy()
    # partial sums beyond the 4 MiB array: 300 streams x 1 split x 4096 x 4 bytes
    shp = S.fc_shape(16, 4096, n=300)
    rng = S.rng_for(77)
    L = rrm.Layer(shp, S.I8, S.draw_i8_weight(rng, shp.w_shape), None)
    x = torch.zeros(shp.x_shape, dtype=torch.int8, device="cuda")
    y = torch.empty(L.y_shape, dtype=torch.int32, device="cuda")
    with pytest.raises(RRMError) as e:
        L.dense_noalloc(x, y)
    assert e.value.status == -2 and "static scratch" in str(e.value)
    L.destroy()
