"""Operation-count formulas of the paper, written from Table 1 and Eq. 6, 9 and 10 (Sec. 3.3, 4).
TEST INFRASTRUCTURE ONLY (part of the oracle).

All counts are multiplications ("adds are trivial", Sec. 3.3).  A layer is anything with the
fields of ``rrm_synth.LayerShape``.
"""
from __future__ import annotations

from typing import Sequence

FC = 1


def layer_macs(shape) -> int:
    """Table 1, dense rows: W*H*C_in*C_out*w_F*h_F for a convolution (W, H the output map; with
    stride 1 and 'same' padding this is the input map, which is the case the paper assumes),
    C_in*C_out for an FC layer.  Grouped convolutions see C_in/groups inputs per output."""
    if shape.kind == FC:
        return shape.n * shape.c_in * shape.c_out
    ho = (shape.h + 2 * shape.pad - shape.kh) // shape.stride + 1
    wo = (shape.w + 2 * shape.pad - shape.kw) // shape.stride + 1
    return shape.n * ho * wo * (shape.c_in // shape.groups) * shape.c_out * shape.kh * shape.kw


def sparse_macs(shape, rho: float) -> float:
    """Table 1, '+ SPMV' rows: the dense count scaled by the input density rho."""
    return rho * layer_macs(shape)


def network_cost(shapes: Sequence, rhos: Sequence[float]) -> float:
    """Eq. 6: sum over layers of rho * dense count."""
    return sum(sparse_macs(s, r) for s, r in zip(shapes, rhos))


def overall_sparsity(shapes: Sequence, sparsities: Sequence[float]) -> float:
    """Eq. 9: operation-weighted share of zero inputs over all linear layers."""
    num = sum(sp * layer_macs(s) for s, sp in zip(shapes, sparsities))
    den = sum(layer_macs(s) for s in shapes)
    return num / den


def speedup_eta(shapes: Sequence, rhos: Sequence[float], rhos_rrm: Sequence[float]) -> float:
    """Eq. 10: cost with the original input densities over cost with the RRM densities."""
    return network_cost(shapes, rhos) / network_cost(shapes, rhos_rrm)


def eta_from_overall(S: float, S_rrm: float) -> float:
    """Eq. 9 and Eq. 10 over the same set of layers give eta = (1 - S) / (1 - S_rrm)."""
    return (1.0 - S) / (1.0 - S_rrm)
