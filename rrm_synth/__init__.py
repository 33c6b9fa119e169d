"""Seeded synthetic inputs for the Recurrent Residual Module (RRM) delta-update path.

This module only *draws numbers and lays them out*: layer shapes, weights, biases and
frame sequences whose frame-to-frame differences have the structure of the paper's
video workloads (a moving patch over a static background, spatial blocks that are
re-drawn, a fraction of a feature vector that changes, clustered sign flips).
It holds none of the method's arithmetic (no convolution, no delta, no accumulation),
so that both the CPU oracle and the HIP library can be fed from it without sharing code.

Conventions
-----------
* activations are NHWC (``[n, h, w, c]``), conv weights ``[c_out, kh, kw, c_in/groups]``,
  FC weights ``[c_out, c_in]``.
* int8 tensors are ``numpy.int8``; bf16 tensors are carried as their 16-bit patterns in
  ``numpy.uint16`` (``bf16_bits``) next to the exactly equal ``float32`` values;
  binary tensors are carried as ``numpy.int8`` arrays of +1/-1 next to their bit-packed
  form (bit = 1 means +1, channels packed LSB-first into ``uint32`` words along c).
* every generator takes an integer ``seed`` and uses ``numpy.random.Generator(PCG64(seed))``.
  ``seed_for(config, case)`` gives the seed convention used by the tests and the bench.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 180209723_00


def seed_for(config: int, case: int = 0) -> int:
    """Seed of (config, case): BASE + 100*config + case."""
    return BASE_SEED + 100 * int(config) + int(case)


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


# --------------------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------------------
CONV, FC = 0, 1
I8, BF16, BIN = 0, 1, 2


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """Mirror of the C ``rrm_shape`` struct (same field order)."""

    kind: int = CONV
    n: int = 1
    h: int = 1
    w: int = 1
    c_in: int = 1
    c_out: int = 1
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1

    @property
    def h_out(self) -> int:
        return (self.h + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def w_out(self) -> int:
        return (self.w + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def x_shape(self) -> Tuple[int, ...]:
        if self.kind == FC:
            return (self.n, self.c_in)
        return (self.n, self.h, self.w, self.c_in)

    @property
    def y_shape(self) -> Tuple[int, ...]:
        if self.kind == FC:
            return (self.n, self.c_out)
        return (self.n, self.h_out, self.w_out, self.c_out)

    @property
    def w_shape(self) -> Tuple[int, ...]:
        if self.kind == FC:
            return (self.c_out, self.c_in)
        return (self.c_out, self.kh, self.kw, self.c_in // self.groups)

    def with_n(self, n: int) -> "LayerShape":
        return dataclasses.replace(self, n=n)


def conv_shape(h, w, c_in, c_out, k, stride=1, pad=0, groups=1, n=1) -> LayerShape:
    return LayerShape(CONV, n, h, w, c_in, c_out, k, k, stride, pad, groups)


def fc_shape(c_in, c_out, n=1) -> LayerShape:
    return LayerShape(FC, n, 1, 1, c_in, c_out, 1, 1, 1, 0, 1)


# --------------------------------------------------------------------------------------
# number formats (layout only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 patterns to float32."""
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def pack_pm1(a: np.ndarray) -> np.ndarray:
    """Pack a +1/-1 int8 array along its last axis into uint32 words.

    Bit k of word j holds channel 32*j+k; bit = 1 means +1. The last axis must be a
    multiple of 32.
    """
    a = np.asarray(a)
    c = a.shape[-1]
    if c % 32:
        raise ValueError("binary channel count must be a multiple of 32")
    bits = (a > 0).astype(np.uint8)
    packed = np.packbits(bits.reshape(a.shape[:-1] + (c // 32, 32)), axis=-1, bitorder="little")
    return np.ascontiguousarray(packed).view(np.uint32).reshape(a.shape[:-1] + (c // 32,))


def unpack_pm1(words: np.ndarray) -> np.ndarray:
    """Inverse of :func:`pack_pm1`: uint32 words -> +1/-1 int8."""
    wds = np.ascontiguousarray(words, dtype=np.uint32)
    by = wds.view(np.uint8).reshape(wds.shape + (4,))
    bits = np.unpackbits(by, axis=-1, bitorder="little").reshape(wds.shape[:-1] + (wds.shape[-1] * 32,))
    return (bits.astype(np.int8) * 2 - 1).astype(np.int8)


# --------------------------------------------------------------------------------------
# value drawers
# --------------------------------------------------------------------------------------
def draw_i8_act(rng, shape) -> np.ndarray:
    """post-ReLU style int8 activations, uniform on [0, 127]."""
    return rng.integers(0, 128, size=shape, dtype=np.int16).astype(np.int8)


def draw_i8_relu(rng, shape) -> np.ndarray:
    """max(0, U[-127,127]) int8 activations (about half the entries are zero)."""
    return np.maximum(rng.integers(-127, 128, size=shape, dtype=np.int16), 0).astype(np.int8)


def draw_i8_weight(rng, shape) -> np.ndarray:
    return rng.integers(-127, 128, size=shape, dtype=np.int16).astype(np.int8)


def draw_i32_bias(rng, n) -> np.ndarray:
    return rng.integers(-1000, 1001, size=(n,), dtype=np.int32)


def draw_bf16_weight(rng, shape, sigma=0.05) -> np.ndarray:
    """N(0, sigma) rounded to bf16; returns the bf16 patterns."""
    return f32_to_bf16_bits(rng.normal(0.0, sigma, size=shape).astype(np.float32))


def draw_bf16_relu(rng, shape) -> np.ndarray:
    """ReLU(N(0,1)) rounded to bf16; returns the bf16 patterns."""
    return f32_to_bf16_bits(np.maximum(rng.normal(0.0, 1.0, size=shape), 0.0).astype(np.float32))


def draw_pm1(rng, shape) -> np.ndarray:
    return (rng.integers(0, 2, size=shape, dtype=np.int8) * 2 - 1).astype(np.int8)


# --------------------------------------------------------------------------------------
# change structure
# --------------------------------------------------------------------------------------
def block_cover_mask(rng, h: int, w: int, block: int, target_frac: float) -> np.ndarray:
    """Boolean [h, w] mask made of randomly placed (unaligned, possibly overlapping)
    block x block squares, added until at least ``target_frac`` of the positions is
    covered. A block larger than the target on its own is shrunk to side
    max(1, floor(sqrt(target_frac*h*w))) and clipped to the map."""
    mask = np.zeros((h, w), dtype=bool)
    if target_frac <= 0:
        return mask
    want = target_frac * h * w
    side = block
    if block * block > want:
        side = max(1, int(math.floor(math.sqrt(want))))
    side = min(side, h, w)
    guard = 0
    while mask.sum() < want - 1e-9 and guard < 100000:
        y0 = int(rng.integers(0, h - side + 1))
        x0 = int(rng.integers(0, w - side + 1))
        mask[y0:y0 + side, x0:x0 + side] = True
        guard += 1
    return mask


def redraw_where(x: np.ndarray, mask_hw: np.ndarray, fresh: np.ndarray) -> np.ndarray:
    """Copy of ``x`` ([h, w, c]) with all channels at masked positions taken from ``fresh``."""
    out = x.copy()
    out[mask_hw] = fresh[mask_hw]
    return out


def density(prev: np.ndarray, cur: np.ndarray) -> Dict[str, float]:
    """Realised change fractions between two frames: per element, and per position (the last
    axis being channels)."""
    ne = prev != cur
    pos = ne.any(axis=-1) if ne.ndim > 1 else ne
    return {"rho_elem": float(ne.mean()), "rho_pos": float(pos.mean())}


# --------------------------------------------------------------------------------------
# a sequence bundle
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class Sequence_:
    """One layer's workload: weights, bias and T frames of input for n streams."""

    shape: LayerShape
    dtype: int
    weights: np.ndarray           # int8 | uint16 (bf16 bits) | int8 +/-1
    bias: Optional[np.ndarray]    # int32 | float32 | None
    frames: List[np.ndarray]      # each of shape.x_shape; int8 | uint16 | int8 +/-1
    name: str = ""
    meta: Dict = dataclasses.field(default_factory=dict)


def _stack_streams(per_stream: List[List[np.ndarray]]) -> List[np.ndarray]:
    T = len(per_stream[0])
    return [np.stack([s[t] for s in per_stream], axis=0) for t in range(T)]


def block_redraw_frames(rng, h, w, c, T, block, frac, draw: Callable) -> List[np.ndarray]:
    """T frames [h, w, c]; frame 0 fully drawn, every later frame re-draws all channels in
    random blocks covering >= frac of the positions."""
    frames = [draw(rng, (h, w, c))]
    for _ in range(1, T):
        m = block_cover_mask(rng, h, w, block, frac)
        frames.append(redraw_where(frames[-1], m, draw(rng, (h, w, c))))
    return frames


# ---- config 0 -------------------------------------------------------------------------
def config0(seed: Optional[int] = None, n: int = 1, T: int = 8) -> Sequence_:
    """Single 3x3 conv, 16->16 channels on 32x32, int8; 4x4 blocks re-drawn over 10 % of
    the positions per frame."""
    seed = seed_for(0) if seed is None else seed
    rng = rng_for(seed)
    shp = conv_shape(32, 32, 16, 16, 3, 1, 1, 1, n)
    wts = draw_i8_weight(rng, shp.w_shape)
    bias = draw_i32_bias(rng, 16)
    streams = [block_redraw_frames(rng, 32, 32, 16, T, 4, 0.10, draw_i8_act) for _ in range(n)]
    return Sequence_(shp, I8, wts, bias, _stack_streams(streams), "cfg0_conv3x3_16_32x32")


# ---- config 1 -------------------------------------------------------------------------
ALEXNET_LAYERS = (
    # name, h, w, c_in, c_out, k, stride, pad, groups, pool_after
    ("conv1", 227, 227, 3, 96, 11, 4, 0, 1, True),
    ("conv2", 27, 27, 96, 256, 5, 1, 2, 2, True),
    ("conv3", 13, 13, 256, 384, 3, 1, 1, 1, False),
    ("conv4", 13, 13, 384, 384, 3, 1, 1, 1, False),
    ("conv5", 13, 13, 384, 256, 3, 1, 1, 1, False),
)


def alexnet_shapes(n: int = 1, groups45: int = 1) -> List[Tuple[str, LayerShape, bool]]:
    out = []
    for name, h, w, ci, co, k, s, p, g, pool in ALEXNET_LAYERS:
        if name in ("conv4", "conv5"):
            g = groups45
        out.append((name, conv_shape(h, w, ci, co, k, s, p, g, n), pool))
    return out


def moving_patch_frames(rng, h, w, c, T) -> List[np.ndarray]:
    """Static random background; one square random-texture patch (side 30..60) that moves
    1..4 px per frame along a fixed random direction, reflecting at the borders; the texture
    moves with the patch."""
    bg = draw_i8_act(rng, (h, w, c))
    side = int(rng.integers(30, 61))
    tex = draw_i8_act(rng, (side, side, c))
    y = int(rng.integers(0, h - side + 1))
    x = int(rng.integers(0, w - side + 1))
    ang = float(rng.uniform(0, 2 * math.pi))
    dy, dx = math.sin(ang), math.cos(ang)
    fy, fx = float(y), float(x)
    frames = []
    for _ in range(T):
        f = bg.copy()
        yy, xx = int(round(fy)), int(round(fx))
        yy = min(max(yy, 0), h - side)
        xx = min(max(xx, 0), w - side)
        f[yy:yy + side, xx:xx + side] = tex
        frames.append(f)
        step = int(rng.integers(1, 5))
        fy += dy * step
        fx += dx * step
        if fy < 0:
            fy, dy = -fy, -dy
        if fy > h - side:
            fy, dy = 2 * (h - side) - fy, -dy
        if fx < 0:
            fx, dx = -fx, -dx
        if fx > w - side:
            fx, dx = 2 * (w - side) - fx, -dx
    return frames


def config1(seed: Optional[int] = None, n: int = 1, T: int = 32, groups45: int = 1) -> Dict:
    """AlexNet-shaped int8 conv stack: per-layer weights and the input frame sequences
    (227x227x3). Inputs of the deeper layers come from running the stack."""
    seed = seed_for(1) if seed is None else seed
    rng = rng_for(seed)
    layers = []
    for name, shp, pool in alexnet_shapes(n, groups45):
        layers.append({
            "name": name, "shape": shp, "pool": pool,
            "weights": draw_i8_weight(rng, shp.w_shape),
            "bias": draw_i32_bias(rng, shp.c_out),
        })
    streams = [moving_patch_frames(rng, 227, 227, 3, T) for _ in range(n)]
    return {"layers": layers, "frames": _stack_streams(streams), "dtype": I8, "name": "cfg1_alexnet_conv_stack"}


# ---- config 2 -------------------------------------------------------------------------
RESNET_LAYERS = (("r56", 56, 64), ("r28", 28, 128), ("r14", 14, 256), ("r7", 7, 512))
RESNET_DENSITIES = (0.02, 0.05, 0.10, 0.25, 0.50)


def config2(layer: str, frac: float, seed: Optional[int] = None, n: int = 1, T: int = 16) -> Sequence_:
    """ResNet-18-shaped 3x3 conv (c_out = c_in), bf16 weights N(0,0.05), inputs
    ReLU(N(0,1)); per frame 8x8 blocks are re-drawn up to the position fraction ``frac``."""
    hw, c = {k: (a, b) for k, a, b in RESNET_LAYERS}[layer]
    li = [k for k, _, _ in RESNET_LAYERS].index(layer)
    di = RESNET_DENSITIES.index(frac) if frac in RESNET_DENSITIES else 9
    seed = seed_for(2, 10 * li + di) if seed is None else seed
    rng = rng_for(seed)
    shp = conv_shape(hw, hw, c, c, 3, 1, 1, 1, n)
    wts = draw_bf16_weight(rng, shp.w_shape)
    streams = [block_redraw_frames(rng, hw, hw, c, T, 8, frac, draw_bf16_relu) for _ in range(n)]
    return Sequence_(shp, BF16, wts, None, _stack_streams(streams), f"cfg2_{layer}_d{int(round(frac * 100))}")


# ---- config 3 -------------------------------------------------------------------------
FC_LAYERS = (("fc6", 9216, 4096), ("fc7", 4096, 4096))
FC_DENSITIES = (0.01, 0.05, 0.10, 0.25)


def subset_redraw_frames(rng, c_in, T, frac, dtype) -> List[np.ndarray]:
    """T vectors; every frame after the first re-draws a uniformly random subset of
    ceil(frac*c_in) entries to values guaranteed different; all other entries stay
    bit-identical."""
    if dtype == I8:
        cur = draw_i8_relu(rng, (c_in,))
    else:
        cur = draw_bf16_relu(rng, (c_in,))
    frames = [cur]
    k = int(math.ceil(frac * c_in - 1e-9))
    for _ in range(1, T):
        nxt = frames[-1].copy()
        idx = rng.choice(c_in, size=k, replace=False)
        if dtype == I8:
            fresh = draw_i8_relu(rng, (k,))
            same = fresh == nxt[idx]
            # a guaranteed-different value: move to another value inside [0,127]
            fresh[same] = ((fresh[same].astype(np.int16) + 1 + rng.integers(0, 126, size=int(same.sum()))) % 128).astype(np.int8)
        else:
            fresh = draw_bf16_relu(rng, (k,))
            same = fresh == nxt[idx]
            while same.any():
                fresh[same] = f32_to_bf16_bits(np.abs(rng.normal(0.0, 1.0, size=int(same.sum()))).astype(np.float32) + np.float32(0.0078125))
                same = fresh == nxt[idx]
        nxt[idx] = fresh
        frames.append(nxt)
    return frames


def config3(layer: str, dtype: int, frac: float, seed: Optional[int] = None, n: int = 1, T: int = 64) -> Sequence_:
    """AlexNet fc6 / fc7-shaped sparse-delta mat-vec."""
    ci, co = {k: (a, b) for k, a, b in FC_LAYERS}[layer]
    li = [k for k, _, _ in FC_LAYERS].index(layer)
    di = FC_DENSITIES.index(frac) if frac in FC_DENSITIES else 9
    seed = seed_for(3, 20 * li + 10 * (1 if dtype == BF16 else 0) + di) if seed is None else seed
    rng = rng_for(seed)
    shp = fc_shape(ci, co, n)
    if dtype == I8:
        wts = draw_i8_weight(rng, shp.w_shape)
        bias = draw_i32_bias(rng, co)
    else:
        wts = draw_bf16_weight(rng, shp.w_shape)
        bias = rng.normal(0.0, 0.1, size=(co,)).astype(np.float32)
    streams = [subset_redraw_frames(rng, ci, T, frac, dtype) for _ in range(n)]
    tag = "i8" if dtype == I8 else "bf16"
    return Sequence_(shp, dtype, wts, bias, _stack_streams(streams), f"cfg3_{layer}_{tag}_d{int(round(frac * 100))}")


# ---- config 4 -------------------------------------------------------------------------
XNOR_LAYERS = (("b28", 28, 256), ("b14", 14, 512))
XNOR_FLIPS = (0.01, 0.05, 0.10, 0.20)


def cluster_flip_frames(rng, h, w, c, T, frac, block=4) -> List[np.ndarray]:
    """T frames of +1/-1; each later frame flips, inside randomly placed block x block
    squares, every channel with probability 1/2; squares are added until the fraction of
    flipped elements reaches ``frac``."""
    frames = [draw_pm1(rng, (h, w, c))]
    total = h * w * c
    for _ in range(1, T):
        flip = np.zeros((h, w, c), dtype=bool)
        guard = 0
        while flip.sum() < frac * total and guard < 100000:
            y0 = int(rng.integers(0, h - block + 1))
            x0 = int(rng.integers(0, w - block + 1))
            flip[y0:y0 + block, x0:x0 + block] |= rng.integers(0, 2, size=(block, block, c)).astype(bool)
            guard += 1
        nxt = frames[-1].copy()
        nxt[flip] = -nxt[flip]
        frames.append(nxt)
    return frames


def config4(layer: str, frac: float, seed: Optional[int] = None, n: int = 1, T: int = 32) -> Sequence_:
    """XNOR-Net-style binary 3x3 conv (c_out = c_in); values are +1/-1 int8 here, use
    :func:`pack_pm1` for the bit-packed boundary format."""
    hw, c = {k: (a, b) for k, a, b in XNOR_LAYERS}[layer]
    li = [k for k, _, _ in XNOR_LAYERS].index(layer)
    di = XNOR_FLIPS.index(frac) if frac in XNOR_FLIPS else 9
    seed = seed_for(4, 10 * li + di) if seed is None else seed
    rng = rng_for(seed)
    shp = conv_shape(hw, hw, c, c, 3, 1, 1, 1, n)
    wts = draw_pm1(rng, shp.w_shape)
    bias = draw_i32_bias(rng, c)
    streams = [cluster_flip_frames(rng, hw, hw, c, T, frac) for _ in range(n)]
    return Sequence_(shp, BIN, wts, bias, _stack_streams(streams), f"cfg4_{layer}_f{int(round(frac * 100))}")


# ---- generic small random layers (parity / property tests) ---------------------------
def random_layer(seed: int, shape: LayerShape, dtype: int, T: int = 4, frac: float = 0.2,
                 block: int = 2, with_bias: bool = True) -> Sequence_:
    """A small random layer of any shape with block-redraw (conv) or subset-redraw (FC)
    frame structure, for property tests over odd sizes, strides, pads and groups."""
    rng = rng_for(seed)
    if dtype == I8:
        wts = draw_i8_weight(rng, shape.w_shape)
        bias = draw_i32_bias(rng, shape.c_out) if with_bias else None
        draw = draw_i8_act
    elif dtype == BF16:
        wts = draw_bf16_weight(rng, shape.w_shape)
        bias = rng.normal(0.0, 0.1, size=(shape.c_out,)).astype(np.float32) if with_bias else None
        draw = draw_bf16_relu
    else:
        wts = draw_pm1(rng, shape.w_shape)
        bias = draw_i32_bias(rng, shape.c_out) if with_bias else None
        draw = draw_pm1
    streams = []
    for _ in range(shape.n):
        if shape.kind == FC:
            if dtype == BIN:
                raise ValueError("binary FC is not a workload of this build")
            streams.append(subset_redraw_frames(rng, shape.c_in, T, frac, dtype))
        elif dtype == BIN:
            streams.append(cluster_flip_frames(rng, shape.h, shape.w, shape.c_in, T, frac, block=min(block, shape.h, shape.w)))
        else:
            streams.append(block_redraw_frames(rng, shape.h, shape.w, shape.c_in, T, min(block, shape.h, shape.w), frac, draw))
    return Sequence_(shape, dtype, wts, bias, _stack_streams(streams), "random")


def pruned(seq: Sequence_, keep: float, seed: int) -> Sequence_:
    """The same sequence with a pruned copy of the weights: a seeded random subset of `keep` of them survives,
    the rest are zero (a stand-in for a compressed model's weights, Sec. 4.3: the paper's own pruned models
    are not available)."""
    rng = rng_for(seed)
    mask = rng.random(seq.weights.shape) < keep
    w = np.where(mask, seq.weights, np.zeros_like(seq.weights))
    return Sequence_(seq.shape, seq.dtype, w, seq.bias, seq.frames, f"{seq.name}_w{int(round(keep * 100))}", dict(seq.meta))
