"""Seeded synthetic video sequences and layer parameters.

This module only draws random numbers and pastes rectangles; it holds none of
the change-based-convolution arithmetic.  It is the one module that both the CPU
oracle's tests and the HIP path's tests/bench import, so that both sides see
bit-identical host arrays.

The sequences stand in for the static-camera recordings the paper evaluates on
(Sec. IV-A: urban surveillance scene labelling, CAVIAR pose detection, traffic
cameras): a fixed background, a few small moving objects touching a few percent
of the pixels per frame, and single-pixel sensor noise well below the change
threshold.  Layer shapes follow Table I (scene-labelling net) and the VGG-style
trunk of the pose network (Sec. IV-A).

All "N(0, s)" below use s as the standard deviation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Iterator, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 180805488


def rng_for(config_index: int, stream: int = 0) -> np.random.Generator:
    """Independent generator per (config, stream) so that e.g. weights do not
    shift when the number of frames changes."""
    return np.random.default_rng([BASE_SEED + config_index, stream])


# --------------------------------------------------------------------------
# layer descriptions
# --------------------------------------------------------------------------
@dataclass
class ConvSpec:
    c_in: int
    c_out: int
    k: int
    stride: int = 1
    pad: int = 0
    relu: bool = False
    pool: bool = False          # 2x2/2 ceil-mode max-pool after this conv
    weight: Optional[np.ndarray] = None   # (c_out, c_in, k, k) float32
    bias: Optional[np.ndarray] = None     # (c_out,) float32


def he_normal(rng: np.random.Generator, c_out: int, c_in: int, k: int) -> np.ndarray:
    std = math.sqrt(2.0 / (c_in * k * k))
    return (rng.standard_normal((c_out, c_in, k, k)) * std).astype(np.float32)


def to_bf16_f32(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them as float32.  Pure bit manipulation; used only to prepare inputs."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 values that are exactly bf16-representable -> uint16 patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


# --------------------------------------------------------------------------
# moving-object sequences
# --------------------------------------------------------------------------
@dataclass
class _Obj:
    y: float
    x: float
    vy: float
    vx: float
    h: int
    w: int
    tex: np.ndarray            # (C, h, w)
    t_on: int = 0
    t_off: int = 1 << 30


def _step(o: _Obj, H: int, W: int) -> None:
    o.y += o.vy
    o.x += o.vx
    if o.y < 0:
        o.y = -o.y
        o.vy = -o.vy
    if o.x < 0:
        o.x = -o.x
        o.vx = -o.vx
    if o.y + o.h > H:
        o.y = 2 * (H - o.h) - o.y
        o.vy = -o.vy
    if o.x + o.w > W:
        o.x = 2 * (W - o.w) - o.x
        o.vx = -o.vx


def _render(bg: np.ndarray, objs: Sequence[_Obj], t: int, noise_std: float,
            rng: np.random.Generator) -> np.ndarray:
    f = bg.copy()
    for o in objs:
        if o.t_on <= t < o.t_off:
            y, x = int(round(o.y)), int(round(o.x))
            f[:, y:y + o.h, x:x + o.w] = o.tex
    if noise_std > 0:
        f += (rng.standard_normal(f.shape, dtype=np.float32) * np.float32(noise_std))
    return f


def moving_rect_sequence(config_index: int, C: int, H: int, W: int, n_frames: int,
                         n_rect: int = 4, rect: int = 40, speed: float = 3.0,
                         noise_std: float = 0.003) -> Iterator[np.ndarray]:
    """Static U[0,1) background, `n_rect` textured squares with axis-aligned
    velocity `speed` px/frame bouncing at the borders, fresh N(0, noise_std)
    noise on every frame."""
    rng = rng_for(config_index, 1)
    bg = rng.random((C, H, W), dtype=np.float32)
    rect = min(rect, H // 2, W // 2)
    objs: List[_Obj] = []
    dirs = [(0.0, speed), (speed, 0.0), (0.0, -speed), (-speed, 0.0)]
    for r in range(n_rect):
        vy, vx = dirs[r % 4]
        objs.append(_Obj(y=float(rng.integers(0, H - rect + 1)),
                         x=float(rng.integers(0, W - rect + 1)),
                         vy=vy, vx=vx, h=rect, w=rect,
                         tex=rng.random((C, rect, rect), dtype=np.float32)))
    nrng = rng_for(config_index, 2)
    for t in range(n_frames):
        yield _render(bg, objs, t, noise_std, nrng)
        for o in objs:
            _step(o, H, W)


def varying_objects_sequence(config_index: int, C: int, H: int, W: int, n_frames: int,
                             max_obj: int = 6, noise_std: float = 0.003) -> Iterator[np.ndarray]:
    """Static background with 1..max_obj moving textured rectangles; objects
    appear and disappear over the sequence (at least one is always present)."""
    rng = rng_for(config_index, 1)
    bg = rng.random((C, H, W), dtype=np.float32)
    objs: List[_Obj] = []
    for r in range(max_obj):
        h = int(rng.integers(max(4, H // 24), max(6, H // 8)))
        w = int(rng.integers(max(4, W // 32), max(6, W // 10)))
        ang = rng.uniform(0, 2 * math.pi)
        sp = rng.uniform(1.0, 4.0)
        t_on = 0 if r == 0 else int(rng.integers(0, max(1, n_frames // 2)))
        t_off = (1 << 30) if r == 0 else t_on + int(rng.integers(max(2, n_frames // 4), n_frames + 1))
        objs.append(_Obj(y=float(rng.integers(0, H - h + 1)), x=float(rng.integers(0, W - w + 1)),
                         vy=sp * math.sin(ang), vx=sp * math.cos(ang), h=h, w=w,
                         tex=rng.random((C, h, w), dtype=np.float32), t_on=t_on, t_off=t_off))
    nrng = rng_for(config_index, 2)
    for t in range(n_frames):
        yield _render(bg, objs, t, noise_std, nrng)
        for o in objs:
            _step(o, H, W)


def articulated_figure_sequence(config_index: int, C: int, H: int, W: int, n_frames: int,
                                n_blobs: int = 8, noise_std: float = 0.003) -> Iterator[np.ndarray]:
    """Static textured background and one figure made of `n_blobs` rectangles
    that share a common drift and swing around it with individual phases."""
    rng = rng_for(config_index, 1)
    bg = rng.random((C, H, W), dtype=np.float32)
    bh, bw = max(4, H // 9), max(4, W // 16)
    cy, cx = H * 0.5, W * 0.3
    offs = rng.uniform(-1.0, 1.0, size=(n_blobs, 2)) * np.array([H * 0.22, W * 0.08])
    phase = rng.uniform(0, 2 * math.pi, size=n_blobs)
    amp = rng.uniform(3.0, 9.0, size=n_blobs)
    texs = [rng.random((C, bh, bw), dtype=np.float32) for _ in range(n_blobs)]
    nrng = rng_for(config_index, 2)
    for t in range(n_frames):
        f = bg.copy()
        fx = cx + 2.5 * t
        span = W - bw - 1
        fx = fx % (2 * span)
        if fx > span:
            fx = 2 * span - fx
        for b in range(n_blobs):
            y = cy + offs[b, 0] + amp[b] * math.sin(0.45 * t + phase[b])
            x = fx + offs[b, 1] + amp[b] * math.cos(0.45 * t + phase[b])
            yi = int(min(max(round(y), 0), H - bh))
            xi = int(min(max(round(x), 0), W - bw))
            f[:, yi:yi + bh, xi:xi + bw] = texs[b]
        if noise_std > 0:
            f += nrng.standard_normal(f.shape, dtype=np.float32) * np.float32(noise_std)
        yield f


def block_change_pair(config_index: int, C: int, H: int, W: int, fraction: float,
                      block: int = 16) -> Tuple[np.ndarray, np.ndarray, int]:
    """Frame A ~ U[0,1); frame B = A with round(fraction*P/block^2) distinct
    aligned block x block cells replaced by fresh U[0,1) in every channel.
    Returns (A, B, n_blocks)."""
    rng = rng_for(config_index, 1)
    A = rng.random((C, H, W), dtype=np.float32)
    gh, gw = H // block, W // block
    n_blocks = int(round(fraction * H * W / (block * block)))
    n_blocks = min(n_blocks, gh * gw)
    crng = rng_for(config_index, 3 + int(round(fraction * 1e6)))
    cells = crng.choice(gh * gw, size=n_blocks, replace=False)
    B = A.copy()
    for cell in np.sort(cells):
        y, x = (int(cell) // gw) * block, (int(cell) % gw) * block
        B[:, y:y + block, x:x + block] = crng.random((C, block, block), dtype=np.float32)
    return A, B, n_blocks


# --------------------------------------------------------------------------
# the five configurations (full size by default; `scale` arguments give the
# same recipe at sizes the CPU oracle finishes in seconds)
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    layers: List[ConvSpec]
    H: int
    W: int
    tau: float
    n_frames: int
    frames: object = field(repr=False, default=None)   # callable -> iterator of (C,H,W) float32


def config1() -> Workload:
    """3->16, 3x3, pad 1, 48x64, two frames; second frame = first + N(0,0.002)
    plus one 8x8 block of fresh U[0,1).  tau = 0.01, weights N(0,0.1), bias 0."""
    ci = 1
    C, O, H, W = 3, 16, 48, 64
    wr = rng_for(ci, 0)
    w = (wr.standard_normal((O, C, 3, 3)) * 0.1).astype(np.float32)
    b = np.zeros(O, np.float32)

    def frames():
        rng = rng_for(ci, 1)
        x0 = rng.random((C, H, W), dtype=np.float32)
        x1 = x0 + rng.standard_normal((C, H, W), dtype=np.float32) * np.float32(0.002)
        y = int(rng.integers(2, H - 10))
        x = int(rng.integers(2, W - 10))
        x1[:, y:y + 8, x:x + 8] = rng.random((C, 8, 8), dtype=np.float32)
        yield x0
        yield x1.astype(np.float32)

    return Workload("c1_3to16_3x3_48x64", [ConvSpec(C, O, 3, 1, 1, False, False, w, b)],
                    H, W, 0.01, 2, frames)


def config2(H: int = 480, W: int = 640, C: int = 64, O: int = 64, n_frames: int = 30,
            rect: int = 40) -> Workload:
    """64->64, 3x3, pad 1, 480x640, 30 frames, 4 moving 40x40 rectangles at
    3 px/frame, N(0,0.003) noise, tau = 0.02.  He-normal weights, zero bias,
    fused ReLU off (single layer)."""
    ci = 2
    wr = rng_for(ci, 0)
    w = he_normal(wr, O, C, 3)
    b = np.zeros(O, np.float32)
    return Workload(f"c2_{C}to{O}_3x3_{H}x{W}", [ConvSpec(C, O, 3, 1, 1, False, False, w, b)],
                    H, W, 0.02, n_frames,
                    lambda: moving_rect_sequence(ci, C, H, W, n_frames, 4, rect, 3.0, 0.003))


def config3(H: int = 480, W: int = 640, n_frames: int = 100,
            widths: Sequence[int] = (16, 64, 256, 64, 8)) -> Workload:
    """Scene-labelling-style net of Table I at 3xHxW: 7x7 3->16 +ReLU+pool,
    7x7 16->64 +ReLU+pool, 7x7 64->256 +ReLU, 1x1 256->64 +ReLU, 1x1 64->8."""
    ci = 3
    wr = rng_for(ci, 0)
    chans = [3] + list(widths)
    ks = [7, 7, 7, 1, 1]
    relu = [True, True, True, True, False]
    pool = [True, True, False, False, False]
    layers = []
    for l in range(5):
        layers.append(ConvSpec(chans[l], chans[l + 1], ks[l], 1, (ks[l] - 1) // 2, relu[l], pool[l],
                               he_normal(wr, chans[l + 1], chans[l], ks[l]),
                               np.zeros(chans[l + 1], np.float32)))
    return Workload(f"c3_seg5_{H}x{W}", layers, H, W, 0.02, n_frames,
                    lambda: varying_objects_sequence(ci, 3, H, W, n_frames, 6, 0.003))


def config4(H: int = 368, W: int = 656, n_frames: int = 60, width_div: int = 1) -> Workload:
    """VGG-style trunk of the pose network at 3xHxW: 3x3 convs 64,64,P,128,128,P,
    256x4,P,512,512, each + ReLU."""
    ci = 4
    wr = rng_for(ci, 0)
    plan = [64, 64, "P", 128, 128, "P", 256, 256, 256, 256, "P", 512, 512]
    layers: List[ConvSpec] = []
    c = 3
    for item in plan:
        if item == "P":
            layers[-1].pool = True
            continue
        o = max(4, int(item) // width_div)
        layers.append(ConvSpec(c, o, 3, 1, 1, True, False, he_normal(wr, o, c, 3),
                               np.zeros(o, np.float32)))
        c = o
    return Workload(f"c4_vgg10_{H}x{W}", layers, H, W, 0.02, n_frames,
                    lambda: articulated_figure_sequence(ci, 3, H, W, n_frames, 8, 0.003))


C5_FRACTIONS = (0.001, 0.005, 0.01, 0.02, 0.05, 0.10, 0.20, 0.50)


def config5(fraction: float, H: int = 1080, W: int = 1920, C: int = 128, O: int = 128) -> Workload:
    """128->128 3x3 pad 1 at 1080x1920; frame B differs from frame A in random
    aligned 16x16 blocks covering `fraction` of the pixels.  tau = 0.02."""
    ci = 5
    wr = rng_for(ci, 0)
    w = he_normal(wr, O, C, 3)
    b = np.zeros(O, np.float32)

    def frames():
        A, B, _ = block_change_pair(ci, C, H, W, fraction)
        yield A
        yield B

    return Workload(f"c5_{C}to{O}_3x3_{H}x{W}_f{fraction:g}",
                    [ConvSpec(C, O, 3, 1, 1, False, False, w, b)], H, W, 0.02, 2, frames)


def random_layer_case(seed: int, C: int, O: int, k: int, stride: int, pad: int, H: int, W: int,
                      n_frames: int, change_prob: float = 0.05, relu: bool = True,
                      noise_std: float = 0.0) -> Tuple[ConvSpec, List[np.ndarray]]:
    """Small random layer + frames with i.i.d. per-pixel changes (all channels
    of a chosen pixel get fresh values); used for geometry sweeps."""
    rng = np.random.default_rng([BASE_SEED, 77, seed])
    w = he_normal(rng, O, C, k)
    b = (rng.standard_normal(O) * 0.1).astype(np.float32)
    x = rng.random((C, H, W), dtype=np.float32)
    frames = [x.copy()]
    for _ in range(1, n_frames):
        sel = rng.random((H, W)) < change_prob
        x = x.copy()
        fresh = rng.random((C, H, W), dtype=np.float32)
        x[:, sel] = fresh[:, sel]
        if noise_std > 0:
            x = x + rng.standard_normal((C, H, W), dtype=np.float32) * np.float32(noise_std)
        frames.append(x.astype(np.float32))
    return ConvSpec(C, O, k, stride, pad, relu, False, w, b), frames
