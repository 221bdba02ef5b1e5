"""GPU parity on randomly drawn layer geometries: the fused back end (float32 and
bfloat16) and the explicit one against the CPU oracle, three frames per case.  The draws are
seeded; they cover all four row-tile shapes of the fused kernels (up to 16 / 32 / 64 / more
output channels), 1x1 ... 7x7 filters, stride 1 and 2, padding 0 and half the filter, maps
from a few dozen pixels (every listed pixel at the border) to more than 8 192 pixels (the
32-column tile of the float32 kernel on the full-update frame), and sparse to dense change.
A second set of draws has power-of-two channel counts only: those layers keep a channel-last
shadow of their state, which change detection updates and the fused kernel gathers from."""
import numpy as np
import pytest
import torch

import synth_inputs as syn

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from parity import Pair


def _draw(rng):
    k = int(rng.choice([1, 3, 3, 3, 5, 7]))
    s = int(rng.choice([1, 1, 1, 2]))
    pad = int(rng.choice([0, k // 2, k // 2]))
    C = int(rng.integers(1, 48))
    O = int(rng.choice([int(rng.integers(1, 17)), int(rng.integers(17, 33)), int(rng.integers(33, 65)),
                        int(rng.integers(65, 150))]))
    H, W = int(rng.integers(max(k, 6), 100)), int(rng.integers(max(k, 6), 140))
    if rng.random() < 0.25:
        H, W = int(rng.integers(80, 130)), int(rng.integers(100, 160))
    bf16 = bool(rng.random() < 0.35)
    prob = float(rng.choice([0.002, 0.02, 0.2]))
    relu = bool(rng.random() < 0.7)
    return C, O, k, s, pad, H, W, bf16, prob, relu


@pytest.mark.parametrize("seed,backend", [(11, 2), (12, 2), (13, 2), (14, 1)])
def test_random_geometries(seed, backend):
    rng = np.random.default_rng(seed)
    for i in range(40):
        C, O, k, s, pad, H, W, bf16, prob, relu = _draw(rng)
        tag = f"seed {seed} case {i}: C={C} O={O} k={k} s={s} pad={pad} H={H} W={W} bf16={bf16} p={prob} backend={backend}"
        print(tag, flush=True)
        spec, frames = syn.random_layer_case(100 * seed + i, C, O, k, s, pad, H, W, 3, change_prob=prob, relu=relu,
                                             noise_std=0.004)
        p = Pair(spec, H, W, bf16=bf16, backend=backend)
        for t, f in enumerate(frames):
            p.step(f, 0.02, tag=f"{tag} frame {t}")


def _draw_shadow(rng):
    k = int(rng.choice([1, 2, 3, 3, 3, 4, 5, 7]))
    s = int(rng.choice([1, 1, 1, 2, 3]))
    pad = int(rng.choice([0, k // 2, k // 2, min(k, 3)]))
    C = int(rng.choice([16, 16, 32, 32, 64, 64, 128, 256, 512]))
    O = int(rng.choice([int(rng.integers(1, 17)), int(rng.integers(17, 33)), int(rng.integers(33, 65)),
                        int(rng.integers(65, 150))]))
    if C * k * k > 3200:
        O = min(O, 40)                                   # keeps the oracle quick
    H, W = int(rng.integers(max(k, 6), 90)), int(rng.integers(max(k, 6), 120))
    if rng.random() < 0.25 and C <= 64 and k <= 3:
        H, W = int(rng.integers(100, 150)), int(rng.integers(130, 180))     # more than 16 384 pixels: the wide tiles
    if C >= 256:
        H, W = min(H, 40), min(W, 50)
    if C * k * k > 12000:
        k = 3                                            # (beyond the fused back end's longest K)
        pad = min(pad, 1)
    bf16 = bool(rng.random() < 0.5)
    prob = float(rng.choice([0.002, 0.02, 0.2]))
    relu = bool(rng.random() < 0.7)
    return C, O, k, s, pad, H, W, bf16, prob, relu


@pytest.mark.parametrize("seed", [21, 22])
def test_random_geometries_with_a_channel_last_shadow(seed):
    rng = np.random.default_rng(seed)
    for i in range(40):
        C, O, k, s, pad, H, W, bf16, prob, relu = _draw_shadow(rng)
        tag = f"seed {seed} case {i}: C={C} O={O} k={k} s={s} pad={pad} H={H} W={W} bf16={bf16} p={prob}"
        print(tag, flush=True)
        spec, frames = syn.random_layer_case(100 * seed + i, C, O, k, s, pad, H, W, 4, change_prob=prob, relu=relu,
                                             noise_std=0.004)
        p = Pair(spec, H, W, bf16=bf16, backend=2)
        for t, f in enumerate(frames):
            p.step(f if t != 2 else f + np.float32(0.5), 0.02, tag=f"{tag} frame {t}")
