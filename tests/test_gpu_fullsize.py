"""GPU parity at the full sizes of the five BASELINE configurations, in the
launch configuration bench.py times.  Maps, index lists and the input state are
compared in full; outputs in full where the oracle finishes in seconds, and on
sampled pixels (which the oracle computes one by one from the state) for the
1080p configuration."""
import numpy as np
import pytest
import torch

import synth_inputs as syn

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_1808_05488_amd as cb
    from oracle import cb_oracle as orc
    from parity import Pair, assert_close, to_dev, to_host, prep
    from test_gpu_parity import _run_chain


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("backend", [1, 2])
def test_config2_full_size(backend):
    wl = syn.config2(n_frames=5)
    _say(f"config2 full size, 5 frames, backend {backend}")
    p = Pair(wl.layers[0], wl.H, wl.W, backend=backend)
    P = wl.H * wl.W
    for t, f in enumerate(wl.frames()):
        _, n = p.step(f, wl.tau, tag=f"c2 frame {t}")
        _say(f"  frame {t}: N = {n}")
        if t:
            assert 0.015 * P < n < 0.06 * P      # the "about 2-5 % changed" regime


@pytest.mark.parametrize("backend", [1, 2])
def test_config3_full_size(backend):
    wl = syn.config3(n_frames=4)
    _say(f"config3 full size, 4 frames, teacher-forced per layer, backend {backend}")
    _run_chain(wl, False, backend=backend)


@pytest.mark.parametrize("backend", [1, 2])
def test_config4_full_size(backend):
    wl = syn.config4(n_frames=3)
    _say(f"config4 full size, 3 frames, teacher-forced per layer, backend {backend}")
    _run_chain(wl, False, backend=backend)


def test_config3_full_size_chained_detection():
    wl = syn.config3(n_frames=4)
    _say("config3 full size, 4 frames, detection at the producer's listed pixels from layer 2 on")
    _run_chain(wl, False, chained=True)


def test_config4_full_size_chained_detection():
    wl = syn.config4(n_frames=3)
    _say("config4 full size, 3 frames, detection at the producer's listed pixels from layer 2 on")
    _run_chain(wl, False, chained=True)


@pytest.mark.parametrize("fraction,bf16,backend", [(0.05, False, 1), (0.05, False, 2), (0.01, True, 1), (0.02, True, 2)])
def test_config5_full_size_sampled(fraction, bf16, backend):
    wl = syn.config5(fraction)
    spec = wl.layers[0]
    _say(f"config5 1080p fraction {fraction} bf16={bf16}")
    A, B = [prep(f, bf16) for f in wl.frames()]
    w = prep(spec.weight, bf16)
    b = prep(spec.bias, bf16)
    g = cb.Layer(to_dev(w, bf16), to_dev(b, bf16), 1, 1, wl.H, wl.W, spec.relu, backend=backend)
    xa, xb = to_dev(A, bf16), to_dev(B, bf16)
    g.process_frame(xa, wl.tau)                     # full update, several column chunks
    m, mt, idx, n = g.changes_host()
    assert n == wl.H * wl.W and m.all() and mt.all() and np.array_equal(idx, np.arange(n, dtype=np.int32))
    rng = np.random.default_rng(7)
    samp = np.sort(rng.choice(wl.H * wl.W, 1500, replace=False)).astype(np.int32)
    out = to_host(g.process_frame(xa, wl.tau)).reshape(spec.c_out, -1)   # same frame again: N = 0
    assert g.stats()["n_changed_out"] == 0
    assert_close(out[:, samp], orc.conv_at(A, w, b, 1, 1, spec.relu, samp, bf16=bf16), bf16, "c5 full update")
    # the change frame
    out = to_host(g.process_frame(xb, wl.tau)).reshape(spec.c_out, -1)
    m, mt, idx, n = g.changes_host()
    S = A.copy()
    om, M = orc.detect(B, S, wl.tau)
    omt = orc.dilate(om, 3, 3, 1, 1)
    oidx = orc.extract(omt)
    _say(f"  M = {M} ({100.0 * M / om.size:.2f} %), N = {oidx.size}")
    assert abs(M / om.size - fraction) < 0.002
    assert np.array_equal(m, om) and np.array_equal(mt, omt) and np.array_equal(idx, oidx) and n == oidx.size
    assert g.stats()["n_changed_in"] == M
    assert np.array_equal(to_host(g.state()), S)
    listed = oidx[np.sort(rng.choice(oidx.size, 1500, replace=False))]
    for name, pix in (("listed", listed), ("any", samp)):
        assert_close(out[:, pix], orc.conv_at(S, w, b, 1, 1, spec.relu, pix, bf16=bf16), bf16, f"c5 {name} pixels")


# ---------------------------------------------------------------- maximum map size of the index extraction
def test_map_beyond_the_single_pass_scan():
    """A map of more than 262 144 bit words (here 4100 x 4100 pixels = 266 500 words) is beyond what the
    one-launch dilation + scan covers: the two-kernel form (dilate, then compact with a block prefix) takes
    over.  Few channels keep the oracle's share at a few seconds; everything is compared element by element."""
    C, O, H, W = 4, 4, 4100, 4100
    _say(f"map of {H * ((W + 63) // 64)} words")
    spec, frames = syn.random_layer_case(9, C, O, 3, 1, 1, H, W, 2, change_prob=0.001, relu=True, noise_std=0.004)
    p = Pair(spec, H, W, bf16=False, backend=2)
    _, n = p.step(frames[0], 0.02, tag="large map, full update")
    assert n == H * W
    _, n = p.step(frames[1], 0.02, tag="large map, sparse frame")
    assert 0 < n < H * W // 20
