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


@pytest.mark.parametrize("fraction,bf16", [(0.05, False), (0.01, True)])
def test_config5_full_size_explicit_back_end(fraction, bf16):
    """The explicit back end on the 1080p layer: the first frame runs in several column chunks."""
    _c5_point_from_scratch(fraction, bf16, backend=1)


def _c5_point_from_scratch(fraction, bf16, backend):
    wl = syn.config5(fraction)
    spec = wl.layers[0]
    _say(f"config5 1080p fraction {fraction} bf16={bf16} backend {backend}")
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


# ---------------------------------------------------------------- config 5: the whole density sweep, both element types
class _C5Sweep:
    """One 128->128 3x3 layer at 1080x1920 on the default back end (the launch configuration of
    `bench.py --workload c5`), kept across the densities of the sweep together with the oracle's own
    copy of the input state: every test plays frame A -> frame B(f) -> frame A on both sides."""

    def __init__(self, bf16):
        self.bf16 = bf16
        wl = syn.config5(syn.C5_FRACTIONS[0])
        self.wl, self.spec = wl, wl.layers[0]
        self.w = prep(self.spec.weight, bf16)
        self.b = prep(self.spec.bias, bf16)
        self.A = prep(syn.block_change_pair(5, self.spec.c_in, wl.H, wl.W, 0.0)[0], bf16)
        self.g = cb.Layer(to_dev(self.w, bf16), to_dev(self.b, bf16), 1, 1, wl.H, wl.W, self.spec.relu)
        self.xa = to_dev(self.A, bf16)
        self.S = self.A.copy()                       # the oracle's input state
        self.out = to_host(self.g.process_frame(self.xa, wl.tau)).reshape(self.spec.c_out, -1)
        m, mt, idx, n = self.g.changes_host()
        assert n == wl.H * wl.W and m.all() and mt.all() and np.array_equal(idx, np.arange(n, dtype=np.int32))
        assert np.array_equal(to_host(self.g.state()), self.S)

    def transition(self, x_host, x_dev, tag, n_sampled, all_listed):
        """One frame on both sides; maps, list, counts and state in full, outputs against the oracle's
        direct convolution of ITS state at listed pixels (all of them, or a sample) and at unlisted ones."""
        wl, spec, bf16 = self.wl, self.spec, self.bf16
        out = to_host(self.g.process_frame(x_dev, wl.tau)).reshape(spec.c_out, -1)
        m, mt, idx, n = self.g.changes_host()
        om, M = orc.detect(x_host, self.S, wl.tau)
        omt = orc.dilate(om, 3, 3, 1, 1)
        oidx = orc.extract(omt)
        _say(f"  {tag}: M = {M} ({100.0 * M / om.size:.3f} %), N = {oidx.size} ({100.0 * oidx.size / om.size:.3f} %)")
        assert n == oidx.size and self.g.stats()["n_changed_in"] == M
        assert np.array_equal(m, om), f"{tag}: change map differs"
        assert np.array_equal(mt, omt), f"{tag}: dilated map differs"
        assert np.array_equal(idx, oidx), f"{tag}: index list differs"
        assert np.array_equal(to_host(self.g.state()), self.S), f"{tag}: input state differs"
        rng = np.random.default_rng(11)
        listed = oidx if all_listed or oidx.size <= n_sampled else \
            oidx[np.sort(rng.choice(oidx.size, n_sampled, replace=False))]
        rest = np.flatnonzero(omt.reshape(-1) == 0).astype(np.int32)
        rest = rest[np.sort(rng.choice(rest.size, min(n_sampled, rest.size), replace=False))]
        for name, pix in (("listed", listed), ("unlisted", rest)):
            ref = orc.conv_at(self.S, self.w, self.b, 1, 1, spec.relu, pix, bf16=bf16)
            assert_close(out[:, pix], ref, bf16, f"{tag}: {pix.size} {name} pixels")
        keep = omt.reshape(-1) == 0
        assert np.array_equal(out[:, keep], self.out[:, keep]), f"{tag}: an unlisted output changed"
        self.out = out
        return M, oidx.size


@pytest.fixture(scope="module", params=[False, True], ids=["f32", "bf16"])
def c5_sweep(request):
    _say(f"config5 sweep layer, bf16={request.param}: full update of frame A")
    s = _C5Sweep(request.param)
    yield s
    del s
    torch.cuda.empty_cache()


@pytest.mark.parametrize("fraction", syn.C5_FRACTIONS)
def test_config5_density_sweep(c5_sweep, fraction):
    """Config 5 as stated: every density of the sweep, float32 and bfloat16.  Maps, index list, N, M and the
    input state are compared in full; the outputs of ALL listed pixels up to 5 % changed, of 20 000 sampled
    listed and 20 000 sampled unlisted pixels above that (the oracle computes each from its own state)."""
    s = c5_sweep
    wl = s.wl
    _say(f"config5 1080p, {100 * fraction:g} % changed, bf16={s.bf16}")
    B = prep(syn.block_change_pair(5, s.spec.c_in, wl.H, wl.W, fraction)[1], s.bf16)
    xb = to_dev(B, s.bf16)
    M, N = s.transition(B, xb, f"A -> B({100 * fraction:g} %)", 20000, all_listed=fraction <= 0.05)
    P = wl.H * wl.W
    assert abs(M / P - fraction) < 0.002 and M <= N <= 1.27 * M
    del xb
    M2, N2 = s.transition(s.A, s.xa, f"B({100 * fraction:g} %) -> A", 5000, all_listed=False)
    assert (M2, N2) == (M, N)
    assert np.array_equal(s.S, s.A)


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
