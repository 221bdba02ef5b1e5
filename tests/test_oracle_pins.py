"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each one checks the oracle against
something other than itself: counts the paper prints, a library convolution /
pooling routine as the textbook special case, the scatter form of the dilation
(the paper's own implementation of Eq. 4) against the oracle's gather form,
exact rational rounding, and the invariants of the closed-loop formulation.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from conftest import golden
from oracle import cb_oracle as orc
import synth_inputs as syn


def lib_conv(x, w, b, s, p, relu):
    """Library dense cross-correlation in float64 (the non-change-based layer)."""
    y = F.conv2d(torch.from_numpy(x.astype(np.float64))[None], torch.from_numpy(w.astype(np.float64)),
                 None if b is None else torch.from_numpy(b.astype(np.float64)), stride=s, padding=p)[0]
    if relu:
        y = torch.relu(y)
    return y.numpy()


def close(a, ref, tol=2e-6):
    scale = max(float(np.sqrt(np.mean(ref.astype(np.float64) ** 2))), 1e-30)
    return np.all(np.abs(a.astype(np.float64) - ref) <= tol * np.maximum(np.abs(ref), scale))


GEOMS = [  # C, O, kh, kw, s, p, H, W
    (3, 4, 3, 3, 1, 1, 9, 11),
    (2, 3, 1, 1, 1, 0, 7, 5),
    (2, 5, 7, 7, 1, 3, 12, 13),
    (3, 2, 5, 5, 2, 2, 11, 14),
    (1, 3, 3, 5, 1, 0, 8, 9),      # kh != kw, no padding
    (4, 2, 3, 3, 2, 0, 10, 9),
    (2, 2, 5, 3, 1, 4, 6, 7),      # padding larger than the half kernel
    (3, 3, 7, 7, 3, 1, 15, 16),
]


# ---------------------------------------------------------------- printed counts
def _single_pixel_layer(k, C=2, O=3, H=31, W=33):
    rng = np.random.default_rng(5)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    L = orc.OracleLayer(w, None, 1, (k - 1) // 2, H, W, relu=False)
    x0 = rng.random((C, H, W), dtype=np.float32)
    x1 = x0.copy()
    x1[1, 15, 16] += 0.5
    L.process(x0, 0.1)
    L.process(x1, 0.1)
    return L, x0, x1


def test_printed_footprint_counts():
    L7, _, _ = _single_pixel_layer(7)
    assert L7.n_in == 1 and L7.count == golden("footprint_7x7")[0]
    L3, _, _ = _single_pixel_layer(3)
    assert L3.count == golden("footprint_3x3")[0]
    # the footprint is the symmetric support {-3..3}^2 around the changed pixel
    lo, hi = golden("support_7x7")
    ys, xs = np.nonzero(L7.mt)
    assert ys.min() == 15 + lo and ys.max() == 15 + hi and xs.min() == 16 + lo and xs.max() == 16 + hi


def test_printed_two_layer_growth():
    """One changed pixel -> 49 outputs after a 7x7 layer -> 169 after a second
    one (threshold zero at the second layer, so every changed value triggers)."""
    L1, x0, x1 = _single_pixel_layer(7, C=2, O=3)
    rng = np.random.default_rng(6)
    w2 = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    L2 = orc.OracleLayer(w2, None, 1, 3, 31, 33, relu=False)
    L1b = orc.OracleLayer(L1._w, None, 1, 3, 31, 33, relu=False)
    L1b.process(x0, 0.1)
    L2.process(L1b.out, 0.0)
    L1b.process(x1, 0.1)
    L2.process(L1b.out, 0.0)
    assert L1b.count == golden("footprint_7x7")[0]
    assert L2.n_in == golden("footprint_7x7")[0]
    assert L2.count == golden("footprint_7x7_then_7x7")[0]


def test_1x1_change_map_is_input_map():
    """Sec. III-E item 2: with a 1x1 filter changes do not propagate."""
    spec, frames = syn.random_layer_case(3, 3, 4, 1, 1, 0, 10, 12, 4, change_prob=0.1)
    L = orc.OracleLayer(spec.weight, spec.bias, 1, 0, 10, 12, relu=True)
    for f in frames:
        L.process(f, 0.02)
        assert np.array_equal(L.m, L.mt)
        assert np.array_equal(L.idx, np.flatnonzero(L.m).astype(np.int32))


# ---------------------------------------------------------------- Eq. 3
def test_detect_strict_threshold_abs_and_whole_pixel_copy():
    C, H, W = 3, 2, 4
    S = np.zeros((C, H, W), np.float32)
    x = np.zeros((C, H, W), np.float32)
    tau = np.float32(0.25)
    x[0, 0, 0] = 0.25            # equal to tau: strict '>' does not trigger
    x[1, 0, 1] = 0.2500001       # just above: triggers
    x[2, 0, 2] = -0.3            # negative difference: absolute value
    x[0, 0, 2] = 0.1             # sub-threshold channel of a triggered pixel
    x[2, 1, 3] = 0.2             # below
    x[0, 1, 0] = np.nan          # NaN difference compares false
    S0 = S.copy()
    m, M = orc.detect(x, S, float(tau))
    exp = np.zeros((H, W), np.uint8)
    exp[0, 1] = 1
    exp[0, 2] = 1
    assert np.array_equal(m, exp) and M == 2
    # all channels of a triggered pixel are copied, the others keep the state
    assert S[0, 0, 2] == np.float32(0.1) and S[2, 0, 2] == np.float32(-0.3)
    assert S[1, 0, 1] == np.float32(0.2500001)
    untouched = exp == 0
    assert np.array_equal(S[:, untouched], S0[:, untouched])


def test_detect_any_channel_brute_force():
    rng = np.random.default_rng(11)
    for C in (1, 2, 5):
        H, W = 6, 7
        S = rng.random((C, H, W), dtype=np.float32)
        x = (S + rng.standard_normal((C, H, W)).astype(np.float32) * np.float32(0.02)).astype(np.float32)
        tau = 0.03
        S_in = S.copy()
        m, M = orc.detect(x, S, tau)
        for y in range(H):
            for xx in range(W):
                ch = False
                for c in range(C):
                    d = np.float32(x[c, y, xx]) - np.float32(S_in[c, y, xx])   # float32 subtract
                    ch = ch or (abs(d) > np.float32(tau))
                assert m[y, xx] == int(ch)
                if ch:
                    assert np.array_equal(S[:, y, xx], x[:, y, xx])
                else:
                    assert np.array_equal(S[:, y, xx], S_in[:, y, xx])
        assert M == int(m.sum())


# ---------------------------------------------------------------- Eq. 4
def scatter_dilate(m, kh, kw, s, p):
    """The paper's implementation of Eq. 4 (Sec. III-A): clear the map, then
    every changed input pixel sets the output pixels whose filter support
    covers it."""
    H, W = m.shape
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    mt = np.zeros((Ho, Wo), np.uint8)
    for yi, xi in zip(*np.nonzero(m)):
        for j in range(kh):
            for i in range(kw):
                ny, nx = yi + p - j, xi + p - i
                if ny % s or nx % s:
                    continue
                yo, xo = ny // s, nx // s
                if 0 <= yo < Ho and 0 <= xo < Wo:
                    mt[yo, xo] = 1
    return mt


@pytest.mark.parametrize("geom", GEOMS)
def test_dilate_matches_scatter_form(geom):
    _, _, kh, kw, s, p, H, W = geom
    rng = np.random.default_rng(hash(geom) % 1000)
    for dens in (0.0, 0.03, 0.3, 1.0):
        m = (rng.random((H, W)) < dens).astype(np.uint8)
        assert np.array_equal(orc.dilate(m, kh, kw, s, p), scatter_dilate(m, kh, kw, s, p))
    for corner in ((0, 0), (0, W - 1), (H - 1, 0), (H - 1, W - 1)):
        m = np.zeros((H, W), np.uint8)
        m[corner] = 1
        assert np.array_equal(orc.dilate(m, kh, kw, s, p), scatter_dilate(m, kh, kw, s, p))


def test_extract_is_ordered_selection():
    rng = np.random.default_rng(2)
    for dens in (0.0, 0.1, 1.0):
        mt = (rng.random((9, 13)) < dens).astype(np.uint8)
        idx = orc.extract(mt)
        assert idx.dtype == np.int32
        assert np.array_equal(idx, np.flatnonzero(mt))


# ---------------------------------------------------------------- Eq. 1/2 and the invariants
@pytest.mark.parametrize("geom", GEOMS)
def test_dense_conv_is_library_cross_correlation(geom):
    C, O, kh, kw, s, p, H, W = geom
    rng = np.random.default_rng(1)
    x = rng.standard_normal((C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, kh, kw)).astype(np.float32)
    b = rng.standard_normal(O).astype(np.float32)
    for relu in (False, True):
        got = orc.dense_conv(x, w, b, s, p, relu)
        assert got.shape == lib_conv(x, w, b, s, p, relu).shape
        assert close(got, lib_conv(x, w, b, s, p, relu), 1e-6)
    assert close(orc.dense_conv(x, w, None, s, p, False), lib_conv(x, w, None, s, p, False), 1e-6)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("feed_forward", [False, True])
def test_threshold_zero_equals_dense_layer(geom, feed_forward):
    """Sec. III-F: a threshold of zero yields the non-change-based result."""
    C, O, kh, kw, s, p, H, W = geom
    spec, frames = syn.random_layer_case(17, C, O, kh, s, p, H, W, 5, change_prob=0.1, noise_std=1e-4)
    rng = np.random.default_rng(3)
    w = rng.standard_normal((O, C, kh, kw)).astype(np.float32)
    L = orc.OracleLayer(w, spec.bias, s, p, H, W, relu=True, feed_forward=feed_forward)
    frames = frames + [frames[-1]]          # an unchanged frame too
    for f in frames:
        L.process(f, 0.0)
        assert close(L.out, lib_conv(f, w, spec.bias, s, p, True), 1e-6)
    assert L.count == 0 and L.n_in == 0     # identical frame: nothing listed


@pytest.mark.parametrize("geom", GEOMS)
def test_closed_loop_invariants(geom):
    """Sec. III-C: the cached output is always the convolution of the input
    state; the state stays within tau of the input; unlisted outputs keep
    their previous bits."""
    C, O, kh, kw, s, p, H, W = geom
    tau = 0.05
    spec, frames = syn.random_layer_case(23, C, O, kh, s, p, H, W, 6, change_prob=0.04, noise_std=0.012)
    rng = np.random.default_rng(4)
    w = rng.standard_normal((O, C, kh, kw)).astype(np.float32)
    L = orc.OracleLayer(w, spec.bias, s, p, H, W, relu=True)
    prev_out, partial = None, False
    for t, f in enumerate(frames):
        N = L.process(f, tau)
        S, out, m, mt, idx = L.state, L.out, L.m, L.mt, L.idx
        assert close(out, lib_conv(S, w, spec.bias, s, p, True), 1e-6)
        assert np.max(np.abs(f - S)) <= np.float32(tau)
        assert np.array_equal(S[:, m == 1], f[:, m == 1])
        assert N == idx.size == int(mt.sum()) and np.all(np.diff(idx) > 0)
        assert np.array_equal(idx, np.flatnonzero(mt))
        if t == 0:
            assert N == L.Ho * L.Wo and np.all(m == 1)
        else:
            keep = mt.reshape(-1) == 0
            assert np.array_equal(out.reshape(O, -1)[:, keep], prev_out.reshape(O, -1)[:, keep])
            partial = partial or 0 < N < L.Ho * L.Wo
        prev_out = out
    assert partial or kh == 7      # the sweep exercises partial updates


def test_all_pixels_changed_equals_dense_and_reset():
    C, O, k, H, W = 2, 3, 3, 8, 9
    rng = np.random.default_rng(8)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    L = orc.OracleLayer(w, None, 1, 1, H, W, relu=False)
    x0 = rng.random((C, H, W), dtype=np.float32)
    L.process(x0, 0.1)
    x1 = x0 + np.float32(0.5)
    assert L.process(x1, 0.1) == H * W
    assert np.array_equal(L.idx, np.arange(H * W))
    assert close(L.out, lib_conv(x1, w, None, 1, 1, False), 1e-6)
    # after a reset the next frame is a full update again, whatever tau is
    L.reset()
    assert L.process(x1, 10.0) == H * W


def test_conv_at_matches_dense_at_listed_pixels():
    C, O, kh, kw, s, p, H, W = 3, 4, 3, 5, 2, 2, 11, 12
    rng = np.random.default_rng(9)
    x = rng.standard_normal((C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, kh, kw)).astype(np.float32)
    b = rng.standard_normal(O).astype(np.float32)
    ref = lib_conv(x, w, b, s, p, True)
    Po = ref.shape[1] * ref.shape[2]
    idx = np.sort(rng.choice(Po, 17, replace=False)).astype(np.int32)
    vals = orc.conv_at(x, w, b, s, p, True, idx)
    assert close(vals, ref.reshape(O, -1)[:, idx], 1e-6)


def test_feed_forward_goes_stale_closed_loop_does_not():
    """Sec. III-C: increments below the threshold never trigger an update in
    the feed-forward form; the closed-loop state follows within tau."""
    C, O, H, W = 1, 1, 5, 5
    w = np.ones((O, C, 1, 1), np.float32)
    ff = orc.OracleLayer(w, None, 1, 0, H, W, relu=False, feed_forward=True)
    cl = orc.OracleLayer(w, None, 1, 0, H, W, relu=False)
    x = np.zeros((C, H, W), np.float32)
    tau = 0.1
    for t in range(12):
        x = x + np.float32(0.04)
        nf = ff.process(x, tau)
        cl.process(x, tau)
        if t > 0:
            assert nf == 0
        assert np.max(np.abs(cl.out - x)) <= np.float32(tau) + 1e-6
    assert np.max(np.abs(ff.out - x)) > 0.4        # stale: still the first frame's result
    assert np.allclose(ff.out, 0.04)


def test_propagated_change_set():
    """Sec. III-E: case 1 propagates the producer's map through Eq. 4; case 2
    (1x1) re-uses the producer's map and index list unchanged."""
    spec, frames = syn.random_layer_case(31, 2, 3, 3, 1, 1, 9, 10, 4, change_prob=0.05)
    prod = orc.OracleLayer(spec.weight, spec.bias, 1, 1, 9, 10, relu=True)
    rng = np.random.default_rng(10)
    w3 = rng.standard_normal((2, 3, 3, 3)).astype(np.float32)
    w1 = rng.standard_normal((4, 3, 1, 1)).astype(np.float32)
    c3 = orc.OracleLayer(w3, None, 1, 1, 9, 10, relu=False)
    c1 = orc.OracleLayer(w1, None, 1, 0, 9, 10, relu=False)
    for t, f in enumerate(frames):
        prod.process(f, 0.02)
        c3.process_propagated(prod.out, prod.mt)
        c1.process_propagated(prod.out, prod.mt)
        assert np.array_equal(c1.idx, prod.idx) and np.array_equal(c1.mt, prod.mt)
        assert np.array_equal(c3.mt, scatter_dilate(prod.mt, 3, 3, 1, 1))
        # no detection threshold is involved, so both track the dense result exactly
        assert close(c3.out, lib_conv(prod.out, w3, None, 1, 1, False), 1e-6)
        assert close(c1.out, lib_conv(prod.out, w1, None, 1, 0, False), 1e-6)


# ---------------------------------------------------------------- bf16 rounding
def exact_bf16(v: float) -> float:
    """Nearest value with 8 significant bits, ties to even, in exact rationals."""
    if v == 0.0:
        return 0.0
    fv = Fraction(v)
    a = abs(fv)
    e = 0
    while a >= 2:
        a /= 2
        e += 1
    while a < 1:
        a *= 2
        e -= 1
    q = Fraction(2) ** (e - 7)
    n = fv / q
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return float(lo * q)


def test_bf16_output_rounding_is_single_and_exact():
    rng = np.random.default_rng(12)
    C, O, H, W = 4, 3, 6, 6
    x = syn.to_bf16_f32(rng.standard_normal((C, H, W)).astype(np.float32))
    w = syn.to_bf16_f32(rng.standard_normal((O, C, 3, 3)).astype(np.float32))
    ref = lib_conv(x, w, None, 1, 1, False)
    got = orc.dense_conv(x, w, None, 1, 1, False, bf16=True)
    exp = np.vectorize(exact_bf16)(ref)
    assert np.array_equal(got.astype(np.float64), exp)
    assert np.array_equal(syn.to_bf16_f32(got), got)
    # a value exactly half way between two bf16 numbers goes to the even one
    wt = np.zeros((1, 1, 1, 1), np.float32)
    wt[0, 0, 0, 0] = 1.0
    for val, want in ((1.00390625, 1.0), (1.01171875, 1.015625)):
        xt = np.full((1, 1, 1), val, np.float32)
        assert orc.dense_conv(xt, wt, None, 1, 0, False, bf16=True)[0, 0, 0] == np.float32(want)


# ---------------------------------------------------------------- pooling
def lib_pool(out, w=2):
    return F.max_pool2d(torch.from_numpy(out)[None], w, w, ceil_mode=True)[0].numpy()


def test_pool_geometry_matches_table_one():
    h1, w1, h2, w2, h3, w3 = golden("pool_chain")
    a = np.zeros((1, h1, w1), np.float32)
    b = orc.pool_dense(a)
    assert b.shape == (1, h2, w2)
    assert orc.pool_dense(b).shape == (1, h3, w3)


def test_pool_dense_is_library_ceil_mode_pool():
    rng = np.random.default_rng(13)
    for shape in ((3, 8, 10), (2, 7, 9), (1, 1, 5), (2, 5, 1)):
        out = rng.standard_normal(shape).astype(np.float32)
        assert np.array_equal(orc.pool_dense(out), lib_pool(out))


@pytest.mark.parametrize("hw", [(10, 12), (9, 11)])
def test_change_based_pool_tracks_dense_pool(hw):
    H, W = hw
    spec, frames = syn.random_layer_case(41, 2, 3, 3, 1, 1, H, W, 6, change_prob=0.05, noise_std=0.001)
    L = orc.OracleLayer(spec.weight, spec.bias, 1, 1, H, W, relu=True)
    POOL = np.zeros((3, -(-H // 2), -(-W // 2)), np.float32)
    for f in frames:
        L.process(f, 0.02)
        pm = orc.pool_update(L.out, L.idx, L.mt, POOL)
        assert np.array_equal(POOL, lib_pool(L.out))
        assert np.array_equal(pm, lib_pool(L.mt.astype(np.float32)[None])[0].astype(np.uint8))
