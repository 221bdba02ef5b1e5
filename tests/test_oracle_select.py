"""Pins of the threshold-selection oracle (oracle/cb_select.py, Sec. III-F) against what the paper
and arithmetic fix: a closed form for an identity layer, the original model as the zero-threshold
reference, the bracketing property of every selected threshold, and the two degenerate limits.
No GPU."""
import importlib.util
import os
import sys

import numpy as np

import synth_inputs as syn
from oracle import cb_oracle as orc


def _load_procedure():
    """oracle/cb_select.py -- or, for tests/test_oracle_select_mutants.py, a deliberately broken copy."""
    path = os.environ.get("CB_SELECT_SRC")
    if not path:
        from oracle import cb_select
        return cb_select
    spec = importlib.util.spec_from_file_location("oracle.cb_select_under_test", path)
    mod = importlib.util.module_from_spec(spec)
    sys.modules[spec.name] = mod
    spec.loader.exec_module(mod)
    return mod


sel = _load_procedure()


def _grid(tau0, factor, steps):
    """tau0, tau0*f, tau0*f*f, ... in float32 arithmetic."""
    out, t = [], np.float32(tau0)
    for _ in range(steps):
        out.append(t)
        t = np.float32(t * np.float32(factor))
    return out


def _identity_spec():
    return syn.ConvSpec(1, 1, 1, 1, 0, False, False, np.ones((1, 1, 1, 1), np.float32), np.zeros(1, np.float32))


def test_identity_layer_closed_form():
    """One 1x1 layer with weight 1: after the full update of frame 0 the output holds frame 0; in
    frame 1 a pixel is rewritten only if its change exceeds tau (Eq. 3), so the squared error of
    the last frame is the sum of d^2 over the pixels with |d| <= tau.  Values are multiples of
    1/64, so every subtraction is exact."""
    rng = np.random.default_rng(11)
    H, W = 6, 8
    a = rng.integers(0, 64, (1, H, W)).astype(np.float32) / 64
    d = rng.integers(-12, 13, (1, H, W)).astype(np.float32) / 64
    seqs = [[a, a + d]]
    tau0, factor, max_loss = 1 / 128, 1.25, 2e-3
    net = sel.OracleNetwork([_identity_spec()], H, W)
    taus, log = sel.select_thresholds(net, seqs, tau0, factor, [max_loss], max_steps=50)
    expected, tried = np.float32(0), 0
    for t in _grid(tau0, factor, 50):
        tried += 1
        loss = float(np.sum(np.where(np.abs(d) <= t, d.astype(np.float64) ** 2, 0.0))) / d.size
        if loss > max_loss:
            break
        expected = t
    assert 0 < expected < 12 / 64                      # the case is not degenerate
    assert taus == [float(expected)]
    assert len(log[0]) == tried
    # "exceeds" is strict: with the limit set to exactly the loss of a threshold whose successor loses
    # more, that threshold is still acceptable.  (Squared multiples of 1/64 over 48 pixels: the sums
    # and their quotient by 48 are the same float64 on both sides only if formed the same way, so the
    # limit is taken from the procedure's own log.)
    losses = [loss for _, loss in log[0]]
    k = next(i for i in range(len(losses) - 1) if losses[i + 1] > losses[i] > 0)
    taus_eq, _ = sel.select_thresholds(sel.OracleNetwork([_identity_spec()], H, W), seqs, tau0, factor, [losses[k]],
                                       max_steps=50)
    assert taus_eq == [log[0][k][0]]
    # the logged losses are the closed form too
    for t, loss in log[0]:
        want = float(np.sum(np.where(np.abs(d) <= np.float32(t), d.astype(np.float64) ** 2, 0.0))) / d.size
        assert abs(loss - want) < 1e-15


def test_two_layers_closed_form():
    """A 1x1 layer with weight 1/2, then an identity layer.  While the first layer's threshold is
    chosen the second one sits at zero and passes everything on, so the loss is sum (d/2)^2 over
    |d| <= tau; the second layer then sees differences d/2 at the pixels the first one let through
    (|d| > tau_a) and drops those with |d/2| <= tau_b: its loss is sum (d/2)^2 over
    tau_a < |d| <= 2 tau_b.  All values are exact."""
    rng = np.random.default_rng(5)
    H, W = 8, 9
    a = rng.integers(0, 64, (1, H, W)).astype(np.float32) / 64
    d = rng.integers(-20, 21, (1, H, W)).astype(np.float32) / 64
    half = syn.ConvSpec(1, 1, 1, 1, 0, False, False, np.full((1, 1, 1, 1), 0.5, np.float32), np.zeros(1, np.float32))
    tau0, factor, limits = 3 / 64, 1.2, [1.2e-4, 6e-4]
    net = sel.OracleNetwork([half, _identity_spec()], H, W)
    taus, log = sel.select_thresholds(net, [[a, a + d]], tau0, factor, limits, max_steps=40)
    d64 = d.astype(np.float64)

    def pick(loss_of, limit):
        kept = np.float32(0)
        for t in _grid(tau0, factor, 40):
            if loss_of(t) > limit:
                break
            kept = t
        return kept

    ta = pick(lambda t: float(np.sum(np.where(np.abs(d) <= t, (d64 / 2) ** 2, 0.0))) / d.size, limits[0])
    tb = pick(lambda t: float(np.sum(np.where((np.abs(d) > ta) & (np.abs(d / 2) <= t), (d64 / 2) ** 2, 0.0))) / d.size, limits[1])
    assert tau0 < ta < 2 * tau0 and 2 * tb > ta            # both layers drop something; the first stays below 2 tau0
    assert taus == [float(ta), float(tb)]


def _dense_network(specs, x):
    """The original model, written with the dense step functions (no change-based state)."""
    for sp in specs:
        x = orc.dense_conv(x, sp.weight, sp.bias, sp.stride, sp.pad, sp.relu)
        if sp.pool:
            x = orc.pool_dense(x, 2)
    return x


def _small_net_and_sequences():
    wl = syn.config3(H=20, W=28, n_frames=8, widths=(4, 6, 8, 4, 2))
    frames = list(wl.frames())
    return wl, [frames[0:4], frames[4:8]]


def test_reference_is_the_original_model():
    wl, seqs = _small_net_and_sequences()
    net = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    refs = sel.reference_outputs(net, seqs)
    for seq, ref in zip(seqs, refs):
        dense = _dense_network(wl.layers, seq[-1])
        assert ref.shape == dense.shape
        assert np.allclose(ref, dense, rtol=1e-5, atol=1e-6)
    assert sel.quality(net, seqs, refs, [0.0] * 5) == 0.0


def test_selected_thresholds_bracket_the_limit():
    """For every layer: the loss it adds at the selected threshold is within the limit, the loss at
    the next value of the sequence is beyond it -- recomputed here with a metric written against
    the DENSE model, earlier layers at their selected values and later ones at zero."""
    wl, seqs = _small_net_and_sequences()
    tau0, factor, limits = 2e-3, 1.3, [2e-6, 2e-6, 1e-6, 1e-6, 1e-6]
    net = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    taus, log = sel.select_thresholds(net, seqs, tau0, factor, limits, max_steps=60)
    dense = [_dense_network(wl.layers, sq[-1]) for sq in seqs]

    def metric(t):
        tot = cnt = 0
        for sq, ref in zip(seqs, dense):
            n2 = sel.OracleNetwork(wl.layers, wl.H, wl.W)
            out = None
            for f in sq:
                out = n2.forward(f, t)
            tot += float(np.sum((out.astype(np.float64) - ref.astype(np.float64)) ** 2))
            cnt += out.size
        return tot / cnt

    assert any(t > 0 for t in taus)
    for l in range(5):
        cur = [taus[i] if i < l else 0.0 for i in range(5)]
        base = metric(cur)
        cur[l] = taus[l]
        assert metric(cur) - base <= limits[l] + 1e-12
        nxt = float(np.float32(np.float32(taus[l]) * np.float32(factor))) if taus[l] > 0 else tau0
        cur[l] = nxt
        assert metric(cur) - base > limits[l] - 1e-12, f"layer {l}: the next threshold would still be acceptable"
        # the values tried form the float32 geometric sequence, and the kept one is the last but one
        assert [t for t, _ in log[l]] == [float(v) for v in _grid(tau0, factor, len(log[l]))]
        assert taus[l] == (log[l][-2][0] if len(log[l]) > 1 else 0.0)


def test_limits_below_zero_keep_every_threshold_at_zero():
    wl, seqs = _small_net_and_sequences()
    net = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    taus, log = sel.select_thresholds(net, seqs, 1e-3, 1.5, [-1.0] * 5, max_steps=10)
    assert taus == [0.0] * 5 and all(len(x) == 1 for x in log)


def test_static_sequences_run_to_the_step_limit():
    """Identical frames: no threshold loses anything, so each layer ends at tau0 * f^(max_steps-1)."""
    wl, seqs = _small_net_and_sequences()
    static = [[sq[0]] * 3 for sq in seqs]
    net = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    taus, log = sel.select_thresholds(net, static, 1e-3, 2.0, [1e-9] * 5, max_steps=6)
    assert taus == [float(_grid(1e-3, 2.0, 6)[-1])] * 5
    assert all(loss == 0.0 for lg in log for _, loss in lg)
