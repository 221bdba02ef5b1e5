"""Chains of layers, the output-comparison metric and the threshold selection of Sec. III-F on the
GPU against the CPU oracle (oracle/cb_select.py)."""
import numpy as np
import pytest
import torch

import paper_1808_05488_amd as cb
import synth_inputs as syn
from oracle import cb_select as sel
from parity import prep, to_dev, to_host

pytestmark = pytest.mark.gpu


def _gpu_network(wl, bf16=False):
    layers, pools = [], []
    h, w = wl.H, wl.W
    for sp in wl.layers:
        layers.append(cb.Layer(to_dev(prep(sp.weight, bf16), bf16), to_dev(prep(sp.bias, bf16), bf16), sp.stride,
                               sp.pad, h, w, sp.relu))
        h, w = layers[-1].Ho, layers[-1].Wo
        pools.append(cb.Pool(layers[-1]) if sp.pool else None)
        if sp.pool:
            h, w = pools[-1].Hp, pools[-1].Wp
    return cb.Network(layers, pools)


@pytest.mark.parametrize("n,bf16", [(1, False), (1000, False), (65536 + 77, False), (300001, True)])
def test_sum_squared_diff(n, bf16):
    rng = np.random.default_rng(n)
    a = prep(rng.standard_normal(n).astype(np.float32), bf16)
    b = prep(rng.standard_normal(n).astype(np.float32), bf16)
    ws = torch.empty(cb.CB_METRIC_WORKSPACE_BYTES + 256, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    got = cb.cb_sum_squared_diff(to_dev(a, bf16), to_dev(b, bf16), n, cb.CB_BF16 if bf16 else cb.CB_F32,
                                 ws[off:], torch.cuda.current_stream().cuda_stream)
    want = float(np.sum((a.astype(np.float64) - b.astype(np.float64)) ** 2))
    assert abs(got - want) <= 1e-12 * max(want, 1.0)           # float64 on both sides, different order


def test_network_forward_is_the_chain_of_calls():
    """cb_network_forward against the same frames put through the layers one call at a time."""
    wl = syn.config3(H=40, W=56, n_frames=5, widths=(8, 12, 16, 8, 4))
    taus = [0.02, 0.03, 0.02, 0.025, 0.02]
    net, ref = _gpu_network(wl), _gpu_network(wl)
    for t, f in enumerate(wl.frames()):
        x = to_dev(f, False)
        got = net.forward(x, taus)
        y = x
        for l in range(ref.n):
            if l == 0:
                y = ref.layers[l].process_frame(y, taus[l])
            else:
                prod = ref.pools[l - 1] if ref.pools[l - 1] is not None else ref.layers[l - 1]
                y = ref.layers[l].process_frame_chained(y, prod, taus[l])
            if ref.pools[l] is not None:
                y = ref.pools[l].process()
        assert torch.equal(got, y), f"frame {t}"
        for l in range(ref.n):
            assert net.layers[l].stats()["n_changed_out"] == ref.layers[l].stats()["n_changed_out"]


def test_network_forward_with_zero_thresholds_is_the_original_model():
    """Sec. III-F: a threshold of zero yields the results of the non-change-based network."""
    wl = syn.config3(H=24, W=40, n_frames=4, widths=(6, 8, 10, 6, 3))
    net = _gpu_network(wl)
    onet = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    for f in wl.frames():
        got = to_host(net.forward(to_dev(f, False), [0.0] * 5))
        want = onet.forward(f, [0.0] * 5)
        assert np.allclose(got, want, rtol=1e-4, atol=1e-5)


@pytest.mark.parametrize("factor,limits", [(1.5, [2e-6, 2e-6, 1e-6, 1e-6, 1e-6]), (1.3, [5e-6] * 5)])
def test_threshold_selection_matches_the_oracle(factor, limits):
    wl = syn.config3(H=20, W=28, n_frames=8, widths=(4, 6, 8, 4, 2))
    frames = list(wl.frames())
    seqs = [frames[0:4], frames[4:8]]
    tau0, max_steps = 2e-3, 40
    onet = sel.OracleNetwork(wl.layers, wl.H, wl.W)
    taus_o, log = sel.select_thresholds(onet, seqs, tau0, factor, limits, max_steps=max_steps)
    # The two sides decide "loss > limit" on losses that differ by rounding (and by the rare pixel
    # whose change lies within rounding of a threshold): the comparison below is meaningful only if
    # no decision of the oracle was a close call -- checked, not assumed.
    margin = min(abs(loss - limits[l]) / limits[l] for l in range(5) for _, loss in log[l])
    assert margin > 0.05, f"oracle decision within {margin:.3f} of the limit: pick another case"

    net = _gpu_network(wl)
    dev_seqs = [[to_dev(f, False) for f in sq] for sq in seqs]
    taus_g, loss_g, steps_g = net.select_thresholds(dev_seqs, tau0, factor, limits, max_steps=max_steps)
    assert [float(np.float32(t)) for t in taus_g] == taus_o, f"gpu {taus_g} oracle {taus_o}"
    assert steps_g == [len(log[l]) for l in range(5)]
    for l in range(5):
        kept = [loss for t, loss in log[l] if t == taus_o[l]]
        want = kept[0] if kept else 0.0
        assert abs(loss_g[l] - want) <= 0.02 * max(abs(want), 1e-9) + 1e-12, f"layer {l}: loss {loss_g[l]} vs {want}"


def test_threshold_selection_limits():
    wl = syn.config3(H=20, W=28, n_frames=4, widths=(4, 6, 8, 4, 2))
    frames = [to_dev(f, False) for f in wl.frames()]
    net = _gpu_network(wl)
    taus, loss, steps = net.select_thresholds([frames], 1e-3, 1.5, [-1.0] * 5, max_steps=10)
    assert taus == [0.0] * 5 and steps == [1] * 5
    static = [[frames[0]] * 3]
    taus, loss, steps = net.select_thresholds(static, 1e-3, 2.0, [1e-9] * 5, max_steps=6)
    t = np.float32(1e-3)
    for _ in range(5):
        t = np.float32(t * np.float32(2.0))
    assert [float(np.float32(v)) for v in taus] == [float(t)] * 5 and steps == [6] * 5 and loss == [0.0] * 5
    with pytest.raises(cb.CBError):
        net.select_thresholds([frames], 0.0, 1.5, [1e-6] * 5)          # tau0 must be positive
    with pytest.raises(cb.CBError):
        net.select_thresholds([frames], 1e-3, 1.0, [1e-6] * 5)          # the factor must exceed 1


@pytest.mark.parametrize("bf16", [False, True])
def test_threshold_selection_exact_case(bf16):
    """Two 1x1 layers (weights 1/2 and 1) on multiples of 1/64: every value, difference and loss is
    exact in both element types, so thresholds, step counts and losses must equal the oracle's."""
    rng = np.random.default_rng(5)
    H, W = 8, 9
    a = rng.integers(0, 64, (1, H, W)).astype(np.float32) / 64
    d = rng.integers(-20, 21, (1, H, W)).astype(np.float32) / 64
    specs = [syn.ConvSpec(1, 1, 1, 1, 0, False, False, np.full((1, 1, 1, 1), w, np.float32), np.zeros(1, np.float32))
             for w in (0.5, 1.0)]
    wl = syn.Workload("two 1x1 layers", specs, H, W, 0.0, 2)
    tau0, factor, limits = 3 / 64, 1.2, [1.2e-4, 6e-4]
    taus_o, log = sel.select_thresholds(sel.OracleNetwork(specs, H, W, bf16=bf16), [[a, a + d]], tau0, factor, limits,
                                        max_steps=40)
    net = _gpu_network(wl, bf16)
    taus_g, loss_g, steps_g = net.select_thresholds([[to_dev(a, bf16), to_dev(a + d, bf16)]], tau0, factor, limits,
                                                    max_steps=40)
    assert [float(np.float32(t)) for t in taus_g] == taus_o and taus_o[0] > 0 and taus_o[1] > 0
    assert steps_g == [len(lg) for lg in log]
    for l in range(2):
        want = [loss for t, loss in log[l] if t == taus_o[l]][0]
        assert abs(loss_g[l] - want) <= 1e-15


def test_chain_ending_in_a_pooling_stage_and_with_a_propagating_layer():
    """The metric is taken on the last stage's output, pooled or not; a CB_PROPAGATE stage has no
    threshold of its own (0 is reported) and takes its change set from the stage before."""
    wl = syn.config3(H=24, W=36, n_frames=6, widths=(4, 6, 5, 4, 2))
    specs = wl.layers[:3]
    specs[2].pool = True                                   # conv+pool, conv+pool, conv+pool
    frames = list(wl.frames())
    seqs = [frames[0:3], frames[3:6]]
    tau0, factor, limits = 2e-3, 1.5, [3e-6, 3e-6, 3e-6]
    taus_o, log = sel.select_thresholds(sel.OracleNetwork(specs, wl.H, wl.W), seqs, tau0, factor, limits, max_steps=30)
    margin = min(abs(loss - limits[l]) / limits[l] for l in range(3) for _, loss in log[l])
    assert margin > 0.05, f"oracle decision within {margin:.3f} of the limit: pick another case"
    sub = syn.Workload("three stages", specs, wl.H, wl.W, wl.tau, 6)
    net = _gpu_network(sub)
    assert net.out_shape == (5, 3, 5)
    dev_seqs = [[to_dev(f, False) for f in sq] for sq in seqs]
    taus_g, _, steps_g = net.select_thresholds(dev_seqs, tau0, factor, limits, max_steps=30)
    assert [float(np.float32(t)) for t in taus_g] == taus_o and steps_g == [len(lg) for lg in log]

    # the same chain with a propagating second stage: selection skips it
    layers, pools = [], []
    h, w = wl.H, wl.W
    for l, sp in enumerate(specs):
        layers.append(cb.Layer(to_dev(sp.weight, False), to_dev(sp.bias, False), sp.stride, sp.pad, h, w, sp.relu,
                               mode=cb.CB_PROPAGATE if l == 1 else cb.CB_CLOSED_LOOP))
        pools.append(cb.Pool(layers[-1]))
        h, w = pools[-1].Hp, pools[-1].Wp
    net2 = cb.Network(layers, pools)
    taus2, loss2, steps2 = net2.select_thresholds(dev_seqs, tau0, factor, limits, max_steps=30)
    assert taus2[1] == 0.0 and steps2[1] == 0 and taus2[0] > 0 and taus2[2] > 0
    # stage 0 must detect for itself
    with pytest.raises(cb.CBError):
        cb.Network(layers[1:], pools[1:]).forward(dev_seqs[0][0][:4].contiguous(), [0.0, 0.0])
