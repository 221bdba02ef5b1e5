"""GPU parity on randomly drawn layer geometries: the fused back end (float32 and
bfloat16) and the explicit one against the CPU oracle, three frames per case.  The draws are
seeded; they cover all four row-tile shapes of the fused kernels (up to 16 / 32 / 64 / more
output channels), 1x1 ... 7x7 filters, stride 1 and 2, padding 0 and half the filter, maps
from a few dozen pixels (every listed pixel at the border) to more than 8 192 pixels (the
32-column tile of the float32 kernel on the full-update frame), and sparse to dense change.
A second set of draws has power-of-two channel counts only: those layers keep a channel-last
shadow of their state, which change detection updates and the fused kernel gathers from.
A third set draws two-stage chains -- producer, optional 2x2 pooling, and two consumers of the same
input: one that detects at the producer's listed pixels and one that propagates the producer's change
map -- and lets the pooling stage and the consumers miss frames at random."""
import numpy as np
import pytest
import torch

import synth_inputs as syn

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_1808_05488_amd as cb
    from oracle import cb_oracle as orc
    from parity import Pair, assert_close, prep, to_dev, to_host


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


def _chain_case(seed, i):
    rng = np.random.default_rng([seed, i])
    bf16 = bool(rng.random() < 0.35)
    kA = int(rng.choice([1, 3, 3, 5]))
    C1 = int(rng.integers(1, 9))
    C2 = int(rng.choice([int(rng.integers(1, 24)), 8, 16, 32, 64, 128, 256]))
    H, W = int(rng.integers(12, 56)), int(rng.integers(12, 72))
    pooled = bool(rng.random() < 0.5)
    kB = int(rng.choice([1, 3, 3]))
    sB = int(rng.choice([1, 1, 2])) if kB > 1 else 1
    padB = kB // 2 if rng.random() < 0.8 else 0
    C3, C4 = int(rng.integers(1, 40)), int(rng.integers(1, 40))
    ff = bool(rng.random() < 0.25)
    prob = float(rng.choice([0.005, 0.03, 0.15]))
    tau = 0.02
    tag = (f"chain seed {seed} case {i}: {C1}->{C2} k{kA} {H}x{W} pool={pooled} consumers k{kB} s{sB} pad{padB} "
           f"->{C3} (detecting, feed_forward={ff}) / ->{C4} (propagating) bf16={bf16} p={prob}")
    # where the channel count allows it, mostly: the producer (and its pooling stage) keeps its output pixel-major
    # as well, and the propagating consumer gathers from that copy
    cl = C2 >= (32 if bf16 else 16) and (C2 & (C2 - 1)) == 0 and bool(rng.random() < 0.7)
    tag += f" channel_last={cl}"
    print(tag, flush=True)
    spec, frames = syn.random_layer_case(1000 * seed + i, C1, C2, kA, 1, kA // 2, H, W, 7, change_prob=prob, noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, keep_output_channel_last=cl)
    Hc, Wc = (-(-H // 2), -(-W // 2)) if pooled else (H, W)
    if Hc + 2 * padB < kB or Wc + 2 * padB < kB:
        return
    pool = cb.Pool(p.g) if pooled else None
    opool = np.zeros((C2, Hc, Wc), np.float32) if pooled else None
    wc = prep(rng.standard_normal((C3, C2, kB, kB)) * np.sqrt(2.0 / (C2 * kB * kB)), bf16)
    wq = prep(rng.standard_normal((C4, C2, kB, kB)) * np.sqrt(2.0 / (C2 * kB * kB)), bf16)
    bq = prep(rng.standard_normal(C4) * 0.1, bf16)
    gc = cb.Layer(to_dev(wc, bf16), None, sB, padB, Hc, Wc, True,
                  mode=cb.CB_FEED_FORWARD if ff else cb.CB_CLOSED_LOOP)
    oc = orc.OracleLayer(wc, None, sB, padB, Hc, Wc, True, bf16=bf16, feed_forward=ff)
    gq = cb.Layer(to_dev(wq, bf16), to_dev(bq, bf16), sB, padB, Hc, Wc, False, mode=cb.CB_PROPAGATE,
                  gather_channel_last=cl)
    pool_seen = q_seen = -2                       # last producer frame the pooling stage / the propagating consumer saw
    for t, f in enumerate(frames):
        p.step(f, tau, tag=f"{tag} producer frame {t}")
        prod_out = to_host(p.g_out)
        m_in = p.o.mt
        if pooled:
            pm = orc.pool_update(prod_out, p.o.idx, p.o.mt, opool)
            if t > 0 and rng.random() < 0.2:
                continue                          # the pooling stage (and with it both consumers) misses this frame
            src = pool.process()
            assert np.array_equal(to_host(src), opool), f"{tag} frame {t}: pooled output differs"
            pool_lock = pool_seen == t - 1
            pool_seen = t
            m_in, prod = pm, pool
        else:
            src, prod, pool_lock = p.g_out, p.g, True
        src_host = to_host(src)
        if t == 0 or rng.random() < 0.8:
            out = gc.process_frame_chained(src, prod, tau)
            n_o = oc.process(src_host, tau)
            m, mt, idx, n = gc.changes_host()
            tg = f"{tag} detecting consumer frame {t}"
            assert n == n_o and np.array_equal(idx, oc.idx) and np.array_equal(m, oc.m) and np.array_equal(mt, oc.mt), tg
            assert gc.stats()["n_changed_in"] == oc.n_in, tg
            assert np.array_equal(to_host(gc.state()), oc.state), tg
            assert_close(to_host(out), oc.out, bf16, tg)
        if t == 0 or rng.random() < 0.8:
            out = gq.process_frame_propagated(src, prod)
            m, mt, idx, n = gq.changes_host()
            tg = f"{tag} propagating consumer frame {t}"
            if q_seen == t - 1 and pool_lock:     # in lockstep: exactly the dilated producer map is recomputed
                want = orc.dilate(m_in, kB, kB, sB, padB)
                assert np.array_equal(mt, want) and np.array_equal(idx, np.flatnonzero(want)), tg
            else:                                 # first frame, or a frame was missed: everything once
                assert n == gq.Ho * gq.Wo, f"{tg}: N = {n}"
            q_seen = t
            assert_close(to_host(out), orc.dense_conv(src_host, wq, bq, sB, padB, False, bf16=bf16), bf16, tg)


@pytest.mark.parametrize("seed", [31, 32])
def test_random_chains(seed):
    for i in range(20):
        _chain_case(seed, i)
