"""Checkpoint and resume (GPU): a layer that imports an exported input state and cached output goes on
exactly where the exporting layer stood -- checked against the oracle, which never stops -- and the
stages that consume an imported layer (pooling, detection at the producer's listed pixels, propagated
change sets) take nothing for granted on their first call afterwards."""
import numpy as np
import pytest
import torch

import paper_1808_05488_amd as cb
from oracle import cb_oracle as orc
import synth_inputs as syn
from parity import Pair, assert_close, prep, to_dev, to_host

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _twin(p: Pair, H, W, mode, backend):
    """A fresh layer of the same description as p.g."""
    return cb.Layer(to_dev(p.w, p.bf16), None if p.b is None else to_dev(p.b, p.bf16), p.spec.stride, p.spec.pad,
                    H, W, p.spec.relu, mode=mode, backend=backend)


@pytest.mark.parametrize("case", [
    # C, O, k, s, pad, H, W, bf16, backend, feed_forward
    (4, 6, 3, 1, 1, 40, 52, False, 2, False),          # channel-first fused kernel, no shadow
    (16, 24, 3, 1, 1, 70, 90, False, 2, False),        # float32 layer with a channel-last shadow
    (32, 40, 3, 2, 1, 64, 80, True, 2, False),         # bfloat16 layer with a shadow
    (64, 16, 1, 1, 0, 50, 70, True, 0, False),         # 1x1, shadow
    (3, 5, 5, 1, 2, 33, 47, False, 1, False),          # explicit back end
    (5, 7, 3, 1, 1, 30, 40, False, 0, True),           # feed-forward: the state is the whole previous input
])
def test_a_layer_resumes_from_an_exported_state(case):
    C, O, k, s, pd, H, W, bf16, backend, ff = case
    _say(f"checkpoint: {case}")
    spec, frames = syn.random_layer_case(sum(case[:7]), C, O, k, s, pd, H, W, 10, change_prob=0.03, noise_std=0.004)
    mode = cb.CB_FEED_FORWARD if ff else cb.CB_CLOSED_LOOP
    tau = 0.02
    p = Pair(spec, H, W, bf16=bf16, feed_forward=ff, backend=backend)
    for t in range(4):
        p.step(frames[t], tau, tag=f"{case} frame {t}")
    state, out = p.g.export_state()
    assert torch.equal(state, p.g.state()) and torch.equal(out, p.g_out)

    # another layer of the same description takes over
    g2 = _twin(p, H, W, mode, backend)
    g2.import_state(state, out)
    m, mt, idx, n = g2.changes_host()
    assert n == 0 and idx.size == 0 and not m.any() and not mt.any(), "an imported layer's last change set is empty"
    assert g2.stats()["n_changed_in"] == 0
    assert torch.equal(g2.state(), state)
    first = p.g
    p.g, p.g_out = g2, out                  # Pair.step checks the unlisted outputs against this `out`
    for t in range(4, 7):
        _, n = p.step(frames[t], tau, tag=f"{case} frame {t} after the import")
        assert n < g2.Ho * g2.Wo, "an imported layer does not start with a full update"

    # back into the layer the state came from, after that layer has seen something else entirely
    state6, out6 = g2.export_state()
    junk = to_dev(prep(frames[0] + np.float32(3.0), bf16), bf16)
    first.process_frame(junk, tau)
    first.import_state(state6, out6)
    p.g, p.g_out = first, out6
    for t in range(7, 10):
        p.step(frames[t], tau, tag=f"{case} frame {t} after the second import")


def test_consumers_of_an_imported_producer_start_from_scratch_once():
    """producer -> 2x2 pool -> {closed-loop consumer with detection at the producer's listed pixels,
    consumer that propagates the pooled change map}: all four stages are replaced by fresh ones that import
    what the old ones exported."""
    H, W = 36, 52
    tau = 0.02
    spec, frames = syn.random_layer_case(33, 3, 16, 3, 1, 1, H, W, 7, change_prob=0.02, noise_std=0.004)
    rng = np.random.default_rng(8)
    wc = (rng.standard_normal((6, 16, 3, 3)) * 0.2).astype(np.float32)
    wq = (rng.standard_normal((5, 16, 3, 3)) * 0.2).astype(np.float32)
    Hp, Wp = H // 2, W // 2

    def stages(prod):
        return (cb.Pool(prod), cb.Layer(to_dev(wc, False), None, 1, 1, Hp, Wp, True),
                cb.Layer(to_dev(wq, False), None, 1, 1, Hp, Wp, False, mode=cb.CB_PROPAGATE))

    p = Pair(spec, H, W)
    pool, gc, gq = stages(p.g)
    oc = orc.OracleLayer(wc, None, 1, 1, Hp, Wp, True)
    oq = orc.OracleLayer(wq, None, 1, 1, Hp, Wp, False)
    opool = np.zeros((16, Hp, Wp), np.float32)

    def frame(t, expect_full):
        p.step(frames[t], tau, tag=f"producer frame {t}")
        pooled = pool.process()
        pm = orc.pool_update(to_host(p.g_out), p.o.idx, p.o.mt, opool)
        assert np.array_equal(to_host(pooled), opool), f"frame {t}: pooled output differs"
        out = gc.process_frame_chained(pooled, pool, tau)
        n_o = oc.process(to_host(pooled), tau)
        m, mt, idx, n = gc.changes_host()
        tag = f"chained consumer frame {t}"
        assert n == n_o and np.array_equal(idx, oc.idx) and np.array_equal(m, oc.m) and np.array_equal(mt, oc.mt), tag
        assert np.array_equal(to_host(gc.state()), oc.state), tag
        assert_close(to_host(out), oc.out, False, tag)
        out = gq.process_frame_propagated(pooled, pool)
        n_o = oq.process_propagated(to_host(pooled), pm)
        n = gq.stats()["n_changed_out"]
        tag = f"propagating consumer frame {t}"
        if expect_full:
            assert n == gq.Ho * gq.Wo, f"{tag}: every output is recomputed once, N = {n}"
        else:
            assert n == n_o and np.array_equal(gq.changes_host()[2], oq.idx), tag
        assert_close(to_host(out), oq.out, False, tag)

    for t in range(3):
        frame(t, expect_full=(t == 0))
    saved = (p.g.export_state(), gc.export_state(), gq.export_state())
    assert saved[2][0] is None
    # fresh stages
    g_new = cb.Layer(to_dev(p.w, False), to_dev(p.b, False), spec.stride, spec.pad, H, W, spec.relu)
    g_new.import_state(*saved[0])
    p.g, p.g_out = g_new, saved[0][1]
    pool, gc, gq = stages(g_new)
    gc.import_state(*saved[1])
    gq.import_state(*saved[2])
    # a pooling stage created on an imported producer pools everything on its first call;
    # a consumer cannot use it before that
    with pytest.raises(cb.binding.CBError) as e:
        gq.process_frame_propagated(torch.zeros((16, Hp, Wp), device="cuda"), pool)
    assert e.value.status == cb.CB_ESTATE
    frame(3, expect_full=True)
    for t in range(4, 7):
        frame(t, expect_full=False)


def test_a_pooling_stage_that_misses_a_producer_frame_pools_everything():
    H, W = 31, 45
    spec, frames = syn.random_layer_case(17, 4, 9, 3, 1, 1, H, W, 6, change_prob=0.03, noise_std=0.002)
    p = Pair(spec, H, W)
    pool = cb.Pool(p.g)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"frame {t}")
        if t in (1, 2, 4):
            continue                                   # the pooling stage is not called for these frames
        got = to_host(pool.process())
        assert np.array_equal(got, orc.pool_dense(to_host(p.g_out))), f"frame {t}: not the pool of the cached output"


def test_export_and_import_argument_checks():
    H, W = 20, 24
    rng = np.random.default_rng(2)
    w = to_dev(rng.standard_normal((4, 3, 3, 3)).astype(np.float32), False)
    g = cb.Layer(w, None, 1, 1, H, W, True)
    gp = cb.Layer(w, None, 1, 1, H, W, True, mode=cb.CB_PROPAGATE)
    st = torch.zeros((3, H, W), device="cuda")
    out = torch.zeros((4, H, W), device="cuda")

    def status(fn, *a):
        with pytest.raises(cb.binding.CBError) as e:
            fn(*a)
        return e.value.status

    assert status(cb.cb_layer_export_state, g.handle, st, out) == cb.CB_ESTATE        # no frame yet
    assert status(cb.cb_layer_import_state, g.handle, None, out) == cb.CB_EINVAL      # a closed-loop layer has a state
    assert status(cb.cb_layer_import_state, g.handle, st, None) == cb.CB_EINVAL
    assert status(cb.cb_layer_import_state, gp.handle, st, out) == cb.CB_EINVAL       # a propagating layer has none
    g.process_frame(torch.rand((3, H, W), device="cuda"), 0.02)
    assert status(cb.cb_layer_export_state, g.handle, None, out) == cb.CB_EINVAL
    assert status(cb.cb_layer_import_state, g.handle, g.state(), out) == cb.CB_EINVAL  # source inside the layer's own buffer
    cb.cb_layer_export_state(g.handle, st, out)
    assert torch.equal(st, g.state())
    cb.cb_layer_import_state(gp.handle, None, out)                                     # output only
