"""Captured frames replay correctly (GPU).  The per-frame path has no host synchronisation, no
allocation and no memset node; the number of listed pixels never leaves the GPU, and which of the
layer's two alternating map buffers a frame uses is decided on the GPU too (a frame count in the
layer's control block), so cb_process_frame can be captured in a HIP graph, any number of frames
per capture -- odd numbers included.  Every replay is checked against the same frames processed
eagerly by a second layer, with eager work and synchronisations between the replays, and eager
frames of the graphed layer itself may come between replays."""
import numpy as np
import pytest
import torch

import paper_1808_05488_amd as cb
import synth_inputs as syn
from parity import to_dev, to_host

pytestmark = pytest.mark.gpu


def test_a_captured_single_frame_replays_and_mixes_with_eager_frames():
    """One frame per capture: consecutive replays use alternate map buffers.  Eager frames of the same
    layer between the replays shift the alternation, which lives on the GPU and therefore stays right."""
    C, O, k, s, pd, H, W = 4, 6, 3, 1, 1, 150, 520
    spec, frames = syn.random_layer_case(91, C, O, k, s, pd, H, W, 9, change_prob=0.02, noise_std=0.004)
    tau = 0.02
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        w, b = to_dev(spec.weight, False), to_dev(spec.bias, False)
        eager = cb.Layer(w, b, s, pd, H, W, spec.relu, stream=st)
        graphed = cb.Layer(w, b, s, pd, H, W, spec.relu, stream=st)
        dev_frames = [to_dev(f, False) for f in frames]
        buf = torch.empty_like(dev_frames[0])
        eager.process_frame(dev_frames[0], tau)
        graphed.process_frame(dev_frames[0], tau)
        st.synchronize()
        res = torch.empty((O, graphed.Ho, graphed.Wo), device="cuda")
        g = torch.cuda.CUDAGraph()
        buf.copy_(dev_frames[1])
        with torch.cuda.graph(g, stream=st):
            res.copy_(graphed.process_frame(buf, tau))
        st.synchronize()
        # (the capture itself ran nothing: frame 1 comes with the first replay)
        plan = ["replay", "replay", "eager", "replay", "eager", "eager", "replay", "replay"]
        for t, how in enumerate(plan, start=1):
            ref = eager.process_frame(dev_frames[t], tau).clone()
            if how == "replay":
                buf.copy_(dev_frames[t])
                g.replay()
                got = res
            else:
                got = graphed.process_frame(dev_frames[t], tau)
            st.synchronize()
            tag = f"frame {t} ({how})"
            assert torch.equal(got, ref), f"{tag}: output differs from the eager layer's"
            m_e, mt_e, idx_e, n_e = eager.changes_host()
            m_g, mt_g, idx_g, n_g = graphed.changes_host()
            assert n_g == n_e and np.array_equal(idx_g, idx_e), f"{tag}: index list differs"
            assert np.array_equal(m_g, m_e) and np.array_equal(mt_g, mt_e), f"{tag}: maps differ"
            assert graphed.stats()["n_changed_in"] == eager.stats()["n_changed_in"], f"{tag}: M differs"
            assert np.array_equal(to_host(graphed.state()), to_host(eager.state())), f"{tag}: input state differs"


@pytest.mark.parametrize("geom,backend", [((8, 16, 3, 1, 1, 40, 132), 2),      # one-workgroup index extraction, fused
                                          ((2, 3, 3, 1, 1, 150, 520), 2),      # single-pass index extraction, fused
                                          ((2, 3, 3, 1, 1, 150, 520), 1)])     # ... and the explicit back end
def test_captured_pair_of_frames_replays(geom, backend):
    C, O, k, s, pd, H, W = geom
    spec, frames = syn.random_layer_case(sum(geom) + 7, C, O, k, s, pd, H, W, 7, change_prob=0.03, noise_std=0.004)
    tau = 0.02
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        w, b = to_dev(spec.weight, False), to_dev(spec.bias, False)
        eager = cb.Layer(w, b, s, pd, H, W, spec.relu, backend=backend, stream=st)
        graphed = cb.Layer(w, b, s, pd, H, W, spec.relu, backend=backend, stream=st)
        dev_frames = [to_dev(f, False) for f in frames]
        buf_a, buf_b = torch.empty_like(dev_frames[0]), torch.empty_like(dev_frames[0])
        # both layers see frame 0 eagerly (full update; also the warm-up torch asks for before a capture)
        eager.process_frame(dev_frames[0], tau)
        graphed.process_frame(dev_frames[0], tau)
        st.synchronize()
        res_a = torch.empty((O, graphed.Ho, graphed.Wo), device="cuda")
        res_b = torch.empty_like(res_a)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            res_a.copy_(graphed.process_frame(buf_a, tau))
            res_b.copy_(graphed.process_frame(buf_b, tau))
        st.synchronize()
        for rep in range(3):
            fa, fb = dev_frames[2 * rep + 1], dev_frames[2 * rep + 2]
            ref_a = eager.process_frame(fa, tau).clone()          # eager work between the replays
            ref_b = eager.process_frame(fb, tau).clone()
            m_e, mt_e, idx_e, n_e = eager.changes_host()
            buf_a.copy_(fa)
            buf_b.copy_(fb)
            g.replay()
            st.synchronize()
            tag = f"{geom} backend {backend} replay {rep}"
            assert torch.equal(res_a, ref_a), f"{tag}: first frame differs from the eager result"
            assert torch.equal(res_b, ref_b), f"{tag}: second frame differs from the eager result"
            m_g, mt_g, idx_g, n_g = graphed.changes_host()
            assert n_g == n_e and np.array_equal(idx_g, idx_e), f"{tag}: index list differs"
            assert np.array_equal(m_g, m_e) and np.array_equal(mt_g, mt_e), f"{tag}: maps differ"
            assert graphed.stats()["n_changed_in"] == eager.stats()["n_changed_in"], f"{tag}: M differs"
            assert np.array_equal(to_host(graphed.state()), to_host(eager.state())), f"{tag}: input state differs"
