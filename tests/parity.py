"""Helpers of the GPU parity tests: run the HIP library and the CPU oracle on
the same host arrays and compare what each step produces.

Bars: change maps, index lists and counts bit-exact; the input state bit-exact;
float32 outputs within 1e-4 and bfloat16 outputs within 1e-2 relative error,
measured as |g - o| <= tol * max(|o|, rms(o)) element by element.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_1808_05488_amd as cb
from oracle import cb_oracle as orc
import synth_inputs as syn

TOL = {False: 1e-4, True: 1e-2}


def assert_close(got: np.ndarray, ref: np.ndarray, bf16: bool, what: str = "out"):
    ref64 = ref.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref64 ** 2))) if ref.size else 0.0
    bound = TOL[bf16] * np.maximum(np.abs(ref64), max(rms, 1e-30))
    err = np.abs(got.astype(np.float64) - ref64)
    bad = err > bound
    if bad.any():
        k = int(np.argmax(err / bound))
        raise AssertionError(f"{what}: {int(bad.sum())} of {ref.size} beyond tol {TOL[bf16]}; worst at flat {k}: "
                             f"got {got.reshape(-1)[k]!r} ref {ref.reshape(-1)[k]!r}")


def to_dev(a: np.ndarray, bf16: bool) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if bf16 else t


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def prep(a, bf16: bool) -> np.ndarray:
    """Host array both sides consume: float32, pre-rounded to bf16 values if needed."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return syn.to_bf16_f32(a) if bf16 else a


class Pair:
    """One layer on both sides."""

    def __init__(self, spec: syn.ConvSpec, H: int, W: int, bf16: bool = False, feed_forward: bool = False,
                 scratch_bytes=None, backend=0, **layer_kw):
        self.spec, self.bf16 = spec, bf16
        w = prep(spec.weight, bf16)
        b = None if spec.bias is None else prep(spec.bias, bf16)
        self.w, self.b = w, b
        self.o = orc.OracleLayer(w, b, spec.stride, spec.pad, H, W, spec.relu, bf16=bf16, feed_forward=feed_forward)
        self.g = cb.Layer(to_dev(w, bf16), None if b is None else to_dev(b, bf16), spec.stride, spec.pad, H, W,
                          spec.relu, mode=cb.CB_FEED_FORWARD if feed_forward else cb.CB_CLOSED_LOOP,
                          scratch_bytes=scratch_bytes, backend=backend, **layer_kw)

    def step(self, frame: np.ndarray, tau: float, check_out: bool = True, tag: str = ""):
        x = prep(frame, self.bf16)
        xd = to_dev(x, self.bf16)
        prev = to_host(self.g_out) if hasattr(self, "g_out") else None
        self.g_out = self.g.process_frame(xd, tau)
        n_o = self.o.process(x, tau)
        m, mt, idx, n = self.g.changes_host()
        st = self.g.stats()
        assert n == n_o, f"{tag} N: gpu {n} oracle {n_o}"
        assert st["n_changed_in"] == self.o.n_in, f"{tag} M: gpu {st['n_changed_in']} oracle {self.o.n_in}"
        assert np.array_equal(m, self.o.m), f"{tag} change map m differs"
        assert np.array_equal(mt, self.o.mt), f"{tag} dilated map differs"
        assert np.array_equal(idx, self.o.idx), f"{tag} index list differs"
        assert st["ops"] == 2 * self.o.O * self.o.C * self.o.kh * self.o.kw * n
        assert np.array_equal(to_host(self.g.state()), self.o.state), f"{tag} input state differs"
        out = to_host(self.g_out)
        if check_out:
            assert_close(out, self.o.out, self.bf16, f"{tag} out")
        if prev is not None:
            keep = mt.reshape(-1) == 0
            assert np.array_equal(out.reshape(out.shape[0], -1)[:, keep], prev.reshape(prev.shape[0], -1)[:, keep]), \
                f"{tag} an unlisted output changed"
        return out, n
