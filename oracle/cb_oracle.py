"""ctypes front end of the CPU oracle (oracle/cb_oracle.c).  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays into the plain-C oracle; holds no arithmetic of its own.
Nothing in the product package imports this module.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cb_oracle.c")
_LIB = os.path.join(_HERE, "libcb_oracle.so")
# tests/test_oracle_mutants.py points this at deliberately broken builds to show that the pins catch them
_LIB_OVERRIDE = os.environ.get("CB_ORACLE_LIB")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over listed pixels, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if _LIB_OVERRIDE:
            L = C.CDLL(_LIB_OVERRIDE)
        else:
            build()
            L = C.CDLL(_LIB)
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.cbo_create.restype = vp
        L.cbo_create.argtypes = [i32] * 11 + [vp, vp]
        L.cbo_destroy.argtypes = [vp]
        L.cbo_reset.argtypes = [vp]
        L.cbo_process.restype = i32
        L.cbo_process.argtypes = [vp, vp, f32]
        L.cbo_process_propagated.restype = i32
        L.cbo_process_propagated.argtypes = [vp, vp, vp]
        for name in ("cbo_state", "cbo_out", "cbo_m", "cbo_mt", "cbo_idx"):
            getattr(L, name).restype = vp
            getattr(L, name).argtypes = [vp]
        for name in ("cbo_count", "cbo_n_in", "cbo_ho", "cbo_wo"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [vp]
        L.cbo_detect.restype = i32
        L.cbo_detect.argtypes = [i32, i32, vp, vp, f32, vp]
        L.cbo_detect_ff.restype = i32
        L.cbo_detect_ff.argtypes = [i32, i32, vp, vp, f32, vp]
        L.cbo_dilate.argtypes = [i32] * 8 + [vp, vp]
        L.cbo_extract.restype = i32
        L.cbo_extract.argtypes = [i32, vp, vp]
        L.cbo_conv_at.argtypes = [i32] * 10 + [vp, vp, vp, vp, i32, vp]
        L.cbo_dense_conv.argtypes = [i32] * 10 + [vp, vp, vp, vp]
        L.cbo_pool_update.argtypes = [i32] * 4 + [vp, vp, i32, vp, vp, vp]
        L.cbo_pool_dense.argtypes = [i32] * 4 + [vp, vp]
        L.cbo_max_threads.restype = i32
        L.cbo_set_threads.argtypes = [i32]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def max_threads() -> int:
    return int(lib().cbo_max_threads())


def set_threads(n: int) -> None:
    lib().cbo_set_threads(int(n))


def _view(ptr, shape, dtype):
    n = int(np.prod(shape))
    if n == 0:
        return np.zeros(shape, dtype)
    ct = {np.float32: C.c_float, np.uint8: C.c_uint8, np.int32: C.c_int32}[dtype]
    buf = (ct * n).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype).reshape(shape)


class OracleLayer:
    """One stateful CBconv layer (Sec. III-A/III-C)."""

    def __init__(self, weight, bias, stride: int, pad: int, H: int, W: int, relu: bool,
                 bf16: bool = False, feed_forward: bool = False):
        w = _f32(weight)
        self.O, self.C, self.kh, self.kw = w.shape
        self.s, self.p, self.H, self.W = int(stride), int(pad), int(H), int(W)
        self.relu, self.bf16 = bool(relu), bool(bf16)
        self._w = w
        self._b = None if bias is None else _f32(bias)
        self._h = lib().cbo_create(self.C, self.O, self.kh, self.kw, self.s, self.p, self.H, self.W,
                                   int(self.relu), int(self.bf16), int(feed_forward),
                                   _p(self._w), _p(self._b))
        if not self._h:
            raise ValueError("invalid layer geometry")
        self.Ho, self.Wo = int(lib().cbo_ho(self._h)), int(lib().cbo_wo(self._h))

    def __del__(self):
        # (at interpreter shutdown module globals may be gone already: then the process ends anyway)
        if getattr(self, "_h", None) and lib is not None:
            try:
                lib().cbo_destroy(self._h)
            except Exception:
                pass
            self._h = None

    def reset(self):
        lib().cbo_reset(self._h)

    def process(self, x, tau: float) -> int:
        x = _f32(x)
        assert x.shape == (self.C, self.H, self.W), x.shape
        return int(lib().cbo_process(self._h, _p(x), C.c_float(tau)))

    def process_propagated(self, x, m_producer) -> int:
        x = _f32(x)
        m = np.ascontiguousarray(m_producer, dtype=np.uint8)
        assert x.shape == (self.C, self.H, self.W) and m.shape == (self.H, self.W)
        return int(lib().cbo_process_propagated(self._h, _p(x), _p(m)))

    # views into the oracle's memory, copied so they survive the next frame
    @property
    def state(self):
        return _view(lib().cbo_state(self._h), (self.C, self.H, self.W), np.float32).copy()

    @property
    def out(self):
        return _view(lib().cbo_out(self._h), (self.O, self.Ho, self.Wo), np.float32).copy()

    @property
    def m(self):
        return _view(lib().cbo_m(self._h), (self.H, self.W), np.uint8).copy()

    @property
    def mt(self):
        return _view(lib().cbo_mt(self._h), (self.Ho, self.Wo), np.uint8).copy()

    @property
    def count(self) -> int:
        return int(lib().cbo_count(self._h))

    @property
    def n_in(self) -> int:
        return int(lib().cbo_n_in(self._h))

    @property
    def idx(self):
        return _view(lib().cbo_idx(self._h), (self.Ho * self.Wo,), np.int32)[: self.count].copy()


# ------------------------------------------------------------------ step functions
def detect(x, S, tau: float, feed_forward: bool = False):
    """Eq. 3 (+ state update).  S is modified in place; returns (m, M)."""
    x = _f32(x)
    assert S.dtype == np.float32 and S.flags.c_contiguous and S.shape == x.shape
    Cc, H, W = x.shape
    m = np.zeros((H, W), np.uint8)
    fn = lib().cbo_detect_ff if feed_forward else lib().cbo_detect
    M = fn(Cc, H * W, _p(x), _p(S), C.c_float(tau), _p(m))
    return m, int(M)


def out_hw(H, W, kh, kw, s, p):
    return (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1


def dilate(m, kh, kw, s, p):
    """Eq. 4."""
    m = np.ascontiguousarray(m, dtype=np.uint8)
    H, W = m.shape
    Ho, Wo = out_hw(H, W, kh, kw, s, p)
    mt = np.zeros((Ho, Wo), np.uint8)
    lib().cbo_dilate(H, W, Ho, Wo, kh, kw, s, p, _p(m), _p(mt))
    return mt


def extract(mt):
    mt = np.ascontiguousarray(mt, dtype=np.uint8)
    idx = np.zeros(mt.size, np.int32)
    n = lib().cbo_extract(mt.size, _p(mt), _p(idx))
    return idx[:n].copy()


def conv_at(S, weight, bias, s, p, relu, idx, bf16=False):
    """Outputs (O, n) at the listed linear output indices, from the state S."""
    S, w = _f32(S), _f32(weight)
    b = None if bias is None else _f32(bias)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    O, Cc, kh, kw = w.shape
    _, H, W = S.shape
    vals = np.zeros((O, idx.size), np.float32)
    lib().cbo_conv_at(Cc, O, H, W, kh, kw, s, p, int(relu), int(bf16), _p(S), _p(w), _p(b),
                      _p(idx), idx.size, _p(vals))
    return vals


def dense_conv(x, weight, bias, s, p, relu, bf16=False):
    x, w = _f32(x), _f32(weight)
    b = None if bias is None else _f32(bias)
    O, Cc, kh, kw = w.shape
    _, H, W = x.shape
    Ho, Wo = out_hw(H, W, kh, kw, s, p)
    out = np.zeros((O, Ho, Wo), np.float32)
    lib().cbo_dense_conv(Cc, O, H, W, kh, kw, s, p, int(relu), int(bf16), _p(x), _p(w), _p(b), _p(out))
    return out


def pool_update(OUT, idx, mt, POOL, w=2):
    """Change-based pooling; POOL is updated in place, returns the pooled map."""
    OUT = _f32(OUT)
    O, Ho, Wo = OUT.shape
    Hp, Wp = -(-Ho // w), -(-Wo // w)
    assert POOL.dtype == np.float32 and POOL.flags.c_contiguous and POOL.shape == (O, Hp, Wp)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    mt = np.ascontiguousarray(mt, dtype=np.uint8)
    pm = np.zeros((Hp, Wp), np.uint8)
    lib().cbo_pool_update(O, Ho, Wo, w, _p(OUT), _p(idx), idx.size, _p(mt), _p(POOL), _p(pm))
    return pm


def pool_dense(OUT, w=2):
    OUT = _f32(OUT)
    O, Ho, Wo = OUT.shape
    Hp, Wp = -(-Ho // w), -(-Wo // w)
    POOL = np.zeros((O, Hp, Wp), np.float32)
    lib().cbo_pool_dense(O, Ho, Wo, w, _p(OUT), _p(POOL))
    return POOL
