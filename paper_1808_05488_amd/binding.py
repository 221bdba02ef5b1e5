"""ctypes binding of libcbconv.so: argument marshalling only.

The functions carry the names of the C ABI (include/cbconv.h).  torch is used
for device memory and streams; every step of the path runs in the library's HIP
kernels.  There is no fallback: if the library is not built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcbconv.so")

CB_OK, CB_EINVAL, CB_ENOMEM, CB_EHIP, CB_ESTATE = 0, -1, -2, -3, -4
CB_F32, CB_BF16 = 0, 1
CB_CLOSED_LOOP, CB_FEED_FORWARD, CB_PROPAGATE = 0, 1, 2
CB_BACKEND_AUTO, CB_BACKEND_EXPLICIT, CB_BACKEND_FUSED = 0, 1, 2
CB_NUM_STEPS = 9
STEP_NAMES = ("detect", "dilate", "compact", "gather", "gemm", "update", "fused", "state", "total")

EXPORTS = (
    "cb_layer_workspace_bytes", "cb_layer_min_scratch_bytes", "cb_layer_create", "cb_process_frame",
    "cb_process_frame_propagated", "cb_process_frame_chained", "cb_layer_changes", "cb_layer_state", "cb_layer_matrices",
    "cb_layer_export_state", "cb_layer_import_state",
    "cb_layer_out_shape", "cb_layer_set_timing", "cb_layer_stats", "cb_set_scan_wait_limit", "cb_layer_reset",
    "cb_layer_destroy",
    "cb_pool_workspace_bytes", "cb_pool_create", "cb_pool_process", "cb_pool_changes", "cb_pool_out_shape",
    "cb_pool_destroy", "cb_strerror", "cb_last_hip_error", "cb_version",
    "cb_network_forward", "cb_sum_squared_diff", "cb_sum_squared_diff_noalloc", "cb_select_workspace_bytes",
    "cb_select_thresholds",
)
CB_METRIC_WORKSPACE_BYTES = 4096


class cb_layer_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("c_in", "c_out", "kh", "kw", "stride", "pad", "h_in", "w_in",
                                         "dtype", "relu", "mode", "backend", "keep_output_channel_last",
                                         "gather_channel_last")] + [("reserved", C.c_int32 * 2)]


class cb_stage(C.Structure):
    _fields_ = [("layer", C.c_void_p), ("pool", C.c_void_p)]


class cb_select_params(C.Structure):
    _fields_ = [("tau0", C.c_float), ("factor", C.c_float), ("max_steps", C.c_int32), ("reserved", C.c_int32)]


class cb_stats(C.Structure):
    _fields_ = [("n_changed_in", C.c_int32), ("n_changed_out", C.c_int32), ("ops", C.c_int64),
                ("us_step", C.c_float * CB_NUM_STEPS), ("scan_recounts", C.c_int32), ("reserved", C.c_int32)]


class CBError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().cb_strerror(status).decode()
        if status == CB_EHIP:
            msg += f" (hipError {lib().cb_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


_lib = None


def lib():
    """Load libcbconv.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1808_05488_amd.build` "
                "(or __graft_entry__.build()); there is no non-HIP fallback")
        L = C.CDLL(LIB_PATH)
        # torch's streams and allocations are only valid in the HIP runtime torch loaded
        with open("/proc/self/maps") as f:
            runtimes = {ln.split()[-1] for ln in f if "libamdhip64" in ln}
        if len(runtimes) > 1:
            raise RuntimeError(f"two HIP runtimes are loaded {sorted(runtimes)}; rebuild libcbconv.so "
                               "with paper_1808_05488_amd.build so that it links torch's runtime")
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        P = C.POINTER
        L.cb_layer_workspace_bytes.argtypes = [P(cb_layer_desc), P(sz), P(sz)]
        L.cb_layer_min_scratch_bytes.argtypes = [P(cb_layer_desc), P(sz)]
        L.cb_layer_create.argtypes = [P(cb_layer_desc), vp, vp, vp, sz, vp, sz, vp, P(vp)]
        L.cb_process_frame.argtypes = [vp, vp, C.c_float, P(vp)]
        L.cb_process_frame_propagated.argtypes = [vp, vp, vp, vp, P(vp)]
        L.cb_process_frame_chained.argtypes = [vp, vp, vp, vp, C.c_float, P(vp)]
        L.cb_layer_changes.argtypes = [vp, P(vp), P(vp), P(vp), P(vp)]
        L.cb_network_forward.argtypes = [P(cb_stage), C.c_int32, vp, P(C.c_float), P(vp)]
        L.cb_sum_squared_diff.argtypes = [vp, vp, sz, C.c_int32, vp, P(C.c_double), vp]
        L.cb_sum_squared_diff_noalloc.argtypes = [vp, vp, sz, C.c_int32, P(C.c_double), vp]
        L.cb_select_workspace_bytes.argtypes = [P(cb_stage), C.c_int32, C.c_int32, P(sz)]
        L.cb_select_thresholds.argtypes = [P(cb_stage), C.c_int32, P(vp), C.c_int32, C.c_int32, P(cb_select_params),
                                           P(C.c_double), vp, sz, P(C.c_float), P(C.c_double), P(C.c_int32)]
        L.cb_layer_state.argtypes = [vp, P(vp)]
        L.cb_layer_matrices.argtypes = [vp, P(vp), P(vp), P(vp)]
        L.cb_layer_export_state.argtypes = [vp, vp, vp]
        L.cb_layer_import_state.argtypes = [vp, vp, vp]
        L.cb_layer_out_shape.argtypes = [vp, P(i32), P(i32), P(i32)]
        L.cb_layer_set_timing.argtypes = [vp, i32]
        L.cb_layer_stats.argtypes = [vp, P(cb_stats)]
        L.cb_set_scan_wait_limit.argtypes = [i32]
        L.cb_layer_reset.argtypes = [vp]
        L.cb_layer_destroy.argtypes = [vp]
        L.cb_pool_workspace_bytes.argtypes = [vp, i32, P(sz)]
        L.cb_pool_create.argtypes = [vp, i32, vp, sz, vp, P(vp)]
        L.cb_pool_process.argtypes = [vp, P(vp)]
        L.cb_pool_changes.argtypes = [vp, P(vp)]
        L.cb_pool_out_shape.argtypes = [vp, P(i32), P(i32), P(i32)]
        L.cb_pool_destroy.argtypes = [vp]
        L.cb_strerror.argtypes = [C.c_int]
        L.cb_strerror.restype = C.c_char_p
        L.cb_last_hip_error.restype = C.c_int
        L.cb_version.restype = C.c_int
        for name in EXPORTS:
            if name not in ("cb_strerror",):
                getattr(L, name).restype = getattr(L, name).restype or C.c_int
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != CB_OK:
        raise CBError(status, where)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def make_desc(c_in, c_out, kh, kw, stride, pad, h_in, w_in, dtype=CB_F32, relu=0, mode=CB_CLOSED_LOOP,
              backend=CB_BACKEND_AUTO, keep_output_channel_last=False, gather_channel_last=False):
    d = cb_layer_desc()
    d.c_in, d.c_out, d.kh, d.kw, d.stride, d.pad, d.h_in, d.w_in = c_in, c_out, kh, kw, stride, pad, h_in, w_in
    d.dtype, d.relu, d.mode, d.backend = dtype, int(relu), mode, backend
    d.keep_output_channel_last, d.gather_channel_last = int(keep_output_channel_last), int(gather_channel_last)
    return d


# ---------------------------------------------------------------- C ABI, one to one
def cb_version() -> int:
    return lib().cb_version()


def cb_layer_workspace_bytes(desc: cb_layer_desc) -> Tuple[int, int]:
    a, b = C.c_size_t(), C.c_size_t()
    _check(lib().cb_layer_workspace_bytes(C.byref(desc), C.byref(a), C.byref(b)), "cb_layer_workspace_bytes")
    return a.value, b.value


def cb_layer_min_scratch_bytes(desc: cb_layer_desc) -> int:
    b = C.c_size_t()
    _check(lib().cb_layer_min_scratch_bytes(C.byref(desc), C.byref(b)), "cb_layer_min_scratch_bytes")
    return b.value


def cb_layer_create(desc, w_dev, bias_dev, state_dev, state_bytes, scratch_dev, scratch_bytes, stream=0) -> int:
    h = C.c_void_p()
    _check(lib().cb_layer_create(C.byref(desc), _ptr(w_dev), _ptr(bias_dev), _ptr(state_dev), state_bytes,
                                 _ptr(scratch_dev), scratch_bytes, stream or None, C.byref(h)), "cb_layer_create")
    return h.value


def cb_process_frame(layer: int, input_dev, tau: float) -> int:
    out = C.c_void_p()
    _check(lib().cb_process_frame(layer, _ptr(input_dev), C.c_float(tau), C.byref(out)), "cb_process_frame")
    return out.value


def cb_process_frame_propagated(layer: int, input_dev, producer_layer=None, producer_pool=None) -> int:
    out = C.c_void_p()
    _check(lib().cb_process_frame_propagated(layer, _ptr(input_dev), producer_layer, producer_pool, C.byref(out)),
           "cb_process_frame_propagated")
    return out.value


def cb_process_frame_chained(layer: int, input_dev, producer_layer=None, producer_pool=None, tau: float = 0.0) -> int:
    out = C.c_void_p()
    _check(lib().cb_process_frame_chained(layer, _ptr(input_dev), producer_layer, producer_pool, C.c_float(tau),
                                          C.byref(out)), "cb_process_frame_chained")
    return out.value


def cb_layer_changes(layer: int) -> Tuple[int, int, int, int]:
    a, b, c, d = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib().cb_layer_changes(layer, C.byref(a), C.byref(b), C.byref(c), C.byref(d)), "cb_layer_changes")
    return a.value, b.value, c.value, d.value


def cb_layer_state(layer: int) -> int:
    a = C.c_void_p()
    _check(lib().cb_layer_state(layer, C.byref(a)), "cb_layer_state")
    return a.value


def cb_layer_export_state(layer: int, state_out, output_out) -> None:
    _check(lib().cb_layer_export_state(layer, _ptr(state_out), _ptr(output_out)), "cb_layer_export_state")


def cb_layer_import_state(layer: int, state_in, output_in) -> None:
    _check(lib().cb_layer_import_state(layer, _ptr(state_in), _ptr(output_in)), "cb_layer_import_state")


def cb_layer_matrices(layer: int) -> Tuple[int, int, int]:
    a, b, c = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib().cb_layer_matrices(layer, C.byref(a), C.byref(b), C.byref(c)), "cb_layer_matrices")
    return a.value, b.value, c.value


def cb_layer_out_shape(layer: int) -> Tuple[int, int, int]:
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().cb_layer_out_shape(layer, C.byref(a), C.byref(b), C.byref(c)), "cb_layer_out_shape")
    return a.value, b.value, c.value


def cb_layer_set_timing(layer: int, on: bool) -> None:
    _check(lib().cb_layer_set_timing(layer, int(on)), "cb_layer_set_timing")


def cb_layer_stats(layer: int) -> dict:
    s = cb_stats()
    _check(lib().cb_layer_stats(layer, C.byref(s)), "cb_layer_stats")
    return {"n_changed_in": s.n_changed_in, "n_changed_out": s.n_changed_out, "ops": s.ops,
            "us_step": {n: float(s.us_step[i]) for i, n in enumerate(STEP_NAMES)}, "scan_recounts": s.scan_recounts}


def cb_set_scan_wait_limit(polls: int) -> None:
    _check(lib().cb_set_scan_wait_limit(int(polls)), "cb_set_scan_wait_limit")


def cb_layer_reset(layer: int) -> None:
    _check(lib().cb_layer_reset(layer), "cb_layer_reset")


def cb_layer_destroy(layer: int) -> None:
    _check(lib().cb_layer_destroy(layer), "cb_layer_destroy")


def cb_pool_workspace_bytes(producer: int, window: int = 2) -> int:
    a = C.c_size_t()
    _check(lib().cb_pool_workspace_bytes(producer, window, C.byref(a)), "cb_pool_workspace_bytes")
    return a.value


def cb_pool_create(producer: int, window, state_dev, state_bytes, stream=0) -> int:
    h = C.c_void_p()
    _check(lib().cb_pool_create(producer, window, _ptr(state_dev), state_bytes, stream or None, C.byref(h)),
           "cb_pool_create")
    return h.value


def cb_pool_process(pool: int) -> int:
    out = C.c_void_p()
    _check(lib().cb_pool_process(pool, C.byref(out)), "cb_pool_process")
    return out.value


def cb_pool_changes(pool: int) -> int:
    a = C.c_void_p()
    _check(lib().cb_pool_changes(pool, C.byref(a)), "cb_pool_changes")
    return a.value


def cb_pool_out_shape(pool: int) -> Tuple[int, int, int]:
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().cb_pool_out_shape(pool, C.byref(a), C.byref(b), C.byref(c)), "cb_pool_out_shape")
    return a.value, b.value, c.value


def cb_pool_destroy(pool: int) -> None:
    _check(lib().cb_pool_destroy(pool), "cb_pool_destroy")


# ---------------------------------------------------------------- device-memory helpers
_TORCH_DT = {CB_F32: torch.float32, CB_BF16: torch.bfloat16}


def _alloc(nbytes: int, device) -> torch.Tensor:
    """256-byte aligned byte buffer from torch's allocator."""
    t = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    off = (-t.data_ptr()) % 256
    return t[off:off + nbytes]


def _view(owner: torch.Tensor, ptr: int, shape, dtype) -> torch.Tensor:
    """Tensor view of memory at `ptr` inside the byte buffer `owner`."""
    n = 1
    for s in shape:
        n *= s
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    off = ptr - owner.data_ptr()
    assert 0 <= off and off + nbytes <= owner.numel(), "pointer outside its owner buffer"
    return owner[off:off + nbytes].view(dtype).view(*shape)


class Layer:
    """A cb_layer with its buffers held by torch tensors (memory plumbing only)."""

    def __init__(self, weight: torch.Tensor, bias: Optional[torch.Tensor], stride: int, pad: int, h_in: int,
                 w_in: int, relu: bool, mode: int = CB_CLOSED_LOOP, scratch: Optional[torch.Tensor] = None,
                 scratch_bytes: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None,
                 backend: int = CB_BACKEND_AUTO, keep_output_channel_last: bool = False,
                 gather_channel_last: bool = False):
        assert weight.is_cuda and weight.is_contiguous()
        self.device = weight.device
        self.dtype = CB_BF16 if weight.dtype == torch.bfloat16 else CB_F32
        assert weight.dtype in (torch.float32, torch.bfloat16)
        O, Cc, kh, kw = weight.shape
        self.desc = make_desc(Cc, O, kh, kw, stride, pad, h_in, w_in, self.dtype, relu, mode, backend,
                              keep_output_channel_last, gather_channel_last)
        state_bytes, rec_scratch = cb_layer_workspace_bytes(self.desc)
        self.state_buf = _alloc(state_bytes, self.device)
        if scratch is None:
            scratch = _alloc(scratch_bytes if scratch_bytes is not None else rec_scratch, self.device)
        self.scratch_buf = scratch
        self.stream = stream
        sh = stream.cuda_stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream
        self.stream_handle = sh
        if bias is not None:
            assert bias.dtype == weight.dtype and bias.is_contiguous()
        self.handle = cb_layer_create(self.desc, weight, bias, self.state_buf, self.state_buf.numel(),
                                      self.scratch_buf, self.scratch_buf.numel(), sh)
        self.C, self.H, self.W = Cc, h_in, w_in
        self.O, self.Ho, self.Wo = cb_layer_out_shape(self.handle)
        self._keep = (weight, bias)

    def close(self):
        if getattr(self, "handle", None):
            cb_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def process_frame(self, x: torch.Tensor, tau: float) -> torch.Tensor:
        assert x.is_cuda and x.is_contiguous() and x.dtype == _TORCH_DT[self.dtype]
        assert tuple(x.shape[-3:]) == (self.C, self.H, self.W), (tuple(x.shape), (self.C, self.H, self.W))
        p = cb_process_frame(self.handle, x, tau)
        return _view(self.state_buf, p, (self.O, self.Ho, self.Wo), _TORCH_DT[self.dtype])

    def process_frame_chained(self, x: torch.Tensor, producer, tau: float) -> torch.Tensor:
        assert x.is_cuda and x.is_contiguous() and x.dtype == _TORCH_DT[self.dtype]
        assert tuple(x.shape[-3:]) == (self.C, self.H, self.W)
        if isinstance(producer, Pool):
            p = cb_process_frame_chained(self.handle, x, None, producer.handle, tau)
        else:
            p = cb_process_frame_chained(self.handle, x, producer.handle, None, tau)
        return _view(self.state_buf, p, (self.O, self.Ho, self.Wo), _TORCH_DT[self.dtype])

    def process_frame_propagated(self, x: torch.Tensor, producer) -> torch.Tensor:
        assert x.is_cuda and x.is_contiguous() and x.dtype == _TORCH_DT[self.dtype]
        assert tuple(x.shape[-3:]) == (self.C, self.H, self.W)
        if isinstance(producer, Pool):
            p = cb_process_frame_propagated(self.handle, x, None, producer.handle)
        else:
            p = cb_process_frame_propagated(self.handle, x, producer.handle, None)
        return _view(self.state_buf, p, (self.O, self.Ho, self.Wo), _TORCH_DT[self.dtype])

    def changes(self):
        """(m, m~, idx, N) of the last frame as device tensors (idx is sliced to N on the host)."""
        m, mt, idx, cnt = cb_layer_changes(self.handle)
        m_t = _view(self.state_buf, m, (self.H, self.W), torch.uint8)
        mt_t = _view(self.state_buf, mt, (self.Ho, self.Wo), torch.uint8)
        return m_t, mt_t, idx, cnt

    def changes_host(self):
        import numpy as np
        m, mt, idx_p, cnt_p = cb_layer_changes(self.handle)
        m_t = _view(self.state_buf, m, (self.H, self.W), torch.uint8).cpu().numpy()
        mt_t = _view(self.state_buf, mt, (self.Ho, self.Wo), torch.uint8).cpu().numpy()
        n = cb_layer_stats(self.handle)["n_changed_out"]
        idx = _raw_to_host(idx_p, n, self.device)
        return m_t, mt_t, idx.astype(np.int32), n

    def state(self) -> torch.Tensor:
        return _view(self.state_buf, cb_layer_state(self.handle), (self.C, self.H, self.W), _TORCH_DT[self.dtype])

    def export_state(self):
        """(input state or None for a CB_PROPAGATE layer, cached output) as new tensors."""
        dt = _TORCH_DT[self.dtype]
        st = None if self.desc.mode == CB_PROPAGATE else torch.empty((self.C, self.H, self.W), dtype=dt, device=self.device)
        out = torch.empty((self.O, self.Ho, self.Wo), dtype=dt, device=self.device)
        cb_layer_export_state(self.handle, st, out)
        return st, out

    def import_state(self, state: Optional[torch.Tensor], out: torch.Tensor):
        dt = _TORCH_DT[self.dtype]
        assert out.is_cuda and out.is_contiguous() and out.dtype == dt and tuple(out.shape) == (self.O, self.Ho, self.Wo)
        if state is not None:
            assert state.is_cuda and state.is_contiguous() and state.dtype == dt
            assert tuple(state.shape) == (self.C, self.H, self.W)
        cb_layer_import_state(self.handle, state, out)

    def stats(self) -> dict:
        return cb_layer_stats(self.handle)

    def set_timing(self, on: bool):
        cb_layer_set_timing(self.handle, on)

    def reset(self):
        cb_layer_reset(self.handle)


def _raw_to_host(ptr: int, n: int, device):
    """Copy n int32 from a raw device pointer to a numpy array (hipMemcpy through torch's HIP runtime)."""
    import numpy as np
    out = np.zeros(n, np.int32)
    if n == 0:
        return out
    hip = _hip_runtime()
    torch.cuda.synchronize(device)
    rc = hip.hipMemcpy(C.c_void_p(out.ctypes.data), C.c_void_p(ptr), C.c_size_t(4 * n), 2)
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed: {rc}")
    return out


_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        for name in ("libamdhip64.so", "libamdhip64.so.7", "libamdhip64.so.6"):
            try:
                _hip = C.CDLL(name)
                break
            except OSError:
                continue
        if _hip is None:
            _hip = C.CDLL(os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib", "libamdhip64.so"))
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemcpy.restype = C.c_int
    return _hip


def cb_sum_squared_diff(a_dev, b_dev, n: int, dtype: int, workspace_dev, stream=0) -> float:
    out = C.c_double()
    _check(lib().cb_sum_squared_diff(_ptr(a_dev), _ptr(b_dev), n, dtype, _ptr(workspace_dev), C.byref(out),
                                     stream or None), "cb_sum_squared_diff")
    return out.value


def cb_sum_squared_diff_noalloc(a_dev, b_dev, n: int, dtype: int, stream=0) -> float:
    out = C.c_double()
    _check(lib().cb_sum_squared_diff_noalloc(_ptr(a_dev), _ptr(b_dev), n, dtype, C.byref(out), stream or None),
           "cb_sum_squared_diff_noalloc")
    return out.value


class Network:
    """A chain of Layer objects, each optionally followed by its Pool (cb_stage array of the C ABI)."""

    def __init__(self, layers, pools=None):
        pools = pools if pools is not None else [None] * len(layers)
        assert len(pools) == len(layers)
        self.layers, self.pools = list(layers), list(pools)
        self.n = len(layers)
        self.stages = (cb_stage * self.n)()
        for s in range(self.n):
            self.stages[s].layer = self.layers[s].handle
            self.stages[s].pool = self.pools[s].handle if self.pools[s] is not None else None
        last = self.pools[-1] if self.pools[-1] is not None else self.layers[-1]
        self.out_shape = (last.O, last.Hp, last.Wp) if self.pools[-1] is not None else (last.O, last.Ho, last.Wo)
        self._out_buf = last.state_buf
        self.dtype = self.layers[-1].dtype
        self.device = self.layers[0].device

    def reset(self):
        for L in self.layers:
            L.reset()

    def forward(self, x: torch.Tensor, taus) -> torch.Tensor:
        assert x.is_cuda and x.is_contiguous() and len(taus) == self.n
        t = (C.c_float * self.n)(*[float(v) for v in taus])
        out = C.c_void_p()
        _check(lib().cb_network_forward(self.stages, self.n, _ptr(x), t, C.byref(out)), "cb_network_forward")
        return _view(self._out_buf, out.value, self.out_shape, _TORCH_DT[self.dtype])

    def select_thresholds(self, sequences, tau0: float, factor: float, max_loss, max_steps: int = 200):
        """Sec. III-F threshold selection over `sequences` (lists of equally many device frames).
        Returns (thresholds, loss at each selected threshold, thresholds tried per stage)."""
        n_seq, n_frames = len(sequences), len(sequences[0])
        assert all(len(sq) == n_frames for sq in sequences) and len(max_loss) == self.n
        ptrs = (C.c_void_p * (n_seq * n_frames))(*[_ptr(f) for sq in sequences for f in sq])
        nbytes = C.c_size_t()
        _check(lib().cb_select_workspace_bytes(self.stages, self.n, n_seq, C.byref(nbytes)),
               "cb_select_workspace_bytes")
        ws = _alloc(nbytes.value, self.device)
        prm = cb_select_params(float(tau0), float(factor), int(max_steps), 0)
        ml = (C.c_double * self.n)(*[float(v) for v in max_loss])
        taus, loss, steps = (C.c_float * self.n)(), (C.c_double * self.n)(), (C.c_int32 * self.n)()
        _check(lib().cb_select_thresholds(self.stages, self.n, ptrs, n_seq, n_frames, C.byref(prm), ml, _ptr(ws),
                                          nbytes.value, taus, loss, steps), "cb_select_thresholds")
        return list(taus), list(loss), list(steps)


class Pool:
    """A cb_pool fed by a Layer."""

    def __init__(self, producer: Layer, window: int = 2):
        self.producer = producer
        nbytes = cb_pool_workspace_bytes(producer.handle, window)
        self.state_buf = _alloc(nbytes, producer.device)
        self.handle = cb_pool_create(producer.handle, window, self.state_buf, self.state_buf.numel(),
                                     producer.stream_handle)
        self.O, self.Hp, self.Wp = cb_pool_out_shape(self.handle)
        self.dtype = producer.dtype
        self.stream_handle = producer.stream_handle
        self.device = producer.device

    def close(self):
        if getattr(self, "handle", None):
            cb_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def process(self) -> torch.Tensor:
        p = cb_pool_process(self.handle)
        return _view(self.state_buf, p, (self.O, self.Hp, self.Wp), _TORCH_DT[self.dtype])

    def changes(self) -> torch.Tensor:
        return _view(self.state_buf, cb_pool_changes(self.handle), (self.Hp, self.Wp), torch.uint8)
