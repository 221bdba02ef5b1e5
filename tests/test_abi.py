"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/cbconv.h declares, validates descriptors and sizes."""
import ctypes as C
import os
import re

import pytest

import paper_1808_05488_amd as cb
from paper_1808_05488_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cbconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cb_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported():
    names = declared_functions()
    assert len(names) >= 20
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in cbconv.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_version_and_strerror():
    assert cb.cb_version() >= 100
    L = binding.lib()
    assert L.cb_strerror(0) == b"success"
    for code in (-1, -2, -3, -4, -99):
        assert len(L.cb_strerror(code)) > 0


def test_workspace_sizes_follow_the_geometry():
    d = cb.make_desc(64, 64, 3, 3, 1, 1, 480, 640, backend=cb.CB_BACKEND_EXPLICIT)
    state, scratch = cb.cb_layer_workspace_bytes(d)
    P = 480 * 640
    # input state + cached output dominate the per-layer state (Fig. 2: variables stored per layer)
    assert state >= 2 * 64 * P * 4
    assert state < 2 * 64 * P * 4 + 16 * P + (1 << 20)
    R = 64 * 9
    assert scratch >= (R + 64) * P * 4            # X' and Y' for a full update in one chunk
    assert cb.cb_layer_min_scratch_bytes(d) < scratch
    # a propagating layer keeps no input state (Sec. III-E)
    dp = cb.make_desc(64, 64, 3, 3, 1, 1, 480, 640, mode=cb.CB_PROPAGATE, backend=cb.CB_BACKEND_EXPLICIT)
    assert cb.cb_layer_workspace_bytes(dp)[0] <= state - 64 * P * 4
    # bf16 halves the tensors
    db = cb.make_desc(64, 64, 3, 3, 1, 1, 480, 640, dtype=cb.CB_BF16, backend=cb.CB_BACKEND_EXPLICIT)
    assert cb.cb_layer_workspace_bytes(db)[0] < 0.6 * state
    # the fused back end needs no X' / Y' scratch; it covers filters of up to 60 taps
    df = cb.make_desc(64, 64, 3, 3, 1, 1, 480, 640, backend=cb.CB_BACKEND_FUSED)
    assert cb.cb_layer_workspace_bytes(df)[1] < (1 << 20)
    dw = cb.make_desc(2, 2, 8, 8, 1, 3, 64, 64, backend=cb.CB_BACKEND_FUSED)
    with pytest.raises(binding.CBError):
        cb.cb_layer_workspace_bytes(dw)
    dw.backend = cb.CB_BACKEND_AUTO          # falls back to the explicit kernels
    assert cb.cb_layer_workspace_bytes(dw)[1] > (1 << 20)


def test_which_layers_keep_a_channel_last_shadow_of_the_state():
    """Closed-loop layers on the fused back end with a power-of-two channel count from 16 (float32) / 32 (bfloat16) on
    keep a second, pixel-major copy of the input state: one more C*P*b bytes."""
    def state_bytes(C, H=120, W=160, **kw):
        return cb.cb_layer_workspace_bytes(cb.make_desc(C, 32, 3, 3, 1, 1, H, W, backend=cb.CB_BACKEND_FUSED, **kw))[0]
    P = 120 * 160
    for C in (16, 32, 64, 128, 256, 512):
        extra = state_bytes(C) - state_bytes(C, mode=cb.CB_FEED_FORWARD)
        assert C * P * 4 <= extra < C * P * 4 + 4096, C
    for C in (3, 8, 24, 48, 96):
        assert state_bytes(C) == state_bytes(C, mode=cb.CB_FEED_FORWARD), C
    # bfloat16 layers from 32 channels on (half the bytes); layers on the explicit back end keep none
    extra = state_bytes(64, dtype=cb.CB_BF16) - state_bytes(64, dtype=cb.CB_BF16, mode=cb.CB_FEED_FORWARD)
    assert 64 * P * 2 <= extra < 64 * P * 2 + 4096
    assert state_bytes(16, dtype=cb.CB_BF16) == state_bytes(16, dtype=cb.CB_BF16, mode=cb.CB_FEED_FORWARD)
    de = [cb.cb_layer_workspace_bytes(cb.make_desc(64, 32, 3, 3, 1, 1, 120, 160, backend=cb.CB_BACKEND_EXPLICIT, mode=m))[0]
          for m in (cb.CB_CLOSED_LOOP, cb.CB_FEED_FORWARD)]
    assert de[0] == de[1]
    # states beyond the last-level cache too (1080p x 128 channels = 1 GB)
    assert state_bytes(128, 1080, 1920) - state_bytes(128, 1080, 1920, mode=cb.CB_FEED_FORWARD) >= 128 * 1080 * 1920 * 4
    assert state_bytes(64, 480, 640) - state_bytes(64, 480, 640, mode=cb.CB_FEED_FORWARD) >= 64 * 480 * 640 * 4


@pytest.mark.parametrize("field,value", [("c_in", 0), ("c_out", -1), ("kh", 0), ("kw", 32), ("stride", 0),
                                         ("pad", -1), ("pad", 32), ("h_in", 0), ("dtype", 2), ("relu", 2),
                                         ("mode", 3), ("backend", 3)])
def test_invalid_descriptors_are_rejected(field, value):
    d = cb.make_desc(3, 4, 3, 3, 1, 1, 16, 16)
    setattr(d, field, value)
    with pytest.raises(binding.CBError) as e:
        cb.cb_layer_workspace_bytes(d)
    assert e.value.status == cb.CB_EINVAL


def test_kernel_larger_than_padded_input_is_rejected():
    d = cb.make_desc(3, 4, 7, 7, 1, 0, 5, 5)
    with pytest.raises(binding.CBError):
        cb.cb_layer_workspace_bytes(d)
    d.reserved[1] = 1
    d.kh = d.kw = 3
    with pytest.raises(binding.CBError):
        cb.cb_layer_workspace_bytes(d)


def test_null_arguments():
    L = binding.lib()
    assert L.cb_layer_workspace_bytes(None, None, None) == cb.CB_EINVAL
    assert L.cb_process_frame(None, None, C.c_float(0.0), None) == cb.CB_EINVAL
    assert L.cb_layer_destroy(None) == cb.CB_EINVAL
    assert L.cb_pool_process(None, None) == cb.CB_EINVAL
    h = C.c_void_p()
    d = cb.make_desc(3, 4, 3, 3, 1, 1, 16, 16)
    assert L.cb_layer_create(C.byref(d), None, None, None, 0, None, 0, None, C.byref(h)) == cb.CB_EINVAL
    assert h.value is None
