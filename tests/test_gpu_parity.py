"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Masks, index lists, counts and the input state must
match bit for bit; outputs within 1e-4 (float32) / 1e-2 (bfloat16)."""
import numpy as np
import pytest
import torch

import synth_inputs as syn

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_1808_05488_amd as cb
    from oracle import cb_oracle as orc
    from parity import Pair, assert_close, to_dev, to_host, prep


def _say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------- config 1 (full size)
# (bf16, back end): 1 = explicit gather / GEMM / update kernels, 2 = fused kernel
VARIANTS = [(False, 1), (False, 2), (True, 1), (True, 2)]


@pytest.mark.parametrize("bf16,backend", VARIANTS)
def test_config1(bf16, backend):
    wl = syn.config1()
    _say(f"config1 bf16={bf16} backend={backend}")
    p = Pair(wl.layers[0], wl.H, wl.W, bf16=bf16, backend=backend)
    ns = []
    for t, f in enumerate(wl.frames()):
        _, n = p.step(f, wl.tau, tag=f"c1 frame {t}")
        ns.append(n)
    assert ns[0] == wl.H * wl.W
    assert 64 <= ns[1] <= 400          # the 8x8 block plus its halo, plus a few noise pixels


# ---------------------------------------------------------------- geometry sweep
GEOMS = [  # C, O, kh(=kw), s, p, H, W
    (3, 4, 3, 1, 1, 9, 11),
    (2, 3, 1, 1, 0, 7, 5),
    (2, 5, 7, 1, 3, 12, 13),
    (3, 2, 5, 2, 2, 11, 14),
    (4, 2, 3, 2, 0, 10, 9),
    (3, 3, 7, 3, 1, 15, 16),
    (8, 16, 3, 1, 1, 37, 83),      # channel-split detect, scalar pixel path (P % 4 != 0)
    (16, 33, 3, 1, 1, 40, 132),    # vector path, O not a multiple of the row tile, W > 128
    (5, 70, 5, 1, 2, 33, 70),
    (12, 8, 1, 1, 0, 64, 64),
    (2, 2, 3, 1, 4, 6, 7),         # padding beyond the half kernel: outputs that only see padding
    (2, 3, 3, 1, 1, 150, 520),     # 1350 words of dilated map: the many-workgroup single-pass index extraction
    (1, 2, 5, 1, 2, 131, 1100),    # 2358 words, ragged last word of every row and a ragged last workgroup
    (2, 2, 3, 2, 1, 300, 1030),    # the same kernel with stride 2
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bf16,backend", VARIANTS)
def test_geometry_sweep(geom, bf16, backend):
    C, O, k, s, pd, H, W = geom
    _say(f"sweep {geom} bf16={bf16} backend={backend}")
    spec, frames = syn.random_layer_case(sum(geom), C, O, k, s, pd, H, W, 5, change_prob=0.04, relu=True,
                                         noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=backend)
    frames = frames + [frames[-1]]                 # identical frame: N = 0
    for t, f in enumerate(frames):
        _, n = p.step(f, 0.02, tag=f"{geom} frame {t}")
    assert n == 0
    # a frame that differs everywhere: every output listed again
    _, n = p.step(frames[-1] + np.float32(0.5), 0.02, tag=f"{geom} all changed")
    if pd <= (k - 1) // 2:              # otherwise some outputs see nothing but padding
        assert n == p.o.Ho * p.o.Wo


@pytest.mark.parametrize("backend", [1, 2])
def test_nonsquare_kernel(backend):
    rng = np.random.default_rng(5)
    C, O, kh, kw, H, W = 3, 6, 3, 5, 20, 31
    spec = syn.ConvSpec(C, O, kh, 1, 1, True, False, rng.standard_normal((O, C, kh, kw)).astype(np.float32),
                        rng.standard_normal(O).astype(np.float32))
    _, frames = syn.random_layer_case(9, C, O, 3, 1, 1, H, W, 4, change_prob=0.05)
    p = Pair(spec, H, W, backend=backend)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"3x5 frame {t}")


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(32, 72, 1, 17, 8, 130, 160),    # more than 16 384 listed pixels: wide tiles
                                   (16, 8, 17, 1, 0, 60, 50),        # up to 16 output channels
                                   (64, 40, 2, 18, 1, 50, 120),      # 33 - 64
                                   (32, 24, 1, 1, 0, 2, 4100)])      # an output row of more than 4 095 pixels
def test_channel_last_layers_beyond_the_double_buffered_kernels_limits(shape, bf16):
    """Filters of more than 16 rows or columns, and maps wider than 4 095 pixels, run the channel-last kernel's
    older body (stages of several units behind a barrier pair; tap masks of 64 bits, a division per column)."""
    C, O, kh, kw, pd, H, W = shape
    _say(f"channel-last, outside the double-buffered body: {shape} bf16={bf16}")
    rng = np.random.default_rng(kh * 100 + kw)
    spec = syn.ConvSpec(C, O, kh, 1, pd, True, False,
                        (rng.standard_normal((O, C, kh, kw)) * np.sqrt(2.0 / (C * kh * kw))).astype(np.float32),
                        (rng.standard_normal(O) * 0.1).astype(np.float32))
    _, frames = syn.random_layer_case(kh + kw, C, O, 3, 1, 1, H, W, 4, change_prob=0.02, noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=2)
    for t, f in enumerate(frames):
        p.step(f if t != 2 else f + np.float32(0.5), 0.02, tag=f"{shape} frame {t}")


def test_threshold_zero_and_no_relu_no_bias():
    spec, frames = syn.random_layer_case(3, 6, 10, 3, 1, 1, 24, 40, 4, change_prob=0.1, relu=False, noise_std=1e-5)
    spec.bias = None
    p = Pair(spec, 24, 40)
    for t, f in enumerate(frames):
        out, _ = p.step(f, 0.0, tag=f"tau0 frame {t}")
        dense = orc.dense_conv(prep(f, False), p.w, None, 1, 1, False)
        assert_close(out, dense, False, "tau=0 vs dense layer")


def test_feed_forward_mode():
    spec, frames = syn.random_layer_case(4, 5, 7, 3, 1, 1, 20, 28, 6, change_prob=0.05, noise_std=0.008)
    p = Pair(spec, 20, 28, feed_forward=True)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"ff frame {t}")


def test_reset_forces_full_update():
    spec, frames = syn.random_layer_case(6, 4, 4, 3, 1, 1, 16, 20, 3, change_prob=0.05)
    p = Pair(spec, 16, 20)
    p.step(frames[0], 0.02)
    p.step(frames[1], 0.02)
    p.g.reset()
    p.o.reset()
    _, n = p.step(frames[2], 5.0, tag="after reset")
    assert n == 16 * 20


# ---------------------------------------------------------------- config 2 recipe, reduced and chunked
@pytest.mark.parametrize("bf16,backend", VARIANTS)
def test_config2_reduced(bf16, backend):
    wl = syn.config2(H=96, W=160, C=64, O=64, n_frames=6, rect=16)
    _say(f"config2 reduced bf16={bf16} backend={backend}")
    p = Pair(wl.layers[0], wl.H, wl.W, bf16=bf16, backend=backend)
    for t, f in enumerate(wl.frames()):
        _, n = p.step(f, wl.tau, tag=f"c2r frame {t}")
        if t:
            assert 0 < n < 0.25 * wl.H * wl.W


# long K (the chunked gather of the fused back end; float32 switches to runs of four taps above 2048 rows)
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", [(128, 40, 3, 24, 32), (48, 200, 7, 21, 30), (260, 16, 3, 30, 44), (40, 24, 5, 17, 23)])
def test_fused_long_k(geom, bf16):
    C, O, k, H, W = geom
    _say(f"long K {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(C + O, C, O, k, 1, k // 2, H, W, 4, change_prob=0.01, relu=True,
                                         noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=2)
    ns = []
    for t, f in enumerate(frames):
        _, n = p.step(f, 0.02, tag=f"long K {geom} frame {t}")
        ns.append(n)
    assert ns[0] == H * W and 0 < min(ns[1:]) < ns[0]


# Kernel variants that the configurations above do not reach: change detection with more channels than the
# register-resident variants hold (more than 512, or more than 128 on maps of 65 536 pixels and more, where a lane
# takes four pixels), and the 64-column tile of the fused kernels for 17 - 32 output channels (16 384 listed pixels
# and more).
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", [(520, 6, 1, 1, 0, 10, 12), (136, 4, 1, 1, 0, 256, 260), (3, 24, 3, 1, 1, 150, 130)])
def test_rarely_taken_kernel_variants(geom, bf16):
    C, O, k, s, pd, H, W = geom
    _say(f"variant {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(sum(geom) + 3, C, O, k, s, pd, H, W, 3, change_prob=0.02, relu=True,
                                         noise_std=0.004)
    for backend in (2, 1):
        p = Pair(spec, H, W, bf16=bf16, backend=backend)
        for t, f in enumerate(frames):
            _, n = p.step(f, 0.02, tag=f"variant {geom} backend {backend} frame {t}")
            assert (n == p.o.Ho * p.o.Wo) if t == 0 else (0 < n < p.o.Ho * p.o.Wo)


# The float32 fused kernel takes a 32-column tile when the filter is short (at most 24 units of 64 rows of K), the
# narrow tiles would number more than 512 and fewer than 16 384 pixels are listed: full-update frames of these maps.
# K = 72 / 100 / 8 leave padding rows in the last unit, which that kernel clears itself when it gathers runs of taps.
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", [(8, 64, 3, 100, 120), (4, 130, 5, 64, 150), (8, 48, 1, 90, 101)])
def test_fused_mid_column_tile(geom, bf16):
    C, O, k, H, W = geom
    _say(f"mid tile {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(C * O + k, C, O, k, 1, k // 2, H, W, 3, change_prob=0.02, relu=True,
                                         noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=2)
    _, n = p.step(frames[0], 0.02, tag=f"mid tile {geom} full update")
    assert n == H * W and 512 * 16 < n < 16384
    _, n = p.step(frames[1], 0.02, tag=f"mid tile {geom} frame 1")
    assert 0 < n < H * W
    _, n = p.step(frames[2] + np.float32(0.5), 0.02, tag=f"mid tile {geom} all changed")
    assert n == H * W


SHADOW_GEOMS = [
    # C, O, k, stride, pad, H, W -- power-of-two channel counts from 16 (float32) / 32 (bfloat16) on: closed-loop layers
    # on the fused back end keep a channel-last shadow of the state.  One case per change-detection variant that updates it
    # (channel groups x channels per lane; four pixels per lane from 65 536 pixels on; 16-pixel workgroups below
    # 8 192 pixels) and per tile shape of the fused kernel that reads it.
    (16, 8, 3, 1, 1, 70, 90), (32, 24, 5, 2, 2, 61, 77), (64, 40, 3, 1, 1, 256, 260), (128, 72, 3, 1, 1, 40, 50),
    (128, 130, 1, 1, 0, 96, 100), (256, 20, 3, 1, 1, 30, 40), (256, 16, 1, 1, 0, 100, 90), (512, 12, 3, 1, 0, 20, 24),
    (512, 8, 1, 1, 0, 92, 90), (16, 70, 7, 1, 3, 50, 60), (32, 33, 3, 1, 1, 64, 64), (128, 8, 1, 1, 0, 256, 260),
    (16, 8, 1, 1, 0, 256, 260), (32, 8, 1, 1, 0, 256, 260), (64, 64, 3, 1, 1, 100, 120),
    (1024, 8, 1, 1, 0, 12, 16),      # more channels than the register-resident detection variants hold: looped variant
    (16, 24, 1, 1, 0, 130, 130),     # 17-32 output channels on more than 16 384 pixels: 32 x 64 tiles
    (32, 130, 3, 1, 1, 60, 100),     # 128 x 32 tiles (6 000 pixels, two row tiles: one round of wide tiles against two)
    # more than 64 output channels on more than 16 384 pixels: bfloat16 runs 128 x 128 tiles with two alternating
    # stage buffers (ragged row tiles, ragged last column tile, several taps per 256-byte unit, stride 2, 1x1)
    (32, 72, 3, 1, 1, 130, 140), (64, 130, 3, 1, 1, 129, 131), (32, 96, 5, 2, 2, 270, 262), (128, 128, 1, 1, 0, 130, 130),
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", SHADOW_GEOMS)
def test_channel_last_shadow(geom, bf16):
    C, O, k, s, pd, H, W = geom
    _say(f"shadow {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(sum(geom) + 7, C, O, k, s, pd, H, W, 5, change_prob=0.03, relu=True,
                                         noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=2)
    _, n = p.step(frames[0], 0.02, tag=f"shadow {geom} full update")
    assert n == p.o.Ho * p.o.Wo
    _, n = p.step(frames[1], 0.02, tag=f"shadow {geom} frame 1")
    assert 0 < n < p.o.Ho * p.o.Wo
    _, n = p.step(frames[2] + np.float32(0.5), 0.02, tag=f"shadow {geom} all changed")
    assert n == p.o.Ho * p.o.Wo
    p.step(frames[3], 0.02, tag=f"shadow {geom} all changed back")
    p.step(frames[4], 0.02, tag=f"shadow {geom} frame 4")


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", [(3, 4, 5, 1, 2, 200, 181), (2, 5, 3, 2, 1, 370, 361), (5, 3, 1, 1, 0, 190, 175)])
def test_explicit_gather_with_many_columns(geom, bf16):
    """From 32 768 listed pixels on the matrix-generation kernel gives every lane four columns
    (full-update frames here; the later frames use the one-column form)."""
    C, O, k, s, pd, H, W = geom
    _say(f"many columns {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(sum(geom) + 1, C, O, k, s, pd, H, W, 3, change_prob=0.03, noise_std=0.004)
    p = Pair(spec, H, W, bf16=bf16, backend=1)
    _, n = p.step(frames[0], 0.02, tag=f"{geom} full update")
    assert n == p.o.Ho * p.o.Wo and n >= 32768
    p.step(frames[1], 0.02, tag=f"{geom} frame 1")
    _, n = p.step(frames[2] + np.float32(0.5), 0.02, tag=f"{geom} all changed")
    assert n == p.o.Ho * p.o.Wo


def test_multiple_column_chunks():
    """A scratch buffer of the minimum size forces the listed pixels through
    many 256-column chunks."""
    wl = syn.config2(H=48, W=80, C=16, O=24, n_frames=4, rect=12)
    spec = wl.layers[0]
    d = cb.make_desc(16, 24, 3, 3, 1, 1, 48, 80, backend=1)
    p = Pair(spec, wl.H, wl.W, scratch_bytes=cb.cb_layer_min_scratch_bytes(d), backend=1)
    for t, f in enumerate(wl.frames()):
        p.step(f, wl.tau, tag=f"chunked frame {t}")


def test_xprime_is_the_listed_columns_of_the_image_matrix():
    """X'(r, n) = S(c, yo*s-p+j, xo*s-p+i) with r = (c*kh+j)*kw+i (construction of X below Eq. 2)."""
    C, O, k, s, pd, H, W = 3, 4, 3, 1, 1, 14, 18
    spec, frames = syn.random_layer_case(8, C, O, k, s, pd, H, W, 3, change_prob=0.05)
    p = Pair(spec, H, W, backend=1)
    for f in frames:
        p.step(f, 0.02)
    xp, yp, ldn = cb.cb_layer_matrices(p.g.handle)
    from paper_1808_05488_amd.binding import _raw_to_host
    ld, ncols, nsplit = [int(v) for v in _raw_to_host(ldn, 3, p.g.device)]
    assert nsplit >= 1
    idx = p.o.idx
    assert ncols == idx.size and ld % 256 == 0 and ld >= ncols
    R = C * k * k
    X = _raw_to_host(xp, R * ld, p.g.device).view(np.float32).reshape(R, ld)
    S = p.o.state
    Sp = np.pad(S, ((0, 0), (pd, pd), (pd, pd)))
    for n, q in enumerate(idx):
        yo, xo = divmod(int(q), p.o.Wo)
        col = Sp[:, yo * s:yo * s + k, xo * s:xo * s + k].reshape(-1)
        assert np.array_equal(X[:, n], col)
    assert np.all(X[:, ncols:] == 0)


# ---------------------------------------------------------------- pooling and chained layers
def _pool_check(pool, layer_out, oracle_pool, oracle_layer):
    got = to_host(pool.process())
    pm = orc.pool_update(oracle_layer.out, oracle_layer.idx, oracle_layer.mt, oracle_pool)
    return got, pm


@pytest.mark.parametrize("hw", [(20, 28), (21, 27)])
@pytest.mark.parametrize("bf16", [False, True])
def test_change_based_pool(hw, bf16):
    H, W = hw
    spec, frames = syn.random_layer_case(12, 4, 9, 3, 1, 1, H, W, 5, change_prob=0.04, noise_std=0.002)
    p = Pair(spec, H, W, bf16=bf16)
    pool = cb.Pool(p.g)
    opool = np.zeros((9, -(-H // 2), -(-W // 2)), np.float32)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"pool frame {t}")
        got = to_host(pool.process())
        # oracle pooling on the GPU layer's own cached output (teacher forcing): bit-exact
        gout = to_host(p.g_out)
        pm = orc.pool_update(gout, p.o.idx, p.o.mt, opool)
        assert np.array_equal(got, opool), f"pooled output differs at frame {t}"
        assert np.array_equal(got, orc.pool_dense(gout)), "pooled output is not the dense pool of the cached output"
        assert np.array_equal(pool.changes().cpu().numpy(), pm)


def _run_chain(wl, bf16, frames_limit=None, backend=0, shared_scratch=False, chained=False):
    """Teacher-forced multi-layer parity: each oracle layer is fed the GPU's
    previous-layer output, so both sides see bit-identical inputs.  shared_scratch: all layers
    use ONE scratch buffer (layers on one stream may share it, Sec. III-B)."""
    H, W = wl.H, wl.W
    glayers, gpools, olayers, opools = [], [], [], []
    h, w = H, W
    scratch = None
    if shared_scratch:
        need, hh, ww = 0, H, W
        for spec in wl.layers:
            d = cb.make_desc(spec.c_in, spec.c_out, spec.k, spec.k, spec.stride, spec.pad, hh, ww,
                             dtype=cb.CB_BF16 if bf16 else cb.CB_F32, relu=spec.relu, backend=backend)
            need = max(need, cb.cb_layer_workspace_bytes(d)[1])
            hh, ww = orc.out_hw(hh, ww, spec.k, spec.k, spec.stride, spec.pad)
            if spec.pool:
                hh, ww = -(-hh // 2), -(-ww // 2)
        scratch = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        scratch = scratch[(-scratch.data_ptr()) % 256:][:need]
    for spec in wl.layers:
        wgt, b = prep(spec.weight, bf16), prep(spec.bias, bf16)
        g = cb.Layer(to_dev(wgt, bf16), to_dev(b, bf16), spec.stride, spec.pad, h, w, spec.relu, backend=backend,
                     scratch=scratch)
        o = orc.OracleLayer(wgt, b, spec.stride, spec.pad, h, w, spec.relu, bf16=bf16)
        glayers.append(g)
        olayers.append(o)
        h, w = g.Ho, g.Wo
        if spec.pool:
            gpools.append(cb.Pool(g))
            opools.append(np.zeros((g.O, -(-h // 2), -(-w // 2)), np.float32))
            h, w = gpools[-1].Hp, gpools[-1].Wp
        else:
            gpools.append(None)
            opools.append(None)
    for t, f in enumerate(wl.frames()):
        if frames_limit is not None and t >= frames_limit:
            break
        x = to_dev(prep(f, bf16), bf16)
        for l, spec in enumerate(wl.layers):
            x_host = to_host(x)
            if chained and l > 0:
                # detection only where the producer rewrote its output; the oracle compares everything
                producer = gpools[l - 1] if gpools[l - 1] is not None else glayers[l - 1]
                out = glayers[l].process_frame_chained(x, producer, wl.tau)
            else:
                out = glayers[l].process_frame(x, wl.tau)
            n_o = olayers[l].process(x_host, wl.tau)
            m, mt, idx, n = glayers[l].changes_host()
            tag = f"{wl.name} frame {t} layer {l}"
            assert n == n_o, f"{tag}: N {n} vs {n_o}"
            assert glayers[l].stats()["n_changed_in"] == olayers[l].n_in, f"{tag}: M differs"
            assert np.array_equal(to_host(glayers[l].state()), olayers[l].state), f"{tag}: input state differs"
            assert np.array_equal(m, olayers[l].m) and np.array_equal(mt, olayers[l].mt), f"{tag}: maps differ"
            assert np.array_equal(idx, olayers[l].idx), f"{tag}: index list differs"
            assert_close(to_host(out), olayers[l].out, bf16, tag)
            x = out
            if gpools[l] is not None:
                x = gpools[l].process()
                gout = to_host(out)
                orc.pool_update(gout, olayers[l].idx, olayers[l].mt, opools[l])
                assert np.array_equal(to_host(x), opools[l]), f"{tag}: pooled output differs"
    return glayers


@pytest.mark.parametrize("backend", [1, 2])
def test_config3_reduced_chain(backend):
    wl = syn.config3(H=64, W=96, n_frames=5, widths=(16, 32, 64, 32, 8))
    _say(f"config3 reduced chain backend={backend}")
    _run_chain(wl, False, backend=backend)


@pytest.mark.parametrize("backend", [1, 2])
def test_config4_reduced_chain(backend):
    wl = syn.config4(H=48, W=64, n_frames=4, width_div=8)
    _say(f"config4 reduced chain backend={backend}")
    _run_chain(wl, False, backend=backend)


# ---------------------------------------------------------------- detection restricted to the producer's change set
@pytest.mark.parametrize("bf16", [False, True])
def test_chained_detection_config3(bf16):
    wl = syn.config3(H=64, W=96, n_frames=6, widths=(16, 32, 80, 32, 8))
    _run_chain(wl, bf16, chained=True)


def test_chained_detection_config4():
    wl = syn.config4(H=48, W=64, n_frames=5, width_div=4)
    _run_chain(wl, False, chained=True)


def test_chained_detection_with_repeated_and_fully_changed_frames():
    """No candidates at all (a frame repeated: N = 0 in every layer) and every pixel a candidate."""
    base = syn.config3(H=48, W=64, n_frames=3, widths=(8, 12, 16, 8, 4))
    fr = list(base.frames())
    seq = [fr[0], fr[1], fr[1], fr[1] + np.float32(0.5), fr[2], fr[2]]
    wl = syn.Workload("repeated and fully changed frames", base.layers, base.H, base.W, base.tau, len(seq),
                      lambda: iter(seq))
    _run_chain(wl, False, chained=True)


@pytest.mark.parametrize("widths", [(1, 1, 2, 3, 1), (2, 3, 1, 2, 2)])
def test_chained_detection_with_very_few_channels(widths):
    """Layers with fewer input channels than the listed-pixel kernel has channel groups."""
    wl = syn.config3(H=40, W=56, n_frames=5, widths=widths)
    _run_chain(wl, False, chained=True)


@pytest.mark.parametrize("feed_forward", [False, True])
def test_chained_detection_falls_back_when_a_frame_is_skipped(feed_forward):
    H, W = 30, 44
    spec, frames = syn.random_layer_case(21, 3, 6, 3, 1, 1, H, W, 8, change_prob=0.04, noise_std=0.006)
    rng = np.random.default_rng(4)
    w2 = rng.standard_normal((5, 6, 3, 3)).astype(np.float32) * 0.3
    p = Pair(spec, H, W)
    mode = cb.CB_FEED_FORWARD if feed_forward else cb.CB_CLOSED_LOOP
    g2 = cb.Layer(to_dev(w2, False), None, 1, 1, H, W, True, mode=mode)
    o2 = orc.OracleLayer(w2, None, 1, 1, H, W, True, feed_forward=feed_forward)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"producer frame {t}")
        if t == 3:
            continue                              # the consumer misses this frame of the producer
        x = p.g_out
        # a threshold that drops (frame 6) also ends the lockstep of a closed-loop consumer: pixels the producer
        # left alone are only known to be within the previous threshold of the state
        tau = {6: 0.004, 7: 0.03}.get(t, 0.02)
        if t == 5:
            out = g2.process_frame(x, tau)        # an ordinary call in between also ends the lockstep
        else:
            out = g2.process_frame_chained(x, p.g, tau)
        n_o = o2.process(to_host(x), tau)
        m, mt, idx, n = g2.changes_host()
        tag = f"consumer frame {t}"
        assert n == n_o and np.array_equal(idx, o2.idx), tag
        assert np.array_equal(m, o2.m) and np.array_equal(mt, o2.mt), tag
        assert g2.stats()["n_changed_in"] == o2.n_in, tag
        assert np.array_equal(to_host(g2.state()), o2.state), tag
        assert_close(to_host(out), o2.out, False, tag)


@pytest.mark.parametrize("backend", [1, 2])
def test_chain_with_one_shared_scratch_buffer(backend):
    wl = syn.config3(H=48, W=80, n_frames=4, widths=(16, 32, 48, 16, 8))
    _run_chain(wl, False, backend=backend, shared_scratch=True)


@pytest.mark.parametrize("backend", [1, 2])
def test_config3_reduced_chain_bf16(backend):
    wl = syn.config3(H=48, W=64, n_frames=3, widths=(16, 32, 32, 16, 8))
    _run_chain(wl, True, backend=backend)


# ---------------------------------------------------------------- propagated change sets (Sec. III-E)
def test_propagated_layers():
    H, W = 24, 36
    spec, frames = syn.random_layer_case(15, 3, 6, 3, 1, 1, H, W, 5, change_prob=0.03)
    rng = np.random.default_rng(3)
    w3 = rng.standard_normal((5, 6, 3, 3)).astype(np.float32)
    w1 = rng.standard_normal((7, 6, 1, 1)).astype(np.float32)
    p = Pair(spec, H, W)
    g3 = cb.Layer(to_dev(w3, False), None, 1, 1, H, W, False, mode=cb.CB_PROPAGATE)
    g1 = cb.Layer(to_dev(w1, False), None, 1, 0, H, W, True, mode=cb.CB_PROPAGATE)
    o3 = orc.OracleLayer(w3, None, 1, 1, H, W, False)
    o1 = orc.OracleLayer(w1, None, 1, 0, H, W, True)
    pool = cb.Pool(p.g)
    wq = rng.standard_normal((4, 6, 3, 3)).astype(np.float32)
    gq = cb.Layer(to_dev(wq, False), None, 1, 1, H // 2, W // 2, False, mode=cb.CB_PROPAGATE)
    oq = orc.OracleLayer(wq, None, 1, 1, H // 2, W // 2, False)
    opool = np.zeros((6, H // 2, W // 2), np.float32)
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"prop frame {t}")
        prod_out = p.g_out
        ph = to_host(prod_out)
        for g, o, name in ((g3, o3, "3x3"), (g1, o1, "1x1")):
            out = g.process_frame_propagated(prod_out, p.g)
            n_o = o.process_propagated(ph, p.o.mt)
            m, mt, idx, n = g.changes_host()
            assert n == n_o and np.array_equal(idx, o.idx), f"{name} frame {t}"
            assert np.array_equal(m, o.m) and np.array_equal(mt, o.mt)
            assert_close(to_host(out), o.out, False, f"propagated {name} frame {t}")
        # through a pooling stage
        pooled = pool.process()
        pm = orc.pool_update(ph, p.o.idx, p.o.mt, opool)
        out = gq.process_frame_propagated(pooled, pool)
        n_o = oq.process_propagated(to_host(pooled), pm)
        m, mt, idx, n = gq.changes_host()
        assert n == n_o and np.array_equal(idx, oq.idx) and np.array_equal(m, pm)
        assert_close(to_host(out), oq.out, False, f"propagated after pool frame {t}")


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("geom", [(3, 32, 28, 44), (5, 64, 33, 37), (2, 128, 140, 150)])
def test_propagating_consumers_that_gather_from_a_pixel_major_output(geom, bf16):
    """The producer keeps its cached output pixel-major as well (and so does the pooling stage behind it); its
    CB_PROPAGATE consumers gather from that copy with the channel-last kernel.  Same results as the oracle's
    propagated layers; the last geometry lists more than 16 384 pixels on its first frame (wide tiles)."""
    C1, C2, H, W = geom
    _say(f"propagated, channel-last: {geom} bf16={bf16}")
    spec, frames = syn.random_layer_case(77 + C2, C1, C2, 3, 1, 1, H, W, 5, change_prob=0.03, noise_std=0.004)
    rng = np.random.default_rng(C2)
    p = Pair(spec, H, W, bf16=bf16, keep_output_channel_last=True)
    pool = cb.Pool(p.g)
    Hp, Wp = -(-H // 2), -(-W // 2)
    opool = np.zeros((C2, Hp, Wp), np.float32)
    cons, cons_w = [], []
    for k, s, pad, pooled, O in ((3, 1, 1, False, 40), (1, 1, 0, False, 7), (3, 1, 1, True, 72), (5, 2, 2, True, 20)):
        hh, ww = (Hp, Wp) if pooled else (H, W)
        w = prep(rng.standard_normal((O, C2, k, k)) * np.sqrt(2.0 / (C2 * k * k)), bf16)
        b = prep(rng.standard_normal(O) * 0.1, bf16)
        g = cb.Layer(to_dev(w, bf16), to_dev(b, bf16), s, pad, hh, ww, True, mode=cb.CB_PROPAGATE, gather_channel_last=True)
        o = orc.OracleLayer(w, b, s, pad, hh, ww, True, bf16=bf16)
        cons.append((g, o, pooled, f"k{k} s{s} {'pooled' if pooled else 'direct'}"))
        cons_w.append((w, b))
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"producer frame {t}")
        pooled_out = pool.process()
        pm = orc.pool_update(to_host(p.g_out), p.o.idx, p.o.mt, opool)
        assert np.array_equal(to_host(pooled_out), opool), f"pooled output differs at frame {t}"
        for g, o, pooled, name in cons:
            src, prod, m_in = (pooled_out, pool, pm) if pooled else (p.g_out, p.g, p.o.mt)
            out = g.process_frame_propagated(src, prod)
            n_o = o.process_propagated(to_host(src), m_in)
            m, mt, idx, n = g.changes_host()
            assert n == n_o and np.array_equal(idx, o.idx) and np.array_equal(mt, o.mt), f"{name} frame {t}"
            assert_close(to_host(out), o.out, bf16, f"{name} frame {t}")
    # the copy of an imported output: a fresh producer that imports the exported state serves the same consumer
    st, out = p.g.export_state()
    fresh = cb.Layer(to_dev(p.w, bf16), to_dev(p.b, bf16), spec.stride, spec.pad, H, W, spec.relu,
                     keep_output_channel_last=True)
    fresh.import_state(st, out)
    fresh_out = fresh.process_frame(to_dev(prep(frames[0], bf16), bf16), 0.02)     # a partial update on top of it
    assert fresh.stats()["n_changed_out"] < fresh.Ho * fresh.Wo
    g, o, _, name = cons[0]
    got = g.process_frame_propagated(fresh_out, fresh)
    assert g.stats()["n_changed_out"] == g.Ho * g.Wo                               # another producer: everything once
    assert_close(to_host(got), orc.dense_conv(to_host(fresh_out), cons_w[0][0], cons_w[0][1], 1, 1, True, bf16=bf16), bf16,
                 "consumer of an imported producer")


def test_channel_last_flags_are_checked():
    H, W = 20, 24
    rng = np.random.default_rng(5)
    w16 = to_dev(rng.standard_normal((16, 3, 3, 3)).astype(np.float32), False)
    w12 = to_dev(rng.standard_normal((12, 3, 3, 3)).astype(np.float32), False)
    wc = to_dev(rng.standard_normal((4, 16, 3, 3)).astype(np.float32), False)

    def status(fn):
        with pytest.raises(cb.binding.CBError) as e:
            fn()
        return e.value.status

    # the copy is written four channels at a time by the fused kernel: power-of-two channel counts from 16 on, fused only
    assert status(lambda: cb.Layer(w12, None, 1, 1, H, W, True, keep_output_channel_last=True)) == cb.CB_EINVAL
    assert status(lambda: cb.Layer(w16, None, 1, 1, H, W, True, backend=1, keep_output_channel_last=True)) == cb.CB_EINVAL
    # only layers without a state of their own gather from a producer's copy
    assert status(lambda: cb.Layer(wc, None, 1, 1, H, W, True, gather_channel_last=True)) == cb.CB_EINVAL
    plain = cb.Layer(w16, None, 1, 1, H, W, True)
    keeps = cb.Layer(w16, None, 1, 1, H, W, True, keep_output_channel_last=True)
    cons = cb.Layer(wc, None, 1, 1, H, W, True, mode=cb.CB_PROPAGATE, gather_channel_last=True)
    x = torch.rand((3, H, W), device="cuda")
    out_plain, out_keeps = plain.process_frame(x, 0.02), keeps.process_frame(x, 0.02)
    assert status(lambda: cons.process_frame_propagated(out_plain, plain)) == cb.CB_EINVAL   # no pixel-major copy there
    got = cons.process_frame_propagated(out_keeps, keeps)
    assert torch.equal(out_plain, out_keeps)
    ref = orc.dense_conv(to_host(out_keeps), to_host(wc), None, 1, 1, True)
    assert_close(to_host(got), ref, False, "consumer of the pixel-major copy")


def test_propagating_consumer_that_misses_a_producer_frame():
    """The producer's change set describes its last frame only.  A consumer that was not called for one of the
    producer's frames must not trust it: every output is recomputed once, so the cached output is again the dense
    result on the producer's output; in lockstep afterwards only the listed pixels are touched."""
    H, W = 30, 44
    spec, frames = syn.random_layer_case(21, 3, 6, 3, 1, 1, H, W, 6, change_prob=0.01)
    rng = np.random.default_rng(4)
    p = Pair(spec, H, W)
    pool = cb.Pool(p.g)
    cons = []
    for k, (hh, ww) in ((3, (H, W)), (1, (H, W)), (3, (H // 2, W // 2))):
        w = rng.standard_normal((5, 6, k, k)).astype(np.float32)
        cons.append((w, k, cb.Layer(to_dev(w, False), None, 1, k // 2, hh, ww, True, mode=cb.CB_PROPAGATE)))
    called = [0, 1, 3, 4, 5]                       # frame 2 is skipped by the consumers
    for t, f in enumerate(frames):
        p.step(f, 0.02, tag=f"producer frame {t}")
        pooled = pool.process()
        if t not in called:
            continue
        for j, (w, k, g) in enumerate(cons):
            src, prod = (pooled, pool) if j == 2 else (p.g_out, p.g)
            out = g.process_frame_propagated(src, prod)
            n = g.stats()["n_changed_out"]
            if t in (0, 3):
                assert n == g.Ho * g.Wo, f"consumer {j} frame {t}: full update expected, N = {n}"
            else:
                assert n < g.Ho * g.Wo, f"consumer {j} frame {t}: N = {n}"
            dense = orc.dense_conv(to_host(src), w, None, 1, k // 2, True)
            assert_close(to_host(out), dense, False, f"consumer {j} frame {t} vs dense on the producer's output")
    # a pooling stage that has not processed its producer's last frame cannot feed a consumer
    p.step(frames[2], 0.02, tag="one more producer frame")
    with pytest.raises(cb.binding.CBError) as e:
        cons[2][2].process_frame_propagated(pooled, pool)
    assert e.value.status == cb.CB_ESTATE


# ---------------------------------------------------------------- error handling at the boundary
def test_error_codes():
    spec, frames = syn.random_layer_case(1, 3, 4, 3, 1, 1, 12, 16, 2)
    p = Pair(spec, 12, 16)
    x = to_dev(frames[0], False)
    for bad in (-0.1, float("nan"), float("inf")):
        with pytest.raises(cb.binding.CBError) as e:
            cb.cb_process_frame(p.g.handle, x, bad)
        assert e.value.status == cb.CB_EINVAL
    with pytest.raises(cb.binding.CBError) as e:
        cb.cb_process_frame(p.g.handle, p.g.state_buf, 0.1)       # input aliases the layer's state
    assert e.value.status == cb.CB_EINVAL
    with pytest.raises(cb.binding.CBError) as e:
        cb.cb_layer_changes(p.g.handle)                           # nothing processed yet
    assert e.value.status == cb.CB_ESTATE
    d = cb.make_desc(3, 4, 3, 3, 1, 1, 12, 16)
    sb, _ = cb.cb_layer_workspace_bytes(d)
    buf = torch.empty(sb + 512, dtype=torch.uint8, device="cuda")
    off = (-buf.data_ptr()) % 256
    w = to_dev(spec.weight, False)
    with pytest.raises(cb.binding.CBError) as e:
        cb.cb_layer_create(d, w, None, buf[off:], sb, buf[off:], 64, 0)
    assert e.value.status == cb.CB_ENOMEM
    with pytest.raises(cb.binding.CBError) as e:
        cb.cb_layer_create(d, w, None, buf[off + 4:], sb, buf[off:], sb, 0)   # misaligned state
    assert e.value.status == cb.CB_EINVAL
    # the layer still works after the rejected calls
    p.step(frames[0], 0.02)
    p.step(frames[1], 0.02)
    # a propagating consumer accepts nothing but its producer's own output buffer
    w2 = to_dev(np.ones((2, 4, 3, 3), np.float32), False)
    cons = cb.Layer(w2, None, 1, 1, p.g.Ho, p.g.Wo, True, mode=cb.CB_PROPAGATE)
    with pytest.raises(cb.binding.CBError) as e:
        cons.process_frame_propagated(p.g_out.clone(), p.g)
    assert e.value.status == cb.CB_EINVAL
    cons.process_frame_propagated(p.g_out, p.g)


def test_timing_stats_are_filled():
    wl = syn.config2(H=64, W=96, C=16, O=16, n_frames=3, rect=10)
    p = Pair(wl.layers[0], wl.H, wl.W)
    p.g.set_timing(True)
    for f in wl.frames():
        p.step(f, wl.tau)
        us = p.g.stats()["us_step"]
        assert us["total"] > 0 and us["detect"] > 0 and us["gemm"] + us["fused"] > 0
        assert us["total"] >= us["detect"]


# ---------------------------------------------------------------- bounded wait of the single-pass index extraction
@pytest.mark.parametrize("geom", [(2, 3, 3, 1, 1, 150, 520), (2, 2, 3, 2, 1, 300, 1030), (1, 2, 5, 1, 2, 700, 4200)])
def test_index_extraction_when_the_wait_for_a_predecessor_runs_out(geom):
    """With a wait limit of zero polls a workgroup never waits for the counts of the workgroups before it:
    whatever is not published yet it recomputes from the change map.  The index list, N and everything
    after them must be what they always are (the oracle's), and the statistics say that the path ran."""
    C, O, k, s, pd, H, W = geom
    _say(f"scan without waiting {geom}")
    spec, frames = syn.random_layer_case(sum(geom) + 1, C, O, k, s, pd, H, W, 4, change_prob=0.03, relu=True)
    cb.cb_set_scan_wait_limit(0)
    try:
        p = Pair(spec, H, W)
        for t, f in enumerate(frames):
            p.step(f, 0.02, tag=f"no-wait scan {geom} frame {t}")
        recounts = p.g.stats()["scan_recounts"]
    finally:
        cb.cb_set_scan_wait_limit(1 << 20)
    _say(f"  predecessor counts recomputed: {recounts}")
    assert recounts > 0
    with pytest.raises(cb.binding.CBError) as e:
        cb.cb_set_scan_wait_limit(-1)
    assert e.value.status == cb.CB_EINVAL
