"""GPU parity: every exported call of libowt against the CPU oracle, element by
element, on the same seeded inputs.  Tolerance (per output tensor):
max|gpu - ref| <= 1e-4 * max|ref| for fp32 storage, 2e-2 * max|ref| for bf16
storage; arg-max indices and pooled maxima bit-exact.

Each backward call gets the forward output y (the ReLU mask source) and the
pooling arg-max as INPUTS, the same arrays on both sides, so every call is a
pure function of its arguments and parity is well-posed.
"""
import sys

import numpy as np
import pytest

import oracle
import synthetic_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import ConvCase, assert_close, empty, force, owt, prep, rel_err, to_dev, to_host, workspace  # noqa: E402


def say(*a):
    print(*a)
    sys.stdout.flush()


def layer_parity(N, C, H, W, K, R, S, stride, pad, dt="f32", bias=True, relu=True, seed=0,
                 tensors=None, alpha=1.0, beta=0.0):
    say("case", dict(N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad, dt=dt, bias=bias, relu=relu,
                     alpha=alpha, beta=beta, seed=seed))
    case = ConvCase(N, C, H, W, K, R, S, stride, pad, dt, bias, relu)
    if tensors is None:
        g = np.random.default_rng(1000 + seed)
        x = g.standard_normal(case.shape_x, dtype=np.float32)
        w = g.standard_normal(case.shape_w, dtype=np.float32) * np.float32(0.05)
        b = g.standard_normal((K,), dtype=np.float32) * np.float32(0.05)
        dy = g.standard_normal(case.shape_y, dtype=np.float32)
    else:
        x, w, b, dy = tensors
    x, w, dy = prep(x, dt), prep(w, dt), prep(dy, dt)
    rnd = (lambda a: oracle.round_bf16(a)) if dt == "bf16" else (lambda a: a)

    y_ref = rnd(oracle.conv_fwd(x, w, b if bias else None, stride, pad, relu))
    y_gpu = case.fwd(x, w, b if bias else None)
    e_f = assert_close(y_gpu, y_ref, dt, "fwd")

    y_in = y_ref if relu else None
    dx_ref = rnd(oracle.conv_bwd_data(dy, w, (H, W), stride, pad, y=y_in))
    dx_gpu = case.bwd_data(dy, y_in, w)
    e_d = assert_close(dx_gpu, dx_ref, dt, "bwd_data")

    dw0 = db0 = None
    if beta != 0.0:
        g2 = np.random.default_rng(2000 + seed)
        dw0 = g2.standard_normal(case.shape_w, dtype=np.float32)
        db0 = g2.standard_normal((K,), dtype=np.float32)
    dw_ref, db_ref = oracle.conv_bwd_filter(x, dy, (R, S), stride, pad, y=y_in, alpha=alpha, beta=beta, dw=dw0, db=db0)
    dw_gpu, db_gpu = case.bwd_filter(x, dy, y_in, alpha, beta, dw0, db0)
    e_w = assert_close(dw_gpu, dw_ref, dt if dt == "f32" else "f32", "bwd_filter dw")   # dw is fp32 either way
    e_b = assert_close(db_gpu, db_ref, "f32", "bwd_filter db")
    say("  rel err fwd %.2e  bwd_data %.2e  dw %.2e  db %.2e" % (e_f, e_d, e_w, e_b))
    return y_gpu, dx_gpu, dw_gpu, db_gpu


# ------------------------------------------------------------ named configs ----

def test_config1_small_layer_fp32():
    geom, x, w, b, dy = si.config1()
    layer_parity(geom["N"], geom["C"], geom["H"], geom["W"], geom["K"], geom["R"], geom["S"],
                 geom["stride"], geom["pad"], tensors=(x, w, b, dy))


def test_config2_batch128_layer_fp32():
    geom, x, w, b, dy = si.config2(128)
    layer_parity(geom["N"], geom["C"], geom["H"], geom["W"], geom["K"], geom["R"], geom["S"],
                 geom["stride"], geom["pad"], tensors=(x, w, b, dy))


def test_config2_shape_bf16_storage():
    geom, x, w, b, dy = si.config2(32)
    layer_parity(32, geom["C"], geom["H"], geom["W"], geom["K"], geom["R"], geom["S"],
                 geom["stride"], geom["pad"], dt="bf16", tensors=(x, w, b, dy))


@pytest.mark.parametrize("K", [384, 256])
def test_paper_filter_count_layers_batch128(K):
    # Section 5's footnote sizes the network at 64, 192, 384, 384, 256 filters: its fourth and fifth layers
    # are 384 -> 384 and 384 -> 256 on 13x13 maps (reduction length 3456), shapes the benchmark
    # configuration does not have.  All three passes, batch 128, every element.
    x = si.normal(3, 60, (128, 13, 13, 384))
    w = si.normal(3, 61 + K, (K, 3, 3, 384), 0.01)
    b = si.normal(3, 62 + K, (K,), 0.01)
    dy = si.upstream_grad(3, 63 + K, (128, 13, 13, K))
    layer_parity(128, 384, 13, 13, K, 3, 3, 1, 1, tensors=(x, w, b, dy))


# ------------------------------------------------------------- shape sweep ----

SWEEP = [
    # N, C, H, W, K, R, S, stride, pad           vector-path shapes (C%4 == 0, K%4 == 0)
    (3, 8, 9, 11, 12, 3, 3, 1, 1),
    (2, 16, 14, 10, 20, 5, 3, (1, 1), (2, 1)),
    (5, 4, 23, 19, 8, 11, 11, 4, 2),              # first-layer geometry, stride 4
    (4, 12, 15, 15, 36, 3, 3, 2, 1),
    (2, 64, 27, 27, 192, 5, 5, 1, 2),             # second-layer shape, several tiles + ragged M
    (130, 32, 6, 6, 72, 1, 1, 1, 0),              # 1x1
    (2, 8, 7, 9, 4, 7, 9, 1, 0),                  # filter covers the whole map (dense layer as a conv)
    (1, 4, 5, 5, 4, 3, 3, (2, 3), (0, 2)),
    # scalar-gather shapes (C%4 != 0 and/or K%4 != 0)
    (2, 3, 12, 12, 5, 3, 3, 1, 1),
    (3, 3, 17, 17, 8, 5, 5, 2, 2),
    (2, 8, 10, 10, 7, 3, 3, 1, 1),                # K odd: vector A in fwd, scalar dz gathers
    (2, 5, 9, 8, 16, 3, 2, (2, 1), (1, 0)),
    (1, 1, 8, 8, 1, 3, 3, 1, 1),
]


@pytest.mark.parametrize("i", range(len(SWEEP)))
def test_layer_sweep_fp32(i):
    N, C, H, W, K, R, S, stride, pad = SWEEP[i]
    layer_parity(N, C, H, W, K, R, S, stride, pad, seed=i)


@pytest.mark.parametrize("i", [0, 3, 4, 8, 10])
def test_layer_sweep_bf16(i):
    N, C, H, W, K, R, S, stride, pad = SWEEP[i]
    layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", seed=100 + i)


def test_flags_and_scaling_variants():
    layer_parity(3, 8, 9, 9, 12, 3, 3, 1, 1, bias=False, relu=False, seed=50)
    layer_parity(3, 8, 9, 9, 12, 3, 3, 1, 1, bias=True, relu=False, seed=51)
    layer_parity(3, 8, 9, 9, 12, 3, 3, 1, 1, bias=False, relu=True, seed=52)
    layer_parity(6, 8, 9, 9, 12, 3, 3, 1, 1, alpha=1.0 / 6, beta=1.0, seed=53)     # batch mean, accumulate
    layer_parity(6, 8, 9, 9, 12, 3, 3, 1, 1, alpha=0.5, beta=-0.25, seed=54)


@pytest.mark.parametrize("tile,split,direct", [(0, 1, 0), (1, 1, 0), (2, 1, 0), (3, 1, 0), (0, 3, 0), (1, 4, 0),
                                               (2, 2, 0), (3, 8, 0), (0, 1, 1), (1, 1, 1), (0, 2, 1), (1, 3, 1), (2, 5, 1), (4, 1, 1), (4, 2, 1), (5, 1, 1), (5, 3, 1), (6, 1, 1), (6, 2, 1)])
def test_every_tile_shape_and_split_k(tile, split, direct):
    # The planner is overridden so each instantiation of the gather kernel (direct = 0) and of the
    # panel-resident stride-1 kernel (direct = 1), and the two-pass split reduction, are exercised.
    m = owt()
    fl = 0 if direct else m.OWT_FORCE_NO_DIRECT
    with force(tile, split, fl):
        layer_parity(4, 40, 13, 13, 136, 3, 3, 1, 1, seed=60 + tile)     # M = 676, ragged in every tile and chunk
        layer_parity(2, 32, 13, 13, 136, 3, 3, 1, 1, dt="bf16", seed=70 + tile)
    if direct:
        with force(tile, split, m.OWT_FORCE_NO_BF16_MFMA):                # bf16 storage on the fp32 MFMA kernel
            layer_parity(2, 32, 13, 13, 136, 3, 3, 1, 1, dt="bf16", seed=75 + tile)
        with force(tile, split):
            layer_parity(3, 64, 27, 27, 72, 5, 5, 1, 2, seed=80 + tile)      # 240-row panel
            layer_parity(2, 8, 9, 14, 12, 3, 5, 1, (1, 2), seed=84 + tile)   # R != S, H != W
            layer_parity(2, 8, 12, 12, 8, 3, 3, 1, 0, seed=88 + tile)        # pad 0: forward direct, bwd-data gathers


@pytest.mark.parametrize("split", [1, 7, 40])
def test_filter_gradient_with_chunks_cut_per_image(split):
    # 5x5 "same" layer on 27x27 images: 729 pixels = 22 chunks of 32 + one of 25 per image; the variant whose
    # pixel chunks never straddle two images (small panel, three work-groups per CU), forced, fp32 and bf16 storage
    m = owt()
    with force(3, split):
        # (calls that take dz as it is, relu=False, run the form of the kernel with table-driven loaders and buffer loads)
        for (N, C, K), kw in [((3, 64, 72), {}), ((1, 8, 200), dict(relu=False, alpha=0.5, beta=-0.25)), ((5, 36, 64), dict(bias=False)),
                              ((3, 64, 72), dict(relu=False)), ((5, 36, 68), dict(relu=False, bias=False)), ((2, 64, 192), dict(relu=False, alpha=0.5, beta=1.0))]:
            d = m.conv_desc(N, C, 27, 27, K, 5, 5, 1, 2, m.OWT_F32, m.OWT_BIAS | m.OWT_RELU)
            assert "chunks-per-image" in m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER), m.owt_conv_plan_describe(d, 2)
            layer_parity(N, C, 27, 27, K, 5, 5, 1, 2, seed=800 + split, **kw)
    with force(3, split, m.OWT_FORCE_NO_BF16_MFMA):
        layer_parity(2, 64, 27, 27, 72, 5, 5, 1, 2, dt="bf16", seed=810 + split)


@pytest.mark.parametrize("variant,split", [(0, 1), (0, 2), (0, 3), (1, 1), (1, 4), (1, 6), (2, 1), (2, 3), (2, 5)])
def test_filter_gradient_with_the_pixel_split_inside_the_work_group(variant, split):
    # fp32 filter gradient whose work-groups split a chunk of pixels over several wavefronts per filter block, add
    # the parts up through LDS and stream their operands straight into LDS (variants 0, 1: all nine taps of a 3x3
    # layer on maps 13 pixels wide, chunks of 128 / 64 pixels; variant 2: one row of five taps per work-group),
    # forced, alone and split over work-groups: ragged filter and channel tiles, a last chunk with 41 or 1 valid
    # pixels, chunks that straddle two images, alpha / beta, with and without bias gradient.  The kernel takes dz
    # as it is; a call that masks dy itself (OWT_RELU) must be served by another kernel.
    m = owt()
    with force(10 + variant, split, m.OWT_FORCE_ONLY_DIRECT):
        shapes = [((3, 64, 27, 27, 72, 5, 5, 2), {}), ((2, 8, 12, 21, 12, 3, 5, (1, 2)), dict(alpha=0.5, beta=-0.25)),
                  ((1, 36, 13, 21, 64, 5, 5, 2), dict(bias=False))] if variant == 2 else \
                 [((4, 40, 13, 13, 136, 3, 3, 1), {}), ((2, 200, 13, 13, 192, 3, 3, 1), dict(bias=False)),
                  ((1, 8, 13, 13, 8, 3, 3, 1), dict(alpha=1.0 / 3, beta=1.0)), ((7, 32, 13, 13, 64, 3, 3, 1), {}),
                  ((3, 36, 17, 13, 68, 3, 3, 1), dict(alpha=0.5, beta=-0.25))]           # H != W, ragged in K and C
        for (N, C, H, W, K, R, S, pad), kw in shapes:
            d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_F32, m.OWT_BIAS)
            assert m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("dfilter2"), \
                m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER)
            layer_parity(N, C, H, W, K, R, S, 1, pad, relu=False, seed=600 + 10 * variant + split, **kw)
        N, C, H, W, K, R, S, pad = shapes[0][0]
        d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_F32, m.OWT_BIAS | m.OWT_RELU)
        assert not m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("dfilter2")
        layer_parity(N, C, H, W, K, R, S, 1, pad, relu=True, seed=650 + variant)


@pytest.mark.parametrize("tile,split", [(0, 1), (1, 1), (4, 1), (0, 2), (1, 3), (4, 2), (7, 1), (7, 2), (7, 3), (8, 1), (8, 2)])
def test_bf16_mfma_direct_kernel(tile, split):
    # bf16 storage, stride 1, reduction channels a multiple of 8: forward and backward-data run on the
    # bf16 MFMA kernel (64-channel chunks; backward-data reads re-laid-out filters from the workspace)
    m = owt()
    with force(tile, split):
        shapes = [((4, 72, 13, 13, 136, 3, 3, 1), {}),                       # ragged last chunk in both passes
                  ((3, 64, 27, 27, 72, 5, 5, 2), {}),                        # 240-row panel
                  ((2, 8, 9, 14, 16, 3, 5, (1, 2)), dict(relu=False)),       # one short chunk, R != S
                  ((2, 192, 13, 13, 200, 3, 3, 1), dict(bias=False))]        # three / four chunks
        if tile in (7, 8):   # the pipelined 512x64 / 256x64 tiles: channels and filters in whole 32-channel chunks
            shapes = [((4, 64, 13, 13, 160, 3, 3, 1), {}),                   # two M tiles, ragged N tile, 2 / 5 chunks
                      ((3, 64, 27, 27, 96, 5, 5, 2), {}),                    # 624-row panel, 25 taps
                      ((2, 32, 9, 14, 32, 3, 5, (1, 2)), dict(relu=False)),  # one chunk, R != S, half-empty tile
                      ((5, 192, 13, 13, 224, 3, 3, 1), dict(bias=False))]    # six / seven chunks, odd step counts
        for (N, C, H, W, K, R, S, pad), kw in shapes:
            d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_BF16, m.OWT_BIAS | m.OWT_RELU)
            for ps in (m.OWT_PASS_FWD, m.OWT_PASS_BWD_DATA):
                assert m.owt_conv_plan_describe(d, ps).startswith("dconv16"), m.owt_conv_plan_describe(d, ps)
            layer_parity(N, C, H, W, K, R, S, 1, pad, dt="bf16", seed=300 + 10 * tile + split, **kw)


@pytest.mark.parametrize("variant,split", [(0, 1), (1, 1), (2, 1), (3, 1), (4, 1), (5, 1), (6, 1), (7, 1), (0, 3), (1, 4), (2, 7), (3, 5), (4, 2), (5, 6), (6, 3), (7, 4)])
def test_bf16_mfma_filter_gradient_kernel(variant, split):
    # bf16 storage, stride 1, "same" padding, channels and filters multiples of 8: the filter gradient runs on
    # the bf16 MFMA, one filter row per work-group (3-tap variants 0, 2, 4, 5; 5-tap variants 1, 3, 6)
    m = owt()
    with force(variant, split):
        shapes = [((3, 64, 27, 27, 72, 5, 5, 2), {}), ((2, 8, 9, 14, 16, 3, 5, (1, 2)), dict(relu=False, alpha=0.5, beta=-0.25))] \
            if variant in (1, 3, 6) else \
            [((4, 72, 13, 13, 136, 3, 3, 1), {}), ((2, 200, 13, 13, 192, 3, 3, 1), dict(bias=False)),
             ((3, 8, 6, 11, 8, 3, 3, 1), dict(relu=False, alpha=1.0 / 3, beta=1.0))]
        for (N, C, H, W, K, R, S, pad), kw in shapes:
            d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_BF16, m.OWT_BIAS | m.OWT_RELU)
            assert m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("dfilter16"), \
                m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER)
            layer_parity(N, C, H, W, K, R, S, 1, pad, dt="bf16", seed=500 + 10 * variant + split, **kw)


@pytest.mark.parametrize("variant,split", [(0, 1), (1, 1), (2, 1), (3, 1), (4, 1), (5, 1), (6, 1),
                                           (0, 3), (1, 4), (2, 7), (3, 5), (4, 2), (5, 6), (6, 3)])
def test_bf16_mfma_filter_gradient_kernel_with_operands_streamed_into_lds(variant, split):
    # the bf16-MFMA filter gradient whose chunks go from global memory straight into LDS (per-block LDS layout,
    # loader tables, chunks that may straddle two images), forced, alone and split over work-groups: ragged filter
    # and channel tiles, a last chunk with few valid pixels, H != W, alpha / beta, with and without bias gradient
    # (3-tap variants 0-3, 5-tap variants 4-6).  The kernel takes dz as it is; a call that masks dy itself
    # (OWT_RELU) must be served by another kernel.
    m = owt()
    with force(30 + variant, split, m.OWT_FORCE_ONLY_DIRECT):
        shapes = [((3, 64, 27, 27, 72, 5, 5, 2), {}), ((2, 8, 12, 21, 16, 3, 5, (1, 2)), dict(alpha=0.5, beta=-0.25)),
                  ((1, 40, 13, 21, 64, 5, 5, 2), dict(bias=False))] if variant >= 4 else \
                 [((4, 72, 13, 13, 136, 3, 3, 1), {}), ((2, 200, 13, 13, 192, 3, 3, 1), dict(bias=False)),
                  ((7, 32, 13, 13, 64, 3, 3, 1), dict(alpha=1.0 / 3, beta=1.0)), ((3, 40, 17, 13, 72, 3, 3, 1), {}),
                  ((3, 8, 6, 11, 8, 3, 3, 1), dict(alpha=0.5, beta=-0.25))]
        for (N, C, H, W, K, R, S, pad), kw in shapes:
            d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_BF16, m.OWT_BIAS)
            assert m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("dfilter16b"), \
                m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER)
            layer_parity(N, C, H, W, K, R, S, 1, pad, dt="bf16", relu=False, seed=700 + 10 * variant + split, **kw)
        N, C, H, W, K, R, S, pad = shapes[0][0]
        d = m.conv_desc(N, C, H, W, K, R, S, 1, pad, m.OWT_BF16, m.OWT_BIAS | m.OWT_RELU)
        assert not m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("dfilter16b")


@pytest.mark.parametrize("shape,split", [
    ((5, 4, 23, 20, 8, 7, 7, 4, 2), 3), ((2, 3, 24, 24, 72, 7, 7, 4, 3), 0), ((3, 3, 36, 28, 64, 11, 11, 4, 2), 5),
    ((2, 8, 17, 12, 20, 5, 3, (2, 2), (2, 1)), 2), ((2, 3, 224, 224, 64, 11, 11, 4, 2), 0),
    # six 4-row bands over 2 and over 6 work-groups: three bands or one band each, so the second half of a
    # work-group's wavefronts (the bf16 forward kernel runs two bands half a round apart) ends a round early
    # or has no band at all
    ((3, 3, 36, 28, 64, 11, 11, 4, 2), 2), ((3, 3, 36, 28, 64, 11, 11, 4, 2), 6)])
def test_strided_small_channel_kernels(shape, split):
    # first-layer style geometry: the row-panel forward and filter-gradient kernels, forced, with and
    # without a forced work-group count
    m = owt()
    N, C, H, W, K, R, S, stride, pad = shape
    with force(-1, split, m.OWT_FORCE_ONLY_DIRECT):
        d = m.conv_desc(N, C, H, W, K, R, S, stride, pad, m.OWT_F32, m.OWT_BIAS | m.OWT_RELU)
        assert m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("sfilter")
        assert m.owt_conv_plan_describe(d, m.OWT_PASS_FWD).startswith("sconv")
        layer_parity(N, C, H, W, K, R, S, stride, pad, seed=200 + split)
        layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", relu=False, alpha=0.25, beta=1.0, seed=210 + split)
        if K % 4 == 0:       # bf16 storage takes the bf16-MFMA forward kernel; the line above ran it
            db = m.conv_desc(N, C, H, W, K, R, S, stride, pad, m.OWT_BF16, m.OWT_BIAS | m.OWT_RELU)
            assert m.owt_conv_plan_describe(db, m.OWT_PASS_FWD).startswith("sconv16"), m.owt_conv_plan_describe(db, 0)
            if K % 8 == 0:   # ... and the bf16-MFMA filter-gradient kernel
                assert m.owt_conv_plan_describe(db, m.OWT_PASS_BWD_FILTER).startswith("sfilter16"), m.owt_conv_plan_describe(db, 2)
            layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", seed=220 + split)
    with force(-1, split, m.OWT_FORCE_ONLY_DIRECT | m.OWT_FORCE_NO_BF16_MFMA):   # ... and the fp32-MFMA kernels on bf16 storage
        layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", relu=False, seed=230 + split)
    # the two fp32 forward kernels, each forced: filters streamed in slices / the whole bank of 32 filters in LDS
    for tile, name in ((20, "sconv "), (21, "sconv2 ")):
        with force(tile, split, m.OWT_FORCE_ONLY_DIRECT):
            assert m.owt_conv_plan_describe(d, m.OWT_PASS_FWD).startswith(name), m.owt_conv_plan_describe(d, 0)
            layer_parity(N, C, H, W, K, R, S, stride, pad, seed=240 + split)
            layer_parity(N, C, H, W, K, R, S, stride, pad, relu=False, bias=False, seed=250 + split)
    # the two fp32 filter-gradient kernels, each forced: units staged through registers / streamed straight into LDS
    # (the second takes dz as it is: a call that passes y for the ReLU' mask is served by the first)
    dn = m.conv_desc(N, C, H, W, K, R, S, stride, pad, m.OWT_F32, m.OWT_BIAS)
    for tile, name in ((22, "sfilter "), (23, "sfilter2 ")):
        with force(tile, split, m.OWT_FORCE_ONLY_DIRECT):
            assert m.owt_conv_plan_describe(dn, m.OWT_PASS_BWD_FILTER).startswith(name), m.owt_conv_plan_describe(dn, 2)
            layer_parity(N, C, H, W, K, R, S, stride, pad, relu=False, seed=260 + split)
            layer_parity(N, C, H, W, K, R, S, stride, pad, relu=False, bias=False, alpha=0.5, beta=-0.25, seed=270 + split)
            if tile == 23:
                assert not m.owt_conv_plan_describe(d, m.OWT_PASS_BWD_FILTER).startswith("sfilter2")
                layer_parity(N, C, H, W, K, R, S, stride, pad, seed=280 + split)
    # ... and the two bf16-MFMA filter-gradient kernels (the second one when the row data is 16-byte aligned in LDS)
    if K % 8 == 0:
        dbn = m.conv_desc(N, C, H, W, K, R, S, stride, pad, m.OWT_BF16, m.OWT_BIAS)
        for tile, name in ((24, "sfilter16 "), (25, "sfilter16b ")):
            with force(tile, split, m.OWT_FORCE_ONLY_DIRECT):
                got = m.owt_conv_plan_describe(dbn, m.OWT_PASS_BWD_FILTER)
                pw = pad[1] if isinstance(pad, tuple) else pad
                fits_b = (pw * C + (4 - (pw * C) % 4) % 4) % 8 == 0 and (W * C) % 8 == 0
                if tile == 24 or fits_b:
                    assert got.startswith(name), got
                else:
                    assert not got.startswith("sfilter16b"), got
                layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", relu=False, seed=290 + split)
                layer_parity(N, C, H, W, K, R, S, stride, pad, dt="bf16", relu=False, bias=False, alpha=0.5, beta=-0.25, seed=295 + split)


def test_autotune_keeps_results_and_is_remembered():
    m = owt()
    geom, x, w, b, dy = si.config2(16)
    case = ConvCase(16, 192, 13, 13, 384, 3, 3, 1, 1)
    y0 = case.fwd(x, w, b)
    dx0 = case.bwd_data(dy, y0, w)
    dw0, db0 = case.bwd_filter(x, dy, y0)
    before = [m.owt_conv_plan_describe(case.desc, p) for p in range(3)]
    xd, wd, bd, dyd, yd = to_dev(x), to_dev(w), to_dev(b), to_dev(dy), to_dev(y0)
    out_y, out_dx = empty(case.shape_y), empty(case.shape_x)
    out_dw, out_db = empty(case.shape_w), empty((384,))
    for p in range(3):
        m.owt_conv_autotune(case.desc, p, xd, wd, bd, out_y if p == 0 else yd, dyd, out_dx, out_dw, out_db, case.ws(p))
    after = [m.owt_conv_plan_describe(case.desc, p) for p in range(3)]
    say("plans before", before)
    say("plans after ", after)
    assert after == [m.owt_conv_plan_describe(case.desc, p) for p in range(3)]
    assert_close(case.fwd(x, w, b), y0, "f32", "fwd after tuning")
    assert_close(case.bwd_data(dy, y0, w), dx0, "f32", "bwd_data after tuning")
    dw1, db1 = case.bwd_filter(x, dy, y0)
    assert_close(dw1, dw0, "f32", "dw after tuning")
    assert_close(db1, db0, "f32", "db after tuning")
    ref = oracle.conv_fwd(x, w, b, 1, 1, True)
    assert_close(to_host(out_y), ref, "f32", "y written by the tuning runs")


def test_run_to_run_bit_equality():
    # no floating-point atomics anywhere: identical bits on repeated runs, split-K included
    geom, x, w, b, dy = si.config2(16)
    case = ConvCase(16, 192, 13, 13, 384, 3, 3, 1, 1)
    y = case.fwd(x, w, b)
    a = case.bwd_filter(x, dy, y)
    c = case.bwd_filter(x, dy, y)
    np.testing.assert_array_equal(a[0], c[0])
    np.testing.assert_array_equal(a[1], c[1])
    np.testing.assert_array_equal(case.bwd_data(dy, y, w), case.bwd_data(dy, y, w))
    np.testing.assert_array_equal(case.fwd(x, w, b), y)


def test_beta_zero_never_reads_old_gradient():
    case = ConvCase(2, 8, 6, 6, 8, 3, 3, 1, 1, relu=False, bias=False)
    g = np.random.default_rng(5)
    x = g.standard_normal(case.shape_x, dtype=np.float32)
    dy = g.standard_normal(case.shape_y, dtype=np.float32)
    nan_w = np.full(case.shape_w, np.nan, dtype=np.float32)
    dw, db = case.bwd_filter(x, dy, None, 1.0, 0.0, nan_w, np.full((8,), np.nan, dtype=np.float32))
    assert np.isfinite(dw).all() and np.isfinite(db).all()


# ------------------------------------------------------ fully-connected shard ----

def fc_parity(N, I, O_total, workers, relu, dt="f32", seed=0, tensors=None, alpha=1.0, beta=0.0):
    m = owt()
    O = O_total // workers
    say("fc case", dict(N=N, I=I, O_total=O_total, workers=workers, O_local=O, relu=relu, dt=dt))
    if tensors is None:
        g = np.random.default_rng(3000 + seed)
        x = g.standard_normal((N, I), dtype=np.float32)
        w = g.standard_normal((O, I), dtype=np.float32) * np.float32(0.02)
        b = g.standard_normal((O,), dtype=np.float32) * np.float32(0.02)
        dy = g.standard_normal((N, O), dtype=np.float32)
    else:
        x, w, b, dy = tensors
    x, w, dy = prep(x, dt), prep(w, dt), prep(dy, dt)
    rnd = (lambda a: oracle.round_bf16(a)) if dt == "bf16" else (lambda a: a)
    flags = m.OWT_BIAS | (m.OWT_RELU if relu else 0)
    d = m.fc_desc(N, I, O_total, workers, 0, m.OWT_BF16 if dt == "bf16" else m.OWT_F32, flags)

    y_ref = rnd(oracle.fc_fwd(x, w, b, relu))
    y = empty((N, O), dt)
    m.owt_fc_shard_fwd(d, to_dev(x, dt), to_dev(w, dt), to_dev(b), y, workspace(m.owt_fc_workspace_bytes(d, 0)))
    e_f = assert_close(to_host(y), y_ref, dt, "fc fwd")

    y_in = y_ref if relu else None
    dw0 = db0 = None
    if beta != 0.0:
        g2 = np.random.default_rng(4000 + seed)
        dw0 = g2.standard_normal((O, I), dtype=np.float32); db0 = g2.standard_normal((O,), dtype=np.float32)
    dx_ref, dw_ref, db_ref = oracle.fc_bwd(x, w, dy, y=y_in, alpha=alpha, beta=beta, dw=dw0, db=db0)
    dx_ref = rnd(dx_ref)
    dx = empty((N, I), dt)
    dw = to_dev(dw0) if dw0 is not None else torch.full((O, I), float("nan"), device="cuda")
    db = to_dev(db0) if db0 is not None else torch.full((O,), float("nan"), device="cuda")
    m.owt_fc_shard_bwd(d, to_dev(x, dt), to_dev(w, dt), to_dev(y_in, dt), to_dev(dy, dt), alpha, beta, dx, dw, db,
                       workspace(m.owt_fc_workspace_bytes(d, 1)))
    torch.cuda.synchronize()
    e_d = assert_close(to_host(dx), dx_ref, dt, "fc dx_partial")
    e_w = assert_close(to_host(dw), dw_ref, "f32", "fc dw")
    e_b = assert_close(to_host(db), db_ref, "f32", "fc db")
    say("  rel err fwd %.2e  dx %.2e  dw %.2e  db %.2e" % (e_f, e_d, e_w, e_b))


@pytest.mark.parametrize("layer", [0, 1, 2])
def test_fc_shard_real_shapes_fp32(layer):
    # 9216->4096->4096->1000 over 8 workers: 512 / 512 / 125 columns, batch 128
    L = si.FC_LAYERS[layer]
    ws, bs = si.fc_params(4)
    x = si.normal(4, 60 + layer, (128, L["I"]))
    dy = si.upstream_grad(4, 70 + layer, (128, L["O_local"]))
    fc_parity(128, L["I"], L["O_total"], si.FC_WORKERS, L["relu"], tensors=(x, ws[layer], bs[layer], dy))


def test_fc_shard_small_and_ragged():
    fc_parity(5, 36, 24, 2, True, seed=1)
    fc_parity(7, 33, 15, 3, False, seed=2)                       # I, O_local odd
    fc_parity(130, 260, 140, 1, True, seed=3, alpha=1.0 / 130, beta=1.0)
    fc_parity(16, 64, 1000, 8, False, dt="bf16", seed=4)
    fc_parity(128, 4096, 4096, 8, True, dt="bf16", seed=5)


@pytest.mark.parametrize("tile,split", [(0, 1), (1, 1), (2, 1), (3, 1), (0, 2), (1, 3), (2, 7), (3, 5)])
def test_fc_dense_kernel(tile, split):
    # The dense kernel of the shard (operands streamed straight into LDS), every tile shape, forced, with and
    # without a split reduction: tiles ragged in both directions, 2 to 7 reduction steps, masked dy with bias
    # gradient and accumulation, batch and column counts that are not multiples of 32 or 4 (the backward
    # passes then read a zero-padded copy of dz), and shapes where some or all passes do not qualify (they gather).
    m = owt()
    with force(16 + tile, split):
        for (N, I, O), ok, kw in [((160, 224, 96), (1, 1, 1), dict(relu=True)),
                                  ((128, 256, 192), (1, 1, 1), dict(relu=False, alpha=0.5, beta=-0.25)),
                                  ((100, 64, 40), (1, 1, 1), dict(relu=True)),
                                  ((128, 96, 125), (1, 1, 1), dict(relu=False)),
                                  ((37, 64, 125), (1, 1, 1), dict(relu=True, alpha=0.5, beta=0.5)),
                                  ((96, 36, 64), (0, 1, 1), dict(relu=True, alpha=1.0 / 96, beta=1.0)),
                                  ((64, 30, 32), (0, 0, 0), dict(relu=True))]:
            d = m.conv_desc(N, I, 1, 1, O, 1, 1, 1, 0, m.OWT_F32, m.OWT_BIAS)
            for ps in range(3):
                assert ("fcgemm" in m.owt_conv_plan_describe(d, ps)) == bool(ok[ps]), (ps, m.owt_conv_plan_describe(d, ps))
            fc_parity(N, I, O, 1, seed=900 + tile, **kw)


@pytest.mark.parametrize("mode", ["one_launch", "two_launches", "tuned"])
def test_fc_backward_pair(mode):
    # Both backward products of a shard on the dense kernel share one dz; they run as one launch or as two.
    # Forced either way, and chosen by owt_fc_autotune (whose timing runs must leave results unchanged).
    m = owt()
    fl = {"one_launch": m.OWT_FORCE_FC_ONE_LAUNCH, "two_launches": m.OWT_FORCE_FC_TWO_LAUNCHES, "tuned": 0}[mode]
    with force(-1, 0, fl):
        for (N, I, O), kw in [((128, 512, 125), dict(relu=False)), ((96, 260, 192), dict(relu=True, alpha=0.25, beta=1.0)),
                              ((33, 64, 40), dict(relu=True))]:
            if mode == "tuned":
                d = m.fc_desc(N, I, O, 1, 0, m.OWT_F32, m.OWT_BIAS | (m.OWT_RELU if kw["relu"] else 0))
                g = np.random.default_rng(5)
                t = lambda *sh: to_dev(g.standard_normal(sh, dtype=np.float32))
                wsb = max(m.owt_fc_workspace_bytes(d, 0), m.owt_fc_workspace_bytes(d, 1))
                m.owt_fc_autotune(d, t(N, I), t(O, I), t(O), t(N, O), t(N, O), empty((N, I), "f32"), empty((O, I), "f32"),
                                  empty((O,), "f32"), workspace(wsb))
            fc_parity(N, I, O, 1, seed=950, **kw)


def test_fc_dense_kernel_degenerate_sizes():
    # one image, one column, a single reduction step, a reduction shorter than one step: every operand tile is
    # mostly clamped re-reads and the padded dz copy is mostly padding
    for (N, I, O), relu in [((1, 32, 1), False), ((1, 64, 125), True), ((2, 4, 3), True), ((33, 36, 5), False), ((128, 32, 512), True)]:
        fc_parity(N, I, O, 1, relu, seed=970)
        fc_parity(N, I, O, 1, relu, seed=971, alpha=0.5, beta=1.0)


def test_fc_shard_bwd_without_dx_or_dbias():
    m = owt()
    g = np.random.default_rng(9)
    x = g.standard_normal((8, 32), dtype=np.float32); w = g.standard_normal((16, 32), dtype=np.float32)
    dy = g.standard_normal((8, 16), dtype=np.float32)
    d = m.fc_desc(8, 32, 16, 1, 0, m.OWT_F32, 0)
    dw = torch.full((16, 32), float("nan"), device="cuda")
    m.owt_fc_shard_bwd(d, to_dev(x), to_dev(w), None, to_dev(dy), 1.0, 0.0, None, dw, None,
                       workspace(m.owt_fc_workspace_bytes(d, 1)))
    torch.cuda.synchronize()
    assert_close(to_host(dw), oracle.fc_bwd(x, w, dy, want_dx=False, want_db=False)[1], "f32", "dw only")


# ------------------------------------------------------------------ pooling ----

@pytest.mark.parametrize("N,H,W,C,win,st,dt", [
    (3, 13, 13, 8, 3, 2, "f32"), (2, 55, 55, 64, 3, 2, "f32"), (2, 9, 12, 5, 3, 2, "f32"),
    (2, 10, 7, 4, 2, 2, "f32"), (1, 8, 8, 3, 4, 1, "f32"), (2, 27, 27, 192, 3, 2, "bf16"), (2, 7, 7, 3, 3, 2, "bf16"),
    (2, 10, 7, 12, 2, 2, "bf16"), (1, 9, 9, 8, 4, 1, "bf16"), (2, 12, 10, 8, 3, 2, "f32"), (2, 12, 10, 16, 3, 2, "bf16"), (1, 3, 3, 4, 3, 2, "f32"),
])
def test_maxpool_parity(N, H, W, C, win, st, dt):
    m = owt()
    say("pool case", (N, H, W, C, win, st, dt))
    g = np.random.default_rng(77)
    x = prep(np.maximum(g.standard_normal((N, H, W, C), dtype=np.float32), 0), dt)   # post-ReLU: many exact ties at 0
    y_ref, am_ref = oracle.maxpool_fwd(x, win, st)
    P, Q = y_ref.shape[1:3]
    code = m.OWT_BF16 if dt == "bf16" else m.OWT_F32
    y = empty((N, P, Q, C), dt); am = torch.empty((N, P, Q, C), device="cuda", dtype=torch.uint8)
    m.owt_maxpool_fwd(N, H, W, C, win, st, code, to_dev(x, dt), y, am)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(y), y_ref)             # a max is exact
    np.testing.assert_array_equal(am.cpu().numpy(), am_ref)      # first maximum in scan order
    dy = prep(g.standard_normal((N, P, Q, C), dtype=np.float32), dt)
    dx_ref = oracle.maxpool_bwd(dy, am_ref, (H, W), win, st)
    if dt == "bf16":
        dx_ref = oracle.round_bf16(dx_ref)
    dx = empty((N, H, W, C), dt)
    m.owt_maxpool_bwd(N, H, W, C, win, st, code, to_dev(dy, dt), to_dev(am_ref), dx)
    torch.cuda.synchronize()
    assert_close(to_host(dx), dx_ref, dt, "maxpool bwd")


def test_fused_relu_backward_entry_points():
    # owt_maxpool_bwd_relu == mask(pool_bwd(dy)) and owt_conv_bwd_data_relu_in == mask(bwd_data(dy)),
    # the mask being [input of the ReLU's consumer > 0]; oracle = the unfused definition.
    m = owt()
    g = np.random.default_rng(314)
    for dt in ("f32", "bf16"):
        N, H, W, C, win, st = 3, 13, 13, 24, 3, 2
        y = prep(np.maximum(g.standard_normal((N, H, W, C), dtype=np.float32), 0), dt)      # a ReLU output
        a_ref, am_ref = oracle.maxpool_fwd(y, win, st)
        P, Q = a_ref.shape[1:3]
        da = prep(g.standard_normal((N, P, Q, C), dtype=np.float32), dt)
        ref = oracle.maxpool_bwd(da, am_ref, (H, W), win, st) * (y > 0)
        ref = oracle.round_bf16(ref) if dt == "bf16" else ref
        dx = empty((N, H, W, C), dt)
        code = m.OWT_BF16 if dt == "bf16" else m.OWT_F32
        m.owt_maxpool_bwd_relu(N, H, W, C, win, st, code, to_dev(da, dt), to_dev(am_ref), to_dev(a_ref, dt), dx)
        torch.cuda.synchronize()
        assert_close(to_host(dx), ref, dt, "maxpool_bwd_relu")
        assert (ref[y <= 0] == 0).all() and np.count_nonzero(a_ref <= 0) > 0       # the mask really bites

        for (K, split) in ((40, 0), (136, 3)):
            case = ConvCase(4, 24, 13, 13, K, 3, 3, 1, 1, dt, True, True)
            x = prep(np.maximum(g.standard_normal(case.shape_x, dtype=np.float32), 0), dt)
            w = prep(g.standard_normal(case.shape_w, dtype=np.float32) * np.float32(0.05), dt)
            yy = prep(g.standard_normal(case.shape_y, dtype=np.float32), dt)
            dy = prep(g.standard_normal(case.shape_y, dtype=np.float32), dt)
            ref = oracle.conv_bwd_data(dy, w, (13, 13), 1, 1, y=yy) * (x > 0)
            ref = oracle.round_bf16(ref) if dt == "bf16" else ref
            out = empty(case.shape_x, dt)
            with force(-1, split):
                m.owt_conv_bwd_data_relu_in(case.desc, to_dev(dy, dt), to_dev(yy, dt), to_dev(w, dt), to_dev(x, dt), out, case.ws(1))
            torch.cuda.synchronize()
            assert_close(to_host(out), ref, dt, "conv_bwd_data_relu_in K=%d" % K)


# -------------------------------------------------------------- error paths ----

def test_error_codes_leave_outputs_untouched():
    m = owt()
    d = m.conv_desc(2, 8, 6, 6, 8, 3, 3, 1, 1, m.OWT_F32, m.OWT_BIAS | m.OWT_RELU)
    x = torch.zeros((2, 6, 6, 8), device="cuda"); w = torch.zeros((8, 3, 3, 8), device="cuda")
    b = torch.zeros((8,), device="cuda"); y = torch.full((2, 6, 6, 8), 7.0, device="cuda")
    with pytest.raises(m.OwtError) as ei:
        m.owt_conv_fwd(d, x, w, None, y)                         # OWT_BIAS without a bias pointer
    assert ei.value.status == m.OWT_EINVAL and "bias" in str(ei.value)
    with pytest.raises(m.OwtError) as ei:
        m.owt_conv_bwd_data(d, y, None, w, x)                    # OWT_RELU without y
    assert ei.value.status == m.OWT_EINVAL
    with pytest.raises(m.OwtError) as ei:
        m.owt_conv_fwd(d, x.data_ptr() + 4, w, b, y)             # misaligned
    assert ei.value.status == m.OWT_EINVAL
    big = m.conv_desc(16, 192, 13, 13, 384, 3, 3, 1, 1, m.OWT_F32, 0)
    need = m.owt_conv_workspace_bytes(big, m.OWT_PASS_BWD_FILTER)
    assert need > 0
    with pytest.raises(m.OwtError) as ei:
        m.owt_conv_bwd_filter(big, x, y, None, 1.0, 0.0, w, None, workspace(16))
    assert ei.value.status == m.OWT_EWORKSPACE
    torch.cuda.synchronize()
    assert (y == 7.0).all()
