"""Pins for the CPU oracle: each check ties it to something other than itself --
a library matmul, a closed form, an adjoint identity, finite differences, brute
force, or a number the paper prints.  None of these needs a GPU.

The paper states no convolution formula; it relies on the usual definitions
(Section 4, forward steps 1-3, backward steps 1-2), so the pins are the
mathematics of those definitions.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- forward ----

def test_1x1_conv_is_matmul():
    x = rnd(1, 3, 5, 7, 11)
    w = rnd(2, 6, 1, 1, 11)
    b = rnd(3, 6)
    y = oracle.conv_fwd(x, w, b)
    ref = x.reshape(-1, 11) @ w.reshape(6, 11).T + b
    np.testing.assert_allclose(y.reshape(-1, 6), ref, rtol=1e-12, atol=1e-12)
    y32 = oracle.conv_fwd(x.astype(np.float32), w.astype(np.float32), b.astype(np.float32))
    np.testing.assert_allclose(y32.reshape(-1, 6), ref, rtol=2e-6, atol=2e-6)


def test_fc_is_matmul_and_equals_1x1_conv():
    x = rnd(4, 9, 33)
    w = rnd(5, 13, 33)
    b = rnd(6, 13)
    y = oracle.fc_fwd(x, w, b, relu=True)
    np.testing.assert_allclose(y, np.maximum(x @ w.T + b, 0), rtol=1e-12, atol=1e-12)
    yc = oracle.conv_fwd(x.reshape(9, 1, 1, 33), w.reshape(13, 1, 1, 33), b, relu=True)
    np.testing.assert_array_equal(yc.reshape(9, 13), y)


def test_fc_on_flattened_map_equals_full_window_conv():
    # A dense layer on an HxWxC map flattened in (h,w,c) order is a convolution whose
    # filter covers the whole map: checks the KRSC <-> [o][i] layout claim.
    x = rnd(7, 4, 6, 6, 5)
    w = rnd(8, 10, 6 * 6 * 5)
    y_fc = oracle.fc_fwd(x.reshape(4, -1), w)
    y_cv = oracle.conv_fwd(x, w.reshape(10, 6, 6, 5))
    assert y_cv.shape == (4, 1, 1, 10)
    np.testing.assert_allclose(y_cv.reshape(4, 10), y_fc, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride,pad,r0,s0", [(1, 0, 0, 0), (1, 2, 0, 3), (2, 1, 2, 1), (4, 2, 4, 0), (1, 1, 1, 1)])
def test_delta_filter_shifts_without_flip(stride, pad, r0, s0):
    # w[k,r0,s0,c] = [k == c]  =>  y[n,p,q,k] = x[n, p*st-pad+r0, q*st-pad+s0, k], 0 outside.
    N, H, W, C, R, S = 2, 11, 13, 3, 5, 4
    x = rnd(9, N, H, W, C)
    w = np.zeros((C, R, S, C))
    for c in range(C):
        w[c, r0, s0, c] = 1.0
    y = oracle.conv_fwd(x, w, stride=stride, pad=pad)
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    assert y.shape == (N, P, Q, C)
    ref = np.zeros_like(y)
    for p in range(P):
        for q in range(Q):
            h, ww = p * stride - pad + r0, q * stride - pad + s0
            if 0 <= h < H and 0 <= ww < W:
                ref[:, p, q, :] = x[:, h, ww, :]
    np.testing.assert_array_equal(y, ref)


def test_ones_filter_counts_in_range_taps():
    # constant input 1, all-ones filter: y = (#taps inside the image) * C
    H, W, C, R, S, pad = 6, 7, 3, 3, 5, 2
    x = np.ones((1, H, W, C))
    w = np.ones((1, R, S, C))
    y = oracle.conv_fwd(x, w, pad=(1, 2))[0, :, :, 0]
    for p in range(H):
        for q in range(W):
            nr = sum(0 <= p - 1 + r < H for r in range(R))
            ns = sum(0 <= q - 2 + s < W for s in range(S))
            assert y[p, q] == nr * ns * C
    assert y[2, 3] == R * S * C and y[0, 0] == 2 * 3 * C


def test_conv_fwd_brute_force_python_loops():
    # independent re-derivation with explicit zero padding and numpy slicing
    N, H, W, C, K, R, S = 2, 7, 6, 3, 4, 3, 2
    for stride, pad in [((1, 1), (0, 0)), ((2, 1), (1, 0)), ((1, 3), (2, 1))]:
        x = rnd(10, N, H, W, C); w = rnd(11, K, R, S, C); b = rnd(12, K)
        xp = np.zeros((N, H + 2 * pad[0], W + 2 * pad[1], C))
        xp[:, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = x
        P, Q = oracle.out_hw(H, W, R, S, stride, pad)
        ref = np.zeros((N, P, Q, K))
        for p, q in itertools.product(range(P), range(Q)):
            patch = xp[:, p * stride[0]:p * stride[0] + R, q * stride[1]:q * stride[1] + S, :]
            ref[:, p, q, :] = np.einsum("nrsc,krsc->nk", patch, w) + b
        y = oracle.conv_fwd(x, w, b, stride=stride, pad=pad, relu=True)
        np.testing.assert_allclose(y, np.maximum(ref, 0), rtol=1e-12, atol=1e-12)


def test_linearity_and_translation():
    x1, x2 = rnd(13, 1, 12, 12, 2), rnd(14, 1, 12, 12, 2)
    w = rnd(15, 3, 3, 3, 2)
    a = 0.37
    lhs = oracle.conv_fwd(a * x1 + x2, w, stride=2, pad=1)
    rhs = a * oracle.conv_fwd(x1, w, stride=2, pad=1) + oracle.conv_fwd(x2, w, stride=2, pad=1)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    # shifting the input down/right by the stride shifts the output by one (interior)
    xs = np.zeros_like(x1); xs[:, 2:, 2:] = x1[:, :-2, :-2]
    y, ys = oracle.conv_fwd(x1, w, stride=2, pad=1), oracle.conv_fwd(xs, w, stride=2, pad=1)
    np.testing.assert_allclose(ys[:, 2:, 2:], y[:, 1:-1, 1:-1], rtol=1e-12, atol=1e-12)


def test_output_size_chain_and_fc_flop_count():
    # Section 5: 224x224 crops; map sizes as in the two-tower model -> 55,27,13,13,13 and 6x6x256 = 9216.
    import synthetic_inputs as si
    H = si.STACK_INPUT_HWC[0]
    sizes = []
    for L in si.STACK_LAYERS:
        H = oracle.out_hw(H, H, L["R"], L["R"], L["stride"], L["pad"])[0]
        sizes.append(H)
        if L["pool"]:
            H = (H - si.POOL_WIN) // si.POOL_STRIDE + 1
            sizes.append(H)
    assert sizes == [55, 27, 27, 13, 13, 13, 13, 6]
    assert H * H * si.STACK_LAYERS[-1]["K"] == si.FC_LAYERS[0]["I"] == 9216
    # Section 5.1 footnote: per sample each of 8 GPUs does 4096 x 512 x 2 FLOPs
    L = si.FC_LAYERS[1]
    assert 2 * L["I"] * L["O_local"] == 4096 * 512 * 2 == 4194304
    assert L["O_total"] // si.FC_WORKERS == L["O_local"]
    assert abs(4194304 / 2e12 * 1e6 - 2.09) < 0.01          # 2.09 us at 2 TFLOP/s
    assert abs(4096 * 4 / 6e9 * 1e6 - 2.73) < 0.01          # 2.73 us at 6 GB/s


# --------------------------------------------------------------- backward ----

GEOMS = [
    # N, H, W, C, K, R, S, stride, pad
    (2, 7, 9, 3, 4, 3, 3, (1, 1), (1, 1)),
    (2, 8, 7, 2, 3, 3, 2, (2, 1), (0, 1)),
    (1, 13, 11, 3, 2, 5, 4, (2, 2), (2, 1)),
    (2, 19, 17, 3, 2, 11, 11, (4, 4), (2, 2)),
    (3, 6, 6, 5, 4, 1, 1, (1, 1), (0, 0)),
    (1, 9, 10, 2, 3, 3, 5, (1, 2), (1, 2)),
]


@pytest.mark.parametrize("geom", GEOMS)
def test_adjoint_identities(geom):
    # <conv(x;w), g> = <x, bwd_data(g;w)> = <w, bwd_filter(x,g)>  (no bias, no ReLU)
    N, H, W, C, K, R, S, stride, pad = geom
    x = rnd(20, N, H, W, C); w = rnd(21, K, R, S, C)
    y = oracle.conv_fwd(x, w, stride=stride, pad=pad)
    g = rnd(22, *y.shape)
    lhs = np.sum(y * g)
    dx = oracle.conv_bwd_data(g, w, (H, W), stride, pad)
    dw, db = oracle.conv_bwd_filter(x, g, (R, S), stride, pad)
    assert abs(lhs - np.sum(x * dx)) <= 1e-10 * abs(lhs) + 1e-10
    assert abs(lhs - np.sum(w * dw)) <= 1e-10 * abs(lhs) + 1e-10
    np.testing.assert_allclose(db, g.sum(axis=(0, 1, 2)), rtol=1e-12, atol=1e-12)


def _fd(f, a, eps=1e-5):
    g = np.zeros_like(a)
    flat, gf = a.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + eps; fp = f()
        flat[i] = old - eps; fm = f()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * eps)
    return g


@pytest.mark.parametrize("geom", [(2, 5, 6, 3, 4, 3, 2, (1, 1), (1, 0)), (1, 7, 7, 2, 3, 3, 3, (2, 2), (1, 1))])
def test_finite_differences_conv_bias_relu(geom):
    N, H, W, C, K, R, S, stride, pad = geom
    x = rnd(30, N, H, W, C); w = rnd(31, K, R, S, C); b = rnd(32, K)
    z = oracle.conv_fwd(x, w, b, stride, pad, relu=False)
    y = oracle.conv_fwd(x, w, b, stride, pad, relu=True)
    g = rnd(33, *y.shape)
    # outputs whose pre-activation sits near the kink get no upstream gradient,
    # so the finite difference never straddles it
    near = np.abs(z) < 1e-2
    assert near.mean() < 0.1
    g[near] = 0.0
    loss = lambda: float(np.sum(g * oracle.conv_fwd(x, w, b, stride, pad, relu=True)))
    dx = oracle.conv_bwd_data(g, w, (H, W), stride, pad, y=y)
    dw, db = oracle.conv_bwd_filter(x, g, (R, S), stride, pad, y=y)
    np.testing.assert_allclose(dx, _fd(loss, x), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dw, _fd(loss, w), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(db, _fd(loss, b), rtol=1e-6, atol=1e-7)


def test_relu_mask_is_strictly_positive_y():
    # y == 0 passes no gradient (ReLU'(0) = 0)
    x = np.ones((1, 1, 1, 1)); w = np.ones((2, 1, 1, 1))
    y = np.array([0.0, 2.0]).reshape(1, 1, 1, 2)
    g = np.array([5.0, 7.0]).reshape(1, 1, 1, 2)
    assert oracle.conv_bwd_data(g, w, (1, 1), y=y)[0, 0, 0, 0] == 7.0
    dw, db = oracle.conv_bwd_filter(x, g, (1, 1), y=y)
    assert dw.reshape(-1).tolist() == [0.0, 7.0] and db.tolist() == [0.0, 7.0]


def test_alpha_beta_and_nan_safe_overwrite():
    x = rnd(40, 2, 5, 5, 3); g = rnd(41, 2, 5, 5, 4)
    dw1, db1 = oracle.conv_bwd_filter(x, g, (3, 3), 1, 1)
    old_w, old_b = rnd(42, 4, 3, 3, 3), rnd(43, 4)
    dw2, db2 = oracle.conv_bwd_filter(x, g, (3, 3), 1, 1, alpha=0.5, beta=1.0, dw=old_w, db=old_b)
    np.testing.assert_allclose(dw2, 0.5 * dw1 + old_w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db2, 0.5 * db1 + old_b, rtol=1e-12, atol=1e-12)
    nan_w = np.full((4, 3, 3, 3), np.nan)
    dw3, _ = oracle.conv_bwd_filter(x, g, (3, 3), 1, 1, beta=0.0, dw=nan_w, db=np.full(4, np.nan))
    np.testing.assert_array_equal(dw3, dw1)


def test_bwd_filter_at_matches_full():
    x = rnd(44, 3, 9, 8, 4).astype(np.float32); g = rnd(45, 3, 5, 4, 5).astype(np.float32)
    y = rnd(46, 3, 5, 4, 5).astype(np.float32)
    dw, _ = oracle.conv_bwd_filter(x, g, (3, 3), 2, 1, y=y)
    idx = [(k, r, s, c) for k in range(5) for r in range(3) for s in range(3) for c in range(4)]
    at = oracle.conv_bwd_filter_at(x, g, idx, (3, 3), 2, 1, y=y)
    np.testing.assert_array_equal(at, dw.reshape(-1))


def test_fc_bwd_matches_matmul_and_finite_differences():
    N, I, O = 5, 7, 4
    x = rnd(50, N, I); w = rnd(51, O, I); b = rnd(52, O); g = rnd(53, N, O)
    y = oracle.fc_fwd(x, w, b, relu=True)
    dz = g * (y > 0)
    dx, dw, db = oracle.fc_bwd(x, w, g, y=y)
    np.testing.assert_allclose(dx, dz @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, dz.T @ x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, dz.sum(0), rtol=1e-12, atol=1e-12)
    loss = lambda: float(np.sum(g * oracle.fc_fwd(x, w, b, relu=True)))
    np.testing.assert_allclose(dw, _fd(loss, w), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dx, _fd(loss, x), rtol=1e-6, atol=1e-7)
    # linear layer (no y): plain transposes; alpha/beta
    dx2, dw2, db2 = oracle.fc_bwd(x, w, g, alpha=1.0 / N, beta=1.0, dw=np.ones((O, I)), db=np.ones(O))
    np.testing.assert_allclose(dx2, g @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw2, g.T @ x / N + 1, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db2, g.sum(0) / N + 1, rtol=1e-12, atol=1e-12)


def test_fc_column_shards_concatenate_to_the_full_layer():
    # Section 4: each of K workers owns 1/K of the neurons; stacking the K column
    # shards gives the unsharded layer, and the K partial dX add up to the full dX.
    N, I, O, Kw = 4, 6, 8, 4
    x = rnd(54, N, I); w = rnd(55, O, I); b = rnd(56, O); g = rnd(57, N, O)
    full = oracle.fc_fwd(x, w, b)
    dx_full, dw_full, _ = oracle.fc_bwd(x, w, g)
    cols = O // Kw
    dx_sum = np.zeros_like(x)
    for k in range(Kw):
        sl = slice(k * cols, (k + 1) * cols)
        np.testing.assert_array_equal(oracle.fc_fwd(x, w[sl], b[sl]), full[:, sl])
        dxp, dwp, _ = oracle.fc_bwd(x, w[sl], g[:, sl])
        np.testing.assert_array_equal(dwp, dw_full[sl])
        dx_sum += dxp
    np.testing.assert_allclose(dx_sum, dx_full, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- pooling ----

def test_maxpool_increasing_input_routes_to_last_element():
    H = W = 7
    x = np.arange(H * W, dtype=np.float64).reshape(1, H, W, 1)
    y, am = oracle.maxpool_fwd(x, 3, 2)
    assert y.shape == (1, 3, 3, 1) and (am == 8).all()
    for p in range(3):
        for q in range(3):
            assert y[0, p, q, 0] == x[0, 2 * p + 2, 2 * q + 2, 0]
    dx = oracle.maxpool_bwd(np.ones_like(y), am, (H, W), 3, 2)
    ref = np.zeros((H, W)); ref[2::2, 2::2] = 1
    np.testing.assert_array_equal(dx[0, :, :, 0], ref)


def test_maxpool_ties_go_to_first_in_scan_order():
    x = np.full((1, 7, 7, 2), 3.0)
    y, am = oracle.maxpool_fwd(x, 3, 2)
    assert (am == 0).all() and (y == 3.0).all()
    dx = oracle.maxpool_bwd(np.ones_like(y), am, (7, 7), 3, 2)
    ref = np.zeros((7, 7)); ref[0:6:2, 0:6:2] = 1
    np.testing.assert_array_equal(dx[0, :, :, 1], ref)


def test_maxpool_shared_peak_collects_four_windows():
    x = np.zeros((1, 5, 5, 1)); x[0, 2, 2, 0] = 9.0
    y, am = oracle.maxpool_fwd(x, 3, 2)            # 2x2 windows, all contain (2,2)
    assert (y == 9.0).all()
    assert am[0, :, :, 0].tolist() == [[8, 6], [2, 0]]
    dx = oracle.maxpool_bwd(np.ones_like(y), am, (5, 5), 3, 2)
    assert dx[0, 2, 2, 0] == 4.0 and dx.sum() == 4.0


def test_maxpool_finite_differences_and_brute_force():
    x = rnd(60, 2, 9, 8, 3)
    y, am = oracle.maxpool_fwd(x, 3, 2)
    P, Q = y.shape[1:3]
    for p, q in itertools.product(range(P), range(Q)):
        np.testing.assert_array_equal(y[:, p, q, :], x[:, 2 * p:2 * p + 3, 2 * q:2 * q + 3, :].max(axis=(1, 2)))
    g = rnd(61, *y.shape)
    loss = lambda: float(np.sum(g * oracle.maxpool_fwd(x, 3, 2)[0]))
    np.testing.assert_allclose(oracle.maxpool_bwd(g, am, (9, 8), 3, 2), _fd(loss, x, 1e-6), rtol=1e-5, atol=1e-7)
    # another window/stride
    y2, am2 = oracle.maxpool_fwd(x, 2, 1)
    assert y2.shape == (2, 8, 7, 3)
    np.testing.assert_array_equal(y2[:, 3, 4, :], x[:, 3:5, 4:6, :].max(axis=(1, 2)))


# ------------------------------------------------------------------- bf16 ----

def _bits(u):
    return np.array([u], dtype=np.uint32).view(np.float32)


@pytest.mark.parametrize("inp,out", [
    (0x3F800000, 0x3F800000),   # 1.0 exact
    (0x3F808000, 0x3F800000),   # tie, even mantissa below -> round down
    (0x3F818000, 0x3F820000),   # tie, odd mantissa below -> round up
    (0x3F808001, 0x3F810000),   # just above the tie -> up
    (0x3F807FFF, 0x3F800000),   # just below the tie -> down
    (0x3FFFFFFF, 0x40000000),   # carry ripples into the exponent
    (0x7F7FFFFF, 0x7F800000),   # largest finite rounds to +inf
    (0x80000000, 0x80000000),   # -0
    (0x7F800000, 0x7F800000),   # +inf
    (0xFF800000, 0xFF800000),   # -inf
    (0x00000001, 0x00000000),   # smallest denormal -> 0
    (0xC2F6E979, 0xC2F70000),   # -123.456 -> -123.5
])
def test_bf16_rne_bit_patterns(inp, out):
    r = oracle.round_bf16(_bits(inp)).view(np.uint32)[0]
    assert r == out, hex(r)


def test_bf16_nan_and_idempotent():
    assert np.isnan(oracle.round_bf16(_bits(0x7F800001))[0])
    a = rnd(70, 1000).astype(np.float32)
    r = oracle.round_bf16(a)
    np.testing.assert_array_equal(oracle.round_bf16(r), r)
    assert (r.view(np.uint32) & 0xFFFF == 0).all()
    assert np.max(np.abs(r - a) / np.abs(a)) <= 2.0 ** -8


def test_f32_and_f64_builds_agree():
    x = rnd(80, 2, 9, 9, 5); w = rnd(81, 6, 3, 3, 5) * 0.1; b = rnd(82, 6)
    y64 = oracle.conv_fwd(x, w, b, 2, 1, True)
    y32 = oracle.conv_fwd(x.astype(np.float32), w.astype(np.float32), b.astype(np.float32), 2, 1, True)
    np.testing.assert_allclose(y32, y64, rtol=1e-5, atol=1e-6)


# ------------------------------------------------- update rule (Section 5) ----

def golden():
    vals = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                vals[line[0]] = float(line[1])
    return vals


def test_weight_decay_example_printed_in_the_paper():
    # Section 5 prints omega' for batch 128 -> 1024 to 8 significant digits, and its sqrt(k) approximation
    gv = golden()
    e2, o2 = oracle.scale_hyperparameters(gv["wd_example_k"], gv["wd_example_eps"], gv["wd_example_omega"])
    assert abs(e2 - math.sqrt(8.0) * 0.01) < 1e-15
    assert abs(o2 - gv["wd_example_omega_scaled"]) < 5e-11          # half a unit of the last printed digit
    assert abs(math.sqrt(gv["wd_example_k"]) * gv["wd_example_omega"] - gv["wd_example_omega_sqrtk"]) < 5e-11
    assert abs(o2 - gv["wd_example_omega_sqrtk"]) > 1e-8            # the exact form is not the approximation


def test_update_rule_weight_decay_closed_form_and_batch_equivalence():
    # mu = 0, zero gradient: k applications give w0 (1 - eps omega)^k (derivation in Section 5), and one
    # application with the scaled hyperparameters of a k-times larger batch gives the same weight
    w0 = rnd(300, 50)
    eps, omega, k = 0.01, 0.0005, 8
    w, v = w0.copy(), np.zeros_like(w0)
    for _ in range(k):
        w, v = oracle.sgd_momentum(w, v, np.zeros_like(w0), 0.0, eps, omega)
    np.testing.assert_allclose(w, w0 * (1 - eps * omega) ** k, rtol=1e-14)
    e2, o2 = oracle.scale_hyperparameters(k, eps, omega)
    w1, _ = oracle.sgd_momentum(w0, np.zeros_like(w0), np.zeros_like(w0), 0.0, e2, o2)
    np.testing.assert_allclose(w1, w, rtol=1e-14)


def test_update_rule_momentum_geometric_series():
    # omega = 0, constant gradient g: vel_k = eps g (1 - mu^k)/(1 - mu), w_k = w0 + sum of the velocities;
    # the gradient enters with a plus sign, as the rule is printed
    w0, g = rnd(301, 40), rnd(302, 40)
    mu, eps, k = 0.9, 0.02, 7
    w, v = w0.copy(), np.zeros_like(w0)
    for _ in range(k):
        w, v = oracle.sgd_momentum(w, v, g, mu, eps, 0.0)
    np.testing.assert_allclose(v, eps * g * (1 - mu ** k) / (1 - mu), rtol=1e-13)
    tot = sum(eps * g * (1 - mu ** j) / (1 - mu) for j in range(1, k + 1))
    np.testing.assert_allclose(w, w0 + tot, rtol=1e-13)


def test_update_rule_one_step_all_terms():
    # one step written out with every term non-zero, gscale folding in the batch mean and a descent sign
    w0, v0, g = rnd(303, 30), rnd(304, 30), rnd(305, 30)
    mu, eps, omega, gs = 0.9, 0.01, 0.0005, -1.0 / 128
    w, v = oracle.sgd_momentum(w0, v0, g, mu, eps, omega, gs)
    dv = 0.9 * v0 + 0.01 * (-g / 128 - 0.0005 * w0)
    np.testing.assert_allclose(v, dv, rtol=1e-14, atol=1e-18)
    np.testing.assert_allclose(w, w0 + dv, rtol=1e-14, atol=1e-18)
    # inputs are not modified, and the float32 build agrees
    w32, v32 = oracle.sgd_momentum(w0.astype(np.float32), v0.astype(np.float32), g.astype(np.float32), mu, eps, omega, gs)
    np.testing.assert_allclose(w32, w, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(v32, v, rtol=1e-6, atol=1e-7)


# ------------------------------------- logistic output layer (Section 5) ----

def test_logistic_xent_textbook_formula_and_shard_targets():
    # moderate logits: the plain formulas with s = 1/(1+exp(-z)) written in numpy
    z = rnd(310, 6, 10) * 3.0
    labels = np.array([12, 3, 15, 10, 19, 7])          # shard owns classes 10..19: samples 1 and 5 have no target here
    loss, dz = oracle.logistic_xent(z, labels, col0=10, scale=0.5)
    t = np.zeros_like(z)
    for n, l in enumerate(labels):
        if 10 <= l < 20:
            t[n, l - 10] = 1.0
    s = 1.0 / (1.0 + np.exp(-z))
    np.testing.assert_allclose(loss, -(t * np.log(s) + (1 - t) * np.log(1 - s)).sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(dz, 0.5 * (s - t), rtol=1e-12, atol=1e-15)
    assert t[1].sum() == 0 and t[5].sum() == 0 and t.sum() == 4


def test_logistic_xent_gradient_by_finite_differences():
    z = rnd(311, 4, 7) * 2.0
    labels = np.array([0, 6, 3, 9])
    _, dz = oracle.logistic_xent(z, labels, 0, 1.0)
    h = 1e-6
    for n in range(4):
        for j in range(7):
            zp, zm = z.copy(), z.copy()
            zp[n, j] += h; zm[n, j] -= h
            fd = (oracle.logistic_xent(zp, labels)[0].sum() - oracle.logistic_xent(zm, labels)[0].sum()) / (2 * h)
            assert abs(fd - dz[n, j]) < 1e-8, (n, j, fd, dz[n, j])


def test_logistic_xent_extreme_logits_stay_finite():
    # |z| large: loss -> |z| on the wrong side and -> 0 on the right side, no inf/nan; z = 0 gives log 2 per unit
    z = np.array([[800.0, -800.0, 0.0, 40.0]])
    loss, dz = oracle.logistic_xent(z, np.array([1]), 0, 1.0)     # target on the -800 unit
    assert np.isfinite(loss).all() and np.isfinite(dz).all()
    np.testing.assert_allclose(loss[0], 800.0 + 800.0 + math.log(2.0) + 40.0, rtol=1e-14)
    np.testing.assert_allclose(dz[0], [1.0, -1.0, 0.5, 1.0], rtol=0, atol=1e-15)
    # the shard sums of disjoint column blocks add up to the whole layer's loss
    zz = rnd(312, 5, 12)
    lab = np.array([0, 5, 11, 7, 3])
    whole, _ = oracle.logistic_xent(zz, lab, 0)
    a, _ = oracle.logistic_xent(zz[:, :7], lab, 0)
    b, _ = oracle.logistic_xent(zz[:, 7:], lab, 7)
    np.testing.assert_allclose(a + b, whole, rtol=1e-13)
