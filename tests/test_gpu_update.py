"""GPU parity of the Section 5 pieces that complete a training step: the
momentum / weight-decay update and the logistic cross-entropy output layer,
against the CPU oracle on the same seeded inputs.

Tolerances: fp32 storage max|gpu - ref| <= 1e-4 * max|ref|, bf16 storage 2e-2
(elementwise fp32 arithmetic lands near 1e-7, which the tests also report).
The bf16 copy of the updated weights is an integer decision (rounding): it is
checked bit for bit against nearest-even rounding of the fp32 weights the GPU
itself wrote, i.e. both sides decide in the kernel's precision.
"""
import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import assert_close, empty, owt, to_dev, to_host  # noqa: E402


def say(*a):
    print(*a)
    sys.stdout.flush()


@pytest.mark.parametrize("n", [1, 3, 4, 1000, 4099, 384 * 3 * 3 * 192, 512 * 9216 + 1])
def test_sgd_momentum_update_parity(n):
    m = owt()
    say("case sgd n =", n)
    g = np.random.default_rng(500 + n % 97)
    w0 = g.standard_normal(n, dtype=np.float32) * np.float32(0.01)
    v0 = g.standard_normal(n, dtype=np.float32) * np.float32(0.001)
    gr = g.standard_normal(n, dtype=np.float32)
    mu, eps, omega, gs = 0.9, 0.01, 0.0005, -1.0 / 128
    w_ref, v_ref = oracle.sgd_momentum(w0, v0, gr, mu, eps, omega, gs)
    w, v, gd = to_dev(w0), to_dev(v0), to_dev(gr)
    wb = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
    m.owt_sgd_momentum_update(n, w, v, gd, mu, eps, omega, gs, wb)
    torch.cuda.synchronize()
    e1 = assert_close(to_host(w), w_ref, "f32", "w")
    e2 = assert_close(to_host(v), v_ref, "f32", "vel")
    say("  rel err w %.2e vel %.2e" % (e1, e2))
    assert e1 < 1e-6 and e2 < 1e-6
    np.testing.assert_array_equal(to_host(gd), gr)                       # the gradient is only read
    np.testing.assert_array_equal(to_host(wb), oracle.round_bf16(to_host(w)))


def test_sgd_momentum_several_steps_without_bf16_copy():
    m = owt()
    n = 192 * 5 * 5 * 64
    g = np.random.default_rng(520)
    w_ref = g.standard_normal(n, dtype=np.float32) * np.float32(0.01)
    v_ref = np.zeros(n, dtype=np.float32)
    w, v = to_dev(w_ref), to_dev(v_ref)
    for step in range(6):
        gr = g.standard_normal(n, dtype=np.float32)
        w_ref, v_ref = oracle.sgd_momentum(w_ref, v_ref, gr, 0.9, 0.02, 0.001, 1.0)    # ascent form, as printed
        m.owt_sgd_momentum_update(n, w, v, to_dev(gr), 0.9, 0.02, 0.001)
    torch.cuda.synchronize()
    assert assert_close(to_host(w), w_ref, "f32", "w after 6 steps") < 2e-6
    assert assert_close(to_host(v), v_ref, "f32", "vel after 6 steps") < 2e-6


def test_sgd_momentum_edge_cases_and_errors():
    m = owt()
    w = to_dev(np.ones(8, dtype=np.float32))
    v = to_dev(np.zeros(8, dtype=np.float32))
    g = to_dev(np.ones(8, dtype=np.float32))
    m.owt_sgd_momentum_update(0, None, None, None, 0.9, 0.01, 0.0)         # n == 0: no-op, pointers not looked at
    with pytest.raises(m.OwtError) as ei:
        m.owt_sgd_momentum_update(8, w, None, g, 0.9, 0.01, 0.0)
    assert ei.value.status == m.OWT_EINVAL
    with pytest.raises(m.OwtError) as ei:
        m.owt_sgd_momentum_update(8, w, v, g, float("nan"), 0.01, 0.0)
    assert ei.value.status == m.OWT_EINVAL
    with pytest.raises(m.OwtError) as ei:
        m.owt_sgd_momentum_update(4, w.data_ptr() + 4, v, g, 0.9, 0.01, 0.0)   # misaligned
    assert ei.value.status == m.OWT_EINVAL
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(w), np.ones(8, dtype=np.float32))  # failed calls launched nothing
    # all coefficients zero except eps, gscale: w += eps*g exactly
    m.owt_sgd_momentum_update(8, w, v, g, 0.0, 0.25, 0.0, 2.0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(w), np.full(8, 1.5, dtype=np.float32))
    np.testing.assert_array_equal(to_host(v), np.full(8, 0.5, dtype=np.float32))


@pytest.mark.parametrize("N,O,col0,dt", [(128, 125, 0, "f32"), (128, 125, 875, "f32"), (128, 125, 250, "bf16"),
                                         (5, 1, 3, "f32"), (3, 64, 0, "f32"), (7, 65, 64, "bf16"), (130, 1000, 0, "f32")])
def test_logistic_xent_parity(N, O, col0, dt):
    m = owt()
    say("case xent", N, O, col0, dt)
    g = np.random.default_rng(540 + N + O)
    z = (g.standard_normal((N, O), dtype=np.float32) * np.float32(4.0))
    if dt == "bf16":
        z = oracle.round_bf16(z)
    labels = g.integers(0, 1000, size=N).astype(np.int32)
    labels[: min(N, 3)] = [col0, col0 + O - 1, max(col0 - 1, 0)][: min(N, 3)]    # first / last owned class, one outside
    scale = 1.0 / N
    loss_ref, dz_ref = oracle.logistic_xent(z, labels, col0, scale)
    if dt == "bf16":
        dz_ref = oracle.round_bf16(dz_ref)
    zd, ld = to_dev(z, dt), torch.from_numpy(labels).cuda()
    loss, dz = empty((N,)), empty((N, O), dt)
    m.owt_logistic_xent(N, O, col0, m.OWT_BF16 if dt == "bf16" else m.OWT_F32, zd, ld, scale, loss, dz)
    torch.cuda.synchronize()
    e1 = assert_close(to_host(loss), loss_ref, "f32", "loss")
    e2 = assert_close(to_host(dz), dz_ref, dt, "dz")
    say("  rel err loss %.2e dz %.2e" % (e1, e2))
    assert e1 < 1e-5
    # in place (dz aliases z) gives the same bits
    m.owt_logistic_xent(N, O, col0, m.OWT_BF16 if dt == "bf16" else m.OWT_F32, zd, ld, scale, loss, zd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(zd), to_host(dz))


def test_logistic_xent_extreme_logits_and_errors():
    m = owt()
    z = np.array([[80.0, -80.0, 0.0, 1e4, -1e4, 3.0, -3.0, 20.0]], dtype=np.float32)
    labels = np.array([1], dtype=np.int32)
    loss_ref, dz_ref = oracle.logistic_xent(z, labels, 0, 1.0)
    loss, dz = empty((1,)), empty((1, 8))
    m.owt_logistic_xent(1, 8, 0, m.OWT_F32, to_dev(z), torch.from_numpy(labels).cuda(), 1.0, loss, dz)
    torch.cuda.synchronize()
    assert_close(to_host(loss), loss_ref, "f32", "loss")
    assert_close(to_host(dz), dz_ref, "f32", "dz")
    before = to_host(dz).copy()
    for bad in (dict(N=0), dict(O=0), dict(col0=-1), dict(z=None)):
        with pytest.raises(m.OwtError) as ei:
            m.owt_logistic_xent(bad.get("N", 1), bad.get("O", 8), bad.get("col0", 0), m.OWT_F32,
                                bad.get("z", to_dev(z)), torch.from_numpy(labels).cuda(), 1.0, loss, dz)
        assert ei.value.status == m.OWT_EINVAL
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(dz), before)


def test_fc3_shard_with_logistic_output_chain():
    # the worker's FC3 shard (4096 -> 125 of 1000 units, K = 8) followed by the logistic output layer and
    # its backward pass: logits, loss share, dz, then dx_partial / dw / db of the shard
    m = owt()
    N, I, O, K, rank = 128, 4096, 1000, 8, 3
    Ol, col0 = O // K, rank * (O // K)
    g = np.random.default_rng(560)
    x = np.maximum(g.standard_normal((N, I), dtype=np.float32), 0) * np.float32(0.05)
    w = g.standard_normal((Ol, I), dtype=np.float32) * np.float32(0.005)
    b = g.standard_normal((Ol,), dtype=np.float32) * np.float32(0.005)
    labels = g.integers(0, O, size=N).astype(np.int32)
    z_ref = oracle.fc_fwd(x, w, b, relu=False)
    loss_ref, dz_ref = oracle.logistic_xent(z_ref, labels, col0, 1.0)
    dx_ref, dw_ref, db_ref = oracle.fc_bwd(x, w, dz_ref, None, 1.0 / N, 0.0)

    d = m.fc_desc(N, I, O, K, rank, m.OWT_F32, m.OWT_BIAS)
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    zt, loss, dz = empty((N, Ol)), empty((N,)), empty((N, Ol))
    ws = torch.empty(max(m.owt_fc_workspace_bytes(d, 0), m.owt_fc_workspace_bytes(d, 1), 16), device="cuda", dtype=torch.uint8)
    m.owt_fc_shard_fwd(d, xd, wd, bd, zt, ws)
    m.owt_logistic_xent(N, Ol, col0, m.OWT_F32, zt, torch.from_numpy(labels).cuda(), 1.0, loss, dz)
    dx, dw, db = empty((N, I)), empty((Ol, I)), empty((Ol,))
    m.owt_fc_shard_bwd(d, xd, wd, None, dz, 1.0 / N, 0.0, dx, dw, db, ws)
    torch.cuda.synchronize()
    assert_close(to_host(zt), z_ref, "f32", "logits")
    assert_close(to_host(loss), loss_ref, "f32", "loss")
    assert_close(to_host(dz), dz_ref, "f32", "dz")
    assert_close(to_host(dx), dx_ref, "f32", "dx_partial")
    assert_close(to_host(dw), dw_ref, "f32", "dw")
    assert_close(to_host(db), db_ref, "f32", "db")
