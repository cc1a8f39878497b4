"""owt_conv_bwd_filter_static (the entry point for callers that cannot allocate: its split
reduction's partial sums live in a static device array inside the library) against
owt_conv_bwd_filter with a caller workspace: same inputs, two calls in a row, the second on a
smaller layer, so stale partial sums of the first call sit in the array while the second runs."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import TOL, ConvCase, assert_close, force, owt, to_dev, to_host  # noqa: E402


def say(*a):
    print(*a)
    sys.stdout.flush()


def _one(m, shape, seed, alpha, beta, relu, dt="f32"):
    import oracle
    N, C, H, W, K, R, S, stride, pad = shape
    case = ConvCase(N, C, H, W, K, R, S, stride, pad, dt, True, relu)
    g = np.random.default_rng(seed)
    r = (lambda a: oracle.round_bf16(a)) if dt == "bf16" else (lambda a: a)
    x = r(g.standard_normal(case.shape_x, dtype=np.float32))
    dy = r(g.standard_normal(case.shape_y, dtype=np.float32))
    y = r(g.standard_normal(case.shape_y, dtype=np.float32)) if relu else None
    dw0 = g.standard_normal(case.shape_w, dtype=np.float32)
    db0 = g.standard_normal((K,), dtype=np.float32)
    say("static-scratch case", shape, "plan:", m.owt_conv_plan_describe(case.desc, m.OWT_PASS_BWD_FILTER))
    dw_ref, db_ref = case.bwd_filter(x, dy, y, alpha, beta, dw0, db0)          # caller workspace
    dw, db = to_dev(dw0), to_dev(db0)
    m.owt_conv_bwd_filter_static(case.desc, to_dev(x, dt), to_dev(dy, dt), to_dev(y, dt), alpha, beta, dw, db)
    torch.cuda.synchronize()
    e1 = assert_close(to_host(dw), dw_ref, "f32", "dw (static scratch) %s" % (shape,))
    e2 = assert_close(to_host(db), db_ref, "f32", "db (static scratch) %s" % (shape,))
    say("  rel err vs owt_conv_bwd_filter: dw %.2e db %.2e" % (e1, e2))
    return e1, e2


def test_static_scratch_filter_gradient_equals_the_workspace_call_twice_in_a_row():
    m = owt()
    assert m.owt_static_scratch_bytes() == 64 << 20
    # the benchmark's third layer at batch 128 first: the variant the workspace call runs needs more partial sums
    # than the static array holds once it is split 26 ways or more (384 x 1728 floats per split), so the
    # static call may run another variant (summation order differs); then smaller layers, the last one strided
    # (its split reduction is a different kernel's)
    _one(m, (128, 192, 13, 13, 384, 3, 3, 1, 1), 0, 1.0 / 128, 0.0, True)
    _one(m, (16, 192, 13, 13, 384, 3, 3, 1, 1), 1, 1.0, 0.0, True)
    _one(m, (4, 40, 13, 13, 136, 3, 3, 1, 1), 2, 0.5, -0.25, False)
    with force(-1, 5):
        _one(m, (3, 12, 15, 15, 36, 3, 3, 2, 1), 3, 1.0 / 3, 1.0, True)
    # bf16 storage, dz taken as it is: the kernels that stream their operands straight into LDS
    _one(m, (64, 192, 13, 13, 384, 3, 3, 1, 1), 4, 1.0 / 64, 0.0, False, "bf16")
    _one(m, (4, 3, 64, 64, 64, 11, 11, 4, 2), 5, 0.5, -0.25, False, "bf16")
