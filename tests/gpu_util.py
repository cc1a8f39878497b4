"""Helpers for the GPU parity tests: move seeded host arrays to the device, call
the C ABI through the binding, bring results back, compare with the oracle."""
import numpy as np
import torch

import oracle

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max|gpu - ref| <= TOL * max|ref|, per output tensor


def owt():
    import paper_1404_5997_amd as m
    return m


class force:
    """Context manager around the library's test hook owt_test_force_variant: inside the block the planner
    is restricted to the given tile / variant number, split count and OWT_FORCE_* flags."""

    def __init__(self, tile=-1, splitk=0, flags=0):
        self.args = (tile, splitk, flags)

    def __enter__(self):
        owt().owt_test_force_variant(*self.args)
        return self

    def __exit__(self, *exc):
        owt().owt_test_force_variant(-1, 0, 0)
        return False


def to_dev(a, dt="f32"):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dt == "bf16" and t.dtype == torch.float32:
        t = t.to(torch.bfloat16)       # inputs are already bf16-representable: exact
    return t


def to_host(t):
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def empty(shape, dt="f32"):
    return torch.empty(shape, device="cuda", dtype=torch.bfloat16 if dt == "bf16" else torch.float32)


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 16), device="cuda", dtype=torch.uint8)


def rel_err(gpu, ref):
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.max(np.abs(ref))
    return float(np.max(np.abs(np.asarray(gpu, dtype=np.float64) - ref)) / (denom if denom > 0 else 1.0))


def assert_close(gpu, ref, dt, what=""):
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), what + ": non-finite values"
    e = rel_err(gpu, ref)
    assert e <= TOL[dt], "%s: max abs err / max|ref| = %.3e > %.1e" % (what, e, TOL[dt])
    return e


def prep(a, dt):
    """bf16 cases: both sides consume the bf16-rounded values."""
    return oracle.round_bf16(a) if dt == "bf16" else a


class ConvCase:
    """One convolution layer on the GPU through the C ABI."""

    def __init__(self, N, C, H, W, K, R, S, stride=1, pad=0, dt="f32", bias=True, relu=True):
        m = owt()
        self.m, self.dt = m, dt
        self.flags = (m.OWT_BIAS if bias else 0) | (m.OWT_RELU if relu else 0)
        self.desc = m.conv_desc(N, C, H, W, K, R, S, stride, pad, m.OWT_BF16 if dt == "bf16" else m.OWT_F32, self.flags)
        sh, sw = (stride, stride) if isinstance(stride, int) else stride
        ph, pw = (pad, pad) if isinstance(pad, int) else pad
        self.P, self.Q = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
        self.shape_x, self.shape_y, self.shape_w = (N, H, W, C), (N, self.P, self.Q, K), (K, R, S, C)

    def ws(self, pass_):
        return workspace(self.m.owt_conv_workspace_bytes(self.desc, pass_))

    def fwd(self, x, w, b):
        y = empty(self.shape_y, self.dt)
        self.m.owt_conv_fwd(self.desc, to_dev(x, self.dt), to_dev(w, self.dt), to_dev(b), y, self.ws(0))
        torch.cuda.synchronize()
        return to_host(y)

    def bwd_data(self, dy, y, w):
        dx = empty(self.shape_x, self.dt)
        self.m.owt_conv_bwd_data(self.desc, to_dev(dy, self.dt), to_dev(y, self.dt), to_dev(w, self.dt), dx, self.ws(1))
        torch.cuda.synchronize()
        return to_host(dx)

    def bwd_filter(self, x, dy, y, alpha=1.0, beta=0.0, dw0=None, db0=None, want_db=True):
        K = self.shape_w[0]
        dw = to_dev(dw0) if dw0 is not None else torch.full(self.shape_w, float("nan"), device="cuda")
        db = None
        if want_db:
            db = to_dev(db0) if db0 is not None else torch.full((K,), float("nan"), device="cuda")
        self.m.owt_conv_bwd_filter(self.desc, to_dev(x, self.dt), to_dev(dy, self.dt), to_dev(y, self.dt),
                                   alpha, beta, dw, db, self.ws(2))
        torch.cuda.synchronize()
        return to_host(dw), (to_host(db) if want_db else None)
