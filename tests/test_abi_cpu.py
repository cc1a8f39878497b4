"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, rejects bad arguments before touching the device, and its workspace queries and
host self-test behave."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def m():
    import paper_1404_5997_amd as mod
    return mod


def test_every_declared_symbol_is_exported(m):
    hdr = open(os.path.join(ROOT, "include", "owt.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(owt_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(m.EXPORTS)
    lib = ctypes.CDLL(m.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def test_host_selftest(m):
    assert m.owt_selftest_host() == 0, m.owt_last_error()
    assert m.owt_abi_version() == 3


def test_bad_descriptors_are_rejected_before_any_launch(m):
    ok = dict(N=2, C=8, H=6, W=6, K=8, R=3, S=3, stride=1, pad=1)
    for bad in (dict(N=0), dict(C=-1), dict(R=0), dict(stride=0), dict(pad=3), dict(pad=-1), dict(H=1, pad=0, R=3)):
        g = dict(ok); g.update(bad)
        d = m.conv_desc(g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], g["stride"], g["pad"])
        with pytest.raises(m.OwtError) as ei:
            m.owt_conv_fwd(d, 256, 512, None, 1024, None, 0)
        assert ei.value.status == m.OWT_EINVAL, bad
        with pytest.raises(m.OwtError):
            m.owt_conv_workspace_bytes(d, 0)
    d = m.conv_desc(2, 8, 6, 6, 8, 3, 3, 1, 1, dtype=7)
    with pytest.raises(m.OwtError):
        m.owt_conv_bwd_data(d, 256, None, 512, 1024, None, 0)
    d = m.conv_desc(2, 8, 6, 6, 8, 3, 3, 1, 1, flags=8)
    with pytest.raises(m.OwtError):
        m.owt_conv_bwd_filter(d, 256, 512, None, 1.0, 0.0, 1024, None, None, 0)
    d = m.conv_desc(2, 8, 6, 6, 8, 3, 3, 1, 1)
    for args in ((None, 512, None, 1024), (256, None, None, 1024), (256, 512, None, None), (260, 512, None, 1024)):
        with pytest.raises(m.OwtError) as ei:
            m.owt_conv_fwd(d, *args, None, 0)
        assert ei.value.status == m.OWT_EINVAL
    with pytest.raises(m.OwtError):
        m.owt_conv_workspace_bytes(d, 3)
    # too many elements for 32-bit indexing
    d = m.conv_desc(4096, 64, 224, 224, 64, 3, 3, 1, 1)
    with pytest.raises(m.OwtError) as ei:
        m.owt_conv_fwd(d, 256, 512, None, 1024, None, 0)
    assert ei.value.status == m.OWT_EUNSUPPORTED


def test_fc_descriptor_checks(m):
    for bad in (dict(N=0), dict(I=0), dict(O_total=1001), dict(workers=0), dict(rank=8), dict(rank=-1)):
        g = dict(N=128, I=4096, O_total=1000, workers=8, rank=0); g.update(bad)
        d = m.fc_desc(g["N"], g["I"], g["O_total"], g["workers"], g["rank"])
        with pytest.raises(m.OwtError) as ei:
            m.owt_fc_shard_fwd(d, 256, 512, None, 1024, None, 0)
        assert ei.value.status == m.OWT_EINVAL, bad
    d = m.fc_desc(128, 4096, 1000, 8, flags=m.OWT_RELU)
    with pytest.raises(m.OwtError):       # ReLU mask needs y
        m.owt_fc_shard_bwd(d, 256, 512, None, 1024, 1.0, 0.0, None, 2048, None, None, 0)


def test_pool_argument_checks(m):
    for args in ((0, 8, 8, 4, 3, 2), (1, 8, 8, 4, 1, 2), (1, 8, 8, 4, 16, 2), (1, 8, 8, 4, 3, 0), (1, 2, 8, 4, 3, 2)):
        with pytest.raises(m.OwtError) as ei:
            m.owt_maxpool_fwd(*args, m.OWT_F32, 256, 512, 1024, 0)
        assert ei.value.status == m.OWT_EINVAL
    with pytest.raises(m.OwtError):
        m.owt_maxpool_bwd(1, 8, 8, 4, 3, 2, m.OWT_F32, None, 512, 1024, 0)


def test_workspace_queries_are_stable_and_sized_for_split_k(m):
    d = m.conv_desc(128, 192, 13, 13, 384, 3, 3, 1, 1)
    a = [m.owt_conv_workspace_bytes(d, p) for p in range(3)]
    assert a == [m.owt_conv_workspace_bytes(d, p) for p in range(3)]
    # the filter gradient reduces over N*P*Q = 21632 positions into only 384 x 1728 outputs: it must be split
    assert a[2] > 0 and a[2] % (384 * 1728 * 4) < 384 * 1728 * 4
    f = m.fc_desc(128, 9216, 4096, 8)
    assert m.owt_fc_workspace_bytes(f, 0) > 0     # 128 x 512 outputs cannot fill 256 CUs without split-K
    # a layer's buffer may be sized with the descriptor that carries OWT_RELU and used by calls that pass no y (their
    # candidates include the kernels that take dz as it is): the bound must not depend on the flag
    for dt, shape in ((m.OWT_F32, (128, 192, 13, 13, 384, 3, 3, 1, 1)), (m.OWT_BF16, (1024, 384, 13, 13, 256, 3, 3, 1, 1)),
                      (m.OWT_BF16, (1024, 64, 27, 27, 192, 5, 5, 1, 2)), (m.OWT_F32, (128, 3, 224, 224, 64, 11, 11, 4, 2))):
        masked = m.conv_desc(*shape, dt, m.OWT_BIAS | m.OWT_RELU)
        plain = m.conv_desc(*shape, dt, m.OWT_BIAS)
        for ps in range(3):
            assert m.owt_conv_workspace_bytes(masked, ps) == m.owt_conv_workspace_bytes(plain, ps)


def test_scale_hyperparameters_host_call_matches_the_papers_example(m):
    # host arithmetic only (no GPU): Section 5's worked example, values as printed in the paper
    import math
    vals = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                vals[line[0]] = float(line[1])
    e2, o2 = m.owt_scale_hyperparameters(vals["wd_example_k"], vals["wd_example_eps"], vals["wd_example_omega"])
    assert abs(e2 - math.sqrt(8.0) * 0.01) < 1e-15
    assert abs(o2 - vals["wd_example_omega_scaled"]) < 5e-11
    with pytest.raises(m.OwtError):
        m.owt_scale_hyperparameters(0.0, 0.01, 0.0005)


def test_bench_refuses_more_than_one_gpu():
    # this build runs one worker on one GPU: bench.py must say so and exit before touching a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_static_scratch_entry_rejects_what_does_not_fit_before_any_launch(m):
    # owt_conv_bwd_filter_static keeps its partial sums in a 64 MiB static device array; with every candidate
    # forced to 64 splits of a 1024 x 9216 gradient (2.4 GB of partial sums) nothing fits: clear error, no launch
    assert m.owt_static_scratch_bytes() == 64 << 20
    d = m.conv_desc(64, 1024, 13, 13, 1024, 3, 3, 1, 1, m.OWT_F32, 0)
    m.owt_test_force_variant(-1, 64, 0)
    try:
        with pytest.raises(m.OwtError) as ei:
            m.owt_conv_bwd_filter_static(d, 256, 512, None, 1.0, 0.0, 1024, None, 0)
    finally:
        m.owt_test_force_variant(-1, 0, 0)
    assert ei.value.status == m.OWT_EWORKSPACE and "static buffer" in str(ei.value)
