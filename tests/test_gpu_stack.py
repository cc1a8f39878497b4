"""GPU parity of the chained hot path at the benchmark's full sizes and launch
configuration: the five-layer convolution stack (configs 3 and 5, and the paper's
own filter counts) and the stack plus fully-connected shards (config 4).

The whole batch runs on the GPU and the oracle redoes the WHOLE batch (a
128-image step is a few seconds of host time), so every element of every tensor
of the step is compared:
 * forward: the oracle runs free from the input images and every layer's output
   and pooled map is compared, all images;
 * pooling: the GPU's pooled maxima and arg-max must equal, bit for bit, the
   oracle's pooling of the GPU's own convolution output (all images);
 * backward-data: the oracle back-propagates the same upstream gradient, using
   the GPU's forward outputs as ReLU masks and the GPU's arg-max (both just
   shown valid), and every layer's dz (and dx) is compared, all images.  ReLU
   and arg-max are not smooth, so an element that is +1e-9 on one side and 0 on
   the other would otherwise move gradients by far more than rounding; feeding
   both sides the same mask makes every backward call a pure function of its
   inputs;
 * backward-filter: every entry of every layer's dw and db is recomputed by the
   oracle from the GPU's full-batch inputs of that call.
Each check runs twice: with the variants the library's cost model picks, and
again after ConvStack.autotune(), i.e. with the variants bench.py times.
(`images` restricts the forward / backward-data comparison to a list of image
blocks and dw to sampled entries: used for one of the two bf16 passes at batch
1024, where the oracle's step takes half a minute.)
"""
import sys

import numpy as np
import pytest

import oracle
import synthetic_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import TOL, assert_close, rel_err, to_host  # noqa: E402


def say(*a):
    print(*a)
    sys.stdout.flush()


def build_stack(config, N, dt, with_fc=False, filters=None):
    from paper_1404_5997_amd.stack import ConvStack
    r = (lambda a: oracle.round_bf16(a)) if dt == "bf16" else (lambda a: a)
    x = r(si.stack_input(config, N))
    ws, bs = si.stack_params(config, filters)
    ws = [r(w) for w in ws]
    layers = [dict(L, K=(filters[i] if filters else L["K"])) for i, L in enumerate(si.STACK_LAYERS)]
    st = ConvStack(N, layers, si.STACK_INPUT_HWC, (si.POOL_WIN, si.POOL_STRIDE), dt,
                   fc_layers=si.FC_LAYERS if with_fc else None, fc_workers=si.FC_WORKERS)
    fc = None
    if with_fc:
        fws, fbs = si.fc_params(config)
        fws = [r(w) for w in fws]
        peers = [r(si.fc_peer_columns(config, i, N)) for i in range(2)]
        st.load(x, ws, bs, fws, fbs, peers)
        fc = (fws, fbs, peers)
    else:
        st.load(x, ws, bs)
    g = r(si.upstream_grad(config, 90, tuple(st.top_grad().shape)))
    st.top_grad().copy_(torch.from_numpy(g).to(st.tdt))
    return st, x, ws, bs, g, fc


def describe_plans(st):
    m = __import__("paper_1404_5997_amd")
    for li, e in enumerate(st.L):
        d = e["desc_bwd"] if e["dz_ready"] else e["desc"]
        say("  conv%d plans: %s | %s | %s" % (li + 1, m.owt_conv_plan_describe(e["desc"], 0).split(" grid")[0],
                                             m.owt_conv_plan_describe(d, 1).split(" grid")[0] if li else "-",
                                             m.owt_conv_plan_describe(d, 2).split(" grid")[0]))


def check_conv_stack(st, x, ws, bs, dtop_pooled, dt, images=None, n_dw_samples=96):
    """dtop_pooled: host copy of the gradient w.r.t. the last pooled map, as the GPU backward consumed it.
    images: None = every image and every dw entry; else a list of image indices (forward / backward-data on
    those images only, dw sampled)."""
    N = st.N
    rnd = (lambda a: oracle.round_bf16(a)) if dt == "bf16" else (lambda a: a)
    full = images is None
    sub = slice(0, N) if full else np.asarray(images)
    pick = (lambda t: to_host(t)) if full else (lambda t: to_host(t[torch.as_tensor(sub, device=t.device)]))
    win, pst = si.POOL_WIN, si.POOL_STRIDE
    specs = [dict(stride=s["stride"], pad=s["pad"], pool=s["pool"]) for s in si.STACK_LAYERS]

    # ---- forward, free-running oracle
    cur = x[sub]
    flips = []
    for li, (e, spec) in enumerate(zip(st.L, specs)):
        y_ref = rnd(oracle.conv_fwd(cur, ws[li], bs[li], spec["stride"], spec["pad"], True))
        y_gpu = pick(e["y"])
        err = assert_close(y_gpu, y_ref, dt, "conv%d fwd" % (li + 1))
        flips.append(int(np.sum((y_gpu > 0) != (y_ref > 0))))
        cur = y_ref
        if spec["pool"]:
            a_ref, _ = oracle.maxpool_fwd(y_ref, win, pst)
            assert_close(pick(e["a"]), a_ref, dt, "pool%d fwd" % (li + 1))
            cur = a_ref
        say("  conv%d fwd rel err %.2e on %d images, ReLU mask disagreements %d of %d" %
            (li + 1, err, y_ref.shape[0], flips[-1], y_ref.size))
        del y_gpu, y_ref

    # ---- pooling of the GPU's own conv output: exact, all images
    for li, e in enumerate(st.L):
        if not e["pool"]:
            continue
        y_gpu = to_host(e["y"])
        a_ref, am_ref = oracle.maxpool_fwd(y_gpu, win, pst)
        np.testing.assert_array_equal(to_host(e["a"]), a_ref)
        np.testing.assert_array_equal(e["am"].cpu().numpy(), am_ref)
        del y_gpu, a_ref, am_ref
    say("  pooled maxima and arg-max exact on all images")

    # ---- backward chain, GPU masks / arg-max as inputs.  The stack applies each layer's ReLU mask where the
    # gradient w.r.t. that layer's output is PRODUCED (fused into the pooling backward, or into the store of
    # the next layer's bwd-data), so every e["dy"] holds dz = dy * [y > 0]; the oracle applies the mask as its
    # own elementwise step.
    g = dtop_pooled[sub]
    for li in range(len(st.L) - 1, -1, -1):
        e, spec = st.L[li], specs[li]
        Nn, C, H, W, K, R, stv, pad, P, Q = e["geom"]
        y_mask = pick(e["y"])
        if spec["pool"]:
            g = rnd(oracle.maxpool_bwd(g, pick(e["am"]) if not full else e["am"].cpu().numpy(), (P, Q), win, pst))
        assert e["dz_ready"]
        dz = g * (y_mask > 0)
        err = assert_close(pick(e["dy"]), dz, dt, "conv%d dz" % (li + 1))
        say("  conv%d dz rel err %.2e on %d images" % (li + 1, err, dz.shape[0]))
        if li == 0:
            break
        g = rnd(oracle.conv_bwd_data(dz, ws[li], (H, W), stv, pad))
        prev = st.L[li - 1]
        if prev["pool"]:
            err = assert_close(pick(prev["da"]), g, dt, "conv%d bwd_data" % (li + 1))
            say("  conv%d bwd_data rel err %.2e" % (li + 1, err))
        del y_mask, dz

    # ---- backward-filter from the GPU's full-batch call inputs: all of dw and db (or sampled dw entries)
    rs = np.random.default_rng(123)
    for li, e in enumerate(st.L):
        Nn, C, H, W, K, R, stv, pad, P, Q = e["geom"]
        xin, dyin = to_host(e["x"]), to_host(e["dy"])          # dyin is dz
        dw = e["dw"].cpu().numpy()
        if full:
            dw_ref, db_ref = oracle.conv_bwd_filter(xin, dyin, (R, R), stv, pad, alpha=st.alpha)
            err = assert_close(dw, dw_ref, "f32", "conv%d dw" % (li + 1))
            errb = assert_close(e["db"].cpu().numpy(), db_ref, "f32", "conv%d db" % (li + 1))
            say("  conv%d dw (all %d entries) rel err %.2e, db rel err %.2e" % (li + 1, dw.size, err, errb))
        else:
            idx = np.stack([rs.integers(0, K, n_dw_samples), rs.integers(0, R, n_dw_samples),
                            rs.integers(0, R, n_dw_samples), rs.integers(0, C, n_dw_samples)], axis=1).astype(np.int32)
            idx[0] = (0, 0, 0, 0); idx[1] = (K - 1, R - 1, R - 1, C - 1)
            ref = oracle.conv_bwd_filter_at(xin, dyin, idx, (R, R), stv, pad).astype(np.float64) * st.alpha
            got = dw[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]]
            scale = np.max(np.abs(dw))          # the tensor's max norm (the sample need not contain it)
            err = float(np.max(np.abs(got - ref)) / scale)
            assert np.isfinite(dw).all() and err <= TOL["f32"], "conv%d dw: %.3e" % (li + 1, err)
            # db[k] = alpha * sum dz: the dense-layer oracle on a [N*P*Q, K] matrix with a zero input column
            rows = Nn * P * Q
            _, _, db_ref = oracle.fc_bwd(np.zeros((rows, 1), np.float32), np.zeros((K, 1), np.float32),
                                         dyin.reshape(rows, K), alpha=st.alpha, want_dx=False)
            errb = assert_close(e["db"].cpu().numpy(), db_ref, "f32", "conv%d db" % (li + 1))
            say("  conv%d dw (sampled %d) rel err %.2e, db rel err %.2e" % (li + 1, n_dw_samples, err, errb))
        del xin, dyin
    return flips


def run_and_check_twice(st, x, ws, bs, dt, dtop=None, first_images=None):
    """The step with the cost model's variants, then with the tuned ones (what bench.py times); both compared
    with the oracle.  dtop: callable giving the host gradient of the last pooled map after a step."""
    flips = None
    for tuned in (False, True):
        if tuned:
            st.autotune()
        st.step()
        torch.cuda.synchronize()
        say("%s variants:" % ("tuned" if tuned else "cost-model"))
        describe_plans(st)
        flips = check_conv_stack(st, x, ws, bs, dtop(), dt, images=None if tuned else first_images)
    return flips


def test_config3_conv_stack_fp32_batch128():
    st, x, ws, bs, g, _ = build_stack(3, 128, "f32")
    assert st.out_shape == (128, 6, 6, 256)
    flips = run_and_check_twice(st, x, ws, bs, "f32", lambda: g)
    total = sum(e["y"].numel() for e in st.L)
    say("ReLU mask disagreements of the free-running forward: %d of %d" % (sum(flips), total))
    assert sum(flips) <= 1e-5 * total


def test_paper_filter_counts_conv_stack_fp32_batch128():
    # the network as Section 5's footnote sizes it: 64, 192, 384, 384, 256 filters (conv4 384 -> 384 and
    # conv5 384 -> 256, reduction length 3456 each)
    st, x, ws, bs, g, _ = build_stack(3, 128, "f32", filters=si.PAPER_FILTERS)
    assert st.out_shape == (128, 6, 6, 256) and st.L[3]["geom"][4] == 384 and st.L[4]["geom"][1] == 384
    run_and_check_twice(st, x, ws, bs, "f32", lambda: g)


def test_config5_conv_stack_bf16_batch1024():
    st, x, ws, bs, g, _ = build_stack(5, 1024, "bf16")
    # cost-model variants: first, middle and last image blocks, sampled dw; tuned variants: everything
    run_and_check_twice(st, x, ws, bs, "bf16", lambda: g, first_images=[0, 1, 511, 512, 1022, 1023])


@pytest.mark.parametrize("tuned", [False, True])
def test_config4_stack_plus_fc_shard_fp32(tuned):
    st, x, ws, bs, g, (fws, fbs, peers) = build_stack(4, 128, "f32", with_fc=True)
    if tuned:
        st.autotune()
    st.step()
    torch.cuda.synchronize()
    # every dense call against the oracle on the GPU's inputs of that call (full batch: they are small)
    for i, (f, spec) in enumerate(zip(st.F, si.FC_LAYERS)):
        xin = to_host(f["x"])
        y_ref = oracle.fc_fwd(xin, fws[i], fbs[i], spec["relu"])
        e1 = assert_close(to_host(f["y"]), y_ref, "f32", "fc%d fwd" % (i + 1))
        dyin = to_host(f["dy"])
        dx_ref, dw_ref, db_ref = oracle.fc_bwd(xin, fws[i], dyin, y=to_host(f["y"]) if spec["relu"] else None,
                                               alpha=st.alpha)
        e2 = assert_close(to_host(f["dx"]), dx_ref, "f32", "fc%d dx_partial" % (i + 1))
        e3 = assert_close(to_host(f["dw"]), dw_ref, "f32", "fc%d dw" % (i + 1))
        e4 = assert_close(to_host(f["db"]), db_ref, "f32", "fc%d db" % (i + 1))
        say("  fc%d rel err fwd %.2e dx %.2e dw %.2e db %.2e" % (i + 1, e1, e2, e3, e4))
        if i > 0:   # the hand-over between layers: own columns in front, the peers' columns behind
            own = st.F[i - 1]["O"]
            np.testing.assert_array_equal(xin[:, :own], to_host(st.F[i - 1]["y"]))
            np.testing.assert_array_equal(xin[:, own:], peers[i - 1])
            np.testing.assert_array_equal(to_host(st.F[i - 1]["dy"]), to_host(f["dx"])[:, :own])
    # the convolution part under the gradient the dense shards hand down (= fc1's dx_partial, reshaped): every
    # image, every dw entry
    check_conv_stack(st, x, ws, bs, to_host(st.L[-1]["da"]), "f32")


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_training_step_with_logistic_output_and_weight_update(dt):
    # One worker's whole step: conv stack + dense shards, logistic cross-entropy output layer on the
    # worker's 125 columns, backward, and the Section 5 update over every parameter in one launch.
    # Each added call is checked against the oracle on the GPU's own inputs of that call.
    N = 128 if dt == "f32" else 64
    st, x, ws, bs, g, (fws, fbs, peers) = build_stack(4, N, dt, with_fc=True)
    labels = np.random.default_rng(si.BASE_SEED + 4099).integers(0, 1000, size=N).astype(np.int32)
    labels[:4] = [0, 124, 125, 999]                      # first / last owned class, two outside the shard
    st.set_labels(labels)
    st.step()
    torch.cuda.synchronize()
    f = st.F[-1]
    z = to_host(f["y"])
    loss_ref, dz_ref = oracle.logistic_xent(z, labels, 0, 1.0)
    if dt == "bf16":
        dz_ref = oracle.round_bf16(dz_ref)
    assert_close(to_host(st.loss), loss_ref, "f32", "loss share")
    assert_close(to_host(f["dy"]), dz_ref, dt, "dz of the output layer")
    say("  mean loss share per image %.4f (125 units at logit ~0 -> 125 ln2 = %.4f)" % (loss_ref.mean(), 125 * np.log(2)))
    # the gradients that the update consumes came out of that backward pass
    assert np.isfinite(to_host(st.grads)).all() and float(st.grads.abs().max()) > 0
    p0, v0, g0 = to_host(st.params), to_host(st.vel), to_host(st.grads)
    mu, eps, omega = 0.9, 0.01, 0.0005
    for it in range(2):      # second application has non-zero momentum state
        p_ref, v_ref = oracle.sgd_momentum(p0, v0, g0, mu, eps, omega, -1.0)
        st.update(mu, eps, omega)
        torch.cuda.synchronize()
        p1, v1 = to_host(st.params), to_host(st.vel)
        assert assert_close(p1, p_ref, "f32", "parameters after update %d" % it) < 1e-6
        assert assert_close(v1, v_ref, "f32", "momentum after update %d" % it) < 1e-6
        p0, v0 = p1, v1
    # views alias the arrays: every layer sees its new weights, bf16 stacks their rounded copy
    for e in st.L + st.F:
        w32 = to_host(e["w32"])
        assert w32.shape == tuple(e["wshape"])
        if dt == "bf16":
            np.testing.assert_array_equal(to_host(e["w"]), oracle.round_bf16(w32))
        else:
            assert e["w"].data_ptr() == e["w32"].data_ptr()
    assert not np.array_equal(to_host(st.L[0]["w32"]), ws[0])
    # and the next step runs on them
    st.step()
    torch.cuda.synchronize()
    assert np.isfinite(to_host(st.loss)).all()


def test_hip_graph_replay_of_a_step_equals_eager_launches():
    # the step recorded into a HIP graph (no memset nodes: the library records kernels only) and replayed
    # several times, with eager steps and synchronisations in between, gives the eager step's bits
    st, x, ws, bs, g, _ = build_stack(4, 8, "f32", with_fc=True)
    st.step()
    torch.cuda.synchronize()
    ref_g, ref_y, ref_dx = st.grads.clone(), st.F[-1]["y"].clone(), st.L[1]["dy"].clone()
    st.capture()
    for it in range(4):
        st.grads.zero_(); st.F[-1]["y"].zero_(); st.L[1]["dy"].zero_()
        st.replay()
        torch.cuda.synchronize()
        assert torch.equal(st.grads, ref_g) and torch.equal(st.F[-1]["y"], ref_y) and torch.equal(st.L[1]["dy"], ref_dx), it
        st.step()                                   # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(st.grads, ref_g)


def _kpass_inputs(st, K, seed):
    g = np.random.default_rng(si.BASE_SEED + seed)
    I0 = st.F[0]["I"]
    peer = [np.maximum(g.standard_normal((st.N, I0), dtype=np.float32), 0) * np.float32(0.05) for _ in range(K - 1)]
    labels = [g.integers(0, 1000, size=st.N).astype(np.int32) for _ in range(K)]
    dev = [torch.from_numpy(p).cuda() for p in peer]
    lab = [torch.from_numpy(l).cuda() for l in labels]
    return peer, labels, dev, lab


def _oracle_fc_chain(feats, fws, fbs, peers, labels, alpha):
    """Free-running oracle pass through the three dense shards on `feats` (any number of rows; the
    peers' hidden columns are repeated per block of N rows).  Returns dx of the features and [(dw, db)]."""
    rows = feats.shape[0]
    reps = rows // peers[0].shape[0]
    xs, ys, cur = [], [], feats
    for i, spec in enumerate(si.FC_LAYERS):
        if i > 0:
            cur = np.concatenate([ys[-1], np.tile(peers[i - 1], (reps, 1))], axis=1)
        xs.append(cur)
        ys.append(oracle.fc_fwd(cur, fws[i], fbs[i], spec["relu"]))
    loss, dtop = oracle.logistic_xent(ys[-1], labels, 0, 1.0)
    grads = [None] * 3
    for i in range(2, -1, -1):
        dx, dw, db = oracle.fc_bwd(xs[i], fws[i], dtop, y=ys[i] if si.FC_LAYERS[i]["relu"] else None, alpha=alpha)
        grads[i] = (dw, db)
        dtop = dx[:, :ys[i - 1].shape[1]] if i > 0 else dx
    return dtop, grads, loss


@pytest.mark.parametrize("overlap", [False, True])
def test_kpass_dense_schedule_accumulating_equals_one_big_batch(overlap):
    # Section 4 scheme (b) with K = 8: eight forward+backward iterations of the dense shards, gradients
    # accumulated (beta = 1) with alpha = 1/(8*128), must equal ONE pass over the 1024 examples at once
    # (Section 4.2: the schedule is synchronous SGD on 128K examples).  The oracle does the big batch.
    K = 8
    st, x, ws, bs, g, (fws, fbs, peers) = build_stack(4, 128, "f32", with_fc=True)
    peer, labels, dev, lab = _kpass_inputs(st, K, 4200)
    st.step_kpass(dev, lab, None, overlap)
    torch.cuda.synchronize()
    own = to_host(st.F[0]["x"]) if False else to_host(st.L[-1]["a"]).reshape(st.N, -1)
    big = np.concatenate([own] + peer, axis=0)
    dfeat, grads, _ = _oracle_fc_chain(big, fws, fbs, peers, np.concatenate(labels), 1.0 / (st.N * K))
    for i, f in enumerate(st.F):
        e1 = assert_close(to_host(f["dw"]), grads[i][0], "f32", "fc%d dw accumulated over %d passes" % (i + 1, K))
        e2 = assert_close(to_host(f["db"]), grads[i][1], "f32", "fc%d db accumulated" % (i + 1))
        say("  fc%d accumulated dw %.2e db %.2e" % (i + 1, e1, e2))
    assert_close(to_host(st.L[-1]["da"]).reshape(st.N, -1), dfeat[:st.N], "f32", "gradient of the own batch's activations")
    assert_close(to_host(st.peer_dx), dfeat[-st.N:], "f32", "gradient addend for the last peer's batch")
    # the convolution backward pass ran from the own batch's gradient: same bits as running it again
    conv_g = st.grads[:st.fc_offset].clone()
    assert float(conv_g.abs().max()) > 0
    st.backward_conv()
    torch.cuda.synchronize()
    assert torch.equal(conv_g, st.grads[:st.fc_offset])


@pytest.mark.parametrize("overlap", [False, True])
def test_kpass_dense_schedule_with_an_update_after_every_pass(overlap):
    # the variable batch size of Section 4.2: the dense weights move after each of the K iterations
    # (batch-128 gradient each time); the oracle replays the same sequence with its own arithmetic
    K = 4
    st, x, ws, bs, g, (fws, fbs, peers) = build_stack(4, 128, "f32", with_fc=True)
    peer, labels, dev, lab = _kpass_inputs(st, K, 4300)
    mu, eps, omega = 0.9, 0.01, 0.0005
    p_conv0 = st.params[:st.fc_offset].clone()
    st.step_kpass(dev, lab, (mu, eps, omega), overlap)
    torch.cuda.synchronize()
    own = to_host(st.L[-1]["a"]).reshape(st.N, -1)
    w = [fw.copy() for fw in fws]; b = [fb.copy() for fb in fbs]
    vw = [np.zeros_like(a) for a in w]; vb = [np.zeros_like(a) for a in b]
    for j, feats in enumerate([own] + peer):
        _, grads, _ = _oracle_fc_chain(feats, w, b, peers, labels[j], 1.0 / st.N)
        for i in range(3):
            w[i], vw[i] = oracle.sgd_momentum(w[i], vw[i], grads[i][0], mu, eps, omega, -1.0)
            b[i], vb[i] = oracle.sgd_momentum(b[i], vb[i], grads[i][1], mu, eps, omega, -1.0)
    for i, f in enumerate(st.F):
        e1 = assert_close(to_host(f["w32"]), w[i], "f32", "fc%d weights after %d updates" % (i + 1, K))
        e2 = assert_close(to_host(f["b32"]), b[i], "f32", "fc%d biases after %d updates" % (i + 1, K))
        say("  fc%d weights %.2e biases %.2e" % (i + 1, e1, e2))
        assert e1 < 1e-5
    assert torch.equal(p_conv0, st.params[:st.fc_offset])        # convolution weights wait for the end of the step
