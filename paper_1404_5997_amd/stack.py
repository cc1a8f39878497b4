"""Sequencing of one worker's step through libowt: the five convolution layers
(+ max-pools) forward and backward, and optionally the worker's fully-connected
column shards (Section 4 of the paper, forward steps 1-3 and backward steps 1-2;
model of Section 5).

This file holds buffers and call order only; every arithmetic step runs in the
library's kernels.  torch provides device memory.  The one data movement done
here, copying this worker's 512 hidden columns into the [N, 4096] input of the
next fully-connected layer next to the columns the other workers would have
sent, stands in for the exchange between workers, which is outside a one-GPU
build.
"""
import torch

from . import (OWT_BF16, OWT_BIAS, OWT_F32, OWT_PASS_BWD_DATA, OWT_PASS_BWD_FILTER, OWT_PASS_FWD, OWT_RELU,
               conv_desc, fc_desc, owt_conv_autotune, owt_conv_bwd_data, owt_conv_bwd_data_relu_in, owt_conv_bwd_filter, owt_conv_fwd, owt_conv_workspace_bytes,
               owt_fc_autotune, owt_fc_shard_bwd, owt_fc_shard_fwd, owt_fc_workspace_bytes, owt_logistic_xent, owt_maxpool_bwd_relu,
               owt_maxpool_fwd, owt_sgd_momentum_update)


class ConvStack:
    """layers: sequence of dicts K, R, stride, pad, pool (bool); input_hwc: (H, W, C)."""

    def __init__(self, N, layers, input_hwc, pool=(3, 2), dtype="f32", fc_layers=None, fc_workers=8,
                 skip_first_dx=True):
        self.N, self.dt = N, dtype
        self.code = OWT_BF16 if dtype == "bf16" else OWT_F32
        self.tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.win, self.pst = pool
        self.skip_first_dx = skip_first_dx
        dev = "cuda"
        H, W, C = input_hwc
        self.x = torch.empty((N, H, W, C), device=dev, dtype=self.tdt)
        self.L = []
        ws_bytes = 16
        for spec in layers:
            K, R, st, pad = spec["K"], spec["R"], spec["stride"], spec["pad"]
            d = conv_desc(N, C, H, W, K, R, R, st, pad, self.code, OWT_BIAS | OWT_RELU)
            P, Q = (H + 2 * pad - R) // st + 1, (W + 2 * pad - R) // st + 1
            e = dict(desc=d, desc_bwd=conv_desc(N, C, H, W, K, R, R, st, pad, self.code, OWT_BIAS), geom=(N, C, H, W, K, R, st, pad, P, Q), pool=spec["pool"],
                     wshape=(K, R, R, C), bshape=(K,),
                     y=torch.empty((N, P, Q, K), device=dev, dtype=self.tdt),
                     dy=torch.empty((N, P, Q, K), device=dev, dtype=self.tdt))
            for p in (OWT_PASS_FWD, OWT_PASS_BWD_DATA, OWT_PASS_BWD_FILTER):
                ws_bytes = max(ws_bytes, owt_conv_workspace_bytes(d, p))
            H, W, C = P, Q, K
            if spec["pool"]:
                PP, QQ = (H - self.win) // self.pst + 1, (W - self.win) // self.pst + 1
                e["a"] = torch.empty((N, PP, QQ, K), device=dev, dtype=self.tdt)
                e["am"] = torch.empty((N, PP, QQ, K), device=dev, dtype=torch.uint8)
                e["da"] = torch.empty((N, PP, QQ, K), device=dev, dtype=self.tdt)
                H, W = PP, QQ
            self.L.append(e)
        self.out_shape = (N, H, W, C)
        for li, e in enumerate(self.L):   # does someone upstream of the layer's backward apply its ReLU mask?
            e["dz_ready"] = bool(e["pool"]) or li + 1 < len(self.L)
        # the gradient w.r.t. a layer's output lives in that layer's dy (no pool) or da (pool)
        self.F = []
        if fc_layers:
            I0 = H * W * C
            for i, spec in enumerate(fc_layers):
                assert spec["I"] == (I0 if i == 0 else fc_layers[i - 1]["O_total"])
                flags = OWT_BIAS | (OWT_RELU if spec["relu"] else 0)
                d = fc_desc(N, spec["I"], spec["O_total"], fc_workers, 0, self.code, flags)
                O = spec["O_total"] // fc_workers
                f = dict(desc=d, I=spec["I"], O=O, O_total=spec["O_total"], relu=spec["relu"],
                         wshape=(O, spec["I"]), bshape=(O,),
                         y=torch.empty((N, O), device=dev, dtype=self.tdt),
                         dy=torch.empty((N, O), device=dev, dtype=self.tdt),
                         dx=torch.empty((N, spec["I"]), device=dev, dtype=self.tdt))
                if i > 0:   # input assembled from own columns + the peers' columns
                    f["x"] = torch.zeros((N, spec["I"]), device=dev, dtype=self.tdt)
                for p in (OWT_PASS_FWD, OWT_PASS_BWD_DATA):
                    ws_bytes = max(ws_bytes, owt_fc_workspace_bytes(d, p))
                self.F.append(f)
        if self.F:   # the first dense layer's dx_partial IS the gradient of the last pooled map
            e = self.L[-1]
            self.F[0]["dx"] = (e["da"] if e["pool"] else e["dy"]).view(N, -1)
        self._carve_parameters(dev)
        self.ws = torch.empty((ws_bytes,), device=dev, dtype=torch.uint8)
        self.graph = None
        self.labels = None        # set_labels(): the logistic output layer then produces the top gradient
        self.loss = torch.zeros((N,), device=dev, dtype=torch.float32)
        self.hook = None
        self.alpha = 1.0 / N      # batch-mean weight gradient (update rule of Section 5)
        self.beta = 0.0

    def _carve_parameters(self, dev):
        """All weights and biases of the worker live in ONE fp32 array (each tensor padded to a multiple
        of 8 elements, so every view is 16-byte aligned in fp32 and in bf16), with the gradients and the
        momentum state in two more arrays of the same layout: the update rule is then one launch over
        the whole array.  bf16 stacks read a bf16 copy of the weights that the update rewrites."""
        off, slots = 0, []
        for e in self.L + self.F:
            if self.F and e is self.F[0]:
                self.fc_offset = off
            for key, shape in (("w", e["wshape"]), ("b", e["bshape"])):
                n = 1
                for v in shape:
                    n *= v
                slots.append((e, key, shape, off, n))
                off += (n + 7) // 8 * 8
        self.n_params = off
        if not self.F:
            self.fc_offset = off
        self.params = torch.zeros((off,), device=dev, dtype=torch.float32)
        self.grads = torch.zeros((off,), device=dev, dtype=torch.float32)
        self.vel = torch.zeros((off,), device=dev, dtype=torch.float32)
        self.params_bf16 = torch.zeros((off,), device=dev, dtype=torch.bfloat16) if self.dt == "bf16" else None
        for e, key, shape, o, n in slots:
            e[key + "32"] = self.params[o:o + n].view(shape)                 # fp32 master
            e["d" + key] = self.grads[o:o + n].view(shape)
            if key == "w" and self.dt == "bf16":
                e["w"] = self.params_bf16[o:o + n].view(shape)
            else:
                e[key] = e[key + "32"]

    def update(self, mu, eps, omega, gscale=-1.0, part="all"):
        """Weight update rule of Section 5 over every parameter of the worker (or only the convolution
        / dense part of the array), one launch.  The gradients in self.grads are batch means of a loss
        (alpha = 1/N), so the default gscale = -1 descends."""
        lo, hi = {"all": (0, self.n_params), "conv": (0, self.fc_offset), "fc": (self.fc_offset, self.n_params)}[part]
        if hi > lo:
            self._run("sgd update " + part, owt_sgd_momentum_update, hi - lo, self.params[lo:hi], self.vel[lo:hi],
                      self.grads[lo:hi], mu, eps, omega, gscale,
                      None if self.params_bf16 is None else self.params_bf16[lo:hi])

    # ------------------------------------------------------------------ setup
    def load(self, x, ws, bs, fc_ws=None, fc_bs=None, fc_peers=None):
        """Host numpy arrays (already bf16-representable for bf16 stacks) -> device buffers."""
        self.x.copy_(torch.from_numpy(x).to(self.tdt))
        for e, w, b in zip(self.L, ws, bs):
            e["w32"].copy_(torch.from_numpy(w)); e["w"].copy_(torch.from_numpy(w).to(self.tdt)); e["b"].copy_(torch.from_numpy(b))
        if self.F:
            for f, w, b in zip(self.F, fc_ws, fc_bs):
                f["w32"].copy_(torch.from_numpy(w)); f["w"].copy_(torch.from_numpy(w).to(self.tdt)); f["b"].copy_(torch.from_numpy(b))
            for i, f in enumerate(self.F[1:], start=1):
                own = self.F[i - 1]["O"]
                f["x"][:, own:].copy_(torch.from_numpy(fc_peers[i - 1]).to(self.tdt))

    def set_labels(self, labels):
        """Class index per image (host ints).  From then on backward() starts with the logistic
        cross-entropy output layer of Section 5 on this worker's columns of the last dense layer
        (rank 0: columns from 0) instead of a caller-supplied top gradient."""
        assert self.F, "the output layer sits on the fully-connected shard"
        self.labels = torch.as_tensor(labels, dtype=torch.int32).to(self.loss.device)

    def top_grad(self):
        """Buffer the caller fills with the gradient w.r.t. the stack output."""
        if self.F:
            return self.F[-1]["dy"]
        e = self.L[-1]
        return e["da"] if e["pool"] else e["dy"]

    # --------------------------------------------------------------- one step
    def _run(self, tag, fn, *args):
        """Every library call of a step goes through here; `self.hook`, when set, is called as
        hook(tag, thunk) and must invoke the thunk once (used to bracket calls with events)."""
        if self.hook is None:
            fn(*args)
        else:
            self.hook(tag, lambda: fn(*args))

    def forward_conv(self):
        cur = self.x
        for li, e in enumerate(self.L):
            N, C, H, W, K, R, st, pad, P, Q = e["geom"]
            e["x"] = cur
            self._run("conv%d fwd" % (li + 1), owt_conv_fwd, e["desc"], cur, e["w"], e["b"], e["y"], self.ws)
            cur = e["y"]
            if e["pool"]:
                self._run("pool%d fwd" % (li + 1), owt_maxpool_fwd, N, P, Q, K, self.win, self.pst, self.code, e["y"], e["a"], e["am"])
                cur = e["a"]
        return cur

    def forward_fc(self, feats, ws=None):
        """The worker's dense column shards on one batch of last-stage convolution activations
        feats [N, I] (Section 4, forward step 3)."""
        ws = self.ws if ws is None else ws
        cur = feats
        for i, f in enumerate(self.F):
            if i == 0:
                f["x"] = feats
            else:
                prev = self.F[i - 1]
                f["x"][:, :prev["O"]].copy_(prev["y"])        # own columns (rank 0) beside the peers'
            self._run("fc%d fwd" % (i + 1), owt_fc_shard_fwd, f["desc"], f["x"], f["w"], f["b"], f["y"], ws)
            cur = f["y"]
        return cur

    def backward_fc(self, dx_feats, labels=None, alpha=None, beta=None, ws=None):
        """Backward through the dense shards for the batch forward_fc() last ran on (Section 4, backward
        step 1): this worker's addend of the gradient of the convolution activations goes to dx_feats."""
        ws = self.ws if ws is None else ws
        alpha = self.alpha if alpha is None else alpha
        beta = self.beta if beta is None else beta
        if labels is not None:
            f = self.F[-1]
            self._run("fc%d logistic xent" % len(self.F), owt_logistic_xent, self.N, f["O"], 0, self.code, f["y"],
                      labels, 1.0, self.loss, f["dy"])
        for i in range(len(self.F) - 1, -1, -1):
            f = self.F[i]
            dx = dx_feats if i == 0 else f["dx"]
            self._run("fc%d bwd" % (i + 1), owt_fc_shard_bwd, f["desc"], f["x"], f["w"],
                      f["y"] if f["relu"] else None, f["dy"], alpha, beta, dx, f["dw"], f["db"], ws)
            if i > 0:   # the slice of dx_partial that belongs to this worker's own columns
                self.F[i - 1]["dy"].copy_(f["dx"][:, :self.F[i - 1]["O"]])

    def forward(self):
        cur = self.forward_conv()
        if self.F:
            cur = self.forward_fc(cur.view(self.N, -1))
        return cur

    def backward(self):
        if self.F:
            self.backward_fc(self.F[0]["dx"], self.labels)
        self.backward_conv()

    def backward_conv(self):
        for li in range(len(self.L) - 1, -1, -1):
            e = self.L[li]
            N, C, H, W, K, R, st, pad, P, Q = e["geom"]
            if e["pool"]:
                self._run("pool%d bwd" % (li + 1), owt_maxpool_bwd_relu, N, P, Q, K, self.win, self.pst, self.code,
                          e["da"], e["am"], e["a"], e["dy"])
            # e["dy"] already holds dz = dy*[y > 0] when its producer applied the ReLU mask
            # (the fused pooling backward above, or the next layer's bwd-data below)
            d, ymask = (e["desc_bwd"], None) if e["dz_ready"] else (e["desc"], e["y"])
            self._run("conv%d bwd_filter" % (li + 1), owt_conv_bwd_filter, d, e["x"], e["dy"], ymask, self.alpha, self.beta,
                      e["dw"], e["db"], self.ws)
            if li > 0:
                prev = self.L[li - 1]
                if prev["pool"]:
                    self._run("conv%d bwd_data" % (li + 1), owt_conv_bwd_data, d, e["dy"], ymask, e["w"], prev["da"], self.ws)
                else:   # prev's output feeds this layer directly: fuse prev's ReLU backward into the store
                    self._run("conv%d bwd_data" % (li + 1), owt_conv_bwd_data_relu_in, d, e["dy"], ymask, e["w"], e["x"],
                              prev["dy"], self.ws)
            elif not self.skip_first_dx:
                if "dx0" not in e:
                    e["dx0"] = torch.empty_like(self.x)
                self._run("conv1 bwd_data", owt_conv_bwd_data, d, e["dy"], ymask, e["w"], e["dx0"], self.ws)

    def step(self):
        self.forward()
        self.backward()

    def step_kpass(self, peer_feats, labels=None, per_pass_update=None, overlap=False):
        """One worker's step under scheme (b)/(c) of Section 4 with K = 1 + len(peer_feats) workers:
        convolution forward on the own batch; K forward+backward iterations of the dense shards, the
        first on the own batch's last-stage activations and the others on peer_feats[j] ([N, I] device
        tensors standing in for what the other workers send); then convolution backward from the own
        batch's gradient.  The addends of the peers' activation gradients land in self.peer_dx (they
        would be sent back to their workers).

        per_pass_update = None: the dense weight gradients accumulate over the K iterations with
        alpha = 1/(N*K) (the whole step is then synchronous SGD on N*K examples, Section 4.2).
        per_pass_update = (mu, eps, omega): the dense weights are updated after every iteration from that
        iteration's batch-N gradient (the variable batch size of Section 4.2).
        overlap: run the iterations on the peers' batches on a second stream beside the convolution
        backward pass (they do not depend on each other)."""
        assert self.F and self.hook is None
        K = 1 + len(peer_feats)
        if labels is None:
            labels = [self.labels] * K
        if not hasattr(self, "peer_dx"):
            self.peer_dx = torch.empty_like(peer_feats[0])
            self.side = torch.cuda.Stream(device=self.x.device)
            self.ws_side = torch.empty_like(self.ws)

        def iteration(j, feats, dx, ws):
            self.forward_fc(feats, ws)
            if per_pass_update is None:
                self.backward_fc(dx, labels[j], 1.0 / (self.N * K), 0.0 if j == 0 else 1.0, ws)
            else:
                self.backward_fc(dx, labels[j], 1.0 / self.N, 0.0, ws)
                self.update(*per_pass_update, part="fc")

        own = self.forward_conv().view(self.N, -1)
        iteration(0, own, self.F[0]["dx"], self.ws)
        main = torch.cuda.current_stream()
        if overlap:
            self.side.wait_stream(main)
            with torch.cuda.stream(self.side):
                for j, feats in enumerate(peer_feats, start=1):
                    iteration(j, feats, self.peer_dx, self.ws_side)
            self.backward_conv()
            main.wait_stream(self.side)
        else:
            for j, feats in enumerate(peer_feats, start=1):
                iteration(j, feats, self.peer_dx, self.ws)
            self.backward_conv()

    def capture(self):
        """Record one step into a HIP graph; replay() then runs it with a single launch from the host
        (worth it when the step is launch-bound, i.e. small batches; at batch 128 the kernels are long
        enough that replay and eager launches take the same time).  The graph reads and writes this
        object's buffers."""
        assert self.hook is None
        self.step()                                   # nothing inside the capture runs for the first time
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.step()
        return self.graph

    def replay(self):
        self.graph.replay()

    def autotune(self):
        """Let the library time its kernel variants for every convolution pass of the stack on the
        stack's own buffers (owt_conv_autotune).  Call after load() and after the top gradient is set."""
        self.step()     # gives every buffer the contents a real step leaves in it
        for li, e in enumerate(self.L):
            prev = self.L[li - 1] if li > 0 else None
            dx = (prev["da"] if prev["pool"] else prev["dy"]) if prev is not None else None
            d = e["desc_bwd"] if e["dz_ready"] else e["desc"]
            owt_conv_autotune(e["desc"], OWT_PASS_FWD, e["x"], e["w"], e["b"], e["y"], None, None, None, None, self.ws)
            if dx is not None:
                owt_conv_autotune(d, OWT_PASS_BWD_DATA, None, e["w"], None, e["y"], e["dy"], dx, None, None, self.ws)
            owt_conv_autotune(d, OWT_PASS_BWD_FILTER, e["x"], e["w"], None, e["y"], e["dy"], None, e["dw"], e["db"], self.ws)
        for i, f in enumerate(self.F):
            owt_fc_autotune(f["desc"], f["x"], f["w"], f["b"], f["y"], f["dy"], self.F[0]["dx"] if i == 0 else f["dx"],
                            f["dw"], f["db"], self.ws)
        self.step()

    # ----------------------------------------------------------- work counters
    def conv_flops(self):
        """2*MAC of the dense definition per step: fwd + bwd-filter for every layer, bwd-data for all
        but the first (its input is data) unless skip_first_dx is off."""
        total = 0
        for li, e in enumerate(self.L):
            N, C, H, W, K, R, st, pad, P, Q = e["geom"]
            one = 2 * N * P * Q * K * R * R * C
            total += one * (3 if (li > 0 or not self.skip_first_dx) else 2)
        return total

    def fc_flops(self):
        return sum(2 * self.N * f["I"] * f["O"] * 3 for f in self.F)
