"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds workload geometry and random-number recipes only -- none of
the method's arithmetic.  Both the CPU oracle and the HIP library are fed the
very same host arrays produced here.

The paper trains on 224x224x3 crops of ILSVRC-2012 images in batches of 128 per
worker (Section 4, forward step 1; Section 5).  That dataset is not used: dense
convolution cost and correctness do not depend on pixel values, so seeded
random tensors of the same shapes stand in for it.

Recipe: numpy.random.Generator(PCG64(seed)); tensor number t of config c uses
seed BASE_SEED + 1000*c + t.  For bf16 configs the caller rounds these float32
arrays to bf16 before either side sees them.
"""
import numpy as np

BASE_SEED = 14045997

# The five convolution layers (Section 5 footnote gives 64,192,384,384,256 filters;
# the benchmark configuration uses 256 for the fourth layer).  Each entry:
# K filters, R=S, stride, pad, and whether a 3x3 stride-2 max-pool follows.
STACK_LAYERS = (
    dict(K=64, R=11, stride=4, pad=2, pool=True),
    dict(K=192, R=5, stride=1, pad=2, pool=True),
    dict(K=384, R=3, stride=1, pad=1, pool=False),
    dict(K=256, R=3, stride=1, pad=1, pool=False),
    dict(K=256, R=3, stride=1, pad=1, pool=True),
)
PAPER_FILTERS = (64, 192, 384, 384, 256)
STACK_INPUT_HWC = (224, 224, 3)
POOL_WIN, POOL_STRIDE = 3, 2

# Fully-connected layers 9216 -> 4096 -> 4096 -> 1000 split over K=8 workers by
# output column: this worker owns 512 / 512 / 125 columns.
FC_WORKERS = 8
FC_LAYERS = (
    dict(I=9216, O_total=4096, O_local=512, relu=True),
    dict(I=4096, O_total=4096, O_local=512, relu=True),
    dict(I=4096, O_total=1000, O_local=125, relu=False),
)


def rng(config, tensor):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + tensor))


def normal(config, tensor, shape, std=1.0):
    return (rng(config, tensor).standard_normal(shape, dtype=np.float32) * np.float32(std))


def uniform(config, tensor, shape):
    return rng(config, tensor).random(shape, dtype=np.float32)


def conv_layer_case(config, N, H, W, C, K, R, S, tensor0=0, x_dist="normal"):
    """x, w, bias, dy for one convolution layer; the caller supplies P, Q via dy_shape later."""
    x = uniform(config, tensor0, (N, H, W, C)) if x_dist == "uniform" else normal(config, tensor0, (N, H, W, C))
    w = normal(config, tensor0 + 1, (K, R, S, C), 0.01)
    b = normal(config, tensor0 + 2, (K,), 0.01)
    return x, w, b


def upstream_grad(config, tensor, shape):
    return normal(config, tensor, shape, 1.0)


def config1():
    """Single small layer: N=8, 32x32x3, 16 filters 5x5, stride 1, pad 2, bias+ReLU."""
    geom = dict(N=8, H=32, W=32, C=3, K=16, R=5, S=5, stride=1, pad=2)
    x, w, b = conv_layer_case(1, 8, 32, 32, 3, 16, 5, 5)
    dy = upstream_grad(1, 3, (8, 32, 32, 16))
    return geom, x, w, b, dy


def config2(N=128):
    """One mid-stack layer at batch 128: 13x13x192 -> 384 filters 3x3, stride 1, pad 1."""
    geom = dict(N=N, H=13, W=13, C=192, K=384, R=3, S=3, stride=1, pad=1)
    x, w, b = conv_layer_case(2, N, 13, 13, 192, 384, 3, 3)
    dy = upstream_grad(2, 3, (N, 13, 13, 384))
    return geom, x, w, b, dy


def stack_params(config, filters=None):
    """Weights ~N(0, 0.01) and biases ~N(0, 0.01) of the five layers (tensors 10.., 20..)."""
    C = STACK_INPUT_HWC[2]
    ws, bs = [], []
    for li, L in enumerate(STACK_LAYERS):
        K = L["K"] if filters is None else filters[li]
        ws.append(normal(config, 10 + li, (K, L["R"], L["R"], C), 0.01))
        bs.append(normal(config, 20 + li, (K,), 0.01))
        C = K
    return ws, bs


def stack_input(config, N):
    """Images ~U(0,1), NHWC."""
    return uniform(config, 0, (N,) + STACK_INPUT_HWC)


def fc_params(config):
    """This worker's column shards: W ~N(0, 0.005), b ~N(0, 0.005) (tensors 30.., 40..)."""
    ws = [normal(config, 30 + i, (L["O_local"], L["I"]), 0.005) for i, L in enumerate(FC_LAYERS)]
    bs = [normal(config, 40 + i, (L["O_local"],), 0.005) for i, L in enumerate(FC_LAYERS)]
    return ws, bs


def fc_peer_columns(config, layer, N):
    """Stand-in for the hidden activations the other 7 workers would send:
    max(0, N(0,1)) * 0.05, shape [N, O_total - O_local] (tensors 50..)."""
    L = FC_LAYERS[layer]
    a = normal(config, 50 + layer, (N, L["O_total"] - L["O_local"]))
    return np.maximum(a, 0).astype(np.float32) * np.float32(0.05)
