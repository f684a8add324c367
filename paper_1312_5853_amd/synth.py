"""Seeded synthetic inputs at the shapes of the ConvNet the paper trains.

This module is the only thing the HIP path's callers and the CPU oracle's
callers have in common.  It draws numbers and names shapes; it holds none of
the layer arithmetic (output extents are written out as constants, not
computed).

The paper trains the Krizhevsky et al. ImageNet network (Table 1 caption) on
ImageNet-2012, split either by samples (data parallelism: 128 or 64 samples
per GPU) or by filters (model parallelism: half the filters per GPU).  The
dataset is not needed to time or check convolutions, so seeded Gaussian
tensors of the same shapes stand in for it: activations and output gradients
~ N(0, 1), filters ~ N(0, 0.01^2).
"""
import numpy as np

SEED_BASE = 13125853

# name -> C, H, W (input), K, R, S, stride, pad, P, Q (output extents, stated)
LAYERS = {
    # small case: CPU oracle finishes in well under a second
    "tiny": dict(C=3, H=32, W=32, K=16, R=5, S=5, stride=1, pad=2, P=32, Q=32),
    # first layer on a data-parallel shard
    "conv1": dict(C=3, H=224, W=224, K=96, R=11, S=11, stride=4, pad=2, P=55, Q=55),
    # second layer, one model-parallel column (half the channels and filters)
    "conv2": dict(C=48, H=27, W=27, K=128, R=5, S=5, stride=1, pad=2, P=27, Q=27),
    # third to fifth layers at full width
    "conv3": dict(C=256, H=13, W=13, K=384, R=3, S=3, stride=1, pad=1, P=13, Q=13),
    "conv4": dict(C=384, H=13, W=13, K=384, R=3, S=3, stride=1, pad=1, P=13, Q=13),
    "conv5": dict(C=384, H=13, W=13, K=256, R=3, S=3, stride=1, pad=1, P=13, Q=13),
}

# index of the workload list each layer belongs to (used only to derive seeds)
_CFG_INDEX = {"tiny": 0, "conv1": 1, "conv2": 2, "conv3": 3, "conv4": 3, "conv5": 3}
_SUB_INDEX = {"conv4": 4, "conv5": 8}

STD_ACT = 1.0
STD_FILTER = 0.01


def gaussian(shape, seed, std=1.0):
    """float32 N(0, std^2) tensor from a counter-based generator keyed by seed."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def small_integers(shape, seed, lo=-4, hi=4):
    """float32 tensor of integers in [lo, hi]; sums of products stay exact."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def layer_seed(name, tensor):
    """tensor: 0 = x, 1 = w, 2 = dy."""
    return SEED_BASE + 16 * _CFG_INDEX[name] + _SUB_INDEX.get(name, 0) + tensor


def layer_tensors(name, N):
    """(x, w, dy) float32 numpy arrays for LAYERS[name] at batch size N."""
    L = LAYERS[name]
    x = gaussian((N, L["C"], L["H"], L["W"]), layer_seed(name, 0), STD_ACT)
    w = gaussian((L["K"], L["C"], L["R"], L["S"]), layer_seed(name, 1), STD_FILTER)
    dy = gaussian((N, L["K"], L["P"], L["Q"]), layer_seed(name, 2), STD_ACT)
    return x, w, dy


def to_bf16_grid(a):
    """Round a float32 array to the nearest bfloat16 value (ties to even) and
    return it as float32.  Used to prepare inputs that both sides then read
    exactly; not part of either side's arithmetic."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of an array already on the bfloat16 grid."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def sample_indices(numel, count, seed):
    """`count` distinct flat indices in [0, numel), always including both ends."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    count = min(int(count), int(numel))
    idx = rng.choice(numel, size=count, replace=False) if numel < (1 << 24) else \
        np.unique(rng.integers(0, numel, size=count))
    idx = np.unique(np.concatenate([idx.astype(np.int64), [0, numel - 1]]))
    return idx
