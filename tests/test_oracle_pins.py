"""Pins of the CPU oracle against what the mathematics fixes.

The paper prints no worked example, so every pin here is a closed form, an
identity, a reduction to a textbook routine, a brute force in a different
formulation, or a hand-worked fixture.  They are chosen so that a dropped
term, a flipped filter, a wrong sign of the padding, a transposed index or a
wrong output extent fails at least one of them.
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from paper_1312_5853_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 9, 4, 3, 3, 1, 1),
    (1, 2, 8, 8, 3, 5, 5, 1, 2),
    (2, 3, 11, 10, 2, 3, 2, 2, 1),
    (1, 1, 23, 23, 2, 11, 11, 4, 2),     # first-layer geometry, floor in the extent
    (3, 2, 6, 5, 3, 3, 3, 1, 0),
    (1, 2, 5, 6, 2, 3, 3, 2, 3),         # pad >= R/2 and > 1
    (2, 1, 9, 9, 1, 1, 1, 3, 0),
]


def extent(size, filt, stride, pad):
    # written independently of the oracle's C helper
    return (size + 2 * pad - filt) // stride + 1


def rnd(shape, seed):
    return synth.gaussian(shape, seed).astype(np.float64)


# ---------------------------------------------------------------- fixture ---
def test_handworked_fixture():
    g = json.load(open(os.path.join(GOLDEN, "handworked_3x3.json")))
    x, w, dy = (np.array(g[k], dtype=np.float64) for k in ("x", "w", "dy"))
    a = g["stride1_pad0"]
    np.testing.assert_array_equal(oracle.conv_fwd(x, w, 1, 0), np.array(a["y"], dtype=np.float64))
    np.testing.assert_array_equal(oracle.conv_bwd_data(dy, w, 3, 3, 1, 0), np.array(a["dx"], dtype=np.float64))
    np.testing.assert_array_equal(oracle.conv_bwd_filter(x, dy, 2, 2, 1, 0), np.array(a["dw"], dtype=np.float64))
    b = g["stride2_pad1"]
    np.testing.assert_array_equal(oracle.conv_fwd(x, w, 2, 1), np.array(b["y"], dtype=np.float64))


def test_out_extent_values():
    assert oracle.out_extent(224, 11, 4, 2) == 55       # floor of 217/4, plus 1
    assert oracle.out_extent(27, 5, 1, 2) == 27
    assert oracle.out_extent(13, 3, 1, 1) == 13
    assert oracle.out_extent(32, 5, 1, 2) == 32
    for h in (223, 224, 225, 226):
        assert oracle.out_extent(h, 11, 4, 2) == 55
    assert oracle.out_extent(227, 11, 4, 2) == 56
    assert oracle.pool_extent(55) == 27 and oracle.pool_extent(27) == 13 and oracle.pool_extent(13) == 6


# ------------------------------------------------------------ closed form ---
@pytest.mark.parametrize("shape", SHAPES)
def test_all_ones_closed_form(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    cnt_r = np.array([sum(0 <= p * st - pad + r < H for r in range(R)) for p in range(P)])
    cnt_s = np.array([sum(0 <= q * st - pad + s < W for s in range(S)) for q in range(Q)])
    y = oracle.conv_fwd(np.ones((N, C, H, W)), np.ones((K, C, R, S)), st, pad)
    assert y.shape == (N, K, P, Q)
    np.testing.assert_array_equal(y, np.broadcast_to(C * np.outer(cnt_r, cnt_s), y.shape))

    hit_h = np.array([sum(p * st - pad + r == h for p in range(P) for r in range(R)) for h in range(H)])
    hit_w = np.array([sum(q * st - pad + s == v for q in range(Q) for s in range(S)) for v in range(W)])
    dx = oracle.conv_bwd_data(np.ones((N, K, P, Q)), np.ones((K, C, R, S)), H, W, st, pad)
    np.testing.assert_array_equal(dx, np.broadcast_to(K * np.outer(hit_h, hit_w), dx.shape))

    val_r = np.array([sum(0 <= p * st - pad + r < H for p in range(P)) for r in range(R)])
    val_s = np.array([sum(0 <= q * st - pad + s < W for q in range(Q)) for s in range(S)])
    dw = oracle.conv_bwd_filter(np.ones((N, C, H, W)), np.ones((N, K, P, Q)), R, S, st, pad)
    np.testing.assert_array_equal(dw, np.broadcast_to(N * np.outer(val_r, val_s), dw.shape))


# --------------------------------------- brute force, different formulation ---
def slices_fwd(x, w, st, pad):
    """pad-and-slice formulation: one strided slab of the padded input per tap."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, K, P, Q))
    for c in range(C):          # same (c, r, s) order as the definition so integer sums match exactly
        for r in range(R):
            for s in range(S):
                slab = xp[:, c, r:r + st * (P - 1) + 1:st, s:s + st * (Q - 1) + 1:st]
                y += slab[:, None, :, :] * w[None, :, c, r, s, None, None]
    return y


def gather_dgrad(dy, w, H, W, st, pad):
    """gather formulation: each dx element collects the taps that reach it."""
    N, K, P, Q = dy.shape
    _, C, R, S = w.shape
    dx = np.zeros((N, C, H, W))
    for h in range(H):
        for v in range(W):
            for r in range(R):
                for s in range(S):
                    th, tv = h + pad - r, v + pad - s
                    if th % st or tv % st:
                        continue
                    p, q = th // st, tv // st
                    if 0 <= p < P and 0 <= q < Q:
                        dx[:, :, h, v] += dy[:, :, p, q] @ w[:, :, r, s]
    return dx


def outer_wgrad(x, dy, R, S, st, pad):
    """outer-product formulation: one K x C rank-1 update per (n, p, q, r, s)."""
    N, C, H, W = x.shape
    _, K, P, Q = dy.shape
    dw = np.zeros((K, C, R, S))
    for n, p, q in itertools.product(range(N), range(P), range(Q)):
        for r in range(R):
            for s in range(S):
                h, v = p * st - pad + r, q * st - pad + s
                if 0 <= h < H and 0 <= v < W:
                    dw[:, :, r, s] += np.outer(dy[n, :, p, q], x[n, :, h, v])
    return dw


@pytest.mark.parametrize("shape", SHAPES)
def test_brute_force_small_integers_bitwise(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    x = synth.small_integers((N, C, H, W), 1).astype(np.float64)
    w = synth.small_integers((K, C, R, S), 2).astype(np.float64)
    dy = synth.small_integers((N, K, P, Q), 3).astype(np.float64)
    np.testing.assert_array_equal(oracle.conv_fwd(x, w, st, pad), slices_fwd(x, w, st, pad))
    np.testing.assert_array_equal(oracle.conv_bwd_data(dy, w, H, W, st, pad), gather_dgrad(dy, w, H, W, st, pad))
    np.testing.assert_array_equal(oracle.conv_bwd_filter(x, dy, R, S, st, pad), outer_wgrad(x, dy, R, S, st, pad))


# ------------------------------------------------------------------ deltas ---
def test_delta_filter_is_a_shift():
    N, C, H, W, R, S, pad = 2, 3, 6, 7, 3, 3, 1
    x = rnd((N, C, H, W), 11)
    for r0, s0 in itertools.product(range(R), range(S)):
        w = np.zeros((C, C, R, S))
        for c in range(C):
            w[c, c, r0, s0] = 1.0
        y = oracle.conv_fwd(x, w, 1, pad)
        want = np.zeros_like(x)
        for p in range(H):
            for q in range(W):
                h, v = p - pad + r0, q - pad + s0
                if 0 <= h < H and 0 <= v < W:
                    want[:, :, p, q] = x[:, :, h, v]
        np.testing.assert_array_equal(y, want)
        if (r0, s0) == (pad, pad):
            np.testing.assert_array_equal(y, x)      # centre tap: identity, no flip either way
    # an off-centre tap distinguishes correlation from flipped convolution
    w = np.zeros((C, C, R, S))
    for c in range(C):
        w[c, c, 0, 2] = 1.0
    y = oracle.conv_fwd(x, w, 1, pad)
    assert y[0, 0, 2, 2] == x[0, 0, 1, 3]


def test_delta_input_reads_out_the_filter():
    C, H, W, K, R, S = 2, 12, 12, 3, 5, 5
    w = rnd((K, C, R, S), 12)
    for st, pad, (c0, h0, v0) in [(1, 2, (1, 5, 6)), (2, 2, (0, 6, 4)), (3, 0, (1, 7, 7))]:
        x = np.zeros((1, C, H, W))
        x[0, c0, h0, v0] = 1.0
        y = oracle.conv_fwd(x, w, st, pad)
        P, Q = y.shape[2:]
        want = np.zeros_like(y)
        for p in range(P):
            for q in range(Q):
                r, s = h0 + pad - p * st, v0 + pad - q * st
                if 0 <= r < R and 0 <= s < S:
                    want[0, :, p, q] = w[:, c0, r, s]
        np.testing.assert_array_equal(y, want)


# ----------------------------------------------------------------- adjoint ---
@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identities(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    x, w, g = rnd((N, C, H, W), 21), rnd((K, C, R, S), 22), rnd((N, K, P, Q), 23)
    a = np.sum(oracle.conv_fwd(x, w, st, pad) * g)
    b = np.sum(x * oracle.conv_bwd_data(g, w, H, W, st, pad))
    c = np.sum(w * oracle.conv_bwd_filter(x, g, R, S, st, pad))
    scale = np.sum(np.abs(oracle.conv_fwd(np.abs(x), np.abs(w), st, pad) * np.abs(g)))
    assert abs(a - b) <= 1e-12 * scale
    assert abs(a - c) <= 1e-12 * scale


# ------------------------------------------------------ finite differences ---
def test_finite_differences_every_element():
    """L(x, w) = <conv(x, w), g> is bilinear, so a unit step in one coordinate
    changes L by exactly that coordinate's gradient (no truncation error)."""
    N, C, H, W, K, R, S, st, pad = 1, 2, 6, 5, 3, 3, 3, 2, 1
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    x, w, g = rnd((N, C, H, W), 31), rnd((K, C, R, S), 32), rnd((N, K, P, Q), 33)
    L0 = np.sum(oracle.conv_fwd(x, w, st, pad) * g)
    dx = oracle.conv_bwd_data(g, w, H, W, st, pad)
    dw = oracle.conv_bwd_filter(x, g, R, S, st, pad)
    for i in range(x.size):
        xe = x.copy().ravel()
        xe[i] += 1.0
        L1 = np.sum(oracle.conv_fwd(xe.reshape(x.shape), w, st, pad) * g)
        assert abs((L1 - L0) - dx.ravel()[i]) <= 1e-11 * (1 + abs(L0))
    for i in range(w.size):
        we = w.copy().ravel()
        we[i] += 1.0
        L1 = np.sum(oracle.conv_fwd(x, we.reshape(w.shape), st, pad) * g)
        assert abs((L1 - L0) - dw.ravel()[i]) <= 1e-11 * (1 + abs(L0))


def test_finite_differences_tiny_config_sampled():
    L = synth.LAYERS["tiny"]
    x, w, g = synth.layer_tensors("tiny", 4)
    x, w, g = x.astype(np.float64), w.astype(np.float64), g.astype(np.float64)
    st, pad = L["stride"], L["pad"]
    dx = oracle.conv_bwd_data(g, w, L["H"], L["W"], st, pad)
    dw = oracle.conv_bwd_filter(x, g, L["R"], L["S"], st, pad)
    for i in synth.sample_indices(x.size, 12, 5):
        e = np.zeros(x.size)
        e[i] = 1.0
        dL = np.sum(oracle.conv_fwd(e.reshape(x.shape), w, st, pad) * g)     # L(x+e) - L(x) by linearity
        assert abs(dL - dx.ravel()[i]) <= 1e-12 * max(1.0, np.abs(dx).max())
    for i in synth.sample_indices(w.size, 12, 6):
        e = np.zeros(w.size)
        e[i] = 1.0
        dL = np.sum(oracle.conv_fwd(x, e.reshape(w.shape), st, pad) * g)
        assert abs(dL - dw.ravel()[i]) <= 1e-12 * max(1.0, np.abs(dw).max())


# --------------------------------------------- reductions to textbook ops ---
def test_1x1_is_a_matrix_product():
    N, C, H, W, K = 2, 5, 4, 3, 7
    x, w = rnd((N, C, H, W), 41), rnd((K, C, 1, 1), 42)
    y = oracle.conv_fwd(x, w, 1, 0)
    for n in range(N):
        want = w[:, :, 0, 0] @ x[n].reshape(C, H * W)
        np.testing.assert_allclose(y[n].reshape(K, H * W), want, rtol=1e-13, atol=1e-13)
    g = rnd(y.shape, 43)
    dx = oracle.conv_bwd_data(g, w, H, W, 1, 0)
    dw = oracle.conv_bwd_filter(x, g, 1, 1, 1, 0)
    for n in range(N):
        np.testing.assert_allclose(dx[n].reshape(C, H * W), w[:, :, 0, 0].T @ g[n].reshape(K, H * W),
                                   rtol=1e-13, atol=1e-13)
    want_dw = sum(g[n].reshape(K, H * W) @ x[n].reshape(C, H * W).T for n in range(N))
    np.testing.assert_allclose(dw[:, :, 0, 0], want_dw, rtol=1e-13, atol=1e-13)


def test_full_size_filter_is_a_dot_product():
    N, C, H, W, K = 3, 2, 5, 4, 3
    x, w = rnd((N, C, H, W), 44), rnd((K, C, H, W), 45)
    y = oracle.conv_fwd(x, w, 1, 0)
    assert y.shape == (N, K, 1, 1)
    np.testing.assert_allclose(y[:, :, 0, 0], x.reshape(N, -1) @ w.reshape(K, -1).T, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("st", [2, 3, 4])
def test_stride_is_subsampled_stride_one(st):
    N, C, H, W, K, R, S, pad = 2, 2, 13, 12, 3, 3, 5, 2
    x, w = rnd((N, C, H, W), 46), rnd((K, C, R, S), 47)
    y1 = oracle.conv_fwd(x, w, 1, pad)
    ys = oracle.conv_fwd(x, w, st, pad)
    np.testing.assert_array_equal(ys, y1[:, :, ::st, ::st][:, :, :ys.shape[2], :ys.shape[3]])
    assert ys.shape[2] == extent(H, R, st, pad) and ys.shape[3] == extent(W, S, st, pad)


# -------------------------------------------------- linearity, equivariance ---
def test_linearity_and_shift():
    N, C, H, W, K, R, S, st, pad = 2, 2, 8, 8, 3, 3, 3, 1, 1
    x1, x2, w = rnd((N, C, H, W), 51), rnd((N, C, H, W), 52), rnd((K, C, R, S), 53)
    lhs = oracle.conv_fwd(2.0 * x1 - 0.5 * x2, w, st, pad)
    rhs = 2.0 * oracle.conv_fwd(x1, w, st, pad) - 0.5 * oracle.conv_fwd(x2, w, st, pad)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    # one-pixel shift of an input whose border ring is zero shifts the output
    x = np.zeros((1, C, 10, 10))
    x[:, :, 3:7, 3:7] = rnd((1, C, 4, 4), 54)
    xs = np.roll(x, (1, 1), axis=(2, 3))
    y, ys = oracle.conv_fwd(x, w, 1, 1), oracle.conv_fwd(xs, w, 1, 1)
    np.testing.assert_array_equal(np.roll(y, (1, 1), axis=(2, 3)), ys)


# ------------------- the decompositions the paper's two schemes depend on ---
def test_data_parallel_batch_split():
    """Data parallelism: each GPU sees a slice of the mini-batch; activations and
    input gradients are per sample, filter gradients add over the shards."""
    N, C, H, W, K, R, S, st, pad = 4, 3, 9, 9, 4, 3, 3, 2, 1
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    x, w, g = rnd((N, C, H, W), 61), rnd((K, C, R, S), 62), rnd((N, K, P, Q), 63)
    y = oracle.conv_fwd(x, w, st, pad)
    np.testing.assert_array_equal(y[1:3], oracle.conv_fwd(x[1:3], w, st, pad))
    dx = oracle.conv_bwd_data(g, w, H, W, st, pad)
    np.testing.assert_array_equal(dx[3:], oracle.conv_bwd_data(g[3:], w, H, W, st, pad))
    dw = oracle.conv_bwd_filter(x, g, R, S, st, pad)
    parts = oracle.conv_bwd_filter(x[:1], g[:1], R, S, st, pad) + oracle.conv_bwd_filter(x[1:], g[1:], R, S, st, pad)
    np.testing.assert_allclose(dw, parts, rtol=1e-13, atol=1e-13)


def test_model_parallel_filter_split():
    """Model parallelism: a layer's filters are split in two halves; outputs
    concatenate over channels, input gradients add over the halves, and a
    split of the input channels adds in the forward pass."""
    N, C, H, W, K, R, S, st, pad = 2, 4, 7, 7, 6, 3, 3, 1, 1
    x, w = rnd((N, C, H, W), 64), rnd((K, C, R, S), 65)
    y = oracle.conv_fwd(x, w, st, pad)
    g = rnd(y.shape, 66)
    np.testing.assert_array_equal(y[:, :3], oracle.conv_fwd(x, w[:3], st, pad))
    np.testing.assert_array_equal(y[:, 3:], oracle.conv_fwd(x, w[3:], st, pad))
    dx = oracle.conv_bwd_data(g, w, H, W, st, pad)
    halves = oracle.conv_bwd_data(g[:, :3], w[:3], H, W, st, pad) + oracle.conv_bwd_data(g[:, 3:], w[3:], H, W, st, pad)
    np.testing.assert_allclose(dx, halves, rtol=1e-13, atol=1e-13)
    dw = oracle.conv_bwd_filter(x, g, R, S, st, pad)
    np.testing.assert_array_equal(dw[3:], oracle.conv_bwd_filter(x, g[:, 3:], R, S, st, pad))
    yc = oracle.conv_fwd(x[:, :2], w[:, :2], st, pad) + oracle.conv_fwd(x[:, 2:], w[:, 2:], st, pad)
    np.testing.assert_allclose(y, yc, rtol=1e-13, atol=1e-13)


# ------------------------------------------------- element-wise entry points ---
@pytest.mark.parametrize("shape", SHAPES)
def test_elementwise_entry_points_match_full(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = extent(H, R, st, pad), extent(W, S, st, pad)
    x, w, g = rnd((N, C, H, W), 71), rnd((K, C, R, S), 72), rnd((N, K, P, Q), 73)
    y = oracle.conv_fwd(x, w, st, pad)
    dx = oracle.conv_bwd_data(g, w, H, W, st, pad)
    dw = oracle.conv_bwd_filter(x, g, R, S, st, pad)
    iy = np.arange(y.size)
    np.testing.assert_array_equal(oracle.conv_fwd_at(x, w, st, pad, iy), y.ravel())
    np.testing.assert_array_equal(oracle.conv_bwd_filter_at(x, g, R, S, st, pad, np.arange(dw.size)), dw.ravel())
    # the gather order differs from the scatter order: equal up to rounding only
    np.testing.assert_allclose(oracle.conv_bwd_data_at(g, w, H, W, st, pad, np.arange(dx.size)), dx.ravel(),
                               rtol=1e-12, atol=1e-13)
    xi = synth.small_integers((N, C, H, W), 74)
    wi = synth.small_integers((K, C, R, S), 75)
    gi = synth.small_integers((N, K, P, Q), 76)
    np.testing.assert_array_equal(oracle.conv_bwd_data_at(gi, wi, H, W, st, pad, np.arange(dx.size)),
                                  gather_dgrad(gi.astype(np.float64), wi.astype(np.float64), H, W, st, pad).ravel())


# -------------------------------------------------------------------- glue ---
def test_relu():
    x = np.array([-2.0, -0.0, 0.0, 1e-300, 3.0])
    np.testing.assert_array_equal(oracle.relu_fwd(x), [0.0, 0.0, 0.0, 1e-300, 3.0])
    np.testing.assert_array_equal(oracle.relu_bwd(x, np.full(5, 7.0)), [0.0, 0.0, 0.0, 7.0, 7.0])


def test_maxpool_brute_force_and_ties():
    x = rnd((2, 3, 13, 11), 81)
    y, arg = oracle.maxpool3x3s2_fwd(x, return_arg=True)
    assert y.shape == (2, 3, 6, 5)
    for i in range(6):
        for j in range(5):
            win = x[:, :, 2 * i:2 * i + 3, 2 * j:2 * j + 3].reshape(2, 3, 9)
            np.testing.assert_array_equal(y[:, :, i, j], win.max(axis=2))
            a = win.argmax(axis=2)                       # numpy: first maximum
            np.testing.assert_array_equal(arg[:, :, i, j], (2 * i + a // 3) * 11 + (2 * j + a % 3))
    g = rnd(y.shape, 82)
    dx = oracle.maxpool3x3s2_bwd(x, g)
    want = np.zeros_like(x)
    for n, c, i, j in itertools.product(range(2), range(3), range(6), range(5)):
        a = arg[n, c, i, j]
        want[n, c, a // 11, a % 11] += g[n, c, i, j]
    np.testing.assert_array_equal(dx, want)
    assert abs(dx.sum() - g.sum()) < 1e-12
    # all-equal window: the first element in row-major order takes the gradient
    z = np.zeros((1, 1, 3, 3))
    dz = oracle.maxpool3x3s2_bwd(z, np.ones((1, 1, 1, 1)))
    assert dz[0, 0, 0, 0] == 1.0 and dz.sum() == 1.0
    # overlapping windows sharing one maximum accumulate
    z = np.zeros((1, 1, 5, 5))
    z[0, 0, 2, 2] = 9.0
    dz = oracle.maxpool3x3s2_bwd(z, np.ones((1, 1, 2, 2)))
    assert dz[0, 0, 2, 2] == 4.0


def test_oracle_does_not_import_the_product():
    import subprocess
    import sys
    code = ("import sys, oracle; "
            "bad=[m for m in sys.modules if m.startswith('paper_1312_5853_amd')]; "
            "sys.exit(1 if bad else 0)")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    assert subprocess.run([sys.executable, "-c", code], cwd=root).returncode == 0


# ---------------------------------------------------------------- grouped layers ---
def _block_diagonal(w, groups):
    """Filters of a grouped layer as filters of an ordinary layer over all channels: zero outside the own column."""
    K, Cg, R, S = w.shape
    Kg = K // groups
    full = np.zeros((K, Cg * groups, R, S), dtype=w.dtype)
    for g in range(groups):
        full[g * Kg:(g + 1) * Kg, g * Cg:(g + 1) * Cg] = w[g * Kg:(g + 1) * Kg]
    return full


@pytest.mark.parametrize("groups,st,pad", [(2, 1, 1), (3, 2, 0), (1, 1, 2)])
def test_grouped_layer_is_the_block_diagonal_layer(groups, st, pad):
    """A multi-column layer without cross-connections equals the full layer whose filters are zero outside their
    column -- forward, backward-data, and (restricted to the column blocks) backward-filter.  Small integers: exact."""
    rng = np.random.default_rng(7)
    N, Cg, Kg, H, W, R, S = 2, 3, 4, 7, 6, 3, 3
    x = rng.integers(-3, 4, (N, Cg * groups, H, W)).astype(np.float64)
    w = rng.integers(-3, 4, (Kg * groups, Cg, R, S)).astype(np.float64)
    full = _block_diagonal(w, groups)
    y = oracle.conv_fwd_grouped(x, w, st, pad, groups)
    assert np.array_equal(y, oracle.conv_fwd(x, full, st, pad))
    dy = rng.integers(-3, 4, y.shape).astype(np.float64)
    assert np.array_equal(oracle.conv_bwd_data_grouped(dy, w, H, W, st, pad, groups),
                          oracle.conv_bwd_data(dy, full, H, W, st, pad))
    dw_full = oracle.conv_bwd_filter(x, dy, R, S, st, pad)          # [K, C, R, S]: the column blocks are the grouped dw
    dw = oracle.conv_bwd_filter_grouped(x, dy, R, S, st, pad, groups)
    for g in range(groups):
        assert np.array_equal(dw[g * Kg:(g + 1) * Kg], dw_full[g * Kg:(g + 1) * Kg, g * Cg:(g + 1) * Cg])


def test_grouped_adjoint_identities():
    """<conv_g(x, w), g> = <x, dgrad_g(g, w)> = <w, wgrad_g(x, g)> for the grouped layer as well."""
    rng = np.random.default_rng(8)
    groups, N, Cg, Kg, H, W, R, S, st, pad = 2, 3, 5, 3, 9, 8, 5, 5, 1, 2
    x = rng.standard_normal((N, Cg * groups, H, W))
    w = rng.standard_normal((Kg * groups, Cg, R, S))
    y = oracle.conv_fwd_grouped(x, w, st, pad, groups)
    g = rng.standard_normal(y.shape)
    a = np.sum(y * g)
    b = np.sum(x * oracle.conv_bwd_data_grouped(g, w, H, W, st, pad, groups))
    c = np.sum(w * oracle.conv_bwd_filter_grouped(x, g, R, S, st, pad, groups))
    scale = np.sum(np.abs(y * g))
    assert abs(a - b) <= 1e-12 * scale and abs(a - c) <= 1e-12 * scale


# ------------------------------------------------------------------------- bias ---
def test_bias_closed_forms_and_adjoint():
    rng = np.random.default_rng(9)
    N, K, P, Q = 3, 5, 4, 6
    y = rng.standard_normal((N, K, P, Q))
    b = rng.standard_normal(K)
    out = oracle.bias_fwd(y, b)
    # element by element against the definition, and exact on integers
    for n, k, p, q in [(0, 0, 0, 0), (2, 4, 3, 5), (1, 2, 1, 3)]:
        assert out[n, k, p, q] == y[n, k, p, q] + b[k]
    yi = rng.integers(-5, 6, (N, K, P, Q)).astype(np.float64)
    bi = rng.integers(-5, 6, K).astype(np.float64)
    assert np.array_equal(oracle.bias_fwd(yi, bi) - yi, np.broadcast_to(bi[None, :, None, None], yi.shape))
    # gradient: all-ones closed form, a single non-zero entry, integers against a brute-force loop
    assert np.array_equal(oracle.bias_bwd(np.ones((N, K, P, Q))), np.full(K, N * P * Q, dtype=np.float64))
    d = np.zeros((N, K, P, Q)); d[1, 3, 2, 4] = 2.5
    assert np.array_equal(oracle.bias_bwd(d), np.array([0, 0, 0, 2.5, 0]))
    gi = rng.integers(-5, 6, (N, K, P, Q)).astype(np.float64)
    brute = [sum(gi[n, k, p, q] for n in range(N) for p in range(P) for q in range(Q)) for k in range(K)]
    assert np.array_equal(oracle.bias_bwd(gi), np.array(brute))
    # adjoint of the forward's dependence on b: <bias_fwd(0, b), g> = <b, bias_bwd(g)>
    g = rng.standard_normal((N, K, P, Q))
    lhs = np.sum(oracle.bias_fwd(np.zeros_like(g), b) * g)
    assert abs(lhs - np.dot(b, oracle.bias_bwd(g))) <= 1e-12 * np.sum(np.abs(g))


# ------------------------------------------------- convolution + bias + ReLU chains ---
def test_fused_forward_closed_form_orders_bias_before_relu():
    # x = 1, w = 1, 3x3 pad 1: the sum is C * (taps inside) = 18 inside, 12 on edges, 8 in corners.  A bias of -10
    # leaves 8 / 2 / 0 after the ReLU (ReLU before the bias would give 8 / 2 / -2); filter 1 has bias +1.
    C, H = 2, 5
    x = np.ones((1, C, H, H)); w = np.ones((2, C, 3, 3)); b = np.array([-10.0, 1.0])
    y = oracle.conv_fwd_bias_relu(x, w, b, 1, 1)
    assert y[0, 0, 2, 2] == 8 and y[0, 0, 0, 2] == 2 and y[0, 0, 0, 0] == 0 and y[0, 0, 4, 4] == 0
    assert y[0, 1, 2, 2] == 19 and y[0, 1, 0, 0] == 9
    lin = oracle.conv_fwd_bias_relu(x, w, b, 1, 1, relu=False)
    assert lin[0, 0, 0, 0] == -2 and lin[0, 0, 2, 2] == 8
    nob = oracle.conv_fwd_bias_relu(-x, w, None, 1, 1)
    assert np.array_equal(nob, np.zeros_like(nob))


def test_fused_backward_data_is_the_derivative_through_the_relu():
    # L(a) = <conv_fwd(relu(a), w), g> is piecewise linear in a: away from a = 0 a central difference is exact up to
    # rounding, and it must equal conv_bwd_data_relu(g, w, a); where a <= 0 the gradient is exactly 0.
    rng = np.random.default_rng(21)
    N, C, H, W, K, R, S, st, pad = 2, 3, 7, 6, 4, 3, 3, 2, 1
    a = rng.standard_normal((N, C, H, W))
    a[np.abs(a) < 0.05] = 0.5
    a[0, 1, 2, 3] = 0.0                                   # relu'(0) = 0
    w = rng.standard_normal((K, C, R, S))
    g = rng.standard_normal((N, K, oracle.out_extent(H, R, st, pad), oracle.out_extent(W, S, st, pad)))
    da = oracle.conv_bwd_data_relu(g, w, a, st, pad)
    assert da.shape == a.shape and da[0, 1, 2, 3] == 0.0
    assert np.array_equal(da[a <= 0], np.zeros(np.count_nonzero(a <= 0)))

    def loss(t):
        return float(np.sum(oracle.conv_fwd(np.maximum(t, 0.0), w, st, pad) * g))

    eps = 1e-3
    for _ in range(12):
        i = tuple(int(rng.integers(0, d)) for d in a.shape)
        if a[i] == 0.0:
            continue
        ap, am = a.copy(), a.copy()
        ap[i] += eps; am[i] -= eps
        fd = (loss(ap) - loss(am)) / (2 * eps)
        assert abs(fd - da[i]) <= 1e-8 * max(1.0, abs(da[i])), (i, fd, da[i])


# ------------------------------------------------- fully connected layers and SGD ---
def test_fc_equals_brute_force_and_the_convolution_oracle():
    rng = np.random.default_rng(31)
    N, I, O = 3, 8, 5
    x = rng.integers(-4, 5, (N, I)).astype(np.float64)
    w = rng.integers(-4, 5, (O, I)).astype(np.float64)
    g = rng.integers(-4, 5, (N, O)).astype(np.float64)
    y = oracle.fc_fwd(x, w)
    dx = oracle.fc_bwd_data(g, w)
    dw = oracle.fc_bwd_filter(x, g)
    for n in range(N):
        for o in range(O):
            assert y[n, o] == sum(x[n, i] * w[o, i] for i in range(I))
        for i in range(I):
            assert dx[n, i] == sum(g[n, o] * w[o, i] for o in range(O))
    for o in range(O):
        for i in range(I):
            assert dw[o, i] == sum(g[n, o] * x[n, i] for n in range(N))
    # a fully connected layer is a 1x1 convolution on 1x1 planes ...
    x4, w4, g4 = x.reshape(N, I, 1, 1), w.reshape(O, I, 1, 1), g.reshape(N, O, 1, 1)
    assert np.array_equal(y, oracle.conv_fwd(x4, w4, 1, 0).reshape(N, O))
    assert np.array_equal(dx, oracle.conv_bwd_data(g4, w4, 1, 1, 1, 0).reshape(N, I))
    assert np.array_equal(dw, oracle.conv_bwd_filter(x4, g4, 1, 1, 1, 0).reshape(O, I))
    # ... and, on a flattened [C][H][W] sample, a convolution whose filter covers the whole plane
    C, H, W = 2, 2, 2
    xc, wc = x.reshape(N, C, H, W), w.reshape(O, C, H, W)
    assert np.array_equal(y, oracle.conv_fwd(xc, wc, 1, 0).reshape(N, O))


def test_fc_bias_relu_and_adjoints():
    rng = np.random.default_rng(32)
    N, I, O = 4, 7, 6
    x, w, g = rng.standard_normal((N, I)), rng.standard_normal((O, I)), rng.standard_normal((N, O))
    b = rng.standard_normal(O)
    lin = oracle.fc_fwd(x, w)
    assert np.array_equal(oracle.fc_fwd(x, w, b), lin + b[None, :])
    yr = oracle.fc_fwd(x, w, b, relu=True)
    assert np.array_equal(yr, np.maximum(lin + b[None, :], 0.0)) and (yr >= 0).all()
    # x = 1, w = 1: every output is I; with bias -I-1 the ReLU leaves 0, with bias 1 it leaves I + 1
    one = oracle.fc_fwd(np.ones((2, I)), np.ones((2, I)), np.array([-I - 1.0, 1.0]), relu=True)
    assert np.array_equal(one, np.array([[0.0, I + 1.0]] * 2))
    # <fc(x, w), g> = <x, bwd_data(g, w)> = <w, bwd_filter(x, g)>
    lhs = np.sum(lin * g)
    assert abs(lhs - np.sum(x * oracle.fc_bwd_data(g, w))) <= 1e-12 * abs(lhs) + 1e-12
    assert abs(lhs - np.sum(w * oracle.fc_bwd_filter(x, g))) <= 1e-12 * abs(lhs) + 1e-12
    # not symmetric in its arguments: a transposed operand must fail
    assert oracle.fc_bwd_filter(x, g).shape == (O, I) and oracle.fc_bwd_data(g, w).shape == (N, I)


def test_sgd_update_closed_forms():
    w0 = np.array([1.0, -2.0, 0.5]); g = np.array([0.5, 0.25, -1.0]); z = np.zeros(3)
    # plain SGD: w' = w - lr * dw, velocity is the step
    w1, v1 = oracle.sgd_update(w0, g, z, lr=0.1)
    assert np.allclose(w1, w0 - 0.1 * g, rtol=0, atol=1e-16) and np.allclose(v1, -0.1 * g, rtol=0, atol=1e-16)
    # gradient of the mean: grad_scale = 1/B
    w1, _ = oracle.sgd_update(w0, g, z, lr=0.1, grad_scale=0.25)
    assert np.allclose(w1, w0 - 0.025 * g, rtol=0, atol=1e-16)
    # weight decay alone contracts the weights: w_t = (1 - lr * wd)^t * w_0
    w, v = w0.copy(), z.copy()
    for _ in range(10):
        w, v = oracle.sgd_update(w, z, v, lr=0.1, weight_decay=0.5)
    assert np.allclose(w, (1 - 0.05) ** 10 * w0, rtol=1e-13)
    # constant gradient with momentum: v_t = -lr * g * (1 - mu^t) / (1 - mu), w_t = w_0 + sum of the v
    mu, lr, T = 0.9, 0.01, 25
    w, v = w0.copy(), z.copy()
    for _ in range(T):
        w, v = oracle.sgd_update(w, g, v, lr=lr, momentum=mu)
    assert np.allclose(v, -lr * g * (1 - mu ** T) / (1 - mu), rtol=1e-12)
    total = -lr * g * (T - mu * (1 - mu ** T) / (1 - mu)) / (1 - mu)
    assert np.allclose(w, w0 + total, rtol=1e-12)
    # gradient descent on L = |w|^2 / 2 (dw = w) with lr = 1 lands on the minimum in one step
    w1, _ = oracle.sgd_update(w0, w0, z, lr=1.0)
    assert np.array_equal(w1, z)


# ----------------------------------------------------------- bfloat16 rounding ---
# Hand-written (binary32 pattern -> bfloat16 pattern) pairs, worked from the format: 1 sign, 8 exponent and 7
# fraction bits are kept; the dropped 16 bits decide, 0x8000 being exactly half way (then the even pattern wins).
BF16_BIT_PINS = [
    (0x3F800000, 0x3F80),        # 1.0, exact
    (0x40490FDB, 0x4049),        # pi -> 3.140625 (dropped part 0x0FDB is below half)
    (0x3F808000, 0x3F80),        # 1 + 2^-8: tie, kept pattern even -> down
    (0x3F818000, 0x3F82),        # 1 + 3*2^-8: tie, kept pattern odd -> up
    (0xBF818000, 0xBF82),        # the same tie, negative
    (0x3F808001, 0x3F81),        # just above the tie -> up
    (0x3F807FFF, 0x3F80),        # just below the tie -> down
    (0x3FFFFFFF, 0x4000),        # 1.9999999: the carry runs through the fraction into the exponent -> 2.0
    (0x7F7FFFFF, 0x7F80),        # largest finite binary32 -> +infinity
    (0xFF7FFFFF, 0xFF80),        # ... and -infinity
    (0x7F7F7FFF, 0x7F7F),        # largest value that still rounds to the largest finite bfloat16
    (0x7F7F8000, 0x7F80),        # tie at the top, kept pattern odd -> infinity
    (0x00000000, 0x0000),        # +0
    (0x80000000, 0x8000),        # -0 keeps its sign
    (0x7F800000, 0x7F80),        # infinity stays
    (0x00000001, 0x0000),        # smallest subnormal -> 0
    (0x00008000, 0x0000),        # subnormal tie, even -> 0
    (0x00008001, 0x0001),        # just above -> smallest bfloat16 subnormal
    (0x00018000, 0x0002),        # subnormal tie, odd -> up
    (0x007FFFFF, 0x0080),        # largest subnormal -> smallest normal
]


def test_bf16_rounding_hand_written_bit_patterns():
    bits = np.array([b for b, _ in BF16_BIT_PINS], dtype=np.uint32)
    want = np.array([w for _, w in BF16_BIT_PINS], dtype=np.uint16)
    got = oracle.bf16_bits(bits.view(np.float32))
    assert np.array_equal(got, want), [(hex(b), hex(g), hex(w)) for b, g, w in zip(bits, got, want) if g != w]
    # values, not only patterns
    r = oracle.bf16_round(np.array([1.00390625, 1.01171875, 3.14159265, -0.0], dtype=np.float32))
    assert np.array_equal(r[:3], np.array([1.0, 1.015625, 3.140625], dtype=np.float32))
    assert np.signbit(r[3]) and r[3] == 0.0
    # NaN stays NaN, also when its payload lies wholly in the dropped half (it must not turn into infinity)
    nans = np.array([0x7FC00000, 0x7F800001, 0xFFC00001, 0x7FFFFFFF], dtype=np.uint32)
    out = oracle.bf16_bits(nans.view(np.float32))
    assert np.all((out & 0x7F80) == 0x7F80) and np.all((out & 0x007F) != 0)
    assert np.array_equal(out >> 15, nans >> 31)


def test_bf16_rounding_is_the_nearest_value_with_even_ties():
    """Defining property, checked in exact arithmetic (float64 holds binary32 and bfloat16 values exactly): the
    result is a bfloat16 value at least as close as both of its bfloat16 neighbours, and an exact tie goes to the
    pattern with last bit 0."""
    rng = np.random.default_rng(41)
    bits = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    bits = bits[(bits & 0x7F800000) != 0x7F800000]                        # finite
    bits = bits[(bits & 0x7FFFFFFF) < 0x7F7F0000]                         # neighbours stay finite
    x = bits.view(np.float32)
    out = oracle.bf16_bits(x)
    val = lambda p: (p.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    r = val(out)
    mag = out & 0x7FFF
    # magnitudes one pattern up / down; stepping down from a zero crosses to the other sign's smallest value
    up = val((out & 0x8000) | (mag + 1))
    down_mag = np.where(mag > 0, mag - 1, 1)
    down_sign = np.where(mag > 0, out & 0x8000, (out & 0x8000) ^ 0x8000)
    down = val((down_sign | down_mag).astype(np.uint16))
    x64 = x.astype(np.float64)
    d = np.abs(x64 - r)
    assert np.all(d <= np.abs(x64 - up)) and np.all(d <= np.abs(x64 - down))
    tie = (d == np.abs(x64 - up)) | (d == np.abs(x64 - down))
    assert np.all((out[tie] & 1) == 0)
    # values already on the grid pass unchanged
    assert np.array_equal(oracle.bf16_bits(oracle.bf16_round(x)), out)


def test_bf16_rounding_matches_torch_cpu_conversion():
    import torch
    rng = np.random.default_rng(42)
    bits = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    bits = np.concatenate([bits, np.array([b for b, _ in BF16_BIT_PINS], dtype=np.uint32)])
    notnan = (bits & 0x7FFFFFFF) <= 0x7F800000
    x = bits[notnan].view(np.float32)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.bf16_bits(x), want)
    g = (rng.standard_normal(1 << 18) * 0.01).astype(np.float32)        # the filters' value range
    want = torch.from_numpy(g).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.bf16_round(g), want)


def test_seeded_bf16_inputs_lie_on_the_grid_the_oracle_defines():
    """The input generator's own rounding (used to prepare tensors both sides read) agrees with the oracle's."""
    from paper_1312_5853_amd import synth
    for seed, std in ((1, 1.0), (2, 0.01), (3, 300.0)):
        a = synth.gaussian((50000,), seed, std)
        assert np.array_equal(synth.to_bf16_grid(a), oracle.bf16_round(a))
        assert np.array_equal(synth.bf16_bits(synth.to_bf16_grid(a)), oracle.bf16_bits(a))
