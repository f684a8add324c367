"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Error measure (for every floating-point comparison here): normalised max error
    err = max_i |gpu_i - ref_i| / max_i |ref_i|
over the compared elements, ref = fp64 oracle.  Bars: 1e-4 for fp32 arithmetic,
2e-2 for bf16 inputs with fp32 accumulation (the oracle is fed the same
bf16-rounded values, so only accumulation order and width differ).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1312_5853_amd import binding as hp
from paper_1312_5853_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def norm_err(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    denom = np.abs(ref).max()
    return np.abs(got - ref).max() / (denom if denom > 0 else 1.0)


def dev(a, dtype="f32"):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def nan_like(shape):
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def prepared(x, w, dy, dtype):
    """For bf16 the values are first rounded onto the bf16 grid; both sides then read them exactly."""
    if dtype == "bf16":
        return oracle.bf16_round(x), oracle.bf16_round(w), oracle.bf16_round(dy)
    return x, w, dy


def run_three(x, w, dy, st, pad, dtype="f32"):
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = dy.shape[2:]
    xd, wd, dyd = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    y = hp.conv_fwd(xd, wd, st, pad, y=nan_like((N, K, P, Q)))
    dx = hp.conv_bwd_data(dyd, wd, H, W, st, pad, dx=nan_like((N, C, H, W)))
    dw = hp.conv_bwd_filter(xd, dyd, R, S, st, pad, dw=nan_like((K, C, R, S)))
    torch.cuda.synchronize()
    return y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()


def check_full(x, w, dy, st, pad, dtype="f32"):
    x, w, dy = prepared(x, w, dy, dtype)
    N, C, H, W = x.shape
    R, S = w.shape[2:]
    y, dx, dw = run_three(x, w, dy, st, pad, dtype)
    errs = (norm_err(y, oracle.conv_fwd(x, w, st, pad)),
            norm_err(dx, oracle.conv_bwd_data(dy, w, H, W, st, pad)),
            norm_err(dw, oracle.conv_bwd_filter(x, dy, R, S, st, pad)))
    for name, e in zip(("fwd", "dgrad", "wgrad"), errs):
        assert np.isfinite(e) and e <= TOL[dtype], "%s err %.3e" % (name, e)
    return errs


# ----------------------------------------------------------- tiny config ---
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tiny_config_full_compare(dtype):
    L = synth.LAYERS["tiny"]
    x, w, dy = synth.layer_tensors("tiny", 4)
    check_full(x, w, dy, L["stride"], L["pad"], dtype)


# ------------------------------------------------------ odd small shapes ---
ODD_SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (1, 1, 5, 5, 1, 1, 1, 1, 0),
    (1, 3, 7, 9, 17, 3, 3, 1, 1),
    (3, 17, 9, 7, 3, 3, 2, 1, 1),
    (2, 3, 12, 11, 5, 5, 5, 2, 2),
    (3, 1, 23, 25, 48, 11, 11, 4, 2),
    (1, 48, 6, 6, 17, 3, 3, 1, 0),
    (2, 5, 8, 10, 130, 3, 3, 1, 5),        # pad beyond the filter, K past one row tile
    (1, 2, 9, 9, 2, 9, 9, 1, 0),           # filter as large as the input: 1x1 output
    (3, 4, 10, 10, 100, 2, 3, 3, 1),       # K = 100: ragged 96/128 row tile
    (5, 33, 13, 13, 65, 3, 3, 1, 1),       # columns 5*169 = 845: ragged last column tile
    (2, 2, 40, 3, 3, 4, 1, 4, 0),          # stride 4 along a thin plane
    (3, 48, 9, 9, 40, 3, 3, 1, 1),         # forward with 40 rows: the 48-row tile of 16x16 blocks
    (2, 40, 11, 7, 32, 3, 3, 1, 1),        # backward-data with 40 rows, ragged 256-column tile
    (7, 48, 14, 14, 64, 5, 5, 1, 2),       # backward-data with 48 rows, several column tiles
    # channel count 16 / 32 (fast kernels) on small planes: P*Q = 1, 2, 3 and 0 mod 4, dy tensors of 1 and 3
    # elements, a stride-2 layer
    (2, 16, 5, 5, 3, 3, 3, 1, 1),          # P*Q = 25
    (2, 16, 4, 5, 5, 3, 3, 1, 0),          # P*Q = 6
    (3, 32, 3, 9, 2, 3, 3, 1, 0),          # P*Q = 7
    (2, 16, 6, 6, 130, 3, 3, 1, 0),        # P*Q = 16, K past one row tile
    (1, 16, 3, 3, 1, 3, 3, 1, 0),          # dy has one element
    (3, 16, 1, 1, 1, 1, 1, 1, 0),          # dy has three elements
    (5, 16, 9, 11, 7, 3, 3, 2, 1),         # stride 2: P*Q = 5*6 = 30
    # backward-filter with at most four channels, 49..96 filters and 129..384 taps (input rows staged in LDS,
    # one partial result per work-group): an odd row length (last reduction pair half empty), stride 1 with one
    # new row per step, more (image, row range) units than work-groups, a filter that fills the ring of 16 rows
    (3, 3, 40, 120, 96, 11, 11, 4, 2),
    (2, 4, 14, 17, 64, 5, 7, 1, 2),
    (300, 2, 9, 12, 50, 9, 8, 3, 1),
    (2, 3, 30, 20, 96, 12, 4, 4, 0),
]


@pytest.mark.parametrize("shape", ODD_SHAPES)
def test_odd_shapes_full_compare(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    x = synth.gaussian((N, C, H, W), 101)
    w = synth.gaussian((K, C, R, S), 102, 0.1)
    dy = synth.gaussian((N, K, P, Q), 103)
    check_full(x, w, dy, st, pad)


BF16_SHAPES = [
    # channel counts that select 16, 32, 48 and 64 channels per step of the bf16 kernels, every tile shape,
    # ragged column tiles, a strided forward; passes whose channel count is not a multiple of 16 are widened
    (3, 16, 9, 11, 24, 3, 3, 1, 1),
    (2, 32, 13, 13, 160, 3, 3, 1, 1),
    (5, 48, 10, 7, 96, 5, 5, 1, 2),
    (2, 64, 12, 12, 48, 3, 3, 2, 1),
    (4, 128, 13, 13, 20, 3, 3, 1, 1),
    (3, 80, 7, 7, 64, 1, 1, 1, 0),
    (7, 192, 6, 5, 256, 3, 2, 1, 1),
    # backward-filter on packed copies (stride 1, output extent = input extent): 64-, 96- and 128-row tiles,
    # a reduction that ends inside a 64-position step, and a plane too small for it (falls back)
    (3, 64, 13, 13, 64, 3, 3, 1, 1),
    (2, 32, 27, 27, 128, 5, 5, 1, 2),
    (9, 16, 12, 9, 96, 1, 1, 1, 0),
    (4, 16, 5, 5, 128, 3, 3, 1, 1),
    # few channels, stride 4, row length a multiple of 8: the forward kernel on the bf16 matrix instruction
    # (filter rows padded to 16 columns); 32-, 64- and 128-row filter tiles, a ragged second position tile,
    # more tiles than persistent work-groups
    (2, 3, 24, 32, 40, 11, 11, 4, 2),
    (2, 2, 16, 16, 20, 5, 7, 4, 2),
    (1, 3, 64, 64, 100, 11, 11, 4, 2),
    (70, 1, 56, 40, 33, 8, 16, 4, 0),
    # ... and the backward-filter kernel that stages input rows as shifted copies (stride 4, pad 2, at most four
    # channels, 96 filters, 64 positions per output row): a last group of 8 positions that is part empty and two
    # 16-position blocks, 96 filters, fewer filter rows than the stride, more (image, row range) units than
    # work-groups so that a work-group restarts its ring of rows
    (3, 3, 40, 120, 96, 11, 11, 4, 2),
    (2, 4, 20, 24, 16, 3, 3, 4, 2),
    (300, 1, 16, 16, 8, 5, 5, 4, 2),
]


@pytest.mark.parametrize("shape", BF16_SHAPES)
def test_bf16_shapes_full_compare(shape):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    x = synth.gaussian((N, C, H, W), 104)
    w = synth.gaussian((K, C, R, S), 105, 0.1)
    dy = synth.gaussian((N, K, P, Q), 106)
    check_full(x, w, dy, st, pad, "bf16")


def test_bf16_small_integers_are_exact():
    """Small integers are exact in bf16 and their sums in fp32: the bf16 kernels must return them bit for bit."""
    N, C, H, W, K, R, S, st, pad = 3, 32, 9, 10, 48, 3, 3, 1, 1
    x = synth.small_integers((N, C, H, W), 114)
    w = synth.small_integers((K, C, R, S), 115)
    dy = synth.small_integers((N, K, H, W), 116)
    y, dx, dw = run_three(x, w, dy, st, pad, "bf16")
    np.testing.assert_array_equal(y, oracle.conv_fwd(x, w, st, pad))
    np.testing.assert_array_equal(dx, oracle.conv_bwd_data(dy, w, H, W, st, pad))
    np.testing.assert_array_equal(dw, oracle.conv_bwd_filter(x, dy, R, S, st, pad))


@pytest.mark.parametrize("shape", [(5, 64, 13, 13, 96, 3, 3, 1, 1),      # bf16 kernels
                                   (3, 3, 20, 21, 24, 5, 5, 2, 2),       # widened inputs, fp32 kernels
                                   (4, 48, 9, 9, 40, 3, 3, 1, 1),
                                   # the direct-to-LDS kernels both ways: whole tiles store bf16 pairs (a pair that
                                   # would straddle two samples falls back to single stores), the ragged last tile
                                   # stores one value at a time
                                   (2, 128, 13, 13, 128, 3, 3, 1, 1),
                                   (5, 64, 14, 14, 256, 3, 3, 1, 1),
                                   # the few-channel bf16 forward kernel: a whole 256-position tile and a ragged one
                                   (2, 3, 72, 72, 64, 11, 11, 4, 2),
                                   (3, 3, 64, 72, 96, 11, 11, 4, 2)])
def test_bf16_outputs_are_the_rounded_fp32_results(shape):
    """dtype 2: y and dx come back as bfloat16 = the fp32 results of dtype 1 rounded to nearest even, written
    through batch strides; within the bf16 tolerance of the oracle."""
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    x, w, dy = prepared(synth.gaussian((N, C, H, W), 107), synth.gaussian((K, C, R, S), 108, 0.1),
                        synth.gaussian((N, K, P, Q), 109), "bf16")
    xd, wd, dyd = dev(x, "bf16"), dev(w, "bf16"), dev(dy, "bf16")
    y32 = hp.conv_fwd(xd, wd, st, pad)
    dx32 = hp.conv_bwd_data(dyd, wd, H, W, st, pad)
    # outputs land in channel slices of wider bf16 tensors pre-filled with a marker
    ywide = torch.full((N, K + 8, P, Q), 7.0, dtype=torch.bfloat16, device="cuda")
    dxwide = torch.full((N, C + 8, H, W), 7.0, dtype=torch.bfloat16, device="cuda")
    hp.conv_fwd(xd, wd, st, pad, y=ywide[:, 8:])
    hp.conv_bwd_data(dyd, wd, H, W, st, pad, dx=dxwide[:, 8:])
    y16 = hp.conv_fwd(xd, wd, st, pad, out_bf16=True)
    torch.cuda.synchronize()
    assert y16.dtype == torch.bfloat16 and torch.equal(y16, ywide[:, 8:])
    assert (ywide[:, :8] == 7.0).all() and (dxwide[:, :8] == 7.0).all()
    bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(bits(ywide[:, 8:]), oracle.bf16_bits(y32.cpu().numpy()))
    assert np.array_equal(bits(dxwide[:, 8:]), oracle.bf16_bits(dx32.cpu().numpy()))
    assert norm_err(ywide[:, 8:].float().cpu().numpy(), oracle.conv_fwd(x, w, st, pad)) <= TOL["bf16"]
    assert norm_err(dxwide[:, 8:].float().cpu().numpy(), oracle.conv_bwd_data(dy, w, H, W, st, pad)) <= TOL["bf16"]


def test_small_integers_are_exact():
    """Integer-valued inputs with small sums are exact in fp32: bit-for-bit equality."""
    N, C, H, W, K, R, S, st, pad = 2, 6, 11, 12, 40, 3, 3, 2, 1
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    x = synth.small_integers((N, C, H, W), 111)
    w = synth.small_integers((K, C, R, S), 112)
    dy = synth.small_integers((N, K, P, Q), 113)
    y, dx, dw = run_three(x, w, dy, st, pad)
    np.testing.assert_array_equal(y, oracle.conv_fwd(x, w, st, pad))
    np.testing.assert_array_equal(dx, oracle.conv_bwd_data(dy, w, H, W, st, pad))
    np.testing.assert_array_equal(dw, oracle.conv_bwd_filter(x, dy, R, S, st, pad))


# ---------------------------------------- guard bands and full overwrite ---
def test_guard_bands_untouched():
    N, C, H, W, K, R, S, st, pad = 3, 7, 13, 13, 70, 3, 3, 1, 1
    P, Q = H, W
    x, w, dy = (synth.gaussian(s, i) for i, s in enumerate([(N, C, H, W), (K, C, R, S), (N, K, P, Q)], 121))
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    G = 4096

    def guarded(numel):
        buf = torch.full((numel + 2 * G,), float("nan"), dtype=torch.float32, device="cuda")
        return buf, buf[G:G + numel]

    for op in ("fwd", "dgrad", "wgrad"):
        if op == "fwd":
            buf, out = guarded(N * K * P * Q)
            hp.conv_fwd(xd, wd, st, pad, y=out.view(N, K, P, Q))
        elif op == "dgrad":
            buf, out = guarded(N * C * H * W)
            hp.conv_bwd_data(dyd, wd, H, W, st, pad, dx=out.view(N, C, H, W))
        else:
            buf, out = guarded(K * C * R * S)
            hp.conv_bwd_filter(xd, dyd, R, S, st, pad, dw=out.view(K, C, R, S))
        torch.cuda.synchronize()
        assert torch.isnan(buf[:G]).all() and torch.isnan(buf[-G:]).all(), op
        assert not torch.isnan(out).any(), op


def test_dgrad_rows_no_window_touches_are_zero():
    # H = 226 with an 11x11 stride-4 filter: the last input rows/cols lie beyond every window
    N, C, H, W, K, R, S, st, pad = 1, 2, 30, 30, 3, 11, 11, 4, 0
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    assert (P - 1) * st + R < H
    w = synth.gaussian((K, C, R, S), 131)
    dy = synth.gaussian((N, K, P, Q), 132)
    dx = hp.conv_bwd_data(dev(dy), dev(w), H, W, st, pad, dx=nan_like((N, C, H, W))).cpu().numpy()
    assert (dx[:, :, (P - 1) * st + R:, :] == 0).all() and (dx[:, :, :, (Q - 1) * st + S:] == 0).all()
    assert norm_err(dx, oracle.conv_bwd_data(dy, w, H, W, st, pad)) <= TOL["f32"]


def test_bitwise_determinism():
    x, w, dy = synth.layer_tensors("conv2", 8)
    L = synth.LAYERS["conv2"]
    a = run_three(x, w, dy, L["stride"], L["pad"])
    b = run_three(x, w, dy, L["stride"], L["pad"])
    for u, v in zip(a, b):
        assert np.array_equal(u.view(np.uint32), v.view(np.uint32))


# ------------------------------ decompositions of the two parallel schemes ---
def test_batch_shards_and_filter_halves_on_one_gpu():
    L = synth.LAYERS["conv2"]
    x, w, dy = synth.layer_tensors("conv2", 6)
    st, pad, H, W, R, S = L["stride"], L["pad"], L["H"], L["W"], L["R"], L["S"]
    y, dx, dw = run_three(x, w, dy, st, pad)
    ya, dxa, dwa = run_three(x[:2], w, dy[:2], st, pad)
    yb, dxb, dwb = run_three(x[2:], w, dy[2:], st, pad)
    assert np.array_equal(np.concatenate([ya, yb]), y)            # per-sample results do not depend on the shard
    assert np.array_equal(np.concatenate([dxa, dxb]), dx)
    assert norm_err(dwa + dwb, dw) <= 1e-5                        # filter gradients add over shards
    K = w.shape[0]
    yh, dxh, dwh = run_three(x, w[:K // 2], dy[:, :K // 2], st, pad)
    yg, dxg, dwg = run_three(x, w[K // 2:], dy[:, K // 2:], st, pad)
    assert norm_err(np.concatenate([yh, yg], axis=1), y) <= 1e-6  # filter halves concatenate
    assert norm_err(dxh + dxg, dx) <= 1e-5                        # and their input gradients add
    assert norm_err(np.concatenate([dwh, dwg]), dw) <= 1e-6


def test_channel_slices_of_wider_tensors():
    """One column reads channels 48..95 of a 96-channel tensor and writes filters 128..255 of a 256-channel one."""
    L = synth.LAYERS["conv2"]
    N, st, pad = 5, L["stride"], L["pad"]
    xw = synth.gaussian((N, 96, 27, 27), 141)
    w = synth.gaussian((128, 48, 5, 5), 142, 0.01)
    dyw = synth.gaussian((N, 256, 27, 27), 143)
    xwd, wd, dywd = dev(xw), dev(w), dev(dyw)
    ywd = nan_like((N, 256, 27, 27))
    dxwd = nan_like((N, 96, 27, 27))
    hp.conv_fwd(xwd[:, 48:], wd, st, pad, y=ywd[:, 128:])
    hp.conv_bwd_data(dywd[:, 128:], wd, 27, 27, st, pad, dx=dxwd[:, 48:])
    dw = hp.conv_bwd_filter(xwd[:, 48:], dywd[:, 128:], 5, 5, st, pad)
    torch.cuda.synchronize()
    assert torch.isnan(ywd[:, :128]).all() and torch.isnan(dxwd[:, :48]).all()
    xs, dys = xw[:, 48:], dyw[:, 128:]
    assert norm_err(ywd[:, 128:].cpu().numpy(), oracle.conv_fwd(xs, w, st, pad)) <= TOL["f32"]
    assert norm_err(dxwd[:, 48:].cpu().numpy(), oracle.conv_bwd_data(dys, w, 27, 27, st, pad)) <= TOL["f32"]
    assert norm_err(dw.cpu().numpy(), oracle.conv_bwd_filter(xs, dys, 5, 5, st, pad)) <= TOL["f32"]


@pytest.mark.parametrize("c0,c1,k0,k1", [(48, 96, 128, 256),      # channel counts the bf16 kernels take
                                         (8, 29, 8, 41)])          # widened to dense fp32 copies first
def test_bf16_channel_slices_of_wider_tensors(c0, c1, k0, k1):
    N, st, pad = 3, 1, 2
    xw = oracle.bf16_round(synth.gaussian((N, 96, 27, 27), 151))
    w = oracle.bf16_round(synth.gaussian((k1 - k0, c1 - c0, 5, 5), 152, 0.01))
    dyw = oracle.bf16_round(synth.gaussian((N, 256, 27, 27), 153))
    xwd, wd, dywd = (dev(a).to(torch.bfloat16) for a in (xw, w, dyw))
    ywd = nan_like((N, 256, 27, 27))
    dxwd = nan_like((N, 96, 27, 27))
    hp.conv_fwd(xwd[:, c0:c1], wd, st, pad, y=ywd[:, k0:k1])
    hp.conv_bwd_data(dywd[:, k0:k1], wd, 27, 27, st, pad, dx=dxwd[:, c0:c1])
    dw = hp.conv_bwd_filter(xwd[:, c0:c1], dywd[:, k0:k1], 5, 5, st, pad)
    torch.cuda.synchronize()
    assert torch.isnan(ywd[:, :k0]).all() and torch.isnan(ywd[:, k1:]).all()
    assert torch.isnan(dxwd[:, :c0]).all() and torch.isnan(dxwd[:, c1:]).all()
    xs, dys = xw[:, c0:c1], dyw[:, k0:k1]
    assert norm_err(ywd[:, k0:k1].cpu().numpy(), oracle.conv_fwd(xs, w, st, pad)) <= TOL["bf16"]
    assert norm_err(dxwd[:, c0:c1].cpu().numpy(), oracle.conv_bwd_data(dys, w, 27, 27, st, pad)) <= TOL["bf16"]
    assert norm_err(dw.cpu().numpy(), oracle.conv_bwd_filter(xs, dys, 5, 5, st, pad)) <= TOL["bf16"]


# ------------------------------------------------------------ grouped layers ---
GROUPED = [
    # N, C, H, W, K, R, S, stride, pad, groups, dtype
    (3, 96, 27, 27, 256, 5, 5, 1, 2, 2, "f32"),       # the second layer's two columns: one launch, 48-row backward-data
    (2, 64, 13, 13, 96, 3, 3, 1, 1, 2, "f32"),        # 32 -> 48 per column
    (5, 48, 9, 9, 192, 3, 3, 1, 1, 3, "f32"),         # three columns of 16 -> 64, ragged column tiles
    (2, 32, 12, 12, 64, 3, 3, 2, 1, 2, "f32"),        # strided: forward / backward-filter fused, backward-data in turn
    (2, 6, 10, 10, 16, 3, 3, 1, 1, 2, "f32"),         # few channels: columns one after the other (16-byte aligned slices)
    (3, 96, 27, 27, 256, 5, 5, 1, 2, 2, "bf16"),      # bf16 kernels, columns in turn
    (4, 64, 13, 13, 64, 3, 3, 1, 1, 1, "f32"),        # one group = the ordinary layer
]


@pytest.mark.parametrize("shape", GROUPED)
def test_grouped_layers_full_compare(shape):
    N, C, H, W, K, R, S, st, pad, groups, dtype = shape
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    x, w, dy = prepared(synth.gaussian((N, C, H, W), 131), synth.gaussian((K, C // groups, R, S), 132, 0.1),
                        synth.gaussian((N, K, P, Q), 133), dtype)
    xd, wd, dyd = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    y = hp.conv_fwd_grouped(xd, wd, st, pad, groups, y=nan_like((N, K, P, Q)))
    dx = hp.conv_bwd_data_grouped(dyd, wd, H, W, st, pad, groups, dx=nan_like((N, C, H, W)))
    dw = hp.conv_bwd_filter_grouped(xd, dyd, R, S, st, pad, groups, dw=nan_like((K, C // groups, R, S)))
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert norm_err(y.cpu().numpy(), oracle.conv_fwd_grouped(x, w, st, pad, groups)) <= tol
    assert norm_err(dx.cpu().numpy(), oracle.conv_bwd_data_grouped(dy, w, H, W, st, pad, groups)) <= tol
    assert norm_err(dw.cpu().numpy(), oracle.conv_bwd_filter_grouped(x, dy, R, S, st, pad, groups)) <= tol
    if groups > 1 and dtype == "f32":
        # the columns in one launch give bit for bit what the same columns give as separate calls on channel slices
        Cg, Kg = C // groups, K // groups
        for g in range(groups):
            yg = hp.conv_fwd(xd[:, g * Cg:(g + 1) * Cg], wd[g * Kg:(g + 1) * Kg].contiguous(), st, pad)
            assert torch.equal(yg, y[:, g * Kg:(g + 1) * Kg])
            dwg = hp.conv_bwd_filter(xd[:, g * Cg:(g + 1) * Cg], dyd[:, g * Kg:(g + 1) * Kg], R, S, st, pad)
            assert torch.equal(dwg, dw[g * Kg:(g + 1) * Kg])


# ------------------------------- full-size layers, whole tensors against the oracle ---
FULL = [
    # layer, N, passes (the passes the workload list names for the layer)
    ("conv1", 128, ("fwd", "wgrad")),
    ("conv2", 128, ("fwd", "dgrad", "wgrad")),
    ("conv3", 256, ("fwd", "dgrad", "wgrad")),
    ("conv4", 256, ("fwd", "dgrad", "wgrad")),
    ("conv5", 256, ("fwd", "dgrad", "wgrad")),
]


def edge_indices(shape):
    """Flat indices of the corners of every axis combination (first/last along each axis)."""
    idx = []
    for corner in np.ndindex(*(2,) * len(shape)):
        pos = tuple((s - 1) if c else 0 for c, s in zip(corner, shape))
        idx.append(np.ravel_multi_index(pos, shape))
    return np.array(idx, dtype=np.int64)


def host64(t):
    """A device tensor (fp32 or bfloat16) as a float64 numpy array, exactly."""
    return t.float().cpu().numpy().astype(np.float64)


def check_close(tag, got_t, ref, tol, record):
    """Every element of the device tensor against the oracle's tensor: normalised max error within tol."""
    assert tuple(got_t.shape) == tuple(ref.shape), tag
    got = host64(got_t)
    assert np.isfinite(got).all(), tag + ": not every element written"
    e = norm_err(got, ref)
    record(tag, e, tol)
    assert e <= tol, "%s err %.3e > %.1e" % (tag, e, tol)
    return e


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layer,N,passes", FULL)
def test_full_size_layers_whole_tensors(layer, N, passes, dtype, parity_record):
    """The layers of the workload list at their full sizes (first layer and one second-layer column on a 128-image
    shard, third to fifth layer at 256 images), fp32 and bf16-in / fp32-accumulate: EVERY output element of each
    pass is compared with the oracle's full-tensor result on the same inputs."""
    L = synth.LAYERS[layer]
    st, pad, H, W, R, S, C, K, P, Q = (L[k] for k in ("stride", "pad", "H", "W", "R", "S", "C", "K", "P", "Q"))
    x, w, dy = prepared(*synth.layer_tensors(layer, N), dtype)
    xd, wd, dyd = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    tag = "%s N=%d %s " % (layer, N, dtype)
    if "fwd" in passes:
        y = hp.conv_fwd(xd, wd, st, pad, y=nan_like((N, K, P, Q)))
        check_close(tag + "fwd", y, oracle.conv_fwd(x, w, st, pad), TOL[dtype], parity_record)
        del y
    if "dgrad" in passes:
        dx = hp.conv_bwd_data(dyd, wd, H, W, st, pad, dx=nan_like((N, C, H, W)))
        check_close(tag + "dgrad", dx, oracle.conv_bwd_data(dy, w, H, W, st, pad), TOL[dtype], parity_record)
        del dx
    if "wgrad" in passes:
        dw = hp.conv_bwd_filter(xd, dyd, R, S, st, pad, dw=nan_like((K, C, R, S)))
        check_close(tag + "wgrad", dw, oracle.conv_bwd_filter(x, dy, R, S, st, pad), TOL[dtype], parity_record)


# -------------------------------------------------------------------- glue ---
def test_relu_and_pool_match_oracle():
    for (N, C, H, W) in [(3, 5, 55, 55), (2, 7, 27, 27), (4, 3, 13, 13), (1, 1, 3, 3), (2, 2, 8, 5)]:
        x = synth.gaussian((N, C, H, W), 151)
        x[0, 0, :3, :3] = 0.0                                  # an all-tie window
        xd = dev(x)
        r = hp.relu_fwd(xd)
        assert np.array_equal(r.cpu().numpy(), oracle.relu_fwd(x).astype(np.float32))
        y = hp.maxpool3x3s2_fwd(xd)
        yo = oracle.maxpool3x3s2_fwd(x)
        assert np.array_equal(y.cpu().numpy(), yo.astype(np.float32))
        g = synth.gaussian(yo.shape, 152)
        gd = dev(g)
        dxp = hp.maxpool3x3s2_bwd(xd, gd, dx=nan_like(x.shape))
        assert norm_err(dxp.cpu().numpy(), oracle.maxpool3x3s2_bwd(x, g)) <= 1e-6
        g2 = synth.gaussian(x.shape, 153)
        drelu = hp.relu_bwd(xd, dev(g2))
        assert np.array_equal(drelu.cpu().numpy(), oracle.relu_bwd(x, g2).astype(np.float32))
    # post-ReLU planes: many all-zero windows, ties resolved to the first element on both sides
    x = np.maximum(synth.gaussian((2, 3, 13, 13), 154), 0)
    g = synth.gaussian((2, 3, 6, 6), 155)
    got = hp.maxpool3x3s2_bwd(dev(x), dev(g)).cpu().numpy()
    assert norm_err(got, oracle.maxpool3x3s2_bwd(x, g)) <= 1e-6


def test_fused_relu_pool_matches_separate_oracle_calls():
    """relu_maxpool3x3s2_fwd/bwd take the pre-activation and must equal ReLU then pooling (and back)."""
    # after the layer shapes: even extents (a last row / column that no window reaches), planes that fill a wavefront
    # exactly (width 127, 128), the wide-plane fallback (129), and plane counts that leave lanes of the last wave idle
    for (N, C, H, W) in [(3, 5, 55, 55), (2, 7, 27, 27), (9, 33, 13, 13), (1, 1, 3, 3), (2, 2, 8, 5), (1, 3, 90, 100),
                         (1, 2, 120, 115), (1, 2, 9, 127), (1, 3, 10, 128), (1, 2, 6, 129), (20, 83, 55, 55),
                         (32, 251, 27, 27)]:
        x = synth.gaussian((N, C, H, W), 161)
        x[0, 0, :3, :3] = -1.0                                  # a window with no positive entry
        x[0, 0, 0, 0] = -0.5
        xd = dev(x)
        y = hp.relu_maxpool3x3s2_fwd(xd)
        r = oracle.relu_fwd(x)
        yo = oracle.maxpool3x3s2_fwd(r)
        assert np.array_equal(y.cpu().numpy(), yo.astype(np.float32))
        g = synth.gaussian(yo.shape, 162)
        dx = hp.relu_maxpool3x3s2_bwd(xd, dev(g), dx=nan_like(x.shape))
        want = oracle.relu_bwd(x, oracle.maxpool3x3s2_bwd(r, g))
        assert norm_err(dx.cpu().numpy(), want) <= 1e-6
        # the unfused entry points on the same planes
        dxp = hp.maxpool3x3s2_bwd(xd, dev(g), dx=nan_like(x.shape))
        assert norm_err(dxp.cpu().numpy(), oracle.maxpool3x3s2_bwd(x, g)) <= 1e-6


def test_relu_vector_and_tail_paths():
    for n in (1, 3, 4, 5, 1023, 4099):
        x = synth.gaussian((n + 1,), 171)
        g = synth.gaussian((n + 1,), 172)
        for off in (0, 1):                                      # off = 1 breaks the 16-byte alignment
            xd, gd = dev(x)[off:off + n], dev(g)[off:off + n]
            y = torch.full((n + 2,), float("nan"), device="cuda")
            hp.lib().relu_fwd(hp._ptr(xd), y[1:].data_ptr(), n, hp.DTYPE_F32, None)
            hp.lib().relu_bwd(hp._ptr(xd), hp._ptr(gd), y[1:].data_ptr(), 0, hp.DTYPE_F32, None)
            torch.cuda.synchronize()
            assert torch.isnan(y[0]) and torch.isnan(y[n + 1])
            assert np.array_equal(y[1:n + 1].cpu().numpy(), oracle.relu_fwd(x[off:off + n]).astype(np.float32))
            d = hp.relu_bwd(xd.contiguous(), gd.contiguous())
            assert np.array_equal(d.cpu().numpy(), oracle.relu_bwd(x[off:off + n], g[off:off + n]).astype(np.float32))


def stack_step_parity(N, dtype, record):
    """One forward+backward step of the five-layer stack: EVERY element of every tensor a call writes is compared
    with the oracle applied to the tensors that call read on the GPU (so errors do not compound from layer to
    layer).  fp32: convolutions within 1e-4, ReLU / pooling forward exact, pooling backward (a sum of up to four
    gradients) within 1e-6.  bf16: tensors are bfloat16 in memory (filter gradients fp32); convolution outputs are
    fp32 sums rounded once, within 2e-2; pooling backward rounds a sum once, within 2^-8."""
    from paper_1312_5853_amd.stack import ConvStack
    st = ConvStack(N, dtype=dtype)
    st.step()
    torch.cuda.synchronize()
    tol = TOL[dtype]
    glue_tol = 1e-6 if dtype == "f32" else 2.0 ** -8
    tag = "stack N=%d %s " % (N, dtype)
    want_t = torch.float32 if dtype == "f32" else torch.bfloat16
    assert st.y1.dtype == want_t and st.dy1.dtype == want_t and st.dw["conv1"].dtype == torch.float32

    def conv(name, got_t, ref):
        check_close(tag + name, got_t, ref, tol, record)

    def exact(name, got_t, ref):
        assert np.array_equal(host64(got_t), ref), tag + name
        record(tag + name, 0.0, 0.0)

    x0, w = host64(st.x0), {k: host64(v) for k, v in st.w.items()}
    # forward
    y1 = host64(st.y1)
    conv("conv1.fwd", st.y1, oracle.conv_fwd(x0, w["conv1"], 4, 2))
    a1 = host64(st.a1)
    exact("pool1.fwd", st.a1, oracle.maxpool3x3s2_fwd(oracle.relu_fwd(y1)))
    y2 = host64(st.y2)
    conv("conv2.fwd (two columns)", st.y2, oracle.conv_fwd_grouped(a1, w["conv2"], 1, 2, 2))
    a2 = host64(st.a2)
    exact("pool2.fwd", st.a2, oracle.maxpool3x3s2_fwd(oracle.relu_fwd(y2)))
    # y3, y4 hold relu(conv): the ReLU is applied where the convolution stores
    y3 = host64(st.y3)
    conv("conv3.fwd+relu", st.y3, oracle.relu_fwd(oracle.conv_fwd(a2, w["conv3"], 1, 1)))
    y4 = host64(st.y4)
    conv("conv4.fwd+relu", st.y4, oracle.relu_fwd(oracle.conv_fwd(y3, w["conv4"], 1, 1)))
    assert y3.min() >= 0.0 and y4.min() >= 0.0
    y5 = host64(st.y5)
    conv("conv5.fwd", st.y5, oracle.conv_fwd(y4, w["conv5"], 1, 1))
    exact("pool5.fwd", st.a5, oracle.maxpool3x3s2_fwd(oracle.relu_fwd(y5)))
    # backward
    g5 = host64(st.g5)
    dy5 = host64(st.dy5)
    check_close(tag + "pool5.bwd", st.dy5, oracle.relu_bwd(y5, oracle.maxpool3x3s2_bwd(oracle.relu_fwd(y5), g5)),
                glue_tol, record)
    conv("conv5.wgrad", st.dw["conv5"], oracle.conv_bwd_filter(y4, dy5, 3, 3, 1, 1))
    # dy4, dy3: backward-data with the mask of the ReLU below applied at the store
    dy4 = host64(st.dy4)
    conv("conv5.dgrad+relu", st.dy4, oracle.relu_bwd(y4, oracle.conv_bwd_data(dy5, w["conv5"], 13, 13, 1, 1)))
    conv("conv4.wgrad", st.dw["conv4"], oracle.conv_bwd_filter(y3, dy4, 3, 3, 1, 1))
    dy3 = host64(st.dy3)
    conv("conv4.dgrad+relu", st.dy3, oracle.relu_bwd(y3, oracle.conv_bwd_data(dy4, w["conv4"], 13, 13, 1, 1)))
    conv("conv3.wgrad", st.dw["conv3"], oracle.conv_bwd_filter(a2, dy3, 3, 3, 1, 1))
    da2 = host64(st.da2)
    conv("conv3.dgrad", st.da2, oracle.conv_bwd_data(dy3, w["conv3"], 13, 13, 1, 1))
    dy2 = host64(st.dy2)
    check_close(tag + "pool2.bwd", st.dy2, oracle.relu_bwd(y2, oracle.maxpool3x3s2_bwd(oracle.relu_fwd(y2), da2)),
                glue_tol, record)
    conv("conv2.wgrad (two columns)", st.dw["conv2"], oracle.conv_bwd_filter_grouped(a1, dy2, 5, 5, 1, 2, 2))
    da1 = host64(st.da1)
    conv("conv2.dgrad (two columns)", st.da1, oracle.conv_bwd_data_grouped(dy2, w["conv2"], 27, 27, 1, 2, 2))
    dy1 = host64(st.dy1)
    check_close(tag + "pool1.bwd", st.dy1, oracle.relu_bwd(y1, oracle.maxpool3x3s2_bwd(oracle.relu_fwd(y1), da1)),
                glue_tol, record)
    conv("conv1.wgrad", st.dw["conv1"], oracle.conv_bwd_filter(x0, dy1, 11, 11, 4, 2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stack_step_small_batch(dtype, parity_record):
    stack_step_parity(2, dtype, parity_record)


def test_convert_f32_to_bf16_is_round_to_nearest_even():
    x = synth.gaussian((100003,), 181)
    # exact, ties to even (down / up), a carry into the exponent, the largest finite value (-> infinity), subnormals
    special = np.array([0x00000000, 0x80000000, 0x3F800000, 0x3F808000, 0x3F818000, 0xBF818000, 0x3FFFFFFF,
                        0x7F7FFFFF, 0xFF7FFFFF, 0x7F7F7FFF, 0x00008001, 0x00018000, 0x7F800000], dtype=np.uint32)
    x[:special.size] = special.view(np.float32)
    got = hp.convert_f32_to_bf16(dev(x))
    want = oracle.bf16_bits(x)
    assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), want)


def test_bf16_glue_matches_oracle():
    """Glue on bfloat16 tensors: ReLU and pooling forward return input values (exact); pooling backward adds up to
    four bf16 gradients in fp32 and rounds once."""
    for (N, C, H, W) in [(3, 5, 55, 55), (2, 7, 27, 27), (9, 33, 13, 13), (1, 1, 3, 3), (2, 2, 8, 5), (1, 3, 90, 100),
                         (1, 2, 120, 115), (1, 2, 9, 127), (1, 3, 10, 128), (1, 1, 7, 1003)]:
        x = oracle.bf16_round(synth.gaussian((N, C, H, W), 171))
        x[0, 0, :3, :3] = 0.0
        xd = dev(x, "bf16")
        f = lambda t: t.float().cpu().numpy()
        assert np.array_equal(f(hp.relu_fwd(xd)), oracle.relu_fwd(x).astype(np.float32))
        y = hp.maxpool3x3s2_fwd(xd)
        yo = oracle.maxpool3x3s2_fwd(x)
        assert y.dtype == torch.bfloat16 and np.array_equal(f(y), yo.astype(np.float32))
        assert np.array_equal(f(hp.relu_maxpool3x3s2_fwd(xd)), oracle.maxpool3x3s2_fwd(oracle.relu_fwd(x)).astype(np.float32))
        g = oracle.bf16_round(synth.gaussian(yo.shape, 172))
        gd = dev(g, "bf16")
        marker = torch.full(x.shape, 7.0, dtype=torch.bfloat16, device="cuda")
        dxp = hp.maxpool3x3s2_bwd(xd, gd, dx=marker)
        want = oracle.maxpool3x3s2_bwd(x, g)
        assert norm_err(f(dxp), want) <= 2.0 ** -8
        # where a single window contributes the result is that gradient, exactly; where none does, zero
        single = np.isin(want, g) | (want == 0)
        assert np.array_equal(f(dxp)[single], want[single].astype(np.float32))
        dxr = hp.relu_maxpool3x3s2_bwd(xd, gd)
        assert norm_err(f(dxr), oracle.relu_bwd(x, oracle.maxpool3x3s2_bwd(oracle.relu_fwd(x), g))) <= 2.0 ** -8
        g2 = oracle.bf16_round(synth.gaussian(x.shape, 173))
        assert np.array_equal(f(hp.relu_bwd(xd, dev(g2, "bf16"))), oracle.relu_bwd(x, g2).astype(np.float32))
    # odd counts and unaligned bases: the vector body, the tail and the scalar form of the ReLU kernels
    for count, off in [(1, 0), (7, 0), (8, 0), (1029, 0), (1029, 1), (4099, 3)]:
        x = oracle.bf16_round(synth.gaussian((count + off,), 174))
        g = oracle.bf16_round(synth.gaussian((count + off,), 175))
        xd, gd = dev(x, "bf16")[off:], dev(g, "bf16")[off:]
        f = lambda t: t.float().cpu().numpy()
        assert np.array_equal(f(hp.relu_fwd(xd)), oracle.relu_fwd(x[off:]).astype(np.float32))
        assert np.array_equal(f(hp.relu_bwd(xd, gd)), oracle.relu_bwd(x[off:], g[off:]).astype(np.float32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bias_forward_and_gradient(dtype):
    for (N, K, P, Q) in [(3, 5, 7, 9), (128, 96, 55, 55), (2, 300, 1, 1), (1, 1, 3, 3), (9, 2500, 2, 3)]:
        y = synth.gaussian((N, K, P, Q), 181)
        b = synth.gaussian((K,), 182)
        if dtype == "bf16":
            y = oracle.bf16_round(y)
        got = hp.bias_fwd(dev(y, dtype), dev(b))
        want = oracle.bias_fwd(y, b)
        if dtype == "f32":
            assert np.array_equal(got.cpu().numpy(), (y + b[None, :, None, None]).astype(np.float32))   # one fp32 add
            assert norm_err(got.cpu().numpy(), want) <= 1e-6
        else:
            assert norm_err(got.float().cpu().numpy(), want) <= 2.0 ** -8                                 # one rounding
        db = hp.bias_bwd(dev(y, dtype))
        ref = oracle.bias_bwd(y)
        scale = np.abs(y.astype(np.float64)).sum(axis=(0, 2, 3)).max()
        assert np.abs(db.cpu().numpy() - ref).max() <= 1e-6 * scale
        assert torch.equal(db, hp.bias_bwd(dev(y, dtype)))                                               # fixed order
    yi = synth.small_integers((4, 6, 5, 5), 183)
    assert np.array_equal(hp.bias_bwd(dev(yi, dtype)).cpu().numpy(), oracle.bias_bwd(yi))


# --------------------------------------------- convolution with its bias / ReLU applied at the store ---
EPILOGUE_SHAPES = [
    (128, 64, 13, 13, 256, 3, 3, 1, 1),    # 32 x 32 tile kernels, enough tiles for a whole-reduction launch
    (200, 64, 13, 13, 256, 3, 3, 1, 1),    # 530 tiles of 128 x 128: more than one round of work-groups, ragged end
    (4, 64, 13, 13, 96, 3, 3, 1, 1),       # few tiles: reduction split, epilogue in the split-sum kernel
    (7, 48, 14, 14, 64, 5, 5, 1, 2),       # backward-data in the 48-row kernel: epilogue as a pass of its own
    (3, 3, 23, 25, 48, 11, 11, 4, 2),      # few-channel forward (patch kernel), strided backward-data (tap table)
    (2, 3, 24, 32, 48, 11, 11, 4, 2),      # the same with rows of 32: the bf16 few-channel kernel applies bias / ReLU itself
    (2, 5, 8, 10, 130, 3, 3, 1, 5),        # tap-table kernels both ways
]


@pytest.mark.parametrize("mode", ["f32", "bf16", "bf16out"])
@pytest.mark.parametrize("shape", EPILOGUE_SHAPES)
def test_conv_with_bias_relu_epilogues(shape, mode):
    N, C, H, W, K, R, S, st, pad = shape
    P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
    dtype = "f32" if mode == "f32" else "bf16"
    out_t = torch.bfloat16 if mode == "bf16out" else torch.float32
    x, w, dy = prepared(synth.gaussian((N, C, H, W), 191), synth.gaussian((K, C, R, S), 192, 0.1),
                        synth.gaussian((N, K, P, Q), 193), dtype)
    b = synth.gaussian((K,), 194)
    act = synth.gaussian((N, C, H, W), 195)
    if mode == "bf16out":
        act = oracle.bf16_round(act)
    xd, wd, dyd, bd = dev(x, dtype), dev(w, dtype), dev(dy, dtype), dev(b)
    actd = dev(act).to(out_t)
    tol = TOL[dtype]

    def fresh(shape_):
        return torch.full(shape_, float("nan"), dtype=out_t, device="cuda")

    for bias, relu in [(b, True), (None, True), (b, False)]:
        got = hp.conv_fwd_bias_relu(xd, wd, bd if bias is not None else None, st, pad, relu=relu,
                                    y=fresh((N, K, P, Q)))
        want = oracle.conv_fwd_bias_relu(x, w, bias, st, pad, relu=relu)
        e = norm_err(got.float().cpu().numpy(), want)
        assert np.isfinite(e) and e <= tol, "fwd bias=%s relu=%s err %.3e" % (bias is not None, relu, e)
        if relu:
            assert float(got.float().min()) >= 0.0
        if mode != "bf16out":
            # the separate calls do the same fp32 operations in the same order
            sep = hp.conv_fwd(xd, wd, st, pad, y=fresh((N, K, P, Q)))
            if bias is not None:
                hp.bias_fwd(sep, bd)
            if relu:
                hp.relu_fwd(sep, y=sep)
            assert torch.equal(got, sep)
        else:
            # bfloat16 output: the fused fp32 result (bias added, ReLU applied) rounded ONCE to nearest even
            f32 = hp.conv_fwd_bias_relu(xd, wd, bd if bias is not None else None, st, pad, relu=relu,
                                        y=nan_like((N, K, P, Q)))
            assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16),
                                  oracle.bf16_bits(f32.cpu().numpy()))
    got = hp.conv_bwd_data_relu(dyd, wd, actd, st, pad, dx=fresh((N, C, H, W)))
    want = oracle.conv_bwd_data_relu(dy, w, act, st, pad)
    e = norm_err(got.float().cpu().numpy(), want)
    assert np.isfinite(e) and e <= tol, "dgrad err %.3e" % e
    assert np.array_equal(got.float().cpu().numpy()[act <= 0], np.zeros(np.count_nonzero(act <= 0), np.float32))
    sep = hp.conv_bwd_data(dyd, wd, H, W, st, pad, dx=fresh((N, C, H, W)))
    assert torch.equal(got, hp.relu_bwd(actd, sep))
    if mode == "bf16out":
        f32 = hp.conv_bwd_data_relu(dyd, wd, actd.float(), st, pad, dx=nan_like((N, C, H, W)))
        assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), oracle.bf16_bits(f32.cpu().numpy()))


def test_epilogue_argument_checks():
    x = torch.zeros((1, 16, 5, 5), device="cuda"); w = torch.zeros((16, 16, 3, 3), device="cuda")
    y = torch.zeros((1, 16, 5, 5), device="cuda")
    L = hp.lib()
    import ctypes
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    need = hp.workspace_bytes(hp.OP_FWD, 1, 16, 5, 5, 16, 3, 3, 1, 1)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    dims = (1, 16, 5, 5, 16, 3, 3, 1, 1)
    assert L.conv_fwd_bias_relu(p(x), p(w), None, p(y), *dims, 2, 0, p(ws), ws.numel(), st) == hp.ERR_INVALID_ARG
    assert L.conv_fwd_bias_relu(p(x), p(w), None, None, *dims, 1, 0, p(ws), ws.numel(), st) == hp.ERR_INVALID_ARG
    assert L.conv_bwd_data_relu(p(y), p(w), None, p(x), *dims, 0, p(ws), ws.numel(), st) == hp.ERR_INVALID_ARG
    assert L.conv_fwd_bias_relu(p(x), p(w), None, p(y), *dims, 1, 0, p(ws), 0, st) == (
        hp.ERR_WORKSPACE if need else hp.OK)
    torch.cuda.synchronize()


# ----------------------------------------------------- fully connected layers, SGD update ---
FC_SHAPES = [
    # N, I, O
    (1, 4, 4),
    (3, 8, 12),
    (5, 100, 36),            # reduction tails of 4 and of 5 samples
    (130, 260, 132),         # two tiles each way, ragged
    (257, 16, 1000),         # three row tiles, last output tile of 104
    (64, 4096, 1000),        # fc8 at a shard of 64
    (128, 9216, 4096),       # fc6 at a shard of 128 (reduction split 16 ways forward)
]


@pytest.mark.parametrize("shape", FC_SHAPES)
def test_fc_layers_full_compare(shape):
    N, I, O = shape
    x = synth.gaussian((N, I), 201)
    w = synth.gaussian((O, I), 202, 0.05)
    dy = synth.gaussian((N, O), 203)
    b = synth.gaussian((O,), 204)
    xd, wd, dyd, bd = dev(x), dev(w), dev(dy), dev(b)
    nan2 = lambda *s: torch.full(s, float("nan"), dtype=torch.float32, device="cuda")
    tol = TOL["f32"]
    y = hp.fc_fwd(xd, wd, y=nan2(N, O))
    assert norm_err(y.cpu().numpy(), oracle.fc_fwd(x, w)) <= tol
    yb = hp.fc_fwd(xd, wd, bias=bd, relu=True, y=nan2(N, O))
    assert norm_err(yb.cpu().numpy(), oracle.fc_fwd(x, w, b, relu=True)) <= tol
    assert float(yb.min()) >= 0.0
    # bias and ReLU are applied to the same fp32 sums the plain call stores
    assert torch.equal(yb, torch.clamp_min(y + bd[None, :], 0.0))
    dx = hp.fc_bwd_data(dyd, wd, dx=nan2(N, I))
    assert norm_err(dx.cpu().numpy(), oracle.fc_bwd_data(dy, w)) <= tol
    dw = hp.fc_bwd_filter(xd, dyd, dw=nan2(O, I))
    assert norm_err(dw.cpu().numpy(), oracle.fc_bwd_filter(x, dy)) <= tol
    # fixed summation order
    assert torch.equal(y, hp.fc_fwd(xd, wd)) and torch.equal(dx, hp.fc_bwd_data(dyd, wd))
    assert torch.equal(dw, hp.fc_bwd_filter(xd, dyd))


def test_fc_small_integers_are_exact_and_guards_untouched():
    N, I, O = 37, 72, 140
    x, w, dy = synth.small_integers((N, I), 211), synth.small_integers((O, I), 212), synth.small_integers((N, O), 213)
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    assert np.array_equal(hp.fc_fwd(xd, wd).cpu().numpy(), oracle.fc_fwd(x, w))
    assert np.array_equal(hp.fc_bwd_data(dyd, wd).cpu().numpy(), oracle.fc_bwd_data(dy, w))
    assert np.array_equal(hp.fc_bwd_filter(xd, dyd).cpu().numpy(), oracle.fc_bwd_filter(x, dy))
    # outputs inside a larger allocation: nothing outside [N][O] / [N][I] / [O][I] is written
    for fn, shape in ((lambda out: hp.fc_fwd(xd, wd, y=out), (N, O)),
                      (lambda out: hp.fc_bwd_data(dyd, wd, dx=out), (N, I)),
                      (lambda out: hp.fc_bwd_filter(xd, dyd, dw=out), (O, I))):
        n = shape[0] * shape[1]
        buf = torch.full((n + 2048,), -7.0, dtype=torch.float32, device="cuda")
        fn(buf[1024:1024 + n].view(shape))
        torch.cuda.synchronize()
        assert bool((buf[:1024] == -7.0).all()) and bool((buf[1024 + n:] == -7.0).all())
        assert not bool(torch.isnan(buf).any())


def test_fc_argument_checks():
    import ctypes
    L = hp.lib()
    t = torch.zeros(4096, device="cuda")
    p = lambda off=0: ctypes.c_void_p(t.data_ptr() + off)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.fc_fwd(p(), p(), None, p(), 4, 6, 8, 0, 0, None, 0, st) == hp.ERR_INVALID_ARG      # I % 4
    assert L.fc_fwd(p(), p(), None, p(), 4, 8, 6, 0, 0, None, 0, st) == hp.ERR_INVALID_ARG      # O % 4
    assert L.fc_fwd(p(), p(), None, None, 4, 8, 8, 0, 0, None, 0, st) == hp.ERR_INVALID_ARG
    assert L.fc_fwd(p(), p(), None, p(), 4, 8, 8, 3, 0, None, 0, st) == hp.ERR_INVALID_ARG      # relu flag
    assert L.fc_fwd(p(), p(), None, p(), 4, 8, 8, 0, 1, None, 0, st) == hp.ERR_BAD_DTYPE
    assert L.fc_fwd(p(4), p(), None, p(), 4, 8, 8, 0, 0, None, 0, st) == hp.ERR_MISALIGNED
    assert L.fc_bwd_data(p(), p(), p(), 0, 8, 8, 0, None, 0, st) == hp.ERR_INVALID_ARG
    need = L.fc_workspace_bytes(hp.OP_FWD, 8, 4096, 8, 0)
    assert need > 0 and L.fc_workspace_bytes(hp.OP_FWD, 8, 4095, 8, 0) == 0
    big = torch.zeros(8 * 4096, device="cuda")
    assert L.fc_fwd(ctypes.c_void_p(big.data_ptr()), ctypes.c_void_p(big.data_ptr()), None, p(), 8, 4096, 8, 0, 0,
                    None, 0, st) == hp.ERR_WORKSPACE
    assert L.sgd_update(None, p(), p(), 4, 0.1, 0.0, 0.0, 1.0, st) == hp.ERR_INVALID_ARG
    assert L.sgd_update(p(), p(), p(), -1, 0.1, 0.0, 0.0, 1.0, st) == hp.ERR_INVALID_ARG
    assert L.sgd_update(None, None, None, 0, 0.1, 0.0, 0.0, 1.0, st) == hp.OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("count", [1, 3, 4, 5, 1003, 1 << 20, 37748736 // 8 + 1])
def test_sgd_update_matches_oracle(count):
    w = synth.gaussian((count,), 221)
    g = synth.gaussian((count,), 222)
    v = synth.gaussian((count,), 223, 0.1)
    for off in (0, 1):                       # off = 1: pointers 4 bytes past a 16-byte boundary (scalar path)
        store = [torch.zeros(count + 4, device="cuda") for _ in range(3)]
        wd, gd, vd = (s[off:off + count] for s in store)
        wd.copy_(dev(w)); gd.copy_(dev(g)); vd.copy_(dev(v))
        rw, rv = w.astype(np.float64), v.astype(np.float64)
        for step in range(2):
            hp.sgd_update(wd, gd, vd, lr=0.01, momentum=0.9, weight_decay=5e-4, grad_scale=1.0 / 128)
            rw, rv = oracle.sgd_update(rw, g, rv, 0.01, 0.9, 5e-4, 1.0 / 128)
            # the reference continues from the fp32 state the device holds, so each step is compared on its own
            assert norm_err(vd.cpu().numpy(), rv) <= 1e-6 and norm_err(wd.cpu().numpy(), rw) <= 1e-6
            rw, rv = wd.cpu().numpy().astype(np.float64), vd.cpu().numpy().astype(np.float64)
        assert torch.equal(gd, dev(g))                                   # gradients only read
        for s in store:                                                  # nothing outside the arrays touched
            assert float(s[:off].abs().sum()) == 0.0 and float(s[off + count:].abs().sum()) == 0.0
    # plain SGD is exactly w - lr * dw in fp32
    wd, gd, vd = dev(w), dev(g), torch.zeros(count, device="cuda")
    hp.sgd_update(wd, gd, vd, lr=0.5)
    want = (w - (np.float32(0.5) * g).astype(np.float32)).astype(np.float32)
    assert np.array_equal(wd.cpu().numpy(), want)


def test_full_network_step_fc_part_and_update():
    """One whole training step (conv stack, three fully connected layers, SGD update) at a small batch: the fully
    connected part and the update are checked call by call against the oracle on the tensors each call read (the
    convolutional part has its own test above)."""
    from paper_1312_5853_amd.stack import FullNetwork, FC_LAYERS, CONV_ORDER
    N = 2
    net = FullNetwork(N)
    c = lambda t: t.detach().cpu().numpy().copy()
    before = [c(p) for p, _ in net.params]
    net.forward()
    net.backward()
    torch.cuda.synchronize()
    tol = TOL["f32"]
    a = c(net.a5).reshape(N, -1)
    acts = {}
    for name, _, _ in FC_LAYERS:
        want = oracle.fc_fwd(a, c(net.fc_w[name]), c(net.fc_b[name]), relu=name != "fc8")
        got = c(net.fc_y[name])
        assert norm_err(got, want) <= tol, name
        acts[name] = a
        a = got
    d = c(net.g8)
    for name, _, _ in reversed(FC_LAYERS):
        if name != "fc8":
            d_ref = oracle.relu_bwd(c(net.fc_y[name]), d)
            d = c(net.fc_dy[name])                         # holds the gradient after the in-place ReLU backward
            assert norm_err(d, d_ref) <= tol, name
        assert norm_err(c(net.fc_dw[name]), oracle.fc_bwd_filter(acts[name], d)) <= tol, name
        assert norm_err(c(net.fc_db[name]), d.astype(np.float64).sum(axis=0)) <= 1e-6, name
        d_next = oracle.fc_bwd_data(d, c(net.fc_w[name]))
        d = d_next                                         # compared one layer down, after that layer's ReLU
    assert norm_err(c(net.g5).reshape(N, -1), d) <= tol
    # the convolutional backward consumed g5: its last filter gradient is finite and non-zero
    assert np.isfinite(c(net.dw["conv1"])).all() and np.abs(c(net.dw["conv1"])).max() > 0
    grads = [c(g) for _, g in net.params]
    net.update()
    torch.cuda.synchronize()
    assert len(net.params) == len(CONV_ORDER) + 2 * len(FC_LAYERS)
    for (p, _), w0, g, v in zip(net.params, before, grads, net.vel):
        w_ref, v_ref = oracle.sgd_update(w0, g, np.zeros_like(w0), net.lr, net.momentum, net.weight_decay, 1.0 / N)
        assert norm_err(c(p), w_ref) <= 1e-6 and norm_err(c(v), v_ref) <= 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N", [64, 128, 256])
def test_stack_step_full_batch_whole_tensors(N, dtype, parity_record):
    """The benchmarked step at every batch size and element type of the workload list (a 64-image shard: four-GPU
    data parallelism; 128: two GPUs; 256: the whole mini-batch on one GPU).  Tile shapes, reduction splits and the
    occupancy cap change with N, so each configuration is checked on its own, whole tensors, call by call."""
    stack_step_parity(N, dtype, parity_record)


# ------------------------------------------------------------ seeded random small shapes ---
def _random_shapes(count, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    shapes = []
    while len(shapes) < count:
        N = int(rng.integers(1, 5))
        C = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 32, 33, 48, 64]))
        K = int(rng.choice([1, 3, 16, 31, 32, 33, 47, 48, 64, 96, 100, 129]))
        H, W = int(rng.integers(1, 15)), int(rng.integers(1, 15))
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        st, pad = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        shapes.append((N, C, H, W, K, R, S, st, pad))
    return shapes


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_small_shapes_full_compare(dtype):
    """Sixty seeded random layer shapes per element type (channel counts on and off the multiples of 16 that select
    the kernels, strides 1-3, padding up to 3, planes down to 1x1): all three passes against the oracle."""
    for i, shape in enumerate(_random_shapes(60, 4242 if dtype == "f32" else 4343)):
        N, C, H, W, K, R, S, st, pad = shape
        P, Q = hp.out_extent(H, R, st, pad), hp.out_extent(W, S, st, pad)
        x = synth.gaussian((N, C, H, W), 7000 + i)
        w = synth.gaussian((K, C, R, S), 8000 + i, 0.1)
        dy = synth.gaussian((N, K, P, Q), 9000 + i)
        try:
            check_full(x, w, dy, st, pad, dtype)
        except AssertionError as e:
            raise AssertionError("shape %r: %s" % (shape, e))


def test_sgd_update_multi_equals_the_per_tensor_update():
    """One call for many tensors (more than one launch's worth, sizes with and without a multiple of four, an empty
    tensor, a tensor that is not 16-byte aligned): every parameter bit for bit what sgd_update gives, and the oracle's
    value within the fp32 tolerance."""
    rng = np.random.Generator(np.random.Philox(6161))
    sizes = [int(s) for s in rng.integers(1, 5000, size=27)] + [0, 4096, 1 << 20]
    ws, gs, vs, ws1, vs1, host = [], [], [], [], [], []
    for i, n in enumerate(sizes):
        w, g, v = (synth.gaussian((n + 1,), 15000 + 3 * i + k) for k in range(3))
        off = 1 if i % 5 == 2 else 0                              # a view one element in: 4-byte aligned only
        wd, gd, vd = (torch.from_numpy(a).cuda()[off:off + n] for a in (w, g, v))
        ws.append(wd); gs.append(gd); vs.append(vd)
        ws1.append(wd.clone()); vs1.append(vd.clone())
        host.append((w[off:off + n], g[off:off + n], v[off:off + n]))
    hp.sgd_update_multi(ws, gs, vs, lr=0.01, momentum=0.9, weight_decay=5e-4, grad_scale=1.0 / 128)
    for wd, gd, vd, (w, g, v) in zip(ws1, gs, vs1, host):
        if wd.numel():
            hp.sgd_update(wd, gd, vd, lr=0.01, momentum=0.9, weight_decay=5e-4, grad_scale=1.0 / 128)
    torch.cuda.synchronize()
    for i, (a, b, c, d, (w, g, v)) in enumerate(zip(ws, ws1, vs, vs1, host)):
        assert torch.equal(a, b) and torch.equal(c, d), sizes[i]
        if sizes[i]:
            rw, rv = oracle.sgd_update(w, g, v, 0.01, 0.9, 5e-4, 1.0 / 128)
            assert norm_err(a.cpu().numpy(), rw) <= TOL["f32"] and norm_err(c.cpu().numpy(), rv) <= TOL["f32"]
    L = hp.lib()
    assert L.sgd_update_multi(None, None, None, None, 0, 0.1, 0.0, 0.0, 1.0, None) == hp.OK
    assert L.sgd_update_multi(None, None, None, None, 2, 0.1, 0.0, 0.0, 1.0, None) == hp.ERR_INVALID_ARG


def test_random_fc_shapes_full_compare():
    """Forty seeded random fully connected shapes (batch up to 300, widths up to 600 in multiples of 4: one to
    five tiles each way, reductions of one to 38 steps with ragged ends and split ranges)."""
    rng = np.random.Generator(np.random.Philox(5151))
    for i in range(40):
        N = int(rng.integers(1, 301))
        I, O = 4 * int(rng.integers(1, 151)), 4 * int(rng.integers(1, 151))
        x = synth.gaussian((N, I), 11000 + i)
        w = synth.gaussian((O, I), 12000 + i, 0.1)
        dy = synth.gaussian((N, O), 13000 + i)
        b = synth.gaussian((O,), 14000 + i)
        xd, wd, dyd, bd = dev(x), dev(w), dev(dy), dev(b)
        tag = "N=%d I=%d O=%d" % (N, I, O)
        assert norm_err(hp.fc_fwd(xd, wd, bias=bd, relu=bool(i & 1)).cpu().numpy(),
                        oracle.fc_fwd(x, w, b, relu=bool(i & 1))) <= TOL["f32"], tag
        assert norm_err(hp.fc_bwd_data(dyd, wd).cpu().numpy(), oracle.fc_bwd_data(dy, w)) <= TOL["f32"], tag
        assert norm_err(hp.fc_bwd_filter(xd, dyd).cpu().numpy(), oracle.fc_bwd_filter(x, dy)) <= TOL["f32"], tag


def test_step_replayed_from_a_hip_graph_equals_the_eager_step():
    """The stack step captured into a HIP graph: several replays, with eager steps and synchronisations between
    them, each leave exactly the tensors the eager step leaves (the step is deterministic)."""
    from paper_1312_5853_amd.stack import ConvStack
    st = ConvStack(4)
    st.step()
    torch.cuda.synchronize()
    names = ("y1", "a1", "y2", "a2", "y3", "y4", "y5", "a5", "dy5", "dy4", "dy3", "da2", "dy2", "da1", "dy1")
    want = {n: getattr(st, n).clone() for n in names}
    want_dw = {k: v.clone() for k, v in st.dw.items()}
    graph = st.capture()
    for rep in range(3):
        for n in names:
            getattr(st, n).fill_(float("nan"))
        for v in st.dw.values():
            v.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for n in names:
            assert torch.equal(getattr(st, n), want[n]), (rep, n)
        for k in want_dw:
            assert torch.equal(st.dw[k], want_dw[k]), (rep, k)
        st.step()                                  # eager work between the replays
        torch.cuda.synchronize()
        hp.relu_fwd(st.y3, st.y3)
        torch.cuda.synchronize()


def test_largest_tensors_the_boundary_accepts():
    """Tensors of 2047 x 64 x 64 x 64 fp32 elements: 1 MiB short of the 2^31-byte span the boundary allows, so byte
    offsets inside the kernels run up to the top of their 32-bit range.  Inputs are drawn on the device (seeded);
    sampled outputs, the last elements of every tensor among them, are checked against the oracle."""
    N, C, H, W, K, R, S, st, pad = 2047, 64, 64, 64, 64, 3, 3, 1, 1
    assert N * C * H * W * 4 < 2 ** 31 <= (N + 1) * C * H * W * 4
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.SEED_BASE + 4001)
    xd = torch.randn((N, C, H, W), device="cuda", generator=gen)
    dyd = torch.randn((N, K, H, W), device="cuda", generator=gen)
    wd = torch.randn((K, C, R, S), device="cuda", generator=gen) * 0.05
    x64, dy64, w64 = (t.cpu().numpy().astype(np.float64) for t in (xd, dyd, wd))

    def sample(t, count, seed):
        tail = np.arange(t.numel() - 64, t.numel(), dtype=np.int64)          # the highest addresses
        idx = np.unique(np.concatenate([synth.sample_indices(t.numel(), count, seed), edge_indices(t.shape), tail]))
        return idx, t.view(-1)[torch.from_numpy(idx).cuda()].cpu().numpy()

    y = hp.conv_fwd(xd, wd, st, pad)
    idx, got = sample(y, 4000, 31)
    assert norm_err(got, oracle.conv_fwd_at(x64, w64, st, pad, idx)) <= TOL["f32"]
    del y
    dx = hp.conv_bwd_data(dyd, wd, H, W, st, pad)
    idx, got = sample(dx, 2000, 32)
    assert norm_err(got, oracle.conv_bwd_data_at(dy64, w64, H, W, st, pad, idx)) <= TOL["f32"]
    del dx
    dw = hp.conv_bwd_filter(xd, dyd, R, S, st, pad)
    idx, got = sample(dw, 300, 33)
    assert norm_err(got, oracle.conv_bwd_filter_at(x64, dy64, R, S, st, pad, idx)) <= TOL["f32"]
    # one sample more is refused before anything is launched
    big = torch.empty(((N + 1) * C * H * W,), device="cuda")
    with pytest.raises(hp.ConvError) as e:
        hp.conv_fwd(big.view(N + 1, C, H, W), wd, st, pad, y=big.view(N + 1, K, H, W))
    assert e.value.status == hp.ERR_TOO_LARGE
