"""ctypes binding of ``libconvnet_hotpath.so`` (see ``include/convnet_hotpath.h``).

Argument marshalling only: every function here hands device pointers, extents
and a HIP stream to the C ABI entry point of the same name.  PyTorch supplies
device memory and streams; no arithmetic of the convolution path happens in
Python.  If the library has not been built this module raises -- there is no
fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconvnet_hotpath.so")

OK = 0
ERR_INVALID_ARG, ERR_TOO_LARGE, ERR_BAD_DTYPE, ERR_WORKSPACE, ERR_MISALIGNED, ERR_HIP = -1, -2, -3, -4, -5, -6
ERR_SCRATCH_LIMIT = -7
NOALLOC_SCRATCH_BYTES = 48 << 20
DTYPE_F32, DTYPE_BF16, DTYPE_BF16_OUT_BF16 = 0, 1, 2
OP_FWD, OP_BWD_DATA, OP_BWD_FILTER = 0, 1, 2

EXPORTS = (
    "conv_fwd", "conv_bwd_data", "conv_bwd_filter", "conv_bwd_filter_noalloc",
    "conv_fwd_ex", "conv_bwd_data_ex", "conv_bwd_filter_ex", "conv_fwd_bias_relu", "conv_bwd_data_relu",
    "conv_fwd_grouped", "conv_bwd_data_grouped", "conv_bwd_filter_grouped", "conv_workspace_bytes_grouped",
    "conv_workspace_bytes", "conv_output_extent", "conv_status_string", "conv_last_hip_error",
    "relu_fwd", "relu_bwd", "maxpool3x3s2_fwd", "maxpool3x3s2_bwd",
    "relu_maxpool3x3s2_fwd", "relu_maxpool3x3s2_bwd", "convert_f32_to_bf16",
    "bias_fwd", "bias_bwd", "bias_bwd_workspace_bytes",
    "fc_fwd", "fc_bwd_data", "fc_bwd_filter", "fc_workspace_bytes", "sgd_update", "sgd_update_multi",
)

_lib = None


class ConvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().conv_status_string(status).decode()
        if status == ERR_HIP:
            msg += ": " + lib().conv_last_hip_error().decode()
        super().__init__("%s failed with status %d (%s)" % (where, status, msg))


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "%s is missing: build it with `python -m paper_1312_5853_amd.build` "
            "(there is no fallback implementation)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    dims = [i] * 9
    for name in ("conv_fwd", "conv_bwd_data", "conv_bwd_filter"):
        f = getattr(L, name)
        f.argtypes = [vp, vp, vp] + dims + [i, vp, sz, vp]
        f.restype = i
        f = getattr(L, name + "_ex")
        f.argtypes = [vp, vp, vp] + dims + [i64, i64, i, vp, sz, vp]
        f.restype = i
        f = getattr(L, name + "_grouped")
        f.argtypes = [vp, vp, vp] + dims + [i, i, vp, sz, vp]
        f.restype = i
    L.conv_bwd_filter_noalloc.argtypes = [vp, vp, vp] + dims + [i, vp]
    L.conv_bwd_filter_noalloc.restype = i
    L.conv_fwd_bias_relu.argtypes = [vp, vp, vp, vp] + dims + [i, i, vp, sz, vp]
    L.conv_fwd_bias_relu.restype = i
    L.conv_bwd_data_relu.argtypes = [vp, vp, vp, vp] + dims + [i, vp, sz, vp]
    L.conv_bwd_data_relu.restype = i
    L.fc_fwd.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
    L.fc_bwd_data.argtypes = [vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.fc_bwd_filter.argtypes = [vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.fc_workspace_bytes.argtypes = [i, i, i, i, i]
    L.fc_workspace_bytes.restype = sz
    f32 = ctypes.c_float
    L.sgd_update.argtypes = [vp, vp, vp, i64, f32, f32, f32, f32, vp]
    L.sgd_update_multi.argtypes = [vp, vp, vp, vp, i, f32, f32, f32, f32, vp]
    for name in ("fc_fwd", "fc_bwd_data", "fc_bwd_filter", "sgd_update", "sgd_update_multi"):
        getattr(L, name).restype = i
    L.conv_workspace_bytes_grouped.argtypes = [i] + dims + [i, i]
    L.conv_workspace_bytes_grouped.restype = sz
    L.conv_workspace_bytes.argtypes = [i] + dims + [i]
    L.conv_workspace_bytes.restype = sz
    L.bias_fwd.argtypes = [vp, vp, i, i, i, i, vp]
    L.bias_fwd.restype = i
    L.bias_bwd.argtypes = [vp, vp, i, i, i, i, vp, sz, vp]
    L.bias_bwd.restype = i
    L.bias_bwd_workspace_bytes.argtypes = [i, i]
    L.bias_bwd_workspace_bytes.restype = sz
    L.conv_output_extent.argtypes = [i, i, i, i]
    L.conv_output_extent.restype = i
    L.conv_status_string.argtypes = [i]
    L.conv_status_string.restype = ctypes.c_char_p
    L.conv_last_hip_error.argtypes = []
    L.conv_last_hip_error.restype = ctypes.c_char_p
    L.relu_fwd.argtypes = [vp, vp, i64, i, vp]
    L.relu_bwd.argtypes = [vp, vp, vp, i64, i, vp]
    L.maxpool3x3s2_fwd.argtypes = [vp, vp, i64, i, i, i, vp]
    L.maxpool3x3s2_bwd.argtypes = [vp, vp, vp, i64, i, i, i, vp]
    L.convert_f32_to_bf16.argtypes = [vp, vp, i64, vp]
    L.convert_f32_to_bf16.restype = i
    L.relu_maxpool3x3s2_fwd.argtypes = [vp, vp, i64, i, i, i, vp]
    L.relu_maxpool3x3s2_bwd.argtypes = [vp, vp, vp, i64, i, i, i, vp]
    for name in ("relu_fwd", "relu_bwd", "maxpool3x3s2_fwd", "maxpool3x3s2_bwd", "relu_maxpool3x3s2_fwd",
                 "relu_maxpool3x3s2_bwd"):
        getattr(L, name).restype = i
    _lib = L
    return L


def status_string(status):
    return lib().conv_status_string(int(status)).decode()


def workspace_bytes(op, N, C, H, W, K, R, S, stride, pad, dtype=DTYPE_F32):
    return int(lib().conv_workspace_bytes(op, N, C, H, W, K, R, S, stride, pad, dtype))


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _dtype_of(t):
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError("unsupported tensor dtype %s" % t.dtype)


def out_extent(size, filt, stride, pad):
    """P or Q of a layer, asked of the library (conv_output_extent)."""
    return int(lib().conv_output_extent(size, filt, stride, pad))


class Workspace:
    """A growable device scratch buffer handed to the library as `ws`."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = None

    def get(self, nbytes):
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self.buf, self.buf.numel()


_default_ws = None


def _ws(ws):
    global _default_ws
    if ws is not None:
        return ws
    if _default_ws is None:
        _default_ws = Workspace()
    return _default_ws


def _run(name, op, a, b, out, dims, x_bs, y_bs, dtype, ws, stream):
    need = workspace_bytes(op, *dims, dtype)
    buf, nbytes = _ws(ws).get(need)
    wsp = ctypes.c_void_p(buf.data_ptr()) if buf is not None else ctypes.c_void_p(0)
    if x_bs or y_bs:
        rc = getattr(lib(), name + "_ex")(_ptr(a), _ptr(b), _ptr(out), *dims, int(x_bs), int(y_bs), dtype,
                                          wsp, nbytes, _stream_handle(stream))
    else:
        rc = getattr(lib(), name)(_ptr(a), _ptr(b), _ptr(out), *dims, dtype, wsp, nbytes, _stream_handle(stream))
    if rc != OK:
        raise ConvError(rc, name)
    return out


def _batch_stride(t):
    """Batch stride in elements of an NCHW tensor whose samples are dense (a
    channel slice of a wider tensor qualifies); 0 when the whole tensor is."""
    n, c, h, w = t.shape
    if t.stride(3) != 1 or t.stride(2) != w or t.stride(1) != h * w:
        raise ValueError("the [channel][row][col] block of every sample must be dense")
    return 0 if (n == 1 or t.stride(0) == c * h * w) else t.stride(0)


def _io_dtype(src, out):
    """dtype code of a forward / backward-data call from its input and output tensors."""
    d = _dtype_of(src)
    if out.dtype == torch.bfloat16:
        if d != DTYPE_BF16:
            raise TypeError("a bfloat16 output needs bfloat16 inputs")
        return DTYPE_BF16_OUT_BF16
    if out.dtype != torch.float32:
        raise TypeError("unsupported output dtype %s" % out.dtype)
    return d


def conv_fwd(x, w, stride, pad, y=None, ws=None, stream=None, out_bf16=False):
    """x [N,C,H,W], w [K,C,R,S] -> y [N,K,P,Q], fp32 (or bfloat16: pass a bfloat16 y, or out_bf16=True, with
    bfloat16 inputs).  x and y may be channel slices of wider NCHW tensors (their batch strides are passed on)."""
    N, C, H, W = x.shape
    K, Cw, R, S = w.shape
    if C != Cw or not w.is_contiguous():
        raise ValueError("filter tensor does not match the input")
    P, Q = out_extent(H, R, stride, pad), out_extent(W, S, stride, pad)
    if y is None:
        y = torch.empty((N, K, P, Q), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=x.device)
    dims = (N, C, H, W, K, R, S, stride, pad)
    return _run("conv_fwd", OP_FWD, x, w, y, dims, _batch_stride(x), _batch_stride(y), _io_dtype(x, y), ws, stream)


def conv_bwd_data(dy, w, H, W, stride, pad, dx=None, ws=None, stream=None, out_bf16=False):
    """dy [N,K,P,Q], w [K,C,R,S] -> dx [N,C,H,W] fp32 or bfloat16 (H, W: the layer's input extent)."""
    N = dy.shape[0]
    K, C, R, S = w.shape
    if dy.shape[1] != K or not w.is_contiguous():
        raise ValueError("filter tensor does not match the output gradient")
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=dy.device)
    dims = (N, C, H, W, K, R, S, stride, pad)
    return _run("conv_bwd_data", OP_BWD_DATA, dy, w, dx, dims, _batch_stride(dx), _batch_stride(dy),
                _io_dtype(dy, dx), ws, stream)


def _dense(*ts):
    for t in ts:
        if t is not None and not t.is_contiguous():
            raise ValueError("this call takes dense tensors")


def conv_fwd_bias_relu(x, w, bias, stride, pad, relu=True, y=None, ws=None, stream=None, out_bf16=False):
    """y = relu(conv_fwd(x, w) + bias[k]) in one call (bias: fp32 [K] or None; relu=False leaves the sum as it is)."""
    N, C, H, W = x.shape
    K, Cw, R, S = w.shape
    if C != Cw:
        raise ValueError("filter tensor does not match the input")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K):
        raise ValueError("bias must hold one fp32 value per filter")
    P, Q = out_extent(H, R, stride, pad), out_extent(W, S, stride, pad)
    if y is None:
        y = torch.empty((N, K, P, Q), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=x.device)
    _dense(x, w, bias, y)
    dims = (N, C, H, W, K, R, S, stride, pad)
    dtype = _io_dtype(x, y)
    buf, nbytes = _ws(ws).get(workspace_bytes(OP_FWD, *dims, dtype))
    wsp = ctypes.c_void_p(buf.data_ptr()) if buf is not None else ctypes.c_void_p(0)
    bp = _ptr(bias) if bias is not None else ctypes.c_void_p(0)
    rc = lib().conv_fwd_bias_relu(_ptr(x), _ptr(w), bp, _ptr(y), *dims, 1 if relu else 0, dtype, wsp, nbytes,
                                  _stream_handle(stream))
    if rc != OK:
        raise ConvError(rc, "conv_fwd_bias_relu")
    return y


def conv_bwd_data_relu(dy, w, act, stride, pad, dx=None, ws=None, stream=None):
    """dx = conv_bwd_data(dy, w) where act > 0, else 0 (act [N,C,H,W]: output or input of the ReLU that feeds this
    layer, element type of dx)."""
    N, C, H, W = act.shape
    K, Cw, R, S = w.shape
    if dy.shape[1] != K or Cw != C:
        raise ValueError("filter tensor does not match the tensors")
    if dx is None:
        dx = torch.empty_like(act)
    if dx.dtype != act.dtype or dx.shape != act.shape:
        raise ValueError("act must have the shape and element type of dx")
    _dense(dy, w, act, dx)
    dims = (N, C, H, W, K, R, S, stride, pad)
    dtype = _io_dtype(dy, dx)
    buf, nbytes = _ws(ws).get(workspace_bytes(OP_BWD_DATA, *dims, dtype))
    wsp = ctypes.c_void_p(buf.data_ptr()) if buf is not None else ctypes.c_void_p(0)
    rc = lib().conv_bwd_data_relu(_ptr(dy), _ptr(w), _ptr(act), _ptr(dx), *dims, dtype, wsp, nbytes,
                                  _stream_handle(stream))
    if rc != OK:
        raise ConvError(rc, "conv_bwd_data_relu")
    return dx


def conv_bwd_filter(x, dy, R, S, stride, pad, dw=None, ws=None, stream=None):
    """x [N,C,H,W], dy [N,K,P,Q] -> dw [K,C,R,S] fp32."""
    N, C, H, W = x.shape
    K = dy.shape[1]
    if dw is None:
        dw = torch.empty((K, C, R, S), dtype=torch.float32, device=x.device)
    dims = (N, C, H, W, K, R, S, stride, pad)
    return _run("conv_bwd_filter", OP_BWD_FILTER, x, dy, dw, dims, _batch_stride(x), _batch_stride(dy),
                _dtype_of(x), ws, stream)


def conv_bwd_filter_noalloc(x, dy, R, S, stride, pad, dw=None, stream=None):
    """conv_bwd_filter on dense tensors with the library's built-in scratch: no workspace argument.  `dw` must be
    given by callers that may not allocate (this wrapper allocates it only when it is None)."""
    N, C, H, W = x.shape
    K = dy.shape[1]
    _dense(x, dy, dw)
    if dw is None:
        dw = torch.empty((K, C, R, S), dtype=torch.float32, device=x.device)
    rc = lib().conv_bwd_filter_noalloc(_ptr(x), _ptr(dy), _ptr(dw), N, C, H, W, K, R, S, stride, pad, _dtype_of(x),
                                       _stream_handle(stream))
    if rc != OK:
        raise ConvError(rc, "conv_bwd_filter_noalloc")
    return dw


def _run_grouped(name, op, a, b, out, dims, groups, dtype, ws, stream):
    for t in (a, b, out):
        if not t.is_contiguous():
            raise ValueError("grouped calls take dense tensors")
    need = int(lib().conv_workspace_bytes_grouped(op, *dims, groups, dtype))
    buf, nbytes = _ws(ws).get(need)
    wsp = ctypes.c_void_p(buf.data_ptr()) if buf is not None else ctypes.c_void_p(0)
    rc = getattr(lib(), name)(_ptr(a), _ptr(b), _ptr(out), *dims, groups, dtype, wsp, nbytes, _stream_handle(stream))
    if rc != OK:
        raise ConvError(rc, name)
    return out


def conv_fwd_grouped(x, w, stride, pad, groups, y=None, ws=None, stream=None, out_bf16=False):
    """x [N,C,H,W], w [K,C/groups,R,S] -> y [N,K,P,Q]: column g's filters read column g's channels only."""
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    if Cg * groups != C or K % groups:
        raise ValueError("filter tensor does not match the input and the group count")
    P, Q = out_extent(H, R, stride, pad), out_extent(W, S, stride, pad)
    if y is None:
        y = torch.empty((N, K, P, Q), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=x.device)
    return _run_grouped("conv_fwd_grouped", OP_FWD, x, w, y, (N, C, H, W, K, R, S, stride, pad), groups,
                        _io_dtype(x, y), ws, stream)


def conv_bwd_data_grouped(dy, w, H, W, stride, pad, groups, dx=None, ws=None, stream=None, out_bf16=False):
    N = dy.shape[0]
    K, Cg, R, S = w.shape
    C = Cg * groups
    if dy.shape[1] != K or K % groups:
        raise ValueError("filter tensor does not match the output gradient and the group count")
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=dy.device)
    return _run_grouped("conv_bwd_data_grouped", OP_BWD_DATA, dy, w, dx, (N, C, H, W, K, R, S, stride, pad), groups,
                        _io_dtype(dy, dx), ws, stream)


def conv_bwd_filter_grouped(x, dy, R, S, stride, pad, groups, dw=None, ws=None, stream=None):
    N, C, H, W = x.shape
    K = dy.shape[1]
    if C % groups or K % groups:
        raise ValueError("channel counts are not multiples of the group count")
    if dw is None:
        dw = torch.empty((K, C // groups, R, S), dtype=torch.float32, device=x.device)
    return _run_grouped("conv_bwd_filter_grouped", OP_BWD_FILTER, x, dy, dw, (N, C, H, W, K, R, S, stride, pad),
                        groups, _dtype_of(x), ws, stream)


def _check(rc, where):
    if rc != OK:
        raise ConvError(rc, where)


def _glue_dtype(*tensors):
    """All tensors of a glue call share one element type (fp32 or bfloat16)."""
    d = _dtype_of(tensors[0])
    for t in tensors[1:]:
        if t.dtype != tensors[0].dtype:
            raise TypeError("the tensors of a glue call must have one dtype")
    return d


def relu_fwd(x, y=None, stream=None):
    if y is None:
        y = torch.empty_like(x)
    _check(lib().relu_fwd(_ptr(x), _ptr(y), x.numel(), _glue_dtype(x, y), _stream_handle(stream)), "relu_fwd")
    return y


def relu_bwd(x, dy, dx=None, stream=None):
    if dx is None:
        dx = torch.empty_like(dy)
    _check(lib().relu_bwd(_ptr(x), _ptr(dy), _ptr(dx), x.numel(), _glue_dtype(x, dy, dx), _stream_handle(stream)),
           "relu_bwd")
    return dx


def _pool_fwd(name, x, y, stream):
    N, C, H, W = x.shape
    if y is None:
        y = torch.empty((N, C, (H - 3) // 2 + 1, (W - 3) // 2 + 1), dtype=x.dtype, device=x.device)
    _check(getattr(lib(), name)(_ptr(x), _ptr(y), N * C, H, W, _glue_dtype(x, y), _stream_handle(stream)), name)
    return y


def _pool_bwd(name, x, dy, dx, stream):
    N, C, H, W = x.shape
    if dx is None:
        dx = torch.empty_like(x)
    _check(getattr(lib(), name)(_ptr(x), _ptr(dy), _ptr(dx), N * C, H, W, _glue_dtype(x, dy, dx),
                                _stream_handle(stream)), name)
    return dx


def maxpool3x3s2_fwd(x, y=None, stream=None):
    return _pool_fwd("maxpool3x3s2_fwd", x, y, stream)


def maxpool3x3s2_bwd(x, dy, dx=None, stream=None):
    return _pool_bwd("maxpool3x3s2_bwd", x, dy, dx, stream)


def relu_maxpool3x3s2_fwd(x, y=None, stream=None):
    return _pool_fwd("relu_maxpool3x3s2_fwd", x, y, stream)


def relu_maxpool3x3s2_bwd(x, dy, dx=None, stream=None):
    return _pool_bwd("relu_maxpool3x3s2_bwd", x, dy, dx, stream)


def bias_fwd(y, b, stream=None):
    """y [N,K,P,Q] += b[k] in place (b fp32)."""
    N, K, P, Q = y.shape
    if not y.is_contiguous() or b.dtype != torch.float32 or b.numel() != K:
        raise ValueError("bias_fwd takes a dense y and one fp32 value per filter")
    _check(lib().bias_fwd(_ptr(y), _ptr(b), N, K, P * Q, _dtype_of(y), _stream_handle(stream)), "bias_fwd")
    return y


def bias_bwd(dy, db=None, ws=None, stream=None):
    """db[k] = sum of dy [N,K,P,Q] over samples and positions, fp32."""
    N, K, P, Q = dy.shape
    if not dy.is_contiguous():
        raise ValueError("bias_bwd takes a dense dy")
    if db is None:
        db = torch.empty((K,), dtype=torch.float32, device=dy.device)
    buf, nbytes = _ws(ws).get(int(lib().bias_bwd_workspace_bytes(N, K)))
    _check(lib().bias_bwd(_ptr(dy), _ptr(db), N, K, P * Q, _dtype_of(dy), ctypes.c_void_p(buf.data_ptr()), nbytes,
                          _stream_handle(stream)), "bias_bwd")
    return db


def convert_f32_to_bf16(src, dst=None, stream=None):
    """Round an fp32 tensor to bfloat16 (nearest even) into `dst` (same shape, contiguous)."""
    if dst is None:
        dst = torch.empty(src.shape, dtype=torch.bfloat16, device=src.device)
    if not src.is_contiguous() or not dst.is_contiguous():
        raise ValueError("convert_f32_to_bf16 needs contiguous tensors")
    _check(lib().convert_f32_to_bf16(_ptr(src), _ptr(dst), src.numel(), _stream_handle(stream)), "convert_f32_to_bf16")
    return dst


def _fc_ws(op, N, I, O, ws):
    buf, nbytes = _ws(ws).get(int(lib().fc_workspace_bytes(op, N, I, O, DTYPE_F32)))
    return (ctypes.c_void_p(buf.data_ptr()) if buf is not None else ctypes.c_void_p(0)), nbytes


def fc_fwd(x, w, bias=None, relu=False, y=None, ws=None, stream=None):
    """x [N,I], w [O,I] (fp32) -> y [N,O] = f(x w^T + bias)."""
    N, I = x.shape
    O, Iw = w.shape
    if I != Iw or (bias is not None and (bias.dtype != torch.float32 or bias.numel() != O)):
        raise ValueError("operands do not match")
    if y is None:
        y = torch.empty((N, O), dtype=torch.float32, device=x.device)
    _dense(x, w, bias, y)
    wsp, nbytes = _fc_ws(OP_FWD, N, I, O, ws)
    bp = _ptr(bias) if bias is not None else ctypes.c_void_p(0)
    _check(lib().fc_fwd(_ptr(x), _ptr(w), bp, _ptr(y), N, I, O, 1 if relu else 0, _dtype_of(x), wsp, nbytes,
                        _stream_handle(stream)), "fc_fwd")
    return y


def fc_bwd_data(dy, w, dx=None, ws=None, stream=None):
    """dy [N,O], w [O,I] -> dx [N,I]."""
    N, O = dy.shape
    Ow, I = w.shape
    if O != Ow:
        raise ValueError("operands do not match")
    if dx is None:
        dx = torch.empty((N, I), dtype=torch.float32, device=dy.device)
    _dense(dy, w, dx)
    wsp, nbytes = _fc_ws(OP_BWD_DATA, N, I, O, ws)
    _check(lib().fc_bwd_data(_ptr(dy), _ptr(w), _ptr(dx), N, I, O, _dtype_of(dy), wsp, nbytes,
                             _stream_handle(stream)), "fc_bwd_data")
    return dx


def fc_bwd_filter(x, dy, dw=None, ws=None, stream=None):
    """x [N,I], dy [N,O] -> dw [O,I]."""
    N, I = x.shape
    Ny, O = dy.shape
    if N != Ny:
        raise ValueError("operands do not match")
    if dw is None:
        dw = torch.empty((O, I), dtype=torch.float32, device=x.device)
    _dense(x, dy, dw)
    wsp, nbytes = _fc_ws(OP_BWD_FILTER, N, I, O, ws)
    _check(lib().fc_bwd_filter(_ptr(x), _ptr(dy), _ptr(dw), N, I, O, _dtype_of(x), wsp, nbytes,
                               _stream_handle(stream)), "fc_bwd_filter")
    return dw


def sgd_update(w, dw, vel, lr, momentum=0.0, weight_decay=0.0, grad_scale=1.0, stream=None):
    """In place: vel = momentum*vel - lr*(weight_decay*w + grad_scale*dw); w += vel (fp32 tensors of one size)."""
    if not (w.dtype == dw.dtype == vel.dtype == torch.float32) or not (w.numel() == dw.numel() == vel.numel()):
        raise ValueError("sgd_update takes three fp32 tensors of one size")
    _dense(w, dw, vel)
    _check(lib().sgd_update(_ptr(w), _ptr(dw), _ptr(vel), w.numel(), lr, momentum, weight_decay, grad_scale,
                            _stream_handle(stream)), "sgd_update")
    return w


def sgd_update_multi(ws, dws, vels, lr, momentum=0.0, weight_decay=0.0, grad_scale=1.0, stream=None):
    """sgd_update for lists of tensors in one call (one launch per 24 tensors)."""
    n = len(ws)
    if not (len(dws) == len(vels) == n):
        raise ValueError("sgd_update_multi takes three lists of one length")
    for w, dw, vel in zip(ws, dws, vels):
        if not (w.dtype == dw.dtype == vel.dtype == torch.float32) or not (w.numel() == dw.numel() == vel.numel()):
            raise ValueError("sgd_update_multi takes fp32 tensors, each triple of one size")
        _dense(w, dw, vel)
    ptrs = lambda ts: (ctypes.c_void_p * n)(*[t.data_ptr() for t in ts])
    counts = (ctypes.c_int64 * n)(*[w.numel() for w in ws])
    _check(lib().sgd_update_multi(ptrs(ws), ptrs(dws), ptrs(vels), counts, n, lr, momentum, weight_decay, grad_scale,
                                  _stream_handle(stream)), "sgd_update_multi")
    return ws
