"""Thin Python binding of libswitchback (include/switchback.h): argument marshalling only.

torch is used for device memory and the current HIP stream; every step of the layer runs in the library's HIP
kernels.  There is no CPU or eager fallback: if the built library or the GPU is missing, the calls raise.

Names follow the C ABI: quantize_rowwise, quantize_tensorwise, matmul_int8_dequant, forward, backward_input,
backward_weight (Algorithm 1 of arxiv 2304.13013: X [b,n], W [m,n], Y/dY [b,m]).
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswitchback.so")

SB_BF16, SB_F32, SB_I32_RAW = 0, 1, 2
SB_OP_QUANTIZE_TENSORWISE, SB_OP_FORWARD, SB_OP_BACKWARD_INPUT, SB_OP_BACKWARD_WEIGHT, SB_OP_QUANTIZE_COLWISE = 0, 1, 2, 3, 4
SB_OP_STABLE_ADAMW = 5
SB_E4M3, SB_E5M2 = 0, 1

_TORCH_DTYPE = {SB_BF16: torch.bfloat16, SB_F32: torch.float32, SB_I32_RAW: torch.int32}
_SB_DTYPE = {v: k for k, v in _TORCH_DTYPE.items()}


class SbSaved(ctypes.Structure):
    _fields_ = [("xq", ctypes.c_void_p), ("state_x", ctypes.c_void_p), ("wq", ctypes.c_void_p),
                ("wq_t", ctypes.c_void_p), ("state_w", ctypes.c_void_p)]


class SbAdamwTensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("v", ctypes.c_void_p), ("u", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("count", ctypes.c_int64), ("first_block", ctypes.c_int32), ("num_blocks", ctypes.c_int32)]


class SwitchBackError(RuntimeError):
    pass


_lib = None


def load_library():
    """dlopen the in-tree library and declare the C ABI.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise SwitchBackError("libswitchback.so is not built: run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` (or paper_2304_13013_amd/build.py) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
    lib.switchback_quantize_rowwise.argtypes = [vp, i64, i64, vp, vp, vp]
    lib.switchback_quantize_tensorwise.argtypes = [vp, i64, i64, vp, vp, vp, vp, sz, vp]
    lib.switchback_matmul_int8_dequant.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, ci, vp]
    lib.switchback_forward.argtypes = [vp, vp, i64, i64, i64, vp, ci, ctypes.POINTER(SbSaved), vp, sz, vp]
    lib.switchback_matmul_int8_dequant_bias_layerscale.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, ci, vp]
    lib.switchback_forward_bias_layerscale.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, ci, ctypes.POINTER(SbSaved),
                                                       vp, sz, vp]
    lib.switchback_forward_static.argtypes = [vp, vp, i64, i64, i64, vp, ci, ctypes.POINTER(SbSaved), vp]
    lib.switchback_backward_input.argtypes = [vp, ctypes.POINTER(SbSaved), i64, i64, i64, vp, ci, vp, vp, vp]
    lib.switchback_backward_weight.argtypes = [vp, vp, i64, i64, i64, vp, ci, vp, sz, vp]
    lib.switchback_dequantize_rowwise.argtypes = [vp, vp, i64, i64, vp, vp]
    lib.switchback_backward_weight_m.argtypes = [vp, ctypes.POINTER(SbSaved), i64, i64, i64, vp, vp, ci, vp, sz, vp]
    lib.switchback_quantize_colwise_transpose.argtypes = [vp, i64, i64, vp, vp, vp, sz, vp]
    lib.switchback_matmul_int8_dequant_rc.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, ci, vp]
    lib.switchback_forward_q.argtypes = [vp, vp, i64, i64, i64, vp, ci, vp, vp, vp, vp, vp]
    lib.switchback_backward_input_q.argtypes = [vp, vp, i64, i64, i64, vp, ci, vp, vp, vp, vp, vp, sz, vp]
    cf = ctypes.c_float
    lib.switchback_quantize_rowwise_f8.argtypes = [vp, i64, i64, ci, vp, vp, vp]
    lib.switchback_quantize_tensorwise_f8.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp, sz, vp]
    lib.switchback_matmul_f8_dequant.argtypes = [vp, ci, vp, vp, ci, vp, i64, i64, i64, vp, ci, vp]
    lib.switchback_forward_f8.argtypes = [vp, vp, i64, i64, i64, vp, ci, ctypes.POINTER(SbSaved), ci, ci, vp, sz, vp]
    lib.switchback_backward_input_f8.argtypes = [vp, ctypes.POINTER(SbSaved), i64, i64, i64, vp, ci, vp, vp, ci, ci, vp]
    lib.switchback_stable_adamw_step.argtypes = [vp, vp, vp, vp, ci, i64, cf, cf, cf, cf, cf, i64, vp, vp, sz, vp]
    lib.switchback_stable_adamw_plan.argtypes = [ctypes.POINTER(SbAdamwTensor), ci]
    lib.switchback_stable_adamw_plan.restype = i64
    lib.switchback_stable_adamw_step_multi.argtypes = [vp, ci, i64, ci, cf, cf, cf, cf, cf, i64, vp, vp, sz, vp]
    lib.switchback_stable_adamw_step_multi.restype = ci
    lib.switchback_ceiling_mfma.argtypes = [ci, vp, sz, vp, sz, ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.switchback_ceiling_mfma.restype = ci
    lib.switchback_ceiling_copy.argtypes = [vp, vp, sz, vp]
    lib.switchback_ceiling_copy.restype = ci
    lib.switchback_workspace_bytes.argtypes = [ci, i64, i64, i64]
    lib.switchback_workspace_bytes.restype = sz
    lib.switchback_status_string.argtypes = [ci]
    lib.switchback_status_string.restype = ctypes.c_char_p
    for name in ("switchback_quantize_rowwise", "switchback_quantize_tensorwise", "switchback_matmul_int8_dequant",
                 "switchback_forward", "switchback_forward_static", "switchback_backward_input",
                 "switchback_matmul_int8_dequant_bias_layerscale", "switchback_forward_bias_layerscale", "switchback_backward_weight",
                 "switchback_dequantize_rowwise", "switchback_backward_weight_m",
                 "switchback_quantize_colwise_transpose", "switchback_matmul_int8_dequant_rc",
                 "switchback_forward_q", "switchback_backward_input_q", "switchback_stable_adamw_step",
                 "switchback_quantize_rowwise_f8", "switchback_quantize_tensorwise_f8", "switchback_matmul_f8_dequant",
                 "switchback_forward_f8", "switchback_backward_input_f8"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise SwitchBackError("libswitchback: %s (status %d)"
                              % (load_library().switchback_status_string(status).decode(), status))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, ndim=None):
    if not t.is_cuda:
        raise SwitchBackError("tensors must live on the GPU")
    if t.dtype != dtype or not t.is_contiguous() or (ndim is not None and t.dim() != ndim):
        raise SwitchBackError("expected a contiguous %d-d %s tensor, got %s %s"
                              % (ndim or t.dim(), dtype, tuple(t.shape), t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else None)


def _out(t, shape, dtype, device, name):
    """A fresh output tensor, or the caller's after checking that it has exactly the shape the kernels will write."""
    if t is None:
        return torch.empty(tuple(shape), dtype=dtype, device=device)
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype:
        raise SwitchBackError("%s must be a %s tensor of shape %s, got %s %s"
                              % (name, dtype, tuple(shape), t.dtype, tuple(t.shape)))
    return t


def _check_bufs(bufs, b, n, m):
    """The layer buffers were allocated for one (b, n, m); the kernels write b*n, b*m and m*n codes into them."""
    if (bufs.b, bufs.n, bufs.m) != (b, n, m):
        raise SwitchBackError("layer buffers were allocated for (b, n, m) = %s, the call has %s"
                              % ((bufs.b, bufs.n, bufs.m), (b, n, m)))


def _check_ws(ws, need, name="workspace"):
    if ws.numel() * ws.element_size() < need:
        raise SwitchBackError("%s holds %d bytes, the call needs %d" % (name, ws.numel() * ws.element_size(), need))


def workspace_bytes(op, b, n, m):
    return int(load_library().switchback_workspace_bytes(op, b, n, m))


def _workspace(op, b, n, m, device):
    # Never zero-sized, so that the pointer is a valid aligned device address.
    return torch.empty(max(workspace_bytes(op, b, n, m), 16), dtype=torch.uint8, device=device)


def quantize_rowwise(x, q=None, state=None):
    """Q_row(x), state_row(x) for a bf16 [rows, cols] tensor -> (int8 [rows, cols], f32 [rows])."""
    lib = load_library()
    rows, cols = x.shape
    q = _out(q, (rows, cols), torch.int8, x.device, "q")
    state = _out(state, (rows,), torch.float32, x.device, "state")
    xp = _dev(x, torch.bfloat16, 2)
    _check(lib.switchback_quantize_rowwise(xp, rows, cols, _dev(q, torch.int8), _dev(state, torch.float32),
                                           _stream()))
    return q, state


def dequantize_rowwise(q, state, out=None):
    """Row-wise dequantization of SwitchBackM: bf16 [rows, cols] = q * state / 127."""
    lib = load_library()
    rows, cols = q.shape
    out = _out(out, (rows, cols), torch.bfloat16, q.device, "out")
    _out(state, (rows,), torch.float32, q.device, "state")
    _check(lib.switchback_dequantize_rowwise(_dev(q, torch.int8, 2), _dev(state, torch.float32), rows, cols,
                                             _dev(out, torch.bfloat16, 2), _stream()))
    return out


def quantize_tensorwise(w, q=None, q_t=None, state=None, ws=None, transpose=True):
    """Q_tensor(w), Q_tensor(w)^T, state_tensor(w) for a bf16 [rows, cols] tensor."""
    lib = load_library()
    rows, cols = w.shape
    q = _out(q, (rows, cols), torch.int8, w.device, "q")
    if transpose or q_t is not None:
        q_t = _out(q_t, (cols, rows), torch.int8, w.device, "q_t")
    state = _out(state, (1,), torch.float32, w.device, "state")
    wp = _dev(w, torch.bfloat16, 2)
    ws = _workspace(SB_OP_QUANTIZE_TENSORWISE, 0, cols, rows, w.device) if ws is None else ws
    _check(lib.switchback_quantize_tensorwise(wp, rows, cols, _dev(q, torch.int8),
                                              _dev(q_t, torch.int8) if q_t is not None else None,
                                              _dev(state, torch.float32), _ptr(ws), ws.numel(), _stream()))
    return q, q_t, state


def matmul_int8_dequant(aq, state_row, bq, state_tensor, out_dtype=torch.bfloat16, out=None):
    """out[i,j] = state_tensor/127^2 * state_row[i] * sum_k aq[i,k] bq[j,k]; int32 accumulators if out_dtype is
    torch.int32 (the states may then be None)."""
    lib = load_library()
    M, K = aq.shape
    N = bq.shape[0]
    if bq.shape[1] != K:
        raise SwitchBackError("contraction lengths differ")
    out = _out(out, (M, N), out_dtype, aq.device, "out")
    if state_row is not None:
        _out(state_row, (M,), torch.float32, aq.device, "state_row")
    _check(lib.switchback_matmul_int8_dequant(
        _dev(aq, torch.int8, 2), _dev(state_row, torch.float32) if state_row is not None else None,
        _dev(bq, torch.int8, 2), _dev(state_tensor, torch.float32) if state_tensor is not None else None,
        M, N, K, _dev(out, out_dtype, 2), _SB_DTYPE[out_dtype], _stream()))
    return out


class LayerBuffers:
    """Device buffers of one SwitchBack layer of shape (b, n, m), allocated once: what forward saves for
    backward (int8 codes and states), the quantized dY, and the workspaces."""

    def __init__(self, b, n, m, device="cuda"):
        self.b, self.n, self.m = b, n, m
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        self.xq, self.state_x = e((b, n), torch.int8), e((b,), torch.float32)
        self.wq, self.wq_t, self.state_w = e((m, n), torch.int8), e((n, m), torch.int8), e((1,), torch.float32)
        self.gq, self.state_g = e((b, m), torch.int8), e((b,), torch.float32)
        self.ws_fwd = _workspace(SB_OP_FORWARD, b, n, m, device)
        self.ws_dw = _workspace(SB_OP_BACKWARD_WEIGHT, b, n, m, device)
        self.saved = SbSaved(self.xq.data_ptr(), self.state_x.data_ptr(), self.wq.data_ptr(),
                             self.wq_t.data_ptr(), self.state_w.data_ptr())


def forward(x, w, bufs=None, y=None, y_dtype=torch.bfloat16):
    """Algorithm 1 forward.  Returns (y [b,m], bufs); bufs holds xq, state_x, wq, wq_t, state_w."""
    lib = load_library()
    b, n = x.shape
    m = w.shape[0]
    if w.shape[1] != n:
        raise SwitchBackError("x [b,n] and w [m,n] disagree on n")
    bufs = LayerBuffers(b, n, m, x.device) if bufs is None else bufs
    _check_bufs(bufs, b, n, m)
    y = _out(y, (b, m), y_dtype, x.device, "y")
    _check(lib.switchback_forward(_dev(x, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), b, n, m,
                                  _dev(y, y_dtype, 2), _SB_DTYPE[y_dtype], ctypes.byref(bufs.saved),
                                  _ptr(bufs.ws_fwd), bufs.ws_fwd.numel(), _stream()))
    return y, bufs


def _vec(v, n, device, name):
    """An optional f32 [n] device vector -> pointer (None -> NULL)."""
    if v is None:
        return None
    _out(v, (n,), torch.float32, device, name)
    return _dev(v, torch.float32, 1)


def matmul_int8_dequant_bias_layerscale(aq, state_row, bq, state_tensor, bias=None, gamma=None,
                                        out_dtype=torch.bfloat16, out=None):
    """out[i,j] = gamma[j] * (state_tensor/127^2 * state_row[i] * sum_k aq[i,k] bq[j,k] + bias[j]); bias, gamma f32 [N]
    or None."""
    lib = load_library()
    M, K = aq.shape
    N = bq.shape[0]
    if bq.shape[1] != K:
        raise SwitchBackError("contraction lengths differ")
    out = _out(out, (M, N), out_dtype, aq.device, "out")
    _out(state_row, (M,), torch.float32, aq.device, "state_row")
    _check(lib.switchback_matmul_int8_dequant_bias_layerscale(
        _dev(aq, torch.int8, 2), _dev(state_row, torch.float32), _dev(bq, torch.int8, 2),
        _dev(state_tensor, torch.float32), _vec(bias, N, aq.device, "bias"), _vec(gamma, N, aq.device, "gamma"),
        M, N, K, _dev(out, out_dtype, 2), _SB_DTYPE[out_dtype], _stream()))
    return out


def forward_bias_layerscale(x, w, bias=None, gamma=None, bufs=None, y=None, y_dtype=torch.bfloat16):
    """Algorithm 1 forward with the layer's bias and the block's layer-scale in the epilogue: gamma * (X W^T + bias)."""
    lib = load_library()
    b, n = x.shape
    m = w.shape[0]
    if w.shape[1] != n:
        raise SwitchBackError("x [b,n] and w [m,n] disagree on n")
    bufs = LayerBuffers(b, n, m, x.device) if bufs is None else bufs
    _check_bufs(bufs, b, n, m)
    y = _out(y, (b, m), y_dtype, x.device, "y")
    _check(lib.switchback_forward_bias_layerscale(
        _dev(x, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), _vec(bias, m, x.device, "bias"),
        _vec(gamma, m, x.device, "gamma"), b, n, m, _dev(y, y_dtype, 2), _SB_DTYPE[y_dtype], ctypes.byref(bufs.saved),
        _ptr(bufs.ws_fwd), bufs.ws_fwd.numel(), _stream()))
    return y, bufs


def forward_static(x, w, bufs, y=None, y_dtype=torch.bfloat16):
    """switchback_forward_static: Algorithm 1 forward without a workspace (the library's own per-GPU scratch array
    holds the tensor-wise partial maxima); the call itself allocates nothing when bufs and y are given."""
    lib = load_library()
    b, n = x.shape
    m = w.shape[0]
    if w.shape[1] != n:
        raise SwitchBackError("x [b,n] and w [m,n] disagree on n")
    _check_bufs(bufs, b, n, m)
    y = _out(y, (b, m), y_dtype, x.device, "y")
    _check(lib.switchback_forward_static(_dev(x, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), b, n, m,
                                         _dev(y, y_dtype, 2), _SB_DTYPE[y_dtype], ctypes.byref(bufs.saved), _stream()))
    return y, bufs


def backward_input(dy, bufs, dx=None, dx_dtype=torch.bfloat16):
    """Algorithm 1 input gradient.  Returns dx [b,n]; fills bufs.gq and bufs.state_g."""
    lib = load_library()
    b, m = dy.shape
    n = bufs.n
    _check_bufs(bufs, b, n, m)
    dx = _out(dx, (b, n), dx_dtype, dy.device, "dx")
    _check(lib.switchback_backward_input(_dev(dy, torch.bfloat16, 2), ctypes.byref(bufs.saved), b, n, m,
                                         _dev(dx, dx_dtype, 2), _SB_DTYPE[dx_dtype], _ptr(bufs.gq),
                                         _ptr(bufs.state_g), _stream()))
    return dx


def backward_weight(dy, x, bufs=None, dw=None, dw_dtype=torch.bfloat16):
    """Algorithm 1 weight gradient dW = dY^T X (bf16 operands, binary32 accumulation).  Returns dw [m,n]."""
    lib = load_library()
    b, m = dy.shape
    n = x.shape[1]
    if x.shape[0] != b:
        raise SwitchBackError("dy [b,m] and x [b,n] disagree on b")
    if bufs is not None:
        _check_bufs(bufs, b, n, m)
    ws = bufs.ws_dw if bufs is not None else _workspace(SB_OP_BACKWARD_WEIGHT, b, n, m, dy.device)
    dw = _out(dw, (m, n), dw_dtype, dy.device, "dw")
    _check(lib.switchback_backward_weight(_dev(dy, torch.bfloat16, 2), _dev(x, torch.bfloat16, 2), b, n, m,
                                          _dev(dw, dw_dtype, 2), _SB_DTYPE[dw_dtype], _ptr(ws), ws.numel(),
                                          _stream()))
    return dw


def backward_weight_m(dy, bufs, x_hat=None, dw=None, dw_dtype=torch.bfloat16):
    """SwitchBackM weight gradient: X is rebuilt from bufs.xq / bufs.state_x (filled by forward) into x_hat, then
    dW = dY^T X^.  Returns (dw [m,n], x_hat [b,n])."""
    lib = load_library()
    b, m = dy.shape
    n = bufs.n
    _check_bufs(bufs, b, n, m)
    x_hat = _out(x_hat, (b, n), torch.bfloat16, dy.device, "x_hat")
    dw = _out(dw, (m, n), dw_dtype, dy.device, "dw")
    _check(lib.switchback_backward_weight_m(_dev(dy, torch.bfloat16, 2), ctypes.byref(bufs.saved), b, n, m,
                                            _dev(x_hat, torch.bfloat16, 2), _dev(dw, dw_dtype, 2),
                                            _SB_DTYPE[dw_dtype], _ptr(bufs.ws_dw), bufs.ws_dw.numel(), _stream()))
    return dw, x_hat


# ---- SwitchBackQ: row-wise / column-wise weight quantization ---------------------------------------------------

def quantize_colwise_transpose(w, q_t=None, state=None, ws=None):
    """One absmax per column of w [rows, cols]; returns (q_t int8 [cols, rows], state f32 [cols])."""
    lib = load_library()
    rows, cols = w.shape
    q_t = _out(q_t, (cols, rows), torch.int8, w.device, "q_t")
    state = _out(state, (cols,), torch.float32, w.device, "state")
    ws = _workspace(SB_OP_QUANTIZE_COLWISE, 0, cols, rows, w.device) if ws is None else ws
    _check(lib.switchback_quantize_colwise_transpose(_dev(w, torch.bfloat16, 2), rows, cols, _dev(q_t, torch.int8, 2),
                                                     _dev(state, torch.float32), _ptr(ws), ws.numel(), _stream()))
    return q_t, state


def matmul_int8_dequant_rc(aq, state_a, bq, state_b, out_dtype=torch.bfloat16, out=None):
    """out[i,j] = state_a[i] * state_b[j] / 127^2 * sum_k aq[i,k] bq[j,k]."""
    lib = load_library()
    M, K = aq.shape
    N = bq.shape[0]
    if bq.shape[1] != K:
        raise SwitchBackError("contraction lengths differ")
    out = _out(out, (M, N), out_dtype, aq.device, "out")
    _out(state_a, (M,), torch.float32, aq.device, "state_a")
    _out(state_b, (N,), torch.float32, aq.device, "state_b")
    _check(lib.switchback_matmul_int8_dequant_rc(_dev(aq, torch.int8, 2), _dev(state_a, torch.float32),
                                                 _dev(bq, torch.int8, 2), _dev(state_b, torch.float32), M, N, K,
                                                 _dev(out, out_dtype, 2), _SB_DTYPE[out_dtype], _stream()))
    return out


class LayerBuffersQ:
    """Device buffers of one SwitchBackQ layer of shape (b, n, m): codes and states of both passes."""

    def __init__(self, b, n, m, device="cuda"):
        self.b, self.n, self.m = b, n, m
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        self.xq, self.state_x = e((b, n), torch.int8), e((b,), torch.float32)
        self.wq, self.state_w_row = e((m, n), torch.int8), e((m,), torch.float32)
        self.gq, self.state_g = e((b, m), torch.int8), e((b,), torch.float32)
        self.wq_t, self.state_w_col = e((n, m), torch.int8), e((n,), torch.float32)
        self.ws = _workspace(SB_OP_QUANTIZE_COLWISE, 0, n, m, device)


def forward_q(x, w, bufs=None, y=None, y_dtype=torch.bfloat16):
    """SwitchBackQ forward.  Returns (y [b,m], bufs)."""
    lib = load_library()
    b, n = x.shape
    m = w.shape[0]
    if w.shape[1] != n:
        raise SwitchBackError("x [b,n] and w [m,n] disagree on n")
    bufs = LayerBuffersQ(b, n, m, x.device) if bufs is None else bufs
    _check_bufs(bufs, b, n, m)
    y = _out(y, (b, m), y_dtype, x.device, "y")
    _check(lib.switchback_forward_q(_dev(x, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), b, n, m,
                                    _dev(y, y_dtype, 2), _SB_DTYPE[y_dtype], _ptr(bufs.xq), _ptr(bufs.state_x),
                                    _ptr(bufs.wq), _ptr(bufs.state_w_row), _stream()))
    return y, bufs


def backward_input_q(dy, w, bufs, dx=None, dx_dtype=torch.bfloat16):
    """SwitchBackQ input gradient.  Returns dx [b,n]; fills bufs.gq, state_g, wq_t, state_w_col."""
    lib = load_library()
    b, m = dy.shape
    n = w.shape[1]
    if w.shape[0] != m:
        raise SwitchBackError("dy [b,m] and w [m,n] disagree on m")
    _check_bufs(bufs, b, n, m)
    dx = _out(dx, (b, n), dx_dtype, dy.device, "dx")
    _check(lib.switchback_backward_input_q(_dev(dy, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), b, n, m,
                                           _dev(dx, dx_dtype, 2), _SB_DTYPE[dx_dtype], _ptr(bufs.gq),
                                           _ptr(bufs.state_g), _ptr(bufs.wq_t), _ptr(bufs.state_w_col),
                                           _ptr(bufs.ws), bufs.ws.numel(), _stream()))
    return dx


def stable_adamw_step(theta, v, u, grad, alpha, beta1, beta2, eps, lam, t, rms_out=None, ws=None):
    """One StableAdamW step for one tensor, in place on theta, v, u (f32, any shape, contiguous); grad bf16 or f32.
    Returns rms_out (a 1-element f32 device tensor holding RMS_t)."""
    lib = load_library()
    count = theta.numel()
    for name, x in (("theta", theta), ("v", v), ("u", u)):
        _dev(x, torch.float32)
        if x.numel() != count:
            raise SwitchBackError("%s has %d elements, expected %d" % (name, x.numel(), count))
    if grad.dtype not in (torch.bfloat16, torch.float32) or grad.numel() != count:
        raise SwitchBackError("grad must be bf16 or f32 with as many elements as theta")
    rms_out = torch.empty(1, dtype=torch.float32, device=theta.device) if rms_out is None else rms_out
    ws = _workspace(SB_OP_STABLE_ADAMW, 0, 0, 0, theta.device) if ws is None else ws
    _check(lib.switchback_stable_adamw_step(_ptr(theta), _ptr(v), _ptr(u), _dev(grad, grad.dtype),
                                            _SB_DTYPE[grad.dtype], count, alpha, beta1, beta2, eps, lam, t,
                                            _ptr(rms_out), _ptr(ws), ws.numel(), _stream()))
    return rms_out


# ---- float8 SwitchBack: the same layer with float8cast(x / absmax) as the quantizer; codes are uint8 tensors ------

def quantize_rowwise_f8(x, fmt, codes=None, state=None):
    lib = load_library()
    rows, cols = x.shape
    codes = _out(codes, (rows, cols), torch.uint8, x.device, "codes")
    state = _out(state, (rows,), torch.float32, x.device, "state")
    xp = _dev(x, torch.bfloat16, 2)
    _check(lib.switchback_quantize_rowwise_f8(xp, rows, cols, fmt, _ptr(codes), _ptr(state), _stream()))
    return codes, state


def quantize_tensorwise_f8(w, fmt, codes=None, codes_t=None, state=None, ws=None):
    lib = load_library()
    rows, cols = w.shape
    codes = _out(codes, (rows, cols), torch.uint8, w.device, "codes")
    codes_t = _out(codes_t, (cols, rows), torch.uint8, w.device, "codes_t")
    state = _out(state, (1,), torch.float32, w.device, "state")
    wp = _dev(w, torch.bfloat16, 2)
    ws = _workspace(SB_OP_QUANTIZE_TENSORWISE, 0, cols, rows, w.device) if ws is None else ws
    _check(lib.switchback_quantize_tensorwise_f8(wp, rows, cols, fmt, _ptr(codes), _ptr(codes_t), _ptr(state),
                                                 _ptr(ws), ws.numel(), _stream()))
    return codes, codes_t, state


def matmul_f8_dequant(aq, fmt_a, state_row, bq, fmt_b, state_tensor, out=None, out_dtype=torch.bfloat16):
    lib = load_library()
    M, K = aq.shape
    N = bq.shape[0]
    if bq.shape[1] != K:
        raise SwitchBackError("aq [M,K] and bq [N,K] disagree on K")
    out = torch.empty((M, N), dtype=out_dtype, device=aq.device) if out is None else _out(out, (M, N), out.dtype,
                                                                                              aq.device, "out")
    _out(state_row, (M,), torch.float32, aq.device, "state_row")
    _check(lib.switchback_matmul_f8_dequant(_dev(aq, torch.uint8, 2), fmt_a, _ptr(state_row), _dev(bq, torch.uint8, 2),
                                            fmt_b, _ptr(state_tensor), M, N, K, _dev(out, out.dtype, 2),
                                            _SB_DTYPE[out.dtype], _stream()))
    return out


def forward_f8(x, w, bufs=None, y=None, y_dtype=torch.bfloat16, fmt_x=SB_E4M3, fmt_w=SB_E4M3):
    """float8 SwitchBack forward.  Returns (y [b,m], bufs); bufs (a LayerBuffers) then holds float8 bytes."""
    lib = load_library()
    b, n = x.shape
    m = w.shape[0]
    if w.shape[1] != n:
        raise SwitchBackError("x [b,n] and w [m,n] disagree on n")
    bufs = LayerBuffers(b, n, m, x.device) if bufs is None else bufs
    _check_bufs(bufs, b, n, m)
    y = _out(y, (b, m), y_dtype, x.device, "y")
    _check(lib.switchback_forward_f8(_dev(x, torch.bfloat16, 2), _dev(w, torch.bfloat16, 2), b, n, m,
                                     _dev(y, y_dtype, 2), _SB_DTYPE[y_dtype], ctypes.byref(bufs.saved), fmt_x, fmt_w,
                                     _ptr(bufs.ws_fwd), bufs.ws_fwd.numel(), _stream()))
    return y, bufs


def backward_input_f8(dy, bufs, dx=None, dx_dtype=torch.bfloat16, fmt_g=SB_E5M2, fmt_w=SB_E4M3):
    """float8 SwitchBack input gradient.  Returns dx [b,n]; fills bufs.gq (float8 bytes) and bufs.state_g."""
    lib = load_library()
    b, m = dy.shape
    n = bufs.n
    _check_bufs(bufs, b, n, m)
    dx = _out(dx, (b, n), dx_dtype, dy.device, "dx")
    _check(lib.switchback_backward_input_f8(_dev(dy, torch.bfloat16, 2), ctypes.byref(bufs.saved), b, n, m,
                                            _dev(dx, dx_dtype, 2), _SB_DTYPE[dx_dtype], _ptr(bufs.gq),
                                            _ptr(bufs.state_g), fmt_g, fmt_w, _stream()))
    return dx


# ---- measured ceilings (include/switchback_ceilings.h): measurement aids of the benchmark, not part of the layer -----

SB_CEILING_I8, SB_CEILING_BF16, SB_CEILING_F8 = 0, 1, 2


def ceiling_mfma(kind, a_codes, b_codes, workgroups, waves_per_workgroup, iters, sink=None):
    """Enqueue the register-resident matrix-instruction loop on operand bytes taken from a_codes / b_codes (any dtype,
    contiguous).  Returns (operations performed, sink)."""
    lib = load_library()
    lanes = workgroups * waves_per_workgroup * 64
    sink = torch.empty(lanes, dtype=torch.float32, device=a_codes.device) if sink is None else sink
    if sink.numel() < lanes or sink.dtype != torch.float32:
        raise SwitchBackError("sink must hold one f32 per launched lane")
    for t in (a_codes, b_codes, sink):
        if not t.is_cuda or not t.is_contiguous():
            raise SwitchBackError("tensors must be contiguous and live on the GPU")
    ops = ctypes.c_double(0.0)
    _check(lib.switchback_ceiling_mfma(kind, _ptr(a_codes), a_codes.numel() * a_codes.element_size(), _ptr(b_codes),
                                       b_codes.numel() * b_codes.element_size(), workgroups, waves_per_workgroup,
                                       iters, _ptr(sink), ctypes.byref(ops), _stream()))
    return ops.value, sink


def ceiling_copy(src, dst):
    """Enqueue a plain device copy src -> dst (same byte count, a multiple of 16)."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise SwitchBackError("src and dst must be GPU tensors of the same byte count")
    _check(lib.switchback_ceiling_copy(_dev(src, src.dtype), _dev(dst, dst.dtype), nbytes, _stream()))


class AdamwPlan:
    """The device table of a batched StableAdamW step over a fixed list of (theta, v, u, grad) tensors: built once,
    valid while the tensors keep their storage."""

    def __init__(self, tensors):
        lib = load_library()
        self.tensors = [tuple(t) for t in tensors]           # keeps the storage alive
        n = len(self.tensors)
        if n == 0:
            raise SwitchBackError("an optimizer plan needs at least one tensor")
        dtypes = {g.dtype for (_, _, _, g) in self.tensors}
        if len(dtypes) != 1 or next(iter(dtypes)) not in (torch.bfloat16, torch.float32):
            raise SwitchBackError("all gradients of a plan must share one dtype, bf16 or f32")
        self.grad_dtype = next(iter(dtypes))
        table = (SbAdamwTensor * n)()
        for i, (theta, v, u, g) in enumerate(self.tensors):
            for x in (theta, v, u):
                _dev(x, torch.float32)
            if not (theta.numel() == v.numel() == u.numel() == g.numel()) or not g.is_cuda or not g.is_contiguous():
                raise SwitchBackError("tensor %d: theta, v, u and grad must be contiguous GPU tensors of one size" % i)
            table[i] = SbAdamwTensor(theta.data_ptr(), v.data_ptr(), u.data_ptr(), g.data_ptr(), theta.numel(), 0, 0)
        total = lib.switchback_stable_adamw_plan(table, n)
        if total < 0:
            _check(-total)
        self.n, self.total_blocks = n, int(total)
        device = self.tensors[0][0].device
        raw = torch.frombuffer(bytearray(bytes(table)), dtype=torch.uint8)
        self.table = raw.to(device)
        self.ws = torch.empty(max(8 * self.total_blocks, 16), dtype=torch.uint8, device=device)
        self.rms = torch.empty(n, dtype=torch.float32, device=device)


def stable_adamw_step_multi(plan, alpha, beta1, beta2, eps, lam, t):
    """One StableAdamW step for every tensor of the plan (two launches in total).  Returns plan.rms [n]."""
    lib = load_library()
    _check(lib.switchback_stable_adamw_step_multi(_ptr(plan.table), plan.n, plan.total_blocks,
                                                  _SB_DTYPE[plan.grad_dtype], alpha, beta1, beta2, eps, lam, t,
                                                  _ptr(plan.rms), _ptr(plan.ws), plan.ws.numel(), _stream()))
    return plan.rms
