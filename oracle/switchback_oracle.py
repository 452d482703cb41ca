"""ctypes front end of the plain-C SwitchBack oracle (arxiv 2304.13013, Section 2.2.1, Algorithm 1).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's cpu_baseline leg call this; the GPU
library never does, and nothing here imports the GPU package.  Arrays are numpy; bf16 tensors are uint16 arrays
holding the bf16 bit patterns.  Every function allocates and returns its outputs.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "switchback_oracle.c")
_LIB = os.path.join(_HERE, "libswitchback_oracle.so")

# No fast-math, no contraction: every binary32 operation in the C file must round exactly once.
_CFLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-Wall"]


def build(force=False):
    """Compile the oracle with gcc (skipped when the library is newer than its source unless force)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.sbo_matmul_int8.restype = ctypes.c_int
        _lib.sbo_num_threads.restype = ctypes.c_int
        _lib.sbo_stable_adamw_step.restype = ctypes.c_double
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def _bf16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16 and a.ndim == 2, "bf16 tensors are 2-D uint16 arrays of bit patterns"
    return a


def num_threads():
    return int(_load().sbo_num_threads())


def quantize_rowwise(x):
    """Q_row and state_row (row-wise quantization equation): returns (q int8 [r,c], state f32 [r])."""
    x = _bf16(x)
    r, c = x.shape
    q = np.empty((r, c), np.int8)
    state = np.empty(r, np.float32)
    _load().sbo_quantize_rowwise(_p(x), _i64(r), _i64(c), _p(q), _p(state))
    return q, state


def quantize_tensorwise(w):
    """Q_tensor and state_tensor (tensor-wise quantization equation): returns (q [r,c], q_t [c,r], state f32)."""
    w = _bf16(w)
    r, c = w.shape
    q = np.empty((r, c), np.int8)
    q_t = np.empty((c, r), np.int8)
    state = np.empty(1, np.float32)
    _load().sbo_quantize_tensorwise(_p(w), _i64(r), _i64(c), _p(q), _p(q_t), _p(state))
    return q, q_t, state[0]


def dequantize_rowwise(q, state):
    """Row-wise dequantization of SwitchBackM (inverse of the row-wise quantization equation): bf16 patterns
    of fl(q * fl(state/127)), uint16 [r,c]."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    state = np.ascontiguousarray(state, dtype=np.float32)
    r, c = q.shape
    assert state.shape == (r,)
    out = np.empty((r, c), np.uint16)
    _load().sbo_dequantize_rowwise(_p(q), _p(state), _i64(r), _i64(c), _p(out))
    return out


def matmul_int8(a, b):
    """acc = a b^T exactly, a [M,K], b [N,K] int8 -> int32 [M,N].  Raises if a sum leaves int32."""
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.dtype == np.int8 and b.dtype == np.int8 and a.shape[1] == b.shape[1]
    M, K = a.shape
    N = b.shape[0]
    acc = np.empty((M, N), np.int32)
    if _load().sbo_matmul_int8(_p(a), _p(b), _i64(M), _i64(N), _i64(K), _p(acc)):
        raise OverflowError("int8 matmul left the int32 range")
    return acc


def dequantize(acc, state_row, state_tensor, want_f64=False):
    """Forward equation with dequantization: y32 (binary32, in the oracle's operation order) and, optionally,
    the same product evaluated in binary64."""
    acc = np.ascontiguousarray(acc)
    state_row = np.ascontiguousarray(state_row, dtype=np.float32)
    assert acc.dtype == np.int32 and state_row.shape == (acc.shape[0],)
    M, N = acc.shape
    y32 = np.empty((M, N), np.float32)
    y64 = np.empty((M, N), np.float64) if want_f64 else None
    _load().sbo_dequantize(_p(acc), _i64(M), _i64(N), _p(state_row), ctypes.c_float(float(state_tensor)),
                           _p(y32), _p(y64) if want_f64 else None)
    return (y32, y64) if want_f64 else y32


def bias_layerscale(y32, bias=None, gamma=None, y64=None):
    """out[i,j] = gamma[j] * (y[i,j] + bias[j]) in binary32, one rounding per operation, bias first (either vector may
    be None).  With y64 (the binary64 product) also returns the same expression in binary64."""
    y32 = np.ascontiguousarray(y32, dtype=np.float32)
    M, N = y32.shape
    vec = lambda v: None if v is None else np.ascontiguousarray(v, dtype=np.float32)
    bias, gamma = vec(bias), vec(gamma)
    assert (bias is None or bias.shape == (N,)) and (gamma is None or gamma.shape == (N,))
    out = np.empty((M, N), np.float32)
    out64 = None
    if y64 is not None:
        y64 = np.ascontiguousarray(y64, dtype=np.float64)
        out64 = np.empty((M, N), np.float64)
    _load().sbo_bias_layerscale(_p(y32), _p(y64) if y64 is not None else None, _i64(M), _i64(N),
                                _p(bias) if bias is not None else None, _p(gamma) if gamma is not None else None,
                                _p(out), _p(out64) if out64 is not None else None)
    return (out, out64) if y64 is not None else out


def dequantize_rowcol(acc, state_row, state_col, want_f64=False):
    """SwitchBackQ dequantization: y = acc * state_row[i] * state_col[j] / 127^2 (binary32, column constant first)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    state_row = np.ascontiguousarray(state_row, dtype=np.float32)
    state_col = np.ascontiguousarray(state_col, dtype=np.float32)
    assert state_row.shape == (M,) and state_col.shape == (N,)
    y32 = np.empty((M, N), np.float32)
    y64 = np.empty((M, N), np.float64) if want_f64 else None
    _load().sbo_dequantize_rowcol(_p(acc), _i64(M), _i64(N), _p(state_row), _p(state_col), _p(y32),
                                  _p(y64) if want_f64 else None)
    return (y32, y64) if want_f64 else y32


def quantize_colwise_transpose(w):
    """SwitchBackQ's column-wise quantization fused with a transpose: every column of w [rows, cols] gets its own
    absmax; the codes come out transposed, [cols, rows].  By definition this is the row-wise quantization of the
    transposed matrix.  Returns (q_t int8 [cols, rows], state f32 [cols])."""
    w = _bf16(w)
    return quantize_rowwise(np.ascontiguousarray(w.T))


def forward_q(x, w):
    """SwitchBackQ forward: row-wise quantization of X and of W (one state per output feature)."""
    xq, state_x = quantize_rowwise(x)
    wq, state_w = quantize_rowwise(w)
    acc = matmul_int8(xq, wq)
    y32 = dequantize_rowcol(acc, state_x, state_w)
    return dict(xq=xq, state_x=state_x, wq=wq, state_w=state_w, acc=acc, y32=y32, y_bf16=round_to_bf16(y32))


def backward_input_q(dy, w):
    """SwitchBackQ input gradient: row-wise quantization of dY, column-wise (transposed) quantization of W, so the
    contraction over m has one state per token and one per input feature."""
    gq, state_g = quantize_rowwise(dy)
    wq_t, state_wc = quantize_colwise_transpose(w)
    acc = matmul_int8(gq, wq_t)
    dx32 = dequantize_rowcol(acc, state_g, state_wc)
    return dict(gq=gq, state_g=state_g, wq_t=wq_t, state_wc=state_wc, acc=acc, dx32=dx32,
                dx_bf16=round_to_bf16(dx32))


def round_to_bf16(y32):
    """binary32 -> bf16 bit patterns, round-to-nearest-even."""
    y32 = np.ascontiguousarray(y32, dtype=np.float32)
    out = np.empty(y32.shape, np.uint16)
    _load().sbo_round_to_bf16(_p(y32), _i64(y32.size), _p(out))
    return out


def weight_grad(dy, x):
    """dW = dY^T X accumulated in binary64 (Algorithm 1's 16-bit matmul, as its exact definition): f64 [m,n]."""
    dy = _bf16(dy)
    x = _bf16(x)
    assert dy.shape[0] == x.shape[0]
    b, m = dy.shape
    n = x.shape[1]
    dw = np.empty((m, n), np.float64)
    _load().sbo_weight_grad(_p(dy), _p(x), _i64(b), _i64(n), _i64(m), _p(dw))
    return dw


def forward(x, w):
    """Algorithm 1 forward.  Returns a dict with every intermediate: xq, state_x, wq, wq_t, state_w, acc,
    y32 (binary32 before the bf16 cast) and y_bf16."""
    xq, state_x = quantize_rowwise(x)
    wq, wq_t, state_w = quantize_tensorwise(w)
    acc = matmul_int8(xq, wq)
    y32 = dequantize(acc, state_x, state_w)
    return dict(xq=xq, state_x=state_x, wq=wq, wq_t=wq_t, state_w=state_w, acc=acc, y32=y32,
                y_bf16=round_to_bf16(y32))


def backward_input(dy, wq_t, state_w):
    """Algorithm 1 input gradient: dX = dequant(Q_row(dY) Q_tensor(W)); contraction over m, so the right
    operand is the transposed code matrix wq_t [n,m]."""
    gq, state_g = quantize_rowwise(dy)
    acc = matmul_int8(gq, wq_t)
    dx32 = dequantize(acc, state_g, state_w)
    return dict(gq=gq, state_g=state_g, acc=acc, dx32=dx32, dx_bf16=round_to_bf16(dx32))


def backward_weight_m(dy, xq, state_x):
    """Weight gradient of SwitchBackM: X is first rebuilt from its int8 codes (row-wise dequantization), then the
    16-bit matmul as in Algorithm 1."""
    x_hat = dequantize_rowwise(xq, state_x)
    out = backward_weight(dy, x_hat)
    out["x_hat"] = x_hat
    return out


def backward_weight(dy, x):
    """Algorithm 1 weight gradient: binary64 sum, its binary32 rounding and the bf16 rounding of that."""
    dw64 = weight_grad(dy, x)
    dw32 = dw64.astype(np.float32)
    return dict(dw64=dw64, dw32=dw32, dw_bf16=round_to_bf16(dw32))


def stable_adamw_step(theta, v, u, grad, alpha, beta1, beta2, eps, lam, t):
    """One StableAdamW step for one tensor (the optimizer algorithm of the paper), binary64 arithmetic on binary32
    state.  grad: uint16 bf16 patterns or float32.  Returns (theta, v, u, rms) as new arrays."""
    theta = np.array(theta, dtype=np.float32).ravel().copy()
    v = np.array(v, dtype=np.float32).ravel().copy()
    u = np.array(u, dtype=np.float32).ravel().copy()
    grad = np.ascontiguousarray(grad).ravel()
    assert theta.size == v.size == u.size == grad.size
    g16 = _p(grad) if grad.dtype == np.uint16 else None
    g32 = None
    if g16 is None:
        grad = grad.astype(np.float32)
        g32 = _p(grad)
    d = ctypes.c_double
    rms = _load().sbo_stable_adamw_step(_p(theta), _p(v), _p(u), g16, g32, _i64(theta.size), d(alpha), d(beta1),
                                        d(beta2), d(eps), d(lam), _i64(t))
    return theta, v, u, float(rms)


E4M3, E5M2 = 0, 1


def float8_encode(x, fmt):
    """float8cast of binary32 values: uint8 codes of the nearest representable value (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.empty(x.shape, np.uint8)
    _load().sbo_float8_encode(_p(x), _i64(x.size), ctypes.c_int(fmt), _p(codes))
    return codes


def float8_decode(codes, fmt):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, np.float64)
    _load().sbo_float8_decode(_p(codes), _i64(codes.size), ctypes.c_int(fmt), _p(out))
    return out


def quantize_rowwise_f8(x, fmt):
    """float8cast(x / absmax_row(x)): returns (codes uint8 [r,c], state f32 [r])."""
    x = _bf16(x)
    r, c = x.shape
    codes = np.empty((r, c), np.uint8)
    state = np.empty(r, np.float32)
    _load().sbo_quantize_rowwise_f8(_p(x), _i64(r), _i64(c), ctypes.c_int(fmt), _p(codes), _p(state))
    return codes, state


def quantize_tensorwise_f8(w, fmt):
    """float8cast(w / absmax(w)): returns (codes [r,c], codes_t [c,r], state f32)."""
    w = _bf16(w)
    r, c = w.shape
    codes = np.empty((r, c), np.uint8)
    codes_t = np.empty((c, r), np.uint8)
    state = np.empty(1, np.float32)
    _load().sbo_quantize_tensorwise_f8(_p(w), _i64(r), _i64(c), ctypes.c_int(fmt), _p(codes), _p(codes_t), _p(state))
    return codes, codes_t, state[0]


def matmul_f8(a, fmt_a, b, fmt_b, want_abs=False):
    """Exact sum_k value(a[i,k]) value(b[j,k]) in binary64; with want_abs also sum_k |.||.|."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    b = np.ascontiguousarray(b, dtype=np.uint8)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    acc = np.empty((M, N), np.float64)
    abs_acc = np.empty((M, N), np.float64) if want_abs else None
    _load().sbo_matmul_f8(_p(a), ctypes.c_int(fmt_a), _p(b), ctypes.c_int(fmt_b), _i64(M), _i64(N), _i64(K), _p(acc),
                          _p(abs_acc) if want_abs else None)
    return (acc, abs_acc) if want_abs else acc


def dequantize_f8(acc, state_row, state_tensor, want_f64=False):
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    M, N = acc.shape
    state_row = np.ascontiguousarray(state_row, dtype=np.float32)
    y32 = np.empty((M, N), np.float32)
    y64 = np.empty((M, N), np.float64) if want_f64 else None
    _load().sbo_dequantize_f8(_p(acc), _i64(M), _i64(N), _p(state_row), ctypes.c_float(float(state_tensor)), _p(y32),
                              _p(y64) if want_f64 else None)
    return (y32, y64) if want_f64 else y32


def forward_f8(x, w, fmt_x=E4M3, fmt_w=E4M3):
    """float8 SwitchBack forward: Y = dequant(f8_row(X) f8_tensor(W)^T)."""
    xq, state_x = quantize_rowwise_f8(x, fmt_x)
    wq, wq_t, state_w = quantize_tensorwise_f8(w, fmt_w)
    acc, abs_acc = matmul_f8(xq, fmt_x, wq, fmt_w, want_abs=True)
    y32 = dequantize_f8(acc, state_x, state_w)
    return dict(xq=xq, state_x=state_x, wq=wq, wq_t=wq_t, state_w=state_w, acc=acc, abs_acc=abs_acc, y32=y32,
                y_bf16=round_to_bf16(y32))


def backward_input_f8(dy, wq_t, state_w, fmt_g=E5M2, fmt_w=E4M3):
    """float8 SwitchBack input gradient: dX = dequant(f8_row(dY) f8_tensor(W))."""
    gq, state_g = quantize_rowwise_f8(dy, fmt_g)
    acc, abs_acc = matmul_f8(gq, fmt_g, wq_t, fmt_w, want_abs=True)
    dx32 = dequantize_f8(acc, state_g, state_w)
    return dict(gq=gq, state_g=state_g, acc=acc, abs_acc=abs_acc, dx32=dx32, dx_bf16=round_to_bf16(dx32))
