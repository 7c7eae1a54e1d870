"""CPU oracle for the fused-operator hot path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, double-precision definitions of the operators (C, in
oracle_ops.c) plus an independent type checker and an op-by-op graph runner
(graph.py).  Nothing on the product path may import this package; it shares
no code with the HIP library.  Only tests, the smoke check and the benchmark's
CPU-baseline leg use it.

Parity status: the paper defines none of the operators' arithmetic, so parity
of the semantics against the paper is unpinned; parity against the stated
standard definitions is pinned by tests/test_oracle_*.py (brute force on tiny
shapes, closed forms, invariants, a library cross-check).  The typing rules
are the paper's (figure of expression typing rules) and are pinned one rule
at a time.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_ops.c")
_LIB = os.path.join(_HERE, "liboracle_ops.so")


def build(force: bool = False) -> str:
    """Compile oracle_ops.c with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _d(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64, order="C")          # (unlike ascontiguousarray, keeps a rank-0 array rank 0)


def _i(v):
    return ctypes.c_int64(int(v))


# ---- operators on float64 arrays -------------------------------------------------
def dense(x, w):
    x, w = _d(x), _d(w)
    (M, K), (N, K2) = x.shape, w.shape
    assert K == K2
    y = np.empty((M, N))
    lib().oracle_dense(_p(x), _p(w), _p(y), _i(M), _i(N), _i(K))
    return y


def conv2d(x, w, stride=(1, 1), pad=(0, 0)):
    x, w = _d(x), _d(w)
    N, C, H, W = x.shape
    O, C2, KH, KW = w.shape
    assert C == C2
    OH = (H + 2 * pad[0] - KH) // stride[0] + 1
    OW = (W + 2 * pad[1] - KW) // stride[1] + 1
    y = np.empty((N, O, OH, OW))
    lib().oracle_conv2d(_p(x), _p(w), _p(y), _i(N), _i(C), _i(H), _i(W), _i(O), _i(KH), _i(KW),
                        _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]), _i(OH), _i(OW))
    return y


def dense_grad_x(dy, w):
    dy, w = _d(dy), _d(w)
    (M, N), (N2, K) = dy.shape, w.shape
    assert N == N2
    dx = np.empty((M, K))
    lib().oracle_dense_grad_x(_p(dy), _p(w), _p(dx), _i(M), _i(N), _i(K))
    return dx


def dense_grad_w(dy, x):
    dy, x = _d(dy), _d(x)
    (M, N), (M2, K) = dy.shape, x.shape
    assert M == M2
    dw = np.empty((N, K))
    lib().oracle_dense_grad_w(_p(dy), _p(x), _p(dw), _i(M), _i(N), _i(K))
    return dw


def conv2d_grad_x(dy, w, x_shape, stride=(1, 1), pad=(0, 0)):
    dy, w = _d(dy), _d(w)
    N, C, H, W = x_shape
    O, C2, KH, KW = w.shape
    N2, O2, OH, OW = dy.shape
    assert (N, C, O) == (N2, C2, O2)
    assert OH == (H + 2 * pad[0] - KH) // stride[0] + 1 and OW == (W + 2 * pad[1] - KW) // stride[1] + 1
    dx = np.empty((N, C, H, W))
    lib().oracle_conv2d_grad_x(_p(dy), _p(w), _p(dx), _i(N), _i(C), _i(H), _i(W), _i(O), _i(KH), _i(KW),
                               _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]), _i(OH), _i(OW))
    return dx


def conv2d_grad_w(dy, x, kernel, stride=(1, 1), pad=(0, 0)):
    dy, x = _d(dy), _d(x)
    N, C, H, W = x.shape
    N2, O, OH, OW = dy.shape
    KH, KW = kernel
    assert N == N2
    assert OH == (H + 2 * pad[0] - KH) // stride[0] + 1 and OW == (W + 2 * pad[1] - KW) // stride[1] + 1
    dw = np.empty((O, C, KH, KW))
    lib().oracle_conv2d_grad_w(_p(dy), _p(x), _p(dw), _i(N), _i(C), _i(H), _i(W), _i(O), _i(KH), _i(KW),
                               _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]), _i(OH), _i(OW))
    return dw


def bias_add(x, b, axis=1):
    x, b = _d(x), _d(b)
    C = x.shape[axis]
    assert b.shape == (C,)
    outer = int(np.prod(x.shape[:axis], dtype=np.int64))
    inner = int(np.prod(x.shape[axis + 1:], dtype=np.int64))
    y = np.empty_like(x)
    lib().oracle_bias_add(_p(x), _p(b), _p(y), _i(outer), _i(C), _i(inner))
    return y


_BIN = {"add": 0, "sub": 1, "mul": 2, "div": 3}
_UN = {"neg": 0, "sq": 1, "relu": 2, "sigmoid": 3, "tanh": 4}


def binary(op, a, b):
    a, b = _d(a), _d(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().oracle_binary(ctypes.c_int(_BIN[op]), _p(a), _p(b), _p(y), _i(a.size))
    return y


def unary(op, x):
    x = _d(x)
    y = np.empty_like(x)
    lib().oracle_unary(ctypes.c_int(_UN[op]), _p(x), _p(y), _i(x.size))
    return y


def batchnorm(x, gamma, beta, mean, var, eps):
    x = _d(x)
    N, C = x.shape[:2]
    HW = int(np.prod(x.shape[2:], dtype=np.int64))
    y = np.empty_like(x)
    lib().oracle_batchnorm(_p(x), _p(_d(gamma)), _p(_d(beta)), _p(_d(mean)), _p(_d(var)),
                           ctypes.c_double(eps), _p(y), _i(N), _i(C), _i(HW))
    return y


def fold_batchnorm(w, gamma, beta, mean, var, eps):
    w = _d(w)
    O = w.shape[0]
    per_o = w.size // O
    wf = np.empty_like(w)
    bf = np.empty((O,))
    lib().oracle_fold_batchnorm(_p(w), _p(_d(gamma)), _p(_d(beta)), _p(_d(mean)), _p(_d(var)),
                                ctypes.c_double(eps), _p(wf), _p(bf), _i(O), _i(per_o))
    return wf, bf


def maxpool2d(x, kernel, stride, pad):
    x = _d(x)
    N, C, H, W = x.shape
    OH = (H + 2 * pad[0] - kernel[0]) // stride[0] + 1
    OW = (W + 2 * pad[1] - kernel[1]) // stride[1] + 1
    y = np.empty((N, C, OH, OW))
    lib().oracle_maxpool2d(_p(x), _p(y), _i(N), _i(C), _i(H), _i(W), _i(kernel[0]), _i(kernel[1]),
                           _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]), _i(OH), _i(OW))
    return y


def global_avgpool(x):
    x = _d(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, 1, 1))
    lib().oracle_global_avgpool(_p(x), _p(y), _i(N), _i(C), _i(H * W))
    return y


def lstm_gates(z, c):
    z, c = _d(z), _d(c)
    B, H = c.shape
    assert z.shape == (B, 4 * H)
    c2, h2 = np.empty_like(c), np.empty_like(c)
    lib().oracle_lstm_gates(_p(z), _p(c), _p(c2), _p(h2), _i(B), _i(H))
    return c2, h2


def round_to(x, dtype: str):
    """Nearest value representable in `dtype` ("f32" | "bf16"), ties to even."""
    x = _d(x)
    y = np.empty_like(x)
    fn = {"f32": lib().oracle_round_f32, "bf16": lib().oracle_round_bf16}[dtype]
    fn(_p(x), _p(y), _i(x.size))
    return y


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored tensor data (float32 array, or uint16 bf16 bit
    patterns) to float64."""
    if dtype == "bf16":
        a = np.asarray(a, dtype=np.uint16, order="C")
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float32, order="C").astype(np.float64)


def lstm_sequence(x_seq, w, b, h0, c0, h_dtype="bf16"):
    """Reference recurrence: for each t, z = [x_t, h_{t-1}] W^T + b (kept f32),
    then the gate math; h_t is rounded to h_dtype and c_t to f32 when stored,
    exactly where the values cross a fusion-group boundary."""
    T = x_seq.shape[0]
    h, c = _d(h0), _d(c0)
    hs = []
    for t in range(T):
        xh = np.concatenate([_d(x_seq[t]), h], axis=1)
        z = bias_add(dense(xh, w), b, axis=1)
        c2, h2 = lstm_gates(z, c)
        c = round_to(c2, "f32")
        h = round_to(h2, h_dtype)
        hs.append(h)
    return np.stack(hs), c


def num_threads() -> int:
    return int(lib().oracle_num_threads())
