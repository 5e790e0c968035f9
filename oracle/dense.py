"""ctypes front end of oracle/dense.c plus the layer-by-layer MLP recipes.

TEST INFRASTRUCTURE ONLY.  Nothing here is imported by the product path.

The forward recipes follow the workload definitions: every layer is
H_{l+1} = act(H_l . W_l); with bf16 weights each layer's input is rounded to
bf16 (nearest-even) first, the sum is exact (double), the activation is applied
to the unrounded sum and the result is rounded once to float; the last layer's
output stays float.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_DIR, "liboracle_dense.so")

ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def build(force=False):
    if os.environ.get("ORACLE_DENSE_SO"):       # another build of dense.c (the sanitizer build of the tests)
        return os.environ["ORACLE_DENSE_SO"]
    src = os.path.join(_DIR, "dense.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", _SO, src, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        L.orc_bf16_from_f32.restype = ctypes.c_uint16
        L.orc_bf16_from_f32.argtypes = [ctypes.c_float]
        L.orc_f32_from_bf16.restype = ctypes.c_float
        L.orc_f32_from_bf16.argtypes = [ctypes.c_uint16]
        L.orc_round_bf16.argtypes = [vp, vp, i64]
        L.orc_dense_f32.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int]
        L.orc_dense_bf16.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int]
        L.orc_dense_bwd_input_bf16.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_dense_bwd_weight_bf16.argtypes = [vp, vp, vp, i64, i64, i64]
        L.orc_softmax_xent.restype = ctypes.c_double
        L.orc_softmax_xent.argtypes = [vp, vp, vp, i64, i64]
        L.orc_sgd_update.argtypes = [vp, vp, vp, ctypes.c_float, i64]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def round_bf16(x):
    """float32 array -> uint16 array of bf16 bit patterns (nearest, ties to even)."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().orc_round_bf16(_p(x), _p(out), x.size)
    return out


def bf16_to_f32(h):
    h = _c(h, np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)


def dense_f32(X, W, act):
    X, W = _c(X, np.float32), _c(W, np.float32)
    M, K = X.shape
    K2, N = W.shape
    assert K == K2
    Y = np.empty((M, N), np.float32)
    lib().orc_dense_f32(_p(X), _p(W), _p(Y), M, K, N, act)
    return Y


def dense_bf16(Xb, Wb, act):
    Xb, Wb = _c(Xb, np.uint16), _c(Wb, np.uint16)
    M, K = Xb.shape
    K2, N = Wb.shape
    assert K == K2
    Y = np.empty((M, N), np.float32)
    lib().orc_dense_bf16(_p(Xb), _p(Wb), _p(Y), M, K, N, act)
    return Y


def mlp_forward_f32(X, Ws, acts):
    """All layers in float storage.  Returns the list [H_1, ..., H_last]."""
    H, out = X, []
    for W, act in zip(Ws, acts):
        H = dense_f32(H, W, act)
        out.append(H)
    return out


def mlp_forward_bf16(Xb, Wbs, acts):
    """bf16 weights and layer inputs, float results.  ``Xb`` holds bf16 bit
    patterns.  Returns the float outputs of every layer (before the rounding
    that feeds the next one)."""
    Hb, out = Xb, []
    for W, act in zip(Wbs, acts):
        Y = dense_bf16(Hb, W, act)
        out.append(Y)
        Hb = round_bf16(Y)
    return out


def dense_bwd_input_bf16(dYb, Wb):
    dYb, Wb = _c(dYb, np.uint16), _c(Wb, np.uint16)
    M, N = dYb.shape
    K, N2 = Wb.shape
    assert N == N2
    dX = np.empty((M, K), np.float32)
    lib().orc_dense_bwd_input_bf16(_p(dYb), _p(Wb), _p(dX), M, K, N)
    return dX


def dense_bwd_weight_bf16(Hb, dYb):
    Hb, dYb = _c(Hb, np.uint16), _c(dYb, np.uint16)
    M, K = Hb.shape
    M2, N = dYb.shape
    assert M == M2
    dW = np.empty((K, N), np.float32)
    lib().orc_dense_bwd_weight_bf16(_p(Hb), _p(dYb), _p(dW), M, K, N)
    return dW


def softmax_xent(logits, labels):
    logits, labels = _c(logits, np.float32), _c(labels, np.int32)
    M, N = logits.shape
    d = np.empty((M, N), np.float32)
    loss = lib().orc_softmax_xent(_p(logits), _p(labels), _p(d), M, N)
    return loss, d


def sgd_update(Wm, Wb, dW, lr):
    """In place on ``Wm`` (float32) and ``Wb`` (uint16)."""
    assert Wm.dtype == np.float32 and Wb.dtype == np.uint16 and Wm.flags.c_contiguous
    dW = _c(dW, np.float32)
    lib().orc_sgd_update(_p(Wm), _p(Wb), _p(dW), np.float32(lr), Wm.size)
