"""ctypes front end of the CPU checker (oracle/hpct_ref.c) and the five chains
composed from its operator definitions.  Inputs are fp32 numpy arrays (the
exact bits the GPU library is given); every result is fp64.

Test infrastructure only.  Each chain keeps its intermediates in fp64 and is
the composition, in the order the workload states, of the definitions in
hpct_ref.c (paper Table 1 operator classes; Section 5.3 for the convolution).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        _lib = C.CDLL(path)
        i64, dbl, p = C.c_int64, C.c_double, C.c_void_p
        sig = {
            "ref_gemm_bias": [p, p, p, i64, i64, i64, p, p],
            "ref_relu": [p, i64],
            "ref_scale": [p, i64, C.c_float],
            "ref_softmax_rows": [p, i64, i64, p],
            "ref_affine_relu_residual": [p, p, p, p, i64, i64, i64, p],
            "ref_avgpool_planes": [p, i64, i64, p],
            "ref_layernorm_rows": [p, p, p, i64, i64, dbl, p],
            "ref_gelu_tanh": [p, i64],
            "ref_conv2d_nchw_bias": [p, p, p] + [i64] * 10 + [p, p],
            "ref_conv2d_nchw_grouped": [p, p, p] + [i64] * 11 + [p, p],
            "ref_relu6": [p, i64],
            "ref_conv_transpose2d_nchw": [p, p, p] + [i64] * 10 + [p, p],
            "ref_attention": [p, p, p, i64, i64, i64, i64, dbl, p, p],
            "ref_attention_causal": [p, p, p, i64, i64, i64, i64, dbl, p, p],
            "ref_layout_copy": [p, C.c_int32, p, p, p],
            "ref_set_threads": [C.c_int],
            "ref_dropout_hash": [p, i64, i64, C.c_float, C.c_uint64],
            "ref_mean_rows": [p, i64, i64, p],
            "ref_scale_shift_planes": [p, p, p, i64, i64, i64],
            "ref_maxpool2x2_planes": [p, i64, i64, i64, p],
            "ref_maxpool2d_planes": [p, i64, i64, i64, i64, i64, i64, p],
            "ref_avgpool2d_planes": [p, i64, i64, i64, i64, i64, i64, p],
            "ref_groupnorm_nchw": [p, p, p, i64, i64, i64, i64, dbl, p],
            "ref_rmsnorm_rows": [p, p, i64, i64, dbl, p],
            "ref_reduce_axis": [p, C.c_int32, p, p, C.c_int32, C.c_int32, p, p, p],
            "ref_eltwise_binary": [p, p, C.c_int32, p, p, p, C.c_int32, C.c_int32, p],
            "ref_eltwise_map": [p, p, C.c_int32, p, p, p, C.c_int32, C.c_int32, p, C.c_float, p],
        }
        for name, args in sig.items():
            f = getattr(_lib, name)
            f.argtypes, f.restype = args, None
        _lib.ref_max_threads.argtypes, _lib.ref_max_threads.restype = [], C.c_int
        _lib.ref_dropout_rand.argtypes, _lib.ref_dropout_rand.restype = [C.c_uint64], C.c_float
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def max_threads() -> int:
    return int(lib().ref_max_threads())


def set_threads(n: int) -> None:
    lib().ref_set_threads(int(n))


# ----------------------------------------------------------------- operators
def gemm_bias(X, W, bias=None, want_norm=False):
    X, W = _f32(X), _f32(W)
    M, K = X.shape
    K2, N = W.shape
    assert K == K2
    b = None if bias is None else _f32(bias)
    Z = np.empty((M, N), dtype=np.float64)
    Dn = np.empty((M, N), dtype=np.float64) if want_norm else None
    lib().ref_gemm_bias(_ptr(X), _ptr(W), _ptr(b), M, K, N, _ptr(Z), _ptr(Dn))
    return (Z, Dn) if want_norm else Z


def relu(Z):
    Z = np.array(Z, dtype=np.float64, order="C")
    lib().ref_relu(_ptr(Z), Z.size)
    return Z


def scale_const(Z, s):
    """Z * s with s rounded to fp32 first (the constant the GPU path is given)."""
    Z = np.array(Z, dtype=np.float64, order="C")
    lib().ref_scale(_ptr(Z), Z.size, C.c_float(s))
    return Z


def softmax_rows(Z):
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    N = Z.shape[-1]
    rows = Z.size // N if N else 0
    Y = np.empty_like(Z)
    if Z.size:
        lib().ref_softmax_rows(_ptr(Z), rows, N, _ptr(Y))
    return Y


def affine_relu_residual(X, scale, shift, R):
    X, R, scale, shift = _f32(X), _f32(R), _f32(scale), _f32(shift)
    Nb, Cc, H, W = X.shape
    assert R.shape == X.shape and scale.shape == (Cc,) and shift.shape == (Cc,)
    T = np.empty(X.shape, dtype=np.float64)
    lib().ref_affine_relu_residual(_ptr(X), _ptr(scale), _ptr(shift), _ptr(R), Nb, Cc, H * W, _ptr(T))
    return T


def avgpool_hw(T):
    T = np.ascontiguousarray(T, dtype=np.float64)
    Nb, Cc, H, W = T.shape
    out = np.empty((Nb, Cc), dtype=np.float64)
    lib().ref_avgpool_planes(_ptr(T), Nb * Cc, H * W, _ptr(out))
    return out


def layernorm_rows(X, gamma=None, beta=None, eps=1e-5):
    X = _f32(X)
    rows, N = X.shape
    g = None if gamma is None else _f32(gamma)
    b = None if beta is None else _f32(beta)
    Y = np.empty((rows, N), dtype=np.float64)
    lib().ref_layernorm_rows(_ptr(X), _ptr(g), _ptr(b), rows, N, float(eps), _ptr(Y))
    return Y


def rmsnorm_rows(X, gamma=None, eps=1e-6):
    """x / sqrt(mean(x^2) + eps) * gamma over the last dim of an fp32 [rows, N] array."""
    X = _f32(X)
    rows, N = X.shape
    g = None if gamma is None else _f32(gamma)
    Y = np.empty((rows, N), dtype=np.float64)
    lib().ref_rmsnorm_rows(_ptr(X), _ptr(g), rows, N, float(eps), _ptr(Y))
    return Y


def groupnorm_nchw(X, groups, gamma=None, beta=None, eps=1e-5):
    """Group normalisation of an fp32 NCHW array: statistics per image and group of C // groups neighbouring channels,
    gamma / beta per channel.  groups = C: instance normalisation."""
    X = _f32(X)
    Nb, Cc, H, W = X.shape
    assert groups >= 1 and Cc % groups == 0
    g = None if gamma is None else _f32(gamma)
    b = None if beta is None else _f32(beta)
    Y = np.empty(X.shape, dtype=np.float64)
    lib().ref_groupnorm_nchw(_ptr(X), _ptr(g), _ptr(b), Nb, Cc, H * W, groups, float(eps), _ptr(Y))
    return Y


def gelu_tanh(Y):
    Y = np.array(Y, dtype=np.float64, order="C")
    lib().ref_gelu_tanh(_ptr(Y), Y.size)
    return Y


def conv_out_hw(H, W, R, S, stride, pad, dil=1):
    # the filter must fit the padded image (otherwise the floor division below and the C routine's truncation disagree)
    assert H + 2 * pad >= (R - 1) * dil + 1 and W + 2 * pad >= (S - 1) * dil + 1, "filter larger than the padded image"
    return (H + 2 * pad - (R - 1) * dil - 1) // stride + 1, (W + 2 * pad - (S - 1) * dil - 1) // stride + 1


def conv2d_nchw_bias(inp, wt, bias=None, stride=1, pad=1, want_norm=False, dil=1):
    inp, wt = _f32(inp), _f32(wt)
    Nb, Cc, H, W = inp.shape
    K, C2, R, S = wt.shape
    assert Cc == C2
    b = None if bias is None else _f32(bias)
    Ho, Wo = conv_out_hw(H, W, R, S, stride, pad, dil)
    out = np.empty((Nb, K, Ho, Wo), dtype=np.float64)
    Dn = np.empty_like(out) if want_norm else None
    lib().ref_conv2d_nchw_bias(_ptr(inp), _ptr(wt), _ptr(b), Nb, Cc, H, W, K, R, S, stride, pad, dil,
                               _ptr(out), _ptr(Dn))
    return (out, Dn) if want_norm else out


def conv2d_nchw_grouped(inp, wt, bias=None, stride=1, pad=1, groups=1, want_norm=False, dil=1):
    """Grouped conv: wt is [K, C/groups, R, S]; groups = C = K is the depthwise convolution."""
    inp, wt = _f32(inp), _f32(wt)
    Nb, Cc, H, W = inp.shape
    K, Cg, R, S = wt.shape
    assert Cc % groups == 0 and K % groups == 0 and Cg == Cc // groups
    b = None if bias is None else _f32(bias)
    Ho, Wo = conv_out_hw(H, W, R, S, stride, pad, dil)
    out = np.empty((Nb, K, Ho, Wo), dtype=np.float64)
    Dn = np.empty_like(out) if want_norm else None
    lib().ref_conv2d_nchw_grouped(_ptr(inp), _ptr(wt), _ptr(b), Nb, Cc, H, W, K, R, S, stride, pad, dil, groups,
                                  _ptr(out), _ptr(Dn))
    return (out, Dn) if want_norm else out


def conv_transpose_out_hw(H, W, R, S, stride, pad, dil=1):
    return (H - 1) * stride - 2 * pad + (R - 1) * dil + 1, (W - 1) * stride - 2 * pad + (S - 1) * dil + 1


def conv_transpose2d_nchw(inp, wt, bias=None, stride=1, pad=0, want_norm=False, dil=1):
    """Transposed conv: inp [N,C,H,W], wt [C,K,R,S] (input channels first), out [N,K,Ho,Wo]."""
    inp, wt = _f32(inp), _f32(wt)
    Nb, Cc, H, W = inp.shape
    C2, K, R, S = wt.shape
    assert Cc == C2
    b = None if bias is None else _f32(bias)
    Ho, Wo = conv_transpose_out_hw(H, W, R, S, stride, pad, dil)
    assert Ho >= 1 and Wo >= 1
    out = np.empty((Nb, K, Ho, Wo), dtype=np.float64)
    Dn = np.empty_like(out) if want_norm else None
    lib().ref_conv_transpose2d_nchw(_ptr(inp), _ptr(wt), _ptr(b), Nb, Cc, H, W, K, R, S, stride, pad, dil,
                                    _ptr(out), _ptr(Dn))
    return (out, Dn) if want_norm else out


def relu6(Z):
    Z = np.array(Z, dtype=np.float64, order="C")
    lib().ref_relu6(_ptr(Z), Z.size)
    return Z


def attention(Q, K, V, scale, want_norm=False, causal=False):
    """softmax(scale * Q K^T) V per batch; causal=True lets query i see keys j <= i only."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Lq, D = Q.shape
    B2, Lk, D2 = K.shape
    assert V.shape == K.shape and B2 == B and D2 == D and Lk >= 1
    O = np.empty((B, Lq, D), dtype=np.float64)
    Dn = np.empty_like(O) if want_norm else None
    fn = lib().ref_attention_causal if causal else lib().ref_attention
    fn(_ptr(Q), _ptr(K), _ptr(V), B, Lq, Lk, D, float(scale), _ptr(O), _ptr(Dn))
    return (O, Dn) if want_norm else O


def layout_copy(base, shape, stride):
    """Contiguous copy of the strided view (shape, stride in elements) of the
    1-D fp32 array `base`; returned as fp32 with the input's bit patterns."""
    base = np.ascontiguousarray(base, dtype=np.float32).reshape(-1)
    nd = len(shape)
    sh = (C.c_int64 * nd)(*[int(v) for v in shape])
    st = (C.c_int64 * nd)(*[int(v) for v in stride])
    assert all(v > 0 for v in shape) and all(v >= 0 for v in stride)
    assert sum((a - 1) * b for a, b in zip(shape, stride)) < base.size
    out = np.empty(tuple(int(v) for v in shape), dtype=np.float32)
    lib().ref_layout_copy(_ptr(base), nd, sh, st, _ptr(out))
    return out


def dropout_rand(h: int) -> float:
    """rand value the hash of Section 5.3 gives for h = offset + seed (fp32)."""
    return float(lib().ref_dropout_rand(int(h) & 0xFFFFFFFFFFFFFFFF))


def dropout_hash(Z, p, seed):
    """Training-mode dropout of a 2-D fp64 array with the hash mask of Section 5.3."""
    Z = np.array(Z, dtype=np.float64, order="C")
    assert Z.ndim == 2
    lib().ref_dropout_hash(_ptr(Z), Z.shape[0], Z.shape[1], float(np.float32(p)), int(seed) & 0xFFFFFFFFFFFFFFFF)
    return Z


def mean_rows(Z):
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    N = Z.shape[-1]
    out = np.empty(Z.shape[:-1], dtype=np.float64)
    lib().ref_mean_rows(_ptr(Z), Z.size // N, N, _ptr(out))
    return out


def scale_shift_ch(T, scale=None, shift=None):
    """T[n,c,h,w] * scale[c] + shift[c] on an fp64 NCHW array."""
    T = np.array(T, dtype=np.float64, order="C")
    Nb, Cc, H, W = T.shape
    sc = None if scale is None else _f32(scale)
    sh = None if shift is None else _f32(shift)
    lib().ref_scale_shift_planes(_ptr(T), _ptr(sc), _ptr(sh), Nb, Cc, H * W)
    return T


def maxpool2x2(T):
    """2x2 / stride-2 max pooling over the last two dims of an fp64 NCHW array."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    Nb, Cc, H, W = T.shape
    out = np.empty((Nb, Cc, H // 2, W // 2), dtype=np.float64)
    if out.size:
        lib().ref_maxpool2x2_planes(_ptr(T), Nb * Cc, H, W, _ptr(out))
    return out


def maxpool2d(T, k, stride, pad):
    """k x k max pooling with stride and padding (pad < k; padding never wins) over the last two dims of an fp64
    NCHW array; output extent (H + 2 pad - k) // stride + 1."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    Nb, Cc, H, W = T.shape
    assert 0 <= pad < k and stride >= 1 and H + 2 * pad >= k and W + 2 * pad >= k
    out = np.empty((Nb, Cc, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1), dtype=np.float64)
    if out.size:
        lib().ref_maxpool2d_planes(_ptr(T), Nb * Cc, H, W, k, stride, pad, _ptr(out))
    return out


def avgpool2d(T, k, stride, pad):
    """k x k average pooling with stride and padding (pad < k; padding counts as zeros, the divisor is k*k) over the
    last two dims of an fp64 NCHW array; output extent (H + 2 pad - k) // stride + 1."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    Nb, Cc, H, W = T.shape
    assert 0 <= pad < k and stride >= 1 and H + 2 * pad >= k and W + 2 * pad >= k
    out = np.empty((Nb, Cc, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1), dtype=np.float64)
    if out.size:
        lib().ref_avgpool2d_planes(_ptr(T), Nb * Cc, H, W, k, stride, pad, _ptr(out))
    return out


def eltwise_binary(a_base, b_base, shape, sa, sb, op, relu_=False):
    """out = [relu](a_view op b_view), op in {"add", "mul"}; the views (shape, strides in elements, stride 0 =
    broadcast) are taken over the flat fp32 arrays a_base and b_base."""
    a_base, b_base = _f32(a_base).reshape(-1), _f32(b_base).reshape(-1)
    nd = len(shape)
    assert all(s >= 0 for s in sa) and all(s >= 0 for s in sb)
    assert sum((n - 1) * s for n, s in zip(shape, sa)) < a_base.size
    assert sum((n - 1) * s for n, s in zip(shape, sb)) < b_base.size
    sh = (C.c_int64 * nd)(*shape)
    out = np.empty(tuple(shape), dtype=np.float64)
    lib().ref_eltwise_binary(_ptr(a_base), _ptr(b_base), nd, sh, (C.c_int64 * nd)(*sa), (C.c_int64 * nd)(*sb),
                             {"add": 0, "mul": 1}[op], 1 if relu_ else 0, _ptr(out))
    return out


MAP_BINARY = {"add": 0, "mul": 1, "sub": 2, "div": 3}
MAP_UNARY = {"relu": 0, "gelu": 1, "scale": 2, "sqrt": 3, "sin": 4, "cos": 5, "exp": 6, "tanh": 7, "sigmoid": 8, "relu6": 9,
             "abs": 10, "neg": 11, "square": 12, "log": 13, "silu": 14, "hardswish": 15}


def eltwise_map(a_base, shape, sa, unary=(), binary=None, b_base=None, sb=None, scale=1.0):
    """Elementwise chain on strided views (Table 1, Elementwise): v = a_view, or a_view `binary` b_view with
    binary in MAP_BINARY; then the steps named in `unary` (MAP_UNARY), in order ("scale" multiplies by the fp32
    constant `scale`).  Views are (shape, strides in elements, 0 = broadcast) over the flat fp32 arrays."""
    a_base = _f32(a_base).reshape(-1)
    nd = len(shape)
    assert all(s >= 0 for s in sa) and sum((n - 1) * s for n, s in zip(shape, sa)) < a_base.size
    if binary is None:
        b_base, sb, code = a_base, tuple(sa), -1
    else:
        b_base, code = _f32(b_base).reshape(-1), MAP_BINARY[binary]
        assert all(s >= 0 for s in sb) and sum((n - 1) * s for n, s in zip(shape, sb)) < b_base.size
    un = (C.c_int32 * max(1, len(unary)))(*[MAP_UNARY[u] for u in unary])
    out = np.empty(tuple(shape), dtype=np.float64)
    lib().ref_eltwise_map(_ptr(a_base), _ptr(b_base), nd, (C.c_int64 * nd)(*shape), (C.c_int64 * nd)(*sa),
                          (C.c_int64 * nd)(*sb), code, len(unary), un, C.c_float(scale), _ptr(out))
    return out


REDUCE_OPS = {"sum": 0, "mean": 1, "argmax": 2, "argmin": 3, "max": 4, "min": 5}


def reduce_axis(base, shape, stride, axis, op, want_abs=False):
    """Reduction `op` in {"sum","mean","argmax","argmin","max","min"} over dim `axis` of the strided view
    (shape, stride in elements) of the flat fp32 array `base`.  Returns fp64 values (and the
    sum of magnitudes with want_abs) for sum / mean / max / min, int64 indices for the arg-reductions."""
    base = _f32(base).reshape(-1)
    nd = len(shape)
    assert 0 <= axis < nd
    top = sum((n - 1) * s for n, s in zip(shape, stride))
    assert all(s >= 0 for s in stride) and top < base.size
    sh = (C.c_int64 * nd)(*shape)
    st = (C.c_int64 * nd)(*stride)
    oshape = tuple(n for d, n in enumerate(shape) if d != axis)
    code = REDUCE_OPS[op]
    if code <= 1 or code >= 4:
        val = np.empty(oshape, dtype=np.float64)
        ab = np.empty(oshape, dtype=np.float64) if want_abs and code <= 1 else None
        lib().ref_reduce_axis(_ptr(base), nd, sh, st, axis, code, _ptr(val), _ptr(ab), None)
        return (val, ab) if want_abs else val
    idx = np.empty(oshape, dtype=np.int64)
    lib().ref_reduce_axis(_ptr(base), nd, sh, st, axis, code, None, None, _ptr(idx))
    return idx


# -------------------------------------------------------------------- chains
def chain1(X, W, bias):
    """softmax_rows(relu(X @ W + bias))"""
    return softmax_rows(relu(gemm_bias(X, W, bias)))


def chain2(X, scale, shift, R):
    """avgpool_hw(relu(X * scale[c] + shift[c]) + R)"""
    return avgpool_hw(affine_relu_residual(X, scale, shift, R))


def chain3(X, gamma, beta, eps=1e-5):
    """gelu_tanh(layernorm(X) * gamma + beta)"""
    return gelu_tanh(layernorm_rows(X, gamma, beta, eps))


def chain4(inp, wt, bias, stride=1, pad=1):
    """relu(conv2d(inp, wt) + bias) and the contraction's normaliser."""
    out, Dn = conv2d_nchw_bias(inp, wt, bias, stride, pad, want_norm=True)
    return relu(out), Dn


def chain5(Q, K, V, scale=0.125):
    """softmax(scale * Q K^T) V and the second contraction's normaliser."""
    return attention(Q, K, V, scale, want_norm=True)


def chain6(X, W, bias, p, seed, stop_after="softmax"):
    """[Matmul, Dropout, Mean, Softmax] of Section 5.3: dropout(X @ W + bias), mean over the
    feature axis (one value per row), softmax over those M values.  `stop_after` in
    {"dropout", "mean", "softmax"} returns the intermediate of that name."""
    Z = dropout_hash(gemm_bias(X, W, bias), p, seed)
    if stop_after == "dropout":
        return Z
    mu = mean_rows(Z)
    if stop_after == "mean":
        return mu
    return softmax_rows(mu.reshape(1, -1)).reshape(-1)


def chain7(inp, wt, bias, scale, shift, stride=1, pad=1, relu_=True, pool=True, dil=1):
    """VGG-style block: maxpool2x2(relu((conv2d(inp, wt) + bias) * scale[k] + shift[k])) and the
    contraction normaliser of the conv output scaled by |scale[k]| (before pooling)."""
    out, Dn = conv2d_nchw_bias(inp, wt, bias, stride, pad, want_norm=True, dil=dil)
    if scale is not None or shift is not None:
        out = scale_shift_ch(out, scale, shift)
        Dn = scale_shift_ch(Dn, None if scale is None else np.abs(_f32(scale)), None if shift is None else np.abs(_f32(shift)))
    if relu_:
        out = relu(out)
    if pool:
        out = maxpool2x2(out)
    return out, Dn
