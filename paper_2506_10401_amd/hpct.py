"""ctypes binding of the C-ABI operator library (include/hpct.h).

Argument marshalling only: every function here fills an op descriptor, creates
(and caches) a plan and launches it; all arithmetic runs in the HIP kernels of
libhpct.so.  PyTorch is used for device memory (`data_ptr()`) and for the
current stream handle, nothing else.  There is no CPU fallback: if the library
is missing and cannot be built, or no GPU is present at launch, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhpct.so")

# ---- enums (mirror include/hpct.h) -------------------------------------------
HPCT_OK, HPCT_ERR_NULL, HPCT_ERR_BAD_DESC, HPCT_ERR_SHAPE_MISMATCH, HPCT_ERR_ALIGNMENT, \
    HPCT_ERR_UNSUPPORTED, HPCT_ERR_WORKSPACE, HPCT_ERR_HIP = range(8)
STATUS_NAMES = ["HPCT_OK", "HPCT_ERR_NULL", "HPCT_ERR_BAD_DESC", "HPCT_ERR_SHAPE_MISMATCH", "HPCT_ERR_ALIGNMENT",
                "HPCT_ERR_UNSUPPORTED", "HPCT_ERR_WORKSPACE", "HPCT_ERR_HIP"]
HPCT_F32, HPCT_I32 = 0, 1
HPCT_ANCHOR_NONE, HPCT_ANCHOR_GEMM, HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM, HPCT_ANCHOR_CONV2D_NCHW, \
    HPCT_ANCHOR_CONVT2D_NCHW = range(5)
HPCT_EPI_BIAS_COL, HPCT_EPI_SCALE_SHIFT_CH, HPCT_EPI_RELU, HPCT_EPI_ADD_RESIDUAL, HPCT_EPI_GELU_TANH, \
    HPCT_EPI_SCALE_CONST, HPCT_EPI_DROPOUT_HASH, HPCT_EPI_CAUSAL_MASK, HPCT_EPI_ADD_TENSOR, HPCT_EPI_MUL_TENSOR, \
    HPCT_EPI_SUB_TENSOR, HPCT_EPI_DIV_TENSOR, HPCT_EPI_SQRT, HPCT_EPI_SIN, HPCT_EPI_COS, HPCT_EPI_EXP, HPCT_EPI_TANH, \
    HPCT_EPI_SIGMOID, HPCT_EPI_RELU6, HPCT_EPI_ABS, HPCT_EPI_NEG, HPCT_EPI_SQUARE, HPCT_EPI_LOG, HPCT_EPI_SILU, HPCT_EPI_HARDSWISH = range(25)
HPCT_RED_NONE, HPCT_RED_SOFTMAX_LAST, HPCT_RED_LAYERNORM_LAST, HPCT_RED_AVGPOOL_HW, HPCT_RED_MEAN_LAST, \
    HPCT_RED_MAXPOOL2_HW, HPCT_RED_SUM_AXIS, HPCT_RED_MEAN_AXIS, HPCT_RED_ARGMAX_AXIS, HPCT_RED_ARGMIN_AXIS, HPCT_RED_MAX_AXIS, \
    HPCT_RED_MIN_AXIS, HPCT_RED_MAXPOOL_HW, HPCT_RED_GROUPNORM_NCHW, HPCT_RED_AVGPOOL_WIN_HW, HPCT_RED_RMSNORM_LAST = range(16)
HPCT_MAX_DIMS, HPCT_MAX_EPI, HPCT_MAX_IN, HPCT_MAX_OUT = 6, 8, 8, 2


class TensorDesc(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("shape", C.c_int64 * HPCT_MAX_DIMS), ("stride", C.c_int64 * HPCT_MAX_DIMS),
                ("dtype", C.c_int)]


class OpDesc(C.Structure):
    _fields_ = [("anchor", C.c_int), ("n_epi", C.c_int32), ("epi", C.c_int * HPCT_MAX_EPI), ("reduce", C.c_int),
                ("reduce_before_epi", C.c_int32), ("n_in", C.c_int32), ("in_", TensorDesc * HPCT_MAX_IN),
                ("n_out", C.c_int32), ("out", TensorDesc * HPCT_MAX_OUT), ("stride_hw", C.c_int32 * 2),
                ("pad_hw", C.c_int32 * 2), ("eps", C.c_float), ("scale", C.c_float), ("dropout_p", C.c_float),
                ("reduce2", C.c_int), ("dropout_seed", C.c_uint64), ("axis", C.c_int32), ("dilation_hw", C.c_int32 * 2), ("groups", C.c_int32),
                ("window_hw", C.c_int32 * 2)]


class HpctError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, message))
        self.status = status
        self.message = message


_lib = None


def load(path: Optional[str] = None):
    """Load libhpct.so (building it first if it has never been built)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    # torch first: its wheel carries a HIP runtime of its own, and the library must bind to the one that owns the
    # tensors and streams it is handed (loaded in the other order, the two runtimes do not see each other's device)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp = C.c_void_p
    lib.hpct_plan_create.argtypes = [C.POINTER(OpDesc), C.POINTER(vp)]
    lib.hpct_plan_create.restype = C.c_int
    lib.hpct_plan_workspace_bytes.argtypes = [vp]
    lib.hpct_plan_workspace_bytes.restype = C.c_size_t
    lib.hpct_plan_launch.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, C.c_size_t, vp]
    lib.hpct_plan_launch.restype = C.c_int
    lib.hpct_plan_launch_noalloc.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    lib.hpct_plan_launch_noalloc.restype = C.c_int
    lib.hpct_plan_destroy.argtypes = [vp]
    lib.hpct_plan_destroy.restype = None
    lib.hpct_plan_kernel_name.argtypes = [vp]
    lib.hpct_plan_kernel_name.restype = C.c_char_p
    lib.hpct_plan_launch_shape.argtypes = [vp, C.POINTER(C.c_uint32 * 3), C.POINTER(C.c_uint32 * 3), C.POINTER(C.c_uint32)]
    lib.hpct_plan_launch_shape.restype = C.c_int
    lib.hpct_last_error.argtypes = []
    lib.hpct_last_error.restype = C.c_char_p
    lib.hpct_version.argtypes = []
    lib.hpct_version.restype = C.c_char_p
    for fn in (lib.hpct_sizeof_tensor_desc, lib.hpct_sizeof_op_desc):
        fn.argtypes, fn.restype = [], C.c_size_t
    if lib.hpct_sizeof_tensor_desc() != C.sizeof(TensorDesc) or lib.hpct_sizeof_op_desc() != C.sizeof(OpDesc):
        raise RuntimeError("libhpct.so was built from another version of include/hpct.h than this binding mirrors")
    _lib = lib
    return lib


def hpct_version() -> str:
    return load().hpct_version().decode()


def hpct_last_error() -> str:
    return load().hpct_last_error().decode()


def tensor_desc(shape: Sequence[int], stride: Optional[Sequence[int]] = None, dtype: int = HPCT_F32) -> TensorDesc:
    t = TensorDesc()
    t.ndim = len(shape)
    if stride is None:
        stride, acc = [], 1
        for s in reversed(shape):
            stride.insert(0, acc)
            acc *= s
    for i, (s, st) in enumerate(zip(shape, stride)):
        if i < HPCT_MAX_DIMS:
            t.shape[i], t.stride[i] = s, st
    t.dtype = dtype
    return t


def op_desc(anchor=HPCT_ANCHOR_NONE, epi=(), reduce=HPCT_RED_NONE, reduce_before_epi=0, inputs=(), outputs=(),
            stride_hw=(1, 1), pad_hw=(0, 0), eps=0.0, scale=1.0, dropout_p=0.0, dropout_seed=0,
            reduce2=HPCT_RED_NONE, axis=0, dilation_hw=(1, 1), groups=0, window_hw=(0, 0)) -> OpDesc:
    d = OpDesc()
    d.anchor = anchor
    d.n_epi = len(epi)
    for i, e in enumerate(epi[:HPCT_MAX_EPI]):
        d.epi[i] = e
    d.reduce = reduce
    d.reduce_before_epi = reduce_before_epi
    d.n_in = len(inputs)
    for i, t in enumerate(inputs[:HPCT_MAX_IN]):
        d.in_[i] = t if isinstance(t, TensorDesc) else tensor_desc(t)
    d.n_out = len(outputs)
    for i, t in enumerate(outputs[:HPCT_MAX_OUT]):
        d.out[i] = t if isinstance(t, TensorDesc) else tensor_desc(t)
    d.stride_hw[0], d.stride_hw[1] = stride_hw
    d.pad_hw[0], d.pad_hw[1] = pad_hw
    d.eps = eps
    d.scale = scale
    d.dropout_p = dropout_p
    d.dropout_seed = int(dropout_seed) & 0xFFFFFFFFFFFFFFFF
    d.reduce2 = reduce2
    d.axis = axis
    d.dilation_hw[0], d.dilation_hw[1] = dilation_hw
    d.groups = groups
    d.window_hw[0], d.window_hw[1] = window_hw
    return d


class Plan:
    """Owns one hpct_plan."""

    def __init__(self, desc: OpDesc):
        lib = load()
        h = C.c_void_p()
        st = lib.hpct_plan_create(C.byref(desc), C.byref(h))
        if st != HPCT_OK:
            raise HpctError(st, lib.hpct_last_error().decode())
        self._h = h
        self.n_in, self.n_out = desc.n_in, desc.n_out

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.hpct_plan_destroy(h)

    @property
    def kernel_name(self) -> str:
        return load().hpct_plan_kernel_name(self._h).decode()

    @property
    def workspace_bytes(self) -> int:
        return int(load().hpct_plan_workspace_bytes(self._h))

    def launch_shape(self) -> Tuple[Tuple[int, ...], Tuple[int, ...], int]:
        g, b, l = (C.c_uint32 * 3)(), (C.c_uint32 * 3)(), C.c_uint32()
        st = load().hpct_plan_launch_shape(self._h, C.byref(g), C.byref(b), C.byref(l))
        if st != HPCT_OK:
            raise HpctError(st, hpct_last_error())
        return tuple(g), tuple(b), int(l.value)

    def launch_ptrs(self, in_ptrs: Sequence[int], out_ptrs: Sequence[int], stream: int = 0,
                    workspace: int = 0, workspace_bytes: int = 0) -> None:
        ins = (C.c_void_p * max(1, len(in_ptrs)))(*in_ptrs)
        outs = (C.c_void_p * max(1, len(out_ptrs)))(*out_ptrs)
        st = load().hpct_plan_launch(self._h, ins, outs, C.c_void_p(workspace), workspace_bytes, C.c_void_p(stream))
        if st != HPCT_OK:
            raise HpctError(st, hpct_last_error())

    def bind(self, inputs, outputs, stream=None, workspace=None):
        """Marshal the pointer arrays once and return a zero-argument callable
        that enqueues this plan on `stream` (default: the stream current now).
        For launch loops where per-call Python overhead matters."""
        import torch
        for t in list(inputs) + list(outputs):
            if not t.is_cuda or (t.dtype != torch.float32 and not (t.dtype == torch.int32 and any(t is o for o in outputs))):
                raise HpctError(HPCT_ERR_BAD_DESC, "operands must be fp32 tensors (int32 for index outputs) in GPU memory")
        lib = load()
        ins = (C.c_void_p * max(1, len(inputs)))(*[t.data_ptr() for t in inputs])
        outs = (C.c_void_p * max(1, len(outputs)))(*[t.data_ptr() for t in outputs])
        s = C.c_void_p(torch.cuda.current_stream().cuda_stream if stream is None else stream)
        if workspace is not None and (not workspace.is_cuda or not workspace.is_contiguous()):
            raise HpctError(HPCT_ERR_BAD_DESC, "the workspace must be a contiguous tensor in GPU memory")
        ws = C.c_void_p(workspace.data_ptr()) if workspace is not None else None
        ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        h, fn, keep = self._h, lib.hpct_plan_launch, (list(inputs), list(outputs), workspace, self)

        def go(_keep=keep):
            st = fn(h, ins, outs, ws, ws_bytes, s)
            if st != HPCT_OK:
                raise HpctError(st, hpct_last_error())
        return go

    def launch(self, inputs, outputs, stream=None, workspace=None) -> None:
        """inputs / outputs: torch tensors on the GPU (fp32, laid out as described);
        workspace: a contiguous GPU tensor of at least `workspace_bytes` bytes when the plan needs one."""
        import torch
        for t in list(inputs) + list(outputs):
            if not t.is_cuda or (t.dtype != torch.float32 and not (t.dtype == torch.int32 and any(t is o for o in outputs))):
                raise HpctError(HPCT_ERR_BAD_DESC, "operands must be fp32 tensors (int32 for index outputs) in GPU memory")
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        if workspace is not None and (not workspace.is_cuda or not workspace.is_contiguous()):
            raise HpctError(HPCT_ERR_BAD_DESC, "the workspace must be a contiguous tensor in GPU memory")
        self.launch_ptrs([t.data_ptr() for t in inputs], [t.data_ptr() for t in outputs], s,
                         workspace.data_ptr() if workspace is not None else 0,
                         workspace.numel() * workspace.element_size() if workspace is not None else 0)


    def launch_noalloc(self, inputs, outputs, stream=None) -> None:
        """hpct_plan_launch_noalloc: the same launch with the library's built-in scratch array for a workspace (no
        allocation anywhere; refused when the plan needs more than NOALLOC_SCRATCH_BYTES)."""
        import torch
        for t in list(inputs) + list(outputs):
            if not t.is_cuda or (t.dtype != torch.float32 and not (t.dtype == torch.int32 and any(t is o for o in outputs))):
                raise HpctError(HPCT_ERR_BAD_DESC, "operands must be fp32 tensors (int32 for index outputs) in GPU memory")
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        ins = (C.c_void_p * max(1, len(inputs)))(*[t.data_ptr() for t in inputs])
        outs = (C.c_void_p * max(1, len(outputs)))(*[t.data_ptr() for t in outputs])
        st = load().hpct_plan_launch_noalloc(self._h, ins, outs, C.c_void_p(s))
        if st != HPCT_OK:
            raise HpctError(st, hpct_last_error())


NOALLOC_SCRATCH_BYTES = 4 << 20   # HPCT_NOALLOC_SCRATCH_BYTES of include/hpct.h

_plans: Dict[tuple, Plan] = {}


def _cached(key: tuple, make) -> Plan:
    p = _plans.get(key)
    if p is None:
        p = _plans[key] = Plan(make())
    return p


def _sh(t) -> Tuple[int, ...]:
    return tuple(int(s) for s in t.shape)


# ---- the five chains ---------------------------------------------------------
# Each chain has a *_plan function (descriptor -> cached Plan plus the operand
# list in descriptor order) and a convenience function that launches it.
def _activation(relu):
    """the epilogue list for an activation argument: False / None, True (= "relu"), "relu", "relu6", "gelu", "sigmoid", "tanh" """
    return {False: [], None: [], True: [HPCT_EPI_RELU], "relu": [HPCT_EPI_RELU], "relu6": [HPCT_EPI_RELU6],
            "gelu": [HPCT_EPI_GELU_TANH], "sigmoid": [HPCT_EPI_SIGMOID], "tanh": [HPCT_EPI_TANH]}[relu]


def gemm_bias_relu_softmax_plan(X, W, bias, out, relu=True, softmax=True, scale=None):
    """X [M,K] or a batch [B,M,K], row-major or any strided view (e.g. the .t() of a [K,M] tensor: it is then first
    copied to the plan's workspace as a row-major matrix); W [K,N] row-major, the .t() view of an [N,K] row-major tensor (a linear
    layer's weight), or one such matrix per batch [B,K,N].  `scale`: constant multiplied in after the bias (the
    Gemm-Scale operator), None = no such step.  relu: False, True, or the name of another activation:
    "relu6", "gelu", "sigmoid", "tanh"."""
    wst = tuple(int(v) for v in W.stride())
    xst = tuple(int(v) for v in X.stride())
    act = _activation(relu)
    epi = ([HPCT_EPI_BIAS_COL] if bias is not None else []) + ([HPCT_EPI_SCALE_CONST] if scale is not None else []) + act
    ins = [X, W] + ([bias] if bias is not None else [])
    descs = [tensor_desc(_sh(X), xst), tensor_desc(_sh(W), wst)] + ([_sh(bias)] if bias is not None else [])
    plan = _cached(("gemm", _sh(X), xst, _sh(W), wst, tuple(epi), softmax, scale), lambda: op_desc(
        HPCT_ANCHOR_GEMM, epi, HPCT_RED_SOFTMAX_LAST if softmax else HPCT_RED_NONE, 0, descs, [_sh(out)],
        scale=1.0 if scale is None else scale))
    return plan, ins


def gemm_bias_relu_softmax(X, W, bias, out, relu=True, softmax=True, workspace=None, stream=None, scale=None) -> None:
    """out = softmax_rows(relu((X @ W + bias) * scale)); relu / softmax / bias / scale optional.  `workspace`: GPU
    tensor of at least plan.workspace_bytes bytes when that is not 0 (small outputs with a long K are computed in
    K slices)."""
    plan, ins = gemm_bias_relu_softmax_plan(X, W, bias, out, relu, softmax, scale)
    plan.launch(ins, [out], stream, workspace)


def matmul_dropout_mean_softmax_plan(X, W, bias, out, p, seed, stop_after="softmax", relu=False):
    """Plan of the [Matmul, Dropout, Mean, Softmax] group; `stop_after` in {"dropout", "mean", "softmax"}
    ends the chain there (out is [M,N], [M], [M])."""
    M, K = _sh(X)
    N = _sh(W)[1]
    epi = ([HPCT_EPI_BIAS_COL] if bias is not None else []) + ([HPCT_EPI_RELU] if relu else []) + [HPCT_EPI_DROPOUT_HASH]
    ins = [X, W] + ([bias] if bias is not None else [])
    red = HPCT_RED_NONE if stop_after == "dropout" else HPCT_RED_MEAN_LAST
    red2 = HPCT_RED_SOFTMAX_LAST if stop_after == "softmax" else HPCT_RED_NONE
    plan = _cached(("mdms", M, K, N, tuple(epi), float(p), int(seed), stop_after), lambda: op_desc(
        HPCT_ANCHOR_GEMM, epi, red, 0, [_sh(t) for t in ins], [_sh(out)], dropout_p=p, dropout_seed=seed, reduce2=red2))
    return plan, ins


def matmul_dropout_mean_softmax(X, W, bias, out, p, seed, workspace=None, stop_after="softmax", relu=False, stream=None) -> None:
    """out[M] = softmax over the M values mean_n(dropout(X @ W + bias)[m, n]) (Section 5.3 case study).
    `workspace`: GPU tensor of at least plan.workspace_bytes bytes (needed once the chain contains the mean)."""
    plan, ins = matmul_dropout_mean_softmax_plan(X, W, bias, out, p, seed, stop_after, relu)
    plan.launch(ins, [out], stream, workspace)


def scale_shift_relu_add_pool_plan(X, scale, shift, R, out, relu=True, pool=True):
    epi = ([HPCT_EPI_SCALE_SHIFT_CH] if scale is not None else []) + ([HPCT_EPI_RELU] if relu else []) + \
          ([HPCT_EPI_ADD_RESIDUAL] if R is not None else [])
    ins = [X] + ([scale, shift] if scale is not None else []) + ([R] if R is not None else [])
    plan = _cached(("affine", _sh(X), tuple(epi), pool), lambda: op_desc(
        HPCT_ANCHOR_NONE, epi, HPCT_RED_AVGPOOL_HW if pool else HPCT_RED_NONE, 0, [_sh(t) for t in ins], [_sh(out)]))
    return plan, ins


def scale_shift_relu_add_pool(X, scale, shift, R, out, relu=True, pool=True, stream=None) -> None:
    """out[n,c] = mean_hw(relu(X*scale[c]+shift[c]) + R)  (pool=False: the full tensor)."""
    plan, ins = scale_shift_relu_add_pool_plan(X, scale, shift, R, out, relu, pool)
    plan.launch(ins, [out], stream)


def layernorm_gelu_plan(X, gamma, beta, out, eps=1e-5, gelu=True):
    ins = [X] + ([gamma, beta] if gamma is not None else [])
    plan = _cached(("ln", _sh(X), gamma is not None, float(eps), gelu), lambda: op_desc(
        HPCT_ANCHOR_NONE, [HPCT_EPI_GELU_TANH] if gelu else [], HPCT_RED_LAYERNORM_LAST, 1,
        [_sh(t) for t in ins], [_sh(out)], eps=eps))
    return plan, ins


def layernorm_gelu(X, gamma, beta, out, eps=1e-5, gelu=True, stream=None) -> None:
    """out = gelu_tanh(layernorm(X) * gamma + beta)."""
    plan, ins = layernorm_gelu_plan(X, gamma, beta, out, eps, gelu)
    plan.launch(ins, [out], stream)


def softmax_rows_plan(X, out):
    plan = _cached(("softmax", _sh(X)), lambda: op_desc(HPCT_ANCHOR_NONE, [], HPCT_RED_SOFTMAX_LAST, 0, [_sh(X)], [_sh(out)]))
    return plan, [X]


def softmax_rows(X, out, stream=None) -> None:
    """out = softmax over the last dim of the 2-D tensor X."""
    plan, ins = softmax_rows_plan(X, out)
    plan.launch(ins, [out], stream)


def layout_transform_plan(x_view, out):
    """x_view: a (possibly non-contiguous) fp32 GPU tensor view; out: contiguous, same shape."""
    shape, stride = _sh(x_view), tuple(int(v) for v in x_view.stride())
    plan = _cached(("layout", shape, stride), lambda: op_desc(
        HPCT_ANCHOR_NONE, [], HPCT_RED_NONE, 0, [tensor_desc(shape, stride)], [_sh(out)]))
    return plan, [x_view]


def layout_transform(x_view, out, stream=None) -> None:
    """out = contiguous copy of the strided view x_view (transpose, NCHW <-> NHWC, slices, broadcasts)."""
    plan, ins = layout_transform_plan(x_view, out)
    plan.launch(ins, [out], stream)


def maxpool2x2_plan(X, out):
    plan = _cached(("maxpool2", _sh(X)), lambda: op_desc(HPCT_ANCHOR_NONE, [], HPCT_RED_MAXPOOL2_HW, 0, [_sh(X)], [_sh(out)]))
    return plan, [X]


def maxpool2x2(X, out, stream=None) -> None:
    """out[n,c,y,x] = max of the 2x2 window of X[n,c] at (2y, 2x); odd trailing rows / columns are dropped."""
    plan, ins = maxpool2x2_plan(X, out)
    plan.launch(ins, [out], stream)


def rmsnorm_plan(X, gamma, out, eps=1e-6):
    ins = [X] + ([gamma] if gamma is not None else [])
    plan = _cached(("rmsnorm", _sh(X), eps, gamma is not None), lambda: op_desc(
        HPCT_ANCHOR_NONE, [], HPCT_RED_RMSNORM_LAST, 0, [_sh(t) for t in ins], [_sh(out)], eps=eps))
    return plan, ins


def rmsnorm(X, gamma, out, eps=1e-6, stream=None) -> None:
    """out = X / sqrt(mean(X^2 over the last dim) + eps) * gamma (gamma may be None)."""
    plan, ins = rmsnorm_plan(X, gamma, out, eps)
    plan.launch(ins, [out], stream)


def groupnorm_plan(X, gamma, beta, out, groups, eps=1e-5, relu=False):
    """Group normalisation of X[N,C,H,W] (groups = C: instance normalisation) with per-channel gamma / beta (both or
    neither) and an optional ReLU behind it."""
    assert (gamma is None) == (beta is None)
    ins = [X] + ([gamma, beta] if gamma is not None else [])
    plan = _cached(("groupnorm", _sh(X), groups, eps, relu, gamma is not None), lambda: op_desc(
        HPCT_ANCHOR_NONE, [HPCT_EPI_RELU] if relu else [], HPCT_RED_GROUPNORM_NCHW, 1, [_sh(t) for t in ins], [_sh(out)],
        eps=eps, groups=groups))
    return plan, ins


def groupnorm(X, gamma, beta, out, groups, eps=1e-5, relu=False, stream=None) -> None:
    plan, ins = groupnorm_plan(X, gamma, beta, out, groups, eps, relu)
    plan.launch(ins, [out], stream)


def maxpool_plan(X, out, window, stride, pad=0):
    plan = _cached(("maxpool", _sh(X), window, stride, pad), lambda: op_desc(
        HPCT_ANCHOR_NONE, [], HPCT_RED_MAXPOOL_HW, 0, [_sh(X)], [_sh(out)], stride_hw=(stride, stride), pad_hw=(pad, pad),
        window_hw=(window, window)))
    return plan, [X]


def avgpool_plan(X, out, window, stride, pad=0):
    plan = _cached(("avgpool", _sh(X), window, stride, pad), lambda: op_desc(
        HPCT_ANCHOR_NONE, [], HPCT_RED_AVGPOOL_WIN_HW, 0, [_sh(X)], [_sh(out)], stride_hw=(stride, stride), pad_hw=(pad, pad),
        window_hw=(window, window)))
    return plan, [X]


def avgpool(X, out, window, stride, pad=0, stream=None) -> None:
    """out[n,c,y,x] = mean of the window x window positions of X[n,c] from (y stride - pad, x stride - pad), positions
    outside the image counting as zeros (divisor window * window); extents as maxpool."""
    plan, ins = avgpool_plan(X, out, window, stride, pad)
    plan.launch(ins, [out], stream)


def maxpool(X, out, window, stride, pad=0, stream=None) -> None:
    """out[n,c,y,x] = max of the window x window positions of X[n,c] from (y stride - pad, x stride - pad) that lie
    inside the image (pad < window); out extents (H + 2 pad - window) // stride + 1."""
    plan, ins = maxpool_plan(X, out, window, stride, pad)
    plan.launch(ins, [out], stream)


_MAP_BINARY = {"add": HPCT_EPI_ADD_TENSOR, "mul": HPCT_EPI_MUL_TENSOR, "sub": HPCT_EPI_SUB_TENSOR, "div": HPCT_EPI_DIV_TENSOR}
_MAP_UNARY = {"relu": HPCT_EPI_RELU, "gelu": HPCT_EPI_GELU_TANH, "scale": HPCT_EPI_SCALE_CONST, "sqrt": HPCT_EPI_SQRT,
              "sin": HPCT_EPI_SIN, "cos": HPCT_EPI_COS, "exp": HPCT_EPI_EXP, "tanh": HPCT_EPI_TANH,
              "sigmoid": HPCT_EPI_SIGMOID, "relu6": HPCT_EPI_RELU6, "abs": HPCT_EPI_ABS, "neg": HPCT_EPI_NEG,
              "square": HPCT_EPI_SQUARE, "log": HPCT_EPI_LOG, "silu": HPCT_EPI_SILU, "hardswish": HPCT_EPI_HARDSWISH}


def eltwise_map_plan(a_view, out, unary=(), binary=None, b_view=None, scale=1.0):
    """Elementwise chain: a_view [binary b_view], then the steps of `unary` in order.  Views: fp32 GPU tensor views
    of one shape (expand() for broadcasting); out: contiguous, same shape; `scale` is the constant of "scale"."""
    shape = _sh(a_view)
    sa = tuple(int(v) for v in a_view.stride())
    ins, descs, epi = [a_view], [tensor_desc(shape, sa)], []
    sb = None
    if binary is not None:
        sb = tuple(int(v) for v in b_view.stride())
        ins.append(b_view)
        descs.append(tensor_desc(_sh(b_view), sb))
        epi.append(_MAP_BINARY[binary])
    epi += [_MAP_UNARY[u] for u in unary]
    plan = _cached(("eltwise", shape, sa, sb, binary, tuple(unary), float(scale)), lambda: op_desc(
        HPCT_ANCHOR_NONE, epi, HPCT_RED_NONE, 0, descs, [_sh(out)], scale=scale))
    return plan, ins


def eltwise_map(a_view, out, unary=(), binary=None, b_view=None, scale=1.0, stream=None) -> None:
    """out = steps(a_view binary b_view) or steps(a_view); binary in {"add","mul","sub","div"}, steps from
    {"relu","gelu","scale","sqrt","sin","cos","exp","tanh","sigmoid"}."""
    plan, ins = eltwise_map_plan(a_view, out, unary, binary, b_view, scale)
    plan.launch(ins, [out], stream)


def eltwise_plan(a_view, b_view, out, op, relu=False):
    """out = [relu](a_view op b_view): the two-operand case of eltwise_map_plan."""
    return eltwise_map_plan(a_view, out, ("relu",) if relu else (), op, b_view)


def eltwise(a_view, b_view, out, op, relu=False, stream=None) -> None:
    """out = [relu](a_view op b_view); op in {"add", "mul", "sub", "div"}."""
    plan, ins = eltwise_plan(a_view, b_view, out, op, relu)
    plan.launch(ins, [out], stream)


_REDUCE_OPS = {"sum": HPCT_RED_SUM_AXIS, "mean": HPCT_RED_MEAN_AXIS, "argmax": HPCT_RED_ARGMAX_AXIS,
               "argmin": HPCT_RED_ARGMIN_AXIS, "max": HPCT_RED_MAX_AXIS, "min": HPCT_RED_MIN_AXIS}


def reduce_axis_plan(x_view, out, axis, op):
    """x_view: a (possibly non-contiguous) fp32 GPU tensor view; out: contiguous, x_view's shape without dim
    `axis` (shape [1] for a 1-D input); fp32 for op "sum" / "mean" / "max" / "min", int32 for "argmax" / "argmin"."""
    shape, stride = _sh(x_view), tuple(int(v) for v in x_view.stride())
    arg = op in ("argmax", "argmin")
    plan = _cached(("reduce", shape, stride, axis, op), lambda: op_desc(
        HPCT_ANCHOR_NONE, [], _REDUCE_OPS[op], 0, [tensor_desc(shape, stride)],
        [tensor_desc(_sh(out), None, HPCT_I32 if arg else HPCT_F32)], axis=axis))
    return plan, [x_view]


def reduce_axis(x_view, out, axis, op, workspace=None, stream=None) -> None:
    """out = sum / mean / max / min / argmax / argmin of x_view over dim `axis` (ties of the arg ops go to the lowest index).
    `workspace`: GPU tensor of at least plan.workspace_bytes bytes when that is not 0."""
    plan, ins = reduce_axis_plan(x_view, out, axis, op)
    plan.launch(ins, [out], stream, workspace)


def conv2d_bias_relu_plan(inp, wt, bias, out, stride=1, pad=1, relu=True):
    epi = ([HPCT_EPI_BIAS_COL] if bias is not None else []) + ([HPCT_EPI_RELU] if relu else [])
    ins = [inp, wt] + ([bias] if bias is not None else [])
    plan = _cached(("conv", _sh(inp), _sh(wt), tuple(epi), stride, pad), lambda: op_desc(
        HPCT_ANCHOR_CONV2D_NCHW, epi, HPCT_RED_NONE, 0, [_sh(t) for t in ins], [_sh(out)],
        stride_hw=(stride, stride), pad_hw=(pad, pad)))
    return plan, ins


def conv2d_bias_relu(inp, wt, bias, out, stride=1, pad=1, relu=True, stream=None) -> None:
    """out = relu(conv2d_nchw(inp, wt) + bias[k])."""
    plan, ins = conv2d_bias_relu_plan(inp, wt, bias, out, stride, pad, relu)
    plan.launch(ins, [out], stream)


def conv_block_plan(inp, wt, bias, scale, shift, out, stride=1, pad=1, relu=True, pool=True, dilation=1, groups=1):
    """Plan of conv2d [+bias] [+per-channel scale/shift] [+relu] [+2x2 max pool] (a VGG-style block).
    relu: False, True, or "relu6"; groups: 1 (dense) or the channel count (depthwise, wt [C,1,R,R], no pooling)."""
    assert (scale is None) == (shift is None)
    act = _activation(relu)
    epi = ([HPCT_EPI_BIAS_COL] if bias is not None else []) + ([HPCT_EPI_SCALE_SHIFT_CH] if scale is not None else []) + act
    ins = [inp, wt] + ([bias] if bias is not None else []) + ([scale, shift] if scale is not None else [])
    plan = _cached(("convblock", _sh(inp), _sh(wt), tuple(epi), stride, pad, pool, dilation, groups), lambda: op_desc(
        HPCT_ANCHOR_CONV2D_NCHW, epi, HPCT_RED_MAXPOOL2_HW if pool else HPCT_RED_NONE, 0, [_sh(t) for t in ins], [_sh(out)],
        stride_hw=(stride, stride), pad_hw=(pad, pad), dilation_hw=(dilation, dilation), groups=groups))
    return plan, ins


def conv_block(inp, wt, bias, scale, shift, out, stride=1, pad=1, relu=True, pool=True, dilation=1, stream=None,
               groups=1) -> None:
    """out = maxpool2x2(relu((conv2d_nchw(inp, wt) + bias[k]) * scale[k] + shift[k])); every stage after the conv optional."""
    plan, ins = conv_block_plan(inp, wt, bias, scale, shift, out, stride, pad, relu, pool, dilation, groups)
    plan.launch(ins, [out], stream)


def conv_transpose_plan(inp, wt, bias, scale, shift, out, stride=1, pad=0, relu=False, dilation=1):
    """Transposed conv (inp [N,C,H,W], wt [C,K,R,R], out [N,K,(H-1)*stride - 2*pad + (R-1)*dilation + 1, ...])
    [+bias] [+per-channel scale/shift] [+relu / "relu6"].  The plan needs a workspace (plan.workspace_bytes)."""
    assert (scale is None) == (shift is None)
    act = _activation(relu)
    epi = ([HPCT_EPI_BIAS_COL] if bias is not None else []) + ([HPCT_EPI_SCALE_SHIFT_CH] if scale is not None else []) + act
    ins = [inp, wt] + ([bias] if bias is not None else []) + ([scale, shift] if scale is not None else [])
    plan = _cached(("convt", _sh(inp), _sh(wt), tuple(epi), stride, pad, dilation), lambda: op_desc(
        HPCT_ANCHOR_CONVT2D_NCHW, epi, HPCT_RED_NONE, 0, [_sh(t) for t in ins], [_sh(out)],
        stride_hw=(stride, stride), pad_hw=(pad, pad), dilation_hw=(dilation, dilation)))
    return plan, ins


def conv_transpose(inp, wt, bias, scale, shift, out, workspace, stride=1, pad=0, relu=False, dilation=1, stream=None) -> None:
    plan, ins = conv_transpose_plan(inp, wt, bias, scale, shift, out, stride, pad, relu, dilation)
    plan.launch(ins, [out], stream, workspace)


def depthwise_conv_plan(inp, wt, bias, scale, shift, out, stride=1, pad=1, relu="relu6", dilation=1):
    """Depthwise conv (wt [C,1,R,R]) [+bias] [+per-channel scale/shift] [+relu / relu6]: the depthwise layer of a
    MobileNetV2 block."""
    return conv_block_plan(inp, wt, bias, scale, shift, out, stride, pad, relu, False, dilation, groups=_sh(inp)[1])


def depthwise_conv(inp, wt, bias, scale, shift, out, stride=1, pad=1, relu="relu6", dilation=1, stream=None) -> None:
    plan, ins = depthwise_conv_plan(inp, wt, bias, scale, shift, out, stride, pad, relu, dilation)
    plan.launch(ins, [out], stream)


def attention_plan(Q, K, V, out, scale=0.125, causal=False):
    epi = [HPCT_EPI_SCALE_CONST] + ([HPCT_EPI_CAUSAL_MASK] if causal else [])
    plan = _cached(("attn", _sh(Q), _sh(K), float(scale), causal), lambda: op_desc(
        HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM, epi, HPCT_RED_NONE, 0,
        [_sh(Q), _sh(K), _sh(V)], [_sh(out)], scale=scale))
    return plan, [Q, K, V]


def attention(Q, K, V, out, scale=0.125, causal=False, stream=None) -> None:
    """out = softmax(scale * Q K^T) V per batch; causal: query i attends keys j <= i only."""
    plan, ins = attention_plan(Q, K, V, out, scale, causal)
    plan.launch(ins, [out], stream)
