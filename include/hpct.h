/*
 * hpct - fused deep-learning tensor operators for AMD MI355X (gfx950).
 *
 * C ABI of the operator library.  One call describes a fused chain
 *     anchor contraction  ->  elementwise / broadcast epilogues  ->  row reduction
 * (operator classes of the paper's Table 1: ComputeIntensive "matmul, conv",
 * Elementwise "add, sub, mul, div, sqrt, sin, cos, relu", Reduction "sum, mean, softmax", LayoutTransform
 * "reshape, transpose"; fused examples
 * of its Section 5.3) with an op descriptor; the library validates it, picks a
 * hand-written HIP kernel and enqueues it on the caller's stream: one kernel per
 * launch; two or three for the plans that report a workspace (the later ones finish
 * a reduction from the partial results the first left there) and two for a GEMM with a
 * row softmax whose rows are wider than one work-group or whose output has so few rows
 * that the contraction is spread over many work-groups per row (the softmax then runs
 * in place on the stored result).
 *
 * Conventions
 *  - All tensors are fp32 (the index output of an arg-reduction is int32), described by
 *    shape and stride in ELEMENTS.
 *  - Every data pointer passed to hpct_plan_launch is a DEVICE pointer owned
 *    by the caller, 16-byte aligned (4-byte aligned suffices for a layout
 *    transform, an axis reduction or an elementwise chain on views, whose inputs may start anywhere).  Descriptors, plans and the pointer
 *    arrays themselves live in HOST memory.
 *  - The library never allocates, frees, copies or synchronises device memory.
 *    Inputs are never written.  Outputs must not overlap inputs.
 *  - Calls return a status; on failure hpct_last_error() gives a text for the
 *    calling thread.  No exception crosses the boundary.
 *  - Plans are immutable after creation and may be launched from several
 *    threads at once.
 *
 * Operand order in hpct_op_desc.in[] is execution order: the anchor's operands,
 * then the operands of each epilogue / reduction in the order they run.
 *
 *   chain                                             in[]                          out[0]
 *   GEMM [+BIAS_COL] [+SCALE_CONST] [+RELU]           X[M,K], W[K,N], bias[N]       [M,N]
 *         (in every GEMM chain RELU6, GELU_TANH,
 *         SIGMOID or TANH may stand for RELU)
 *         (X: any strided view; one that is not
 *         row-major is first copied to the workspace)
 *         [+DROPOUT_HASH] [+SOFTMAX_LAST] (one        (W row-major, strides (N,1),
 *         kernel for N <= 256 and many rows, else     or stored transposed as an
 *         the GEMM then an in-place row softmax)      [N,K] array: strides (1,K))
 *   GEMM [+BIAS_COL] [+SCALE_CONST] [+RELU]           X[B,M,K], W[B,K,N] (each      [B,M,N]
 *         [+SOFTMAX_LAST]: a batch of products,       W[b] row-major or transposed,
 *         Y[b] = X[b] W[b] (B <= 65535), or one       batch stride K N) or W[K,N],
 *         W for all of X's rows                       bias[N]
 *   GEMM [+BIAS_COL] [+SCALE_CONST] [+RELU]           X[M,K], W[K,N], bias[N]       [M]
 *         [+DROPOUT_HASH] MEAN_LAST [then reduce2 =                                  (needs the
 *         SOFTMAX_LAST over the M means]                                             workspace)
 *   NONE  SCALE_SHIFT_CH [+RELU] [+ADD_RESIDUAL]      X[N,C,H,W], scale[C],         [N,C] (AVGPOOL_HW)
 *         then AVGPOOL_HW or no reduction             shift[C], R[N,C,H,W]          or [N,C,H,W]
 *   NONE  LAYERNORM_LAST (reduce_before_epi=1)        X[M,N], gamma[N], beta[N]     [M,N]
 *         [+GELU_TANH]
 *   NONE  SOFTMAX_LAST                                X[M,N]                        [M,N]
 *   NONE  MAXPOOL2_HW (no epilogue)                   X[N,C,H,W]                    [N,C,H/2,W/2]
 *   NONE  [ADD|MUL|SUB|DIV_TENSOR] then up to 8 of    A [, B]: strided views of     that shape,
 *         RELU GELU_TANH SCALE_CONST SQRT SIN COS     one shape (stride >= 0, 0 =   contiguous
 *         EXP TANH SIGMOID in list order, no          broadcast, up to 6 dims)
 *         reduction: out = steps(A op B) or steps(A)
 *   NONE  (no epilogue, no reduction): layout         X: any strided view (stride   same shape,
 *         transform, out = contiguous copy of X       >= 0, up to 6 dims)           contiguous
 *   NONE  SUM_AXIS | MEAN_AXIS | MAX_AXIS | MIN_AXIS  X: any strided view (stride   X's shape without
 *         | ARGMAX_AXIS | ARGMIN_AXIS over dim        >= 0, up to 6 dims)           dim `axis`, contiguous
 *         `axis`, no epilogue
 *                                                                                   (1-D input: shape [1]);
 *                                                                                   int32 for the arg ops
 *   NONE  RMSNORM_LAST (eps), no epilogue              X[M,N], gamma[N] (or X alone) [M,N]
 *   NONE  GROUPNORM_NCHW (groups, eps) [+RELU]         X[N,C,H,W], gamma[C],         [N,C,H,W]
 *         (reduce_before_epi = 1 with the ReLU)        beta[C] (or X alone)
 *   NONE  MAXPOOL_HW | AVGPOOL_WIN_HW (window_hw,      X[N,C,H,W]                    [N,C,Ho,Wo]
 *         stride_hw, pad_hw, each square), no epilogue
 *   CONVT2D_NCHW [+BIAS_COL] [+SCALE_SHIFT_CH]        in[N,C,H,W], wt[C,K,R,S],     [N,K,Ho,Wo]
 *         [+RELU|RELU6] (needs the workspace: the     bias[K], scale[K], shift[K]
 *         flipped filter and, for stride > 1, the
 *         zero-dilated input; two kernels)
 *   CONV2D_NCHW, groups = C: depthwise                in[N,C,H,W], wt[C,1,R,S],     [N,C,Ho,Wo]
 *         [+BIAS_COL] [+SCALE_SHIFT_CH] [+RELU|RELU6] bias[C], scale[C], shift[C]
 *   CONV2D_NCHW [+BIAS_COL] [+SCALE_SHIFT_CH] [+RELU] in[N,C,H,W], wt[K,C,R,S],     [N,K,Ho,Wo], or
 *         then MAXPOOL2_HW or no reduction            bias[K], scale[K], shift[K]   [N,K,Ho/2,Wo/2]
 *         (square 1/3/5/7 filter, stride and                                         with MAXPOOL2_HW
 *         dilation <= 4, Ho = (H + 2 pad -
 *         (R-1) dilation - 1) / stride + 1;
 *         Ho * Wo <= 2^27, else UNSUPPORTED)
 *   BGEMM_SOFTMAX_BGEMM [+SCALE_CONST: scores scaled  Q[B,L,D], K[B,Lk,D],          [B,L,D]
 *         by `scale`] [+CAUSAL_MASK] (D = 32, 64, 128) V[B,Lk,D]
 */
#ifndef HPCT_H
#define HPCT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HPCT_OK = 0,
    HPCT_ERR_NULL = 1,            /* a required pointer argument is NULL */
    HPCT_ERR_BAD_DESC = 2,        /* malformed descriptor: ndim, shape <= 0, negative stride, counts, overlap */
    HPCT_ERR_SHAPE_MISMATCH = 3,  /* operands of the chain do not agree in shape */
    HPCT_ERR_ALIGNMENT = 4,       /* a device pointer is not aligned as the chain requires */
    HPCT_ERR_UNSUPPORTED = 5,     /* well-formed, but no kernel covers it (chain, layout, size) */
    HPCT_ERR_WORKSPACE = 6,       /* workspace missing or smaller than hpct_plan_workspace_bytes */
    HPCT_ERR_HIP = 7              /* the HIP runtime refused the launch */
} hpct_status;

typedef enum {
    HPCT_F32 = 0,
    HPCT_I32 = 1   /* only as the output of the arg-reductions */
} hpct_dtype;

#define HPCT_MAX_DIMS 6
#define HPCT_MAX_EPI 8
#define HPCT_MAX_IN 8
#define HPCT_MAX_OUT 2

typedef struct {
    int32_t ndim;                    /* 1..HPCT_MAX_DIMS */
    int64_t shape[HPCT_MAX_DIMS];    /* each > 0 */
    int64_t stride[HPCT_MAX_DIMS];   /* in elements, each >= 0 */
    hpct_dtype dtype;
} hpct_tensor_desc;

/* Anchor contraction (Table 1, ComputeIntensive). */
typedef enum {
    HPCT_ANCHOR_NONE = 0,
    HPCT_ANCHOR_GEMM = 1,                 /* Z[m,n] = sum_k X[m,k] W[k,n] */
    HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM = 2,  /* O = softmax_j(scale * Q K^T) V, per batch: two "matmul" (Table 1, ComputeIntensive,
                                             in its batched form) around a "softmax" (Table 1, Reduction), fused */
    HPCT_ANCHOR_CONV2D_NCHW = 3,          /* cross-correlation, zero padding (Section 5.3 case study) */
    HPCT_ANCHOR_CONVT2D_NCHW = 4          /* transposed conv ("Conv-Trans", Section 5.2): in[n][c][ih][iw] is scattered through
                                             wt[c][k][kh][kw] to out[n][k][ih*stride - pad + kh*dilation][iw*stride - pad + kw*dilation];
                                             output size (H-1)*stride - 2*pad + (R-1)*dilation + 1, no extra output padding */
} hpct_anchor;

/* Elementwise / broadcast epilogues (Table 1, Elementwise), applied in list order. */
typedef enum {
    HPCT_EPI_BIAS_COL = 0,        /* + bias[n]: last dim of a GEMM output, channel k of a conv output */
    HPCT_EPI_SCALE_SHIFT_CH = 1,  /* x * scale[c] + shift[c], c = dim 1 of NCHW (of the output, after a conv anchor) */
    HPCT_EPI_RELU = 2,            /* max(x, 0) */
    HPCT_EPI_ADD_RESIDUAL = 3,    /* + R, same shape as the running value */
    HPCT_EPI_GELU_TANH = 4,       /* 0.5 x (1 + tanh(sqrt(2/pi)(x + 0.044715 x^3))): an activation of Table 1's Elementwise class
                                     ("... relu and etc."), as in the activation-then-norm fusions of Section 4.1 */
    HPCT_EPI_SCALE_CONST = 5,     /* * desc.scale (after BIAS_COL in a GEMM chain; a step of an elementwise chain) */
    HPCT_EPI_DROPOUT_HASH = 6,    /* training-mode dropout with the hash mask of the Section 5.3 case study: for
                                     element (i, j) of an [M,N] value, h = i*N + j + dropout_seed (uint64, wrapping),
                                     h ^= h >> 17; h ^= h << 31; h ^= h >> 8; rand = (float)(h % 1000) / 1000.0f;
                                     the element becomes 0 when rand < dropout_p (fp32 compare) and is multiplied
                                     by 1 / (1 - dropout_p) otherwise.  GEMM anchor only. */
    HPCT_EPI_CAUSAL_MASK = 7,     /* on the scores of BGEMM_SOFTMAX_BGEMM: query i attends keys j <= i only */
    HPCT_EPI_ADD_TENSOR = 8,      /* + in[1], a strided view of the same shape (stride 0 = broadcast).  No anchor. */
    HPCT_EPI_MUL_TENSOR = 9,      /* * in[1], likewise */
    HPCT_EPI_SUB_TENSOR = 10,     /* - in[1], likewise */
    HPCT_EPI_DIV_TENSOR = 11,     /* / in[1], likewise (IEEE division, correctly rounded) */
    /* unary steps of an elementwise chain without anchor (RELU, GELU_TANH and SCALE_CONST are steps too): */
    HPCT_EPI_SQRT = 12,           /* sqrt(x), correctly rounded; NaN for x < 0 */
    HPCT_EPI_SIN = 13,            /* sin(x), full-range argument reduction */
    HPCT_EPI_COS = 14,            /* cos(x) */
    HPCT_EPI_EXP = 15,            /* exp(x) */
    HPCT_EPI_TANH = 16,           /* tanh(x) */
    HPCT_EPI_SIGMOID = 17,        /* 1 / (1 + exp(-x)) */
    HPCT_EPI_RELU6 = 18,          /* min(max(x, 0), 6): in place of RELU in a conv chain, or a unary step */
    HPCT_EPI_ABS = 19,            /* unary steps of an elementwise chain: |x| */
    HPCT_EPI_NEG = 20,            /* -x */
    HPCT_EPI_SQUARE = 21,         /* x * x */
    HPCT_EPI_LOG = 22,            /* natural logarithm */
    HPCT_EPI_SILU = 23,           /* x / (1 + exp(-x)) */
    HPCT_EPI_HARDSWISH = 24       /* x * min(max(x + 3, 0), 6) / 6 */
} hpct_epilogue;

/* Row reductions (Table 1, Reduction). */
typedef enum {
    HPCT_RED_NONE = 0,
    HPCT_RED_SOFTMAX_LAST = 1,    /* exp(x - max) / sum exp(x - max) over the last dim */
    HPCT_RED_LAYERNORM_LAST = 2,  /* (x - mean) / sqrt(biased var + eps) * gamma + beta over the last dim: the "norm" of the
                                     activation-followed-by-norm fusions of Section 4.1, built from Table 1's Reduction "mean" */
    HPCT_RED_AVGPOOL_HW = 3,      /* mean over dims 2,3 of NCHW: Table 1, Reduction "mean" over the two spatial axes */
    HPCT_RED_MEAN_LAST = 4,       /* mean over the last dim, which is dropped: [M,N] -> [M].  GEMM anchor only. */
    HPCT_RED_MAXPOOL2_HW = 5,     /* max over non-overlapping 2x2 windows of dims 2,3 (stride 2; an odd last row or
                                     column is dropped): [N,K,Ho,Wo] -> [N,K,Ho/2,Wo/2].  After a conv anchor, or alone. */
    HPCT_RED_SUM_AXIS = 6,        /* sum over dim `axis`, which is dropped */
    HPCT_RED_MEAN_AXIS = 7,       /* mean over dim `axis`, which is dropped */
    HPCT_RED_ARGMAX_AXIS = 8,     /* int32 index of the maximum along dim `axis`; of equal values the lowest index */
    HPCT_RED_ARGMIN_AXIS = 9,     /* int32 index of the minimum along dim `axis`; of equal values the lowest index */
    HPCT_RED_MAX_AXIS = 10,       /* maximum over dim `axis`, which is dropped (fp32) */
    HPCT_RED_MIN_AXIS = 11,       /* minimum over dim `axis`, which is dropped (fp32) */
    HPCT_RED_MAXPOOL_HW = 12,     /* max over window_hw windows of dims 2,3 of NCHW at stride_hw with pad_hw (padding never
                                     wins; pad < window); output extent (H + 2 pad - window) / stride + 1.  No anchor. */
    HPCT_RED_RMSNORM_LAST = 15,   /* x / sqrt(mean(x^2) + eps) * gamma over the last dim of X[M,N] */
    HPCT_RED_AVGPOOL_WIN_HW = 14, /* mean over window_hw windows of dims 2,3 at stride_hw with pad_hw, positions outside the image
                                     counting as zeros (the divisor is always window * window); extents as MAXPOOL_HW.  No anchor. */
    HPCT_RED_GROUPNORM_NCHW = 13, /* group normalisation of X[N,C,H,W] with `groups` groups of C / groups neighbouring channels:
                                     (x - mean) / sqrt(biased var + eps) over each image's group, * gamma[c] + beta[c];
                                     groups = C is instance normalisation.  No anchor; reduce_before_epi = 1 with an epilogue. */
} hpct_reduce;

typedef struct {
    hpct_anchor anchor;
    int32_t n_epi;
    hpct_epilogue epi[HPCT_MAX_EPI];
    hpct_reduce reduce;
    int32_t reduce_before_epi;    /* 1: reduction runs first, epilogues act on its output */
    int32_t n_in;
    hpct_tensor_desc in[HPCT_MAX_IN];
    int32_t n_out;
    hpct_tensor_desc out[HPCT_MAX_OUT];
    int32_t stride_hw[2];         /* conv only */
    int32_t pad_hw[2];            /* conv only */
    float eps;                    /* layernorm */
    float scale;                  /* SCALE_CONST, and the score scale of BGEMM_SOFTMAX_BGEMM */
    float dropout_p;              /* DROPOUT_HASH: drop probability, 0 <= p < 1 */
    hpct_reduce reduce2;          /* a second reduction applied to the result of `reduce`; only SOFTMAX_LAST
                                     after MEAN_LAST (softmax over the M row means), else HPCT_RED_NONE */
    uint64_t dropout_seed;        /* DROPOUT_HASH */
    int32_t axis;                 /* *_AXIS reductions: the dimension of in[0] that is reduced, 0 <= axis < ndim */
    int32_t dilation_hw[2];       /* conv only: tap kh reads input row h*stride - pad + kh*dilation; 0 means 1 */
    int32_t groups;               /* GROUPNORM_NCHW: the number of groups.  Conv: 0 or 1 = dense; C (with K = C and wt[K,1,R,S]) = depthwise, every channel
                                     filtered by its own R x R filter.  Other group counts are not supported. */
    int32_t window_hw[2];         /* MAXPOOL_HW, AVGPOOL_WIN_HW: the pooling window (square: both equal), 1..16 */
} hpct_op_desc;

typedef struct hpct_plan hpct_plan;   /* opaque; host memory */

/* Validate `desc`, choose the kernel variant and launch shape.  Host-only: no
 * HIP call is made, so it works (and is tested) without a GPU.
 * On success *out owns a new plan (release with hpct_plan_destroy); on failure
 * *out is set to NULL.  Errors: NULL, BAD_DESC, SHAPE_MISMATCH, UNSUPPORTED. */
hpct_status hpct_plan_create(const hpct_op_desc *desc, hpct_plan **out);

/* Device workspace the plan needs at launch, in bytes: 0 except for GEMM chains whose X is not row-major, GEMM chains
 * with MEAN_LAST (one float per row and column tile), GEMMs with a small output and
 * a long K (partial products of the K slices) and axis reductions with few outputs
 * and a long strided axis (partial results of the pieces it is cut into).  The launch overwrites it;
 * it needs no initialisation and carries nothing between launches.  0 for a NULL plan. */
size_t hpct_plan_workspace_bytes(const hpct_plan *plan);

/* Enqueue the plan's kernel on `hip_stream` (a hipStream_t; NULL = the default
 * stream) and return without synchronising.
 *   in_ptrs[i]  device pointer of desc.in[i]   (host array of n_in pointers)
 *   out_ptrs[i] device pointer of desc.out[i]  (host array of n_out pointers)
 *   workspace   device pointer, 16-byte aligned, >= hpct_plan_workspace_bytes, disjoint from
 *               inputs and outputs; may be NULL when that is 0.  Launches that share a
 *               workspace must be ordered on one stream.
 * Errors: NULL (plan, arrays or any data pointer), ALIGNMENT, BAD_DESC (an
 * output range overlaps an input range), WORKSPACE, HIP. */
hpct_status hpct_plan_launch(const hpct_plan *plan, const void *const *in_ptrs, void *const *out_ptrs,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same launch for callers that cannot allocate device memory and have none to pass: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation calls.  In place of a caller's workspace the plan's kernels use
 * a scratch array of HPCT_NOALLOC_SCRATCH_BYTES that is part of the library's device image (each GPU the library runs
 * on holds one copy from the first such launch on it until the process ends; the call that looks its address up runs
 * once per device, on the first launch there that needs scratch).  No hipMalloc, hipFree or other allocating routine
 * is called.  Plans whose hpct_plan_workspace_bytes exceeds HPCT_NOALLOC_SCRATCH_BYTES are refused with
 * HPCT_ERR_WORKSPACE before anything is enqueued; plans that need no workspace launch exactly as hpct_plan_launch does.
 * All such launches on one GPU share the one array: the kernels overwrite it and read back only what the same launch
 * wrote, so nothing is cleared between calls, but two launches that overlap in time on one GPU (different streams,
 * or threads without an ordering between them) race on it.  Results are bit-identical to hpct_plan_launch's.
 * Other errors as hpct_plan_launch; HIP also when the scratch cannot be located on the current device. */
#define HPCT_NOALLOC_SCRATCH_BYTES ((size_t)4 << 20)
hpct_status hpct_plan_launch_noalloc(const hpct_plan *plan, const void *const *in_ptrs, void *const *out_ptrs,
                                     void *hip_stream);

/* Release a plan.  NULL is ignored. */
void hpct_plan_destroy(hpct_plan *plan);

/* Name of the kernel variant the plan selected (static string; "" for NULL). */
const char *hpct_plan_kernel_name(const hpct_plan *plan);

/* Launch shape the plan selected: grid[3], block[3] and dynamic LDS bytes.
 * Any output pointer may be NULL.  Returns HPCT_ERR_NULL for a NULL plan. */
hpct_status hpct_plan_launch_shape(const hpct_plan *plan, uint32_t grid[3], uint32_t block[3],
                                   uint32_t *lds_bytes);

/* Text of the last error on the calling thread ("" if none); valid until the
 * next hpct call on this thread. */
const char *hpct_last_error(void);

/* Library version string. */
const char *hpct_version(void);

/* sizeof(hpct_tensor_desc) and sizeof(hpct_op_desc) as this library was
 * compiled, for bindings that mirror the structs to check themselves against. */
size_t hpct_sizeof_tensor_desc(void);
size_t hpct_sizeof_op_desc(void);

#ifdef __cplusplus
}
#endif
#endif /* HPCT_H */
