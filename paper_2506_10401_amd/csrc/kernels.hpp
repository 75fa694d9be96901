// Launch parameters and host-side launchers of the kernel families.  Each
// launcher enqueues one kernel on `stream` (up to three for the chains that finish
// a reduction from a workspace) and returns the HIP status of the launch.
// Shapes have been validated by the caller (the plan layer); launchers assert
// nothing beyond what they state here.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace hpct {

struct LaunchShape {
    uint32_t grid[3];
    uint32_t block[3];
    uint32_t lds_bytes;
    const char* kernel;
};

// ---- layernorm over the last dim, optional tanh-GELU (Table 1: Reduction + Elementwise)
struct LayernormParams {
    const float* X; const float* gamma; const float* beta; float* Y;
    int64_t rows; int32_t N; float eps; int32_t gelu;
    int32_t rms;   // root-mean-square normalisation: no mean, no beta
};
LaunchShape layernorm_shape(int64_t rows, int32_t N, int32_t rms = 0);
hipError_t layernorm_launch(const LayernormParams& p, hipStream_t stream);

// ---- row softmax over the last dim (Table 1: Reduction)
struct SoftmaxParams { const float* X; float* Y; int64_t rows; int32_t N; };
LaunchShape softmax_shape(int64_t rows, int32_t N);
hipError_t softmax_launch(const SoftmaxParams& p, hipStream_t stream);

// ---- per-channel affine / relu / residual over NCHW planes, then either a
//      global average pool (out = [planes]) or the full tensor (out = [planes*HW])
struct AffineParams {
    const float* X; const float* scale; const float* shift; const float* R; float* out;
    int64_t planes; int32_t C; int32_t HW;
    int32_t has_affine, relu, has_residual, pool;
};
LaunchShape affine_shape(int64_t planes, int32_t HW, int32_t pool);
// 2x2 / stride-2 max pooling of [planes, H, W] -> [planes, H/2, W/2]
LaunchShape maxpool2_shape(int64_t planes, int32_t H, int32_t W);
hipError_t maxpool2_launch(const float* X, float* out, int64_t planes, int32_t H, int32_t W, hipStream_t stream);
// k_maxpool.hip: k x k max pooling with stride and padding (pad < k; padding never wins); 2 x 2 / 2 / 0 goes to maxpool2
struct PoolParams { int64_t planes; int32_t H, W, k, stride, pad; int32_t avg; };   // avg: the mean with zero padding (divisor k*k) instead of the maximum
LaunchShape maxpool_shape(const PoolParams& p);
hipError_t maxpool_launch(const PoolParams& p, const float* in, float* out, hipStream_t stream);
hipError_t affine_launch(const AffineParams& p, hipStream_t stream);

// ---- group normalisation of NCHW [+ ReLU] (k_groupnorm.hip); rows of more than 2^31-1 elements are refused by the plan
struct GroupnormParams {
    const float* X; const float* gamma; const float* beta; float* Y;
    int64_t Nb; int32_t G, Cg, HW; float eps; int32_t relu;
};
LaunchShape groupnorm_shape(const GroupnormParams& p);
hipError_t groupnorm_launch(const GroupnormParams& p, hipStream_t stream);

// ---- layout transform: out = contiguous copy of a strided view (Table 1: LayoutTransform)
constexpr int kLayoutDims = 6;
struct LayoutParams {
    const float* in; float* out;
    int32_t nd;                      // collapsed dimensions, 1..kLayoutDims
    int64_t shape[kLayoutDims];      // collapsed extents
    int64_t sin[kLayoutDims];        // input strides (elements)
    int64_t sout[kLayoutDims];       // output strides (contiguous)
    int64_t total;                   // elements
    int32_t kind;                    // 0 rows scalar, 1 rows vec4, 2 tiled transpose
    int32_t bdim;                    // transpose: the dimension with input stride 1
};
LaunchShape layout_shape(const LayoutParams& p);
hipError_t layout_launch(const LayoutParams& p, hipStream_t stream);

// ---- elementwise chain on strided views: v = a or a (+,*,-,/) b, then unary steps in order
// (Table 1: Elementwise "add, sub, mul, div, sqrt, sin, cos, relu and etc.")
constexpr int kEltwiseDims = 6;
constexpr int kEltwiseSteps = 8;
enum : int32_t { kEltAdd = 0, kEltMul = 1, kEltSub = 2, kEltDiv = 3, kEltNone = 4 };
enum : int32_t { kUnRelu = 0, kUnGelu, kUnScale, kUnSqrt, kUnSin, kUnCos, kUnExp, kUnTanh, kUnSigmoid, kUnRelu6,
                 kUnAbs, kUnNeg, kUnSquare, kUnLog, kUnSilu, kUnHardswish };   // 16 codes: four bits each in EltwiseParams::un
struct EltwiseParams {
    const float* a; const float* b; float* out;
    int32_t nd;                      // collapsed dimensions, 1..kEltwiseDims
    int64_t shape[kEltwiseDims];
    int64_t sa[kEltwiseDims];        // strides of a (elements), 0 = broadcast
    int64_t sb[kEltwiseDims];        // strides of b
    int64_t total;                   // elements
    int32_t op;                      // kEltAdd .. kEltNone (b unused)
    int32_t n_un;                    // unary steps, 0..kEltwiseSteps
    uint32_t un;                     // their codes (kUnRelu ..), 4 bits each, first step in the low bits
    float scale;                     // the constant of kUnScale
    int32_t vec;                     // 128-bit access possible by the strides (pointers are checked at launch)
};
LaunchShape eltwise_shape(const EltwiseParams& p);
hipError_t eltwise_launch(const EltwiseParams& p, hipStream_t stream);

// ---- sum / mean / argmax / argmin over one axis of a strided view (Table 1: Reduction)
constexpr int kReduceDims = 5;
struct ReduceParams {
    const float* in; void* out;        // out: float (sum, mean) or int32 (argmax, argmin), contiguous
    int32_t value;                     // op 2 / 3: write the extreme value (fp32) instead of its index
    int32_t nk;                        // kept dimensions after collapsing, 0..kReduceDims
    int64_t shape[kReduceDims];        // their extents
    int64_t stride[kReduceDims];       // their input strides (elements)
    int32_t R; int64_t sR;             // extent and input stride of the reduced axis
    int64_t outputs;                   // product of the kept extents
    int32_t op;                        // 0 sum, 2 argmax, 3 argmin
    int32_t mean;                      // op 0: divide by R
    int32_t kind;                      // 0 reduced axis contiguous, 1 innermost kept dim contiguous, 2 gather
    // kind 1 (set by reduce_plan_cols): columns per thread, log2 of the column threads per group,
    // pieces the reduced axis is split into (> 1: partial results go through `ws`)
    int32_t cols_v, cols_tc_log2, split;
    float* ws;                         // split > 1: split * outputs floats (+ as many ints for the arg ops)
};
bool reduce_rows_per_group(const ReduceParams& p);
void reduce_plan_cols(ReduceParams& p);
size_t reduce_workspace_bytes(const ReduceParams& p);
LaunchShape reduce_shape(const ReduceParams& p);
hipError_t reduce_launch(const ReduceParams& p, hipStream_t stream);

// ---- GEMM + bias + relu + hash dropout, then one of: store [M,N]; row softmax
//      (when the tile spans the whole row); mean over the last dim (-> [M]),
//      optionally followed by a softmax over those M means.  The mean variants
//      enqueue two or three kernels: the GEMM writes one partial row sum per column
//      tile to `ws` ([col_tiles][M] floats), a second kernel adds them into the row
//      means in Y, a one-group kernel turns Y into its softmax.
struct GemmParams {
    const float* X; const float* W; const float* bias; float* Y;
    int32_t M, K, N; int32_t relu, softmax;   // relu: the activation code of prim.hpp's activate() (0 none, 1 ReLU, ...)
    int32_t dropout;      // apply the hash dropout
    uint32_t drop_t;      // an element is dropped iff (hash % 1000) < drop_t
    float keep_scale;     // 1 / (1 - p)
    uint64_t seed;
    int32_t mean;         // reduce over the last dim instead of storing [M,N]
    int32_t softmax2;     // softmax over the M means
    float* ws;            // partial row sums (`mean`) or the K slices' partial products (ksplit > 1)
    int32_t skinny;       // 1: the streaming kernel for a very small N or M (set by the plan from gemm_skinny_ok)
    int32_t ksplit;       // K slices of the tiled kernel, >= 1 (set by the plan from gemm_ksplit)
    float scale;          // (X W + bias) * scale before ReLU; 1 when the chain has no SCALE_CONST
    int32_t wt;           // W is stored transposed: element (k, n) at n * K + k (an [N,K] row-major array)
    int32_t batch;        // >= 1 independent products; matrix b starts at X + b sX, W + b sW, Y + b sY
    int64_t sX, sW, sY;   // element strides between the matrices of a batch (sW = 0: one W for all)
};
constexpr int kGemmSoftmaxMaxN = 256;
bool gemm_use_tile(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t batch = 1);
bool gemm_use_ksplit16(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t wt, int32_t batch = 1);
int32_t gemm_ksplit(int32_t M, int32_t K, int32_t N, int32_t mean, int32_t batch = 1);
size_t gemm_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t batch = 1);
int32_t gemm_col_tiles(int32_t M, int32_t K, int32_t N);
LaunchShape gemm_shape(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t wt, int32_t batch = 1);
hipError_t gemm_launch(const GemmParams& p, hipStream_t stream);
// the tiled kernel (128 x 128 or 64 x 64 tiles) and the finishing kernels (k_gemm_tile.hip)
LaunchShape gemm_tile_shape(int32_t M, int32_t N, int32_t ksplit, int32_t wt, int32_t batch = 1);
int32_t gemm_tile_col_tiles(int32_t M, int32_t N, int32_t batch = 1);
hipError_t gemm_tile_launch(const GemmParams& p, hipStream_t stream);
hipError_t gemm_split_finish_launch(const GemmParams& p, hipStream_t stream);   // sums p.ksplit slices of p.ws, applies the epilogue
// k_gemm_skinny.hip: N <= 8, or M <= 8 with a transposed W: the large operand streamed row by row (HBM-bound)
bool gemm_skinny_ok(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t dropout, int32_t wt, int32_t batch);
LaunchShape gemm_skinny_shape(int32_t M, int32_t K, int32_t N, int32_t wt, int32_t batch);
size_t gemm_skinny_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t wt);
hipError_t gemm_skinny_launch(const GemmParams& p, hipStream_t stream);
// k_gemm_direct.hip: products with a short K, operands loaded straight into the MFMA layout (no LDS)
bool gemm_direct_ok(int32_t M, int32_t K, int32_t N, int32_t mean, int32_t wt, int32_t batch);
LaunchShape gemm_direct_shape(int32_t M, int32_t N, int32_t batch);
hipError_t gemm_direct_launch(const GemmParams& p, hipStream_t stream);
hipError_t rows_finish_launch(const float* ws, float* out, int32_t M, int32_t T, int32_t N, int32_t softmax, hipStream_t stream);

// ---- NCHW conv2d (square 1/3/5/7 filter, stride and dilation up to 4) + bias + per-channel
//      scale/shift + relu, optionally followed by 2x2 / stride-2 max pooling
struct ConvParams {
    const float* in; const float* wt; const float* bias; float* out;
    int32_t Nb, C, H, W, K, R, S, pad; int32_t relu;   // relu: 0 none, 1 max(x, 0), 2 min(max(x, 0), 6)
    int32_t stride;
    const float* scale; const float* shift;   // per output channel, either may be null
    int32_t pool;                             // out is [Nb, K, Ho/2, Wo/2]
    int32_t dil;                              // dilation, >= 1
    int32_t win;                              // 8 x 8 window tiles (set from conv_window_geometry)
};
int32_t conv_window_geometry(const ConvParams& p);   // from C, H, W, K, R, pad, stride, dil, pool
bool conv_supported(int32_t C, int32_t H, int32_t W, int32_t K, int32_t R, int32_t S, int32_t stride_h,
                    int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t dil_h, int32_t dil_w, int32_t pool,
                    const char** why);
LaunchShape conv_shape(const ConvParams& p);
hipError_t conv_launch(const ConvParams& p, hipStream_t stream);
// 1x1, stride 1, no padding: the weight-stationary streaming kernel (k_conv1x1.hip), taken by conv_shape /
// conv_launch whenever conv1x1_stream_ok
bool conv1x1_stream_ok(const ConvParams& p);
LaunchShape conv1x1_shape(const ConvParams& p);
hipError_t conv1x1_launch(const ConvParams& p, hipStream_t stream);
// 3x3, stride 1, pad 1 on at most 4 input channels (a network's first layer): the kernel without LDS (k_conv_fewc.hip),
// taken by conv_shape / conv_launch whenever conv_fewc_ok
bool conv_fewc_ok(const ConvParams& p);
LaunchShape conv_fewc_shape(const ConvParams& p);
hipError_t conv_fewc_launch(const ConvParams& p, hipStream_t stream);
// transposed conv: the operands of the equivalent stride-1 conv, prepared in the workspace (k_convt_prep.hip)
struct ConvTParams {
    int32_t Nb, C, H, W, K, R, stride;   // in [Nb,C,H,W], wt [C,K,R,R]
    int32_t Hd, Wd;                      // zero-dilated input: (H-1)*stride + 1, (W-1)*stride + 1
};
size_t convt_weights_bytes(const ConvTParams& p);     // offset of the dilated input inside the workspace
size_t convt_workspace_bytes(const ConvTParams& p);
hipError_t convt_prep_launch(const ConvTParams& p, const float* in, const float* wt, float* workspace, hipStream_t stream);
// depthwise (groups = C = K, wt[C,1,R,R]): a memory-bound stencil kernel of its own (k_dwconv.hip)
bool dwconv_supported(const ConvParams& p, const char** why);
LaunchShape dwconv_shape(const ConvParams& p);
hipError_t dwconv_launch(const ConvParams& p, hipStream_t stream);

// ---- batched softmax(scale * Q K^T) V
struct AttnParams {
    const float* Q; const float* K; const float* V; float* O;
    int32_t B, Lq, Lk, D; float scale;
    int32_t causal;   // query i sees keys j <= i only
};
bool attn_supported(int32_t D, const char** why);
LaunchShape attn_shape(const AttnParams& p);
hipError_t attn_launch(const AttnParams& p, hipStream_t stream);

}  // namespace hpct
