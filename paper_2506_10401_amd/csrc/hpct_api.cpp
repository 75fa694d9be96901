// Host side of the C ABI: descriptor validation, chain recognition, plan
// objects, launch-time pointer checks and dispatch to the kernel launchers.
// Nothing here touches device memory; hpct_plan_create makes no HIP call.
#include "../../include/hpct.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "kernels.hpp"

using namespace hpct;

namespace {

thread_local char g_err[512] = "";

hpct_status fail(hpct_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

void clear_err() { g_err[0] = 0; }

enum class Kind { Gemm, Affine, Layernorm, Softmax, Conv, Attn, Layout, Reduce, Eltwise, MaxPool, DwConv, ConvT, MaxPoolGen, Groupnorm };

constexpr int64_t kI32Max = 2147483647LL;

// ---- the workspace of hpct_plan_launch_noalloc: one array in every GPU's memory, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t kScratchBytes = HPCT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // per device: that device's copy of `scratch`, looked up on first use

// Address of the current device's scratch array (looked up once per device, with that device current).
hipError_t scratch_address(void** out, int* device) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    *device = dev;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct hpct_plan {
    Kind kind;
    LaunchShape shape;
    int32_t n_in, n_out;
    // byte extents of every operand (max offset + 1 element), for the overlap check
    int64_t in_bytes[HPCT_MAX_IN];
    int64_t out_bytes[HPCT_MAX_OUT];
    // which in[] slot feeds which kernel operand; -1 = absent
    int32_t slot[6];
    int64_t pool_planes; int32_t pool_h, pool_w;   // Kind::MaxPool
    PoolParams pool;                               // Kind::MaxPoolGen
    GroupnormParams gn;                            // Kind::Groupnorm
    int32_t x_copy; LayoutParams x_layout; size_t x_off;   // Kind::Gemm with a strided X: copied to workspace + x_off first
    size_t ws_bytes;  // device workspace needed at launch
    union {
        GemmParams gemm;
        AffineParams affine;
        LayernormParams ln;
        SoftmaxParams sm;
        ConvParams conv;
        AttnParams attn;
        LayoutParams layout;
        ReduceParams red;
        EltwiseParams elt;
    } u;
    ConvTParams convt;   // Kind::ConvT: the preparation step; u.conv is the stride-1 conv that follows it
};

namespace {

// ndim / shape / stride / dtype sanity and the byte extent; overflow-safe.
hpct_status check_tensor(const hpct_tensor_desc& t, const char* what, int idx, bool want_i32, int64_t* count, int64_t* extent_bytes) {
    if (t.ndim < 1 || t.ndim > HPCT_MAX_DIMS)
        return fail(HPCT_ERR_BAD_DESC, "%s[%d]: ndim %d outside 1..%d", what, idx, t.ndim, HPCT_MAX_DIMS);
    if (t.dtype != (want_i32 ? HPCT_I32 : HPCT_F32))
        return fail(HPCT_ERR_UNSUPPORTED, "%s[%d]: dtype %d (%s here)", what, idx, (int)t.dtype, want_i32 ? "int32 indices" : "only fp32");
    int64_t n = 1, maxoff = 0;
    for (int d = 0; d < t.ndim; ++d) {
        if (t.shape[d] <= 0) return fail(HPCT_ERR_BAD_DESC, "%s[%d]: shape[%d] = %lld must be > 0", what, idx, d, (long long)t.shape[d]);
        if (t.stride[d] < 0) return fail(HPCT_ERR_BAD_DESC, "%s[%d]: stride[%d] = %lld must be >= 0", what, idx, d, (long long)t.stride[d]);
        if (__builtin_mul_overflow(n, t.shape[d], &n))
            return fail(HPCT_ERR_BAD_DESC, "%s[%d]: element count overflows 63 bits", what, idx);
        int64_t span;
        if (__builtin_mul_overflow(t.shape[d] - 1, t.stride[d], &span) || __builtin_add_overflow(maxoff, span, &maxoff))
            return fail(HPCT_ERR_BAD_DESC, "%s[%d]: largest offset overflows 63 bits", what, idx);
    }
    int64_t bytes;
    if (__builtin_add_overflow(maxoff, (int64_t)1, &bytes) || __builtin_mul_overflow(bytes, (int64_t)4, &bytes))
        return fail(HPCT_ERR_BAD_DESC, "%s[%d]: byte extent overflows 63 bits", what, idx);
    *count = n;
    *extent_bytes = bytes;
    return HPCT_OK;
}

bool contiguous(const hpct_tensor_desc& t) {
    int64_t want = 1;
    for (int d = t.ndim - 1; d >= 0; --d) {
        if (t.shape[d] != 1 && t.stride[d] != want) return false;
        want *= t.shape[d];
    }
    return true;
}

bool shape_is(const hpct_tensor_desc& t, int nd, const int64_t* dims) {
    if (t.ndim != nd) return false;
    for (int d = 0; d < nd; ++d)
        if (t.shape[d] != dims[d]) return false;
    return true;
}

#define REQUIRE_SHAPE(t, what, ...)                                                              \
    do {                                                                                         \
        const int64_t dims_[] = {__VA_ARGS__};                                                   \
        if (!shape_is((t), (int)(sizeof dims_ / sizeof dims_[0]), dims_))                        \
            return fail(HPCT_ERR_SHAPE_MISMATCH, "%s has the wrong shape for this chain", what); \
    } while (0)

// epilogue list must be a subsequence of `allowed` (in that order, each at most once)
bool parse_epi(const hpct_op_desc& d, const hpct_epilogue* allowed, int n_allowed, bool* present) {
    for (int i = 0; i < n_allowed; ++i) present[i] = false;
    int pos = 0;
    for (int e = 0; e < d.n_epi; ++e) {
        while (pos < n_allowed && allowed[pos] != d.epi[e]) ++pos;
        if (pos == n_allowed) return false;
        present[pos++] = true;
    }
    return true;
}

// Integer form of the dropout decision: rand = (float)u / 1000.0f with u in 0..999 is
// increasing in u, so "rand < p" (fp32) holds exactly for u < t with t counted here.
uint32_t dropout_threshold(float p) {
    uint32_t t = 0;
    for (uint32_t u = 0; u < 1000; ++u)
        if ((float)u / 1000.0f < p) ++t;
    return t;
}

// The activation of a contraction chain: rewrites it to RELU in `dd` (so that the order test sees one name) and
// returns activate()'s code for it: 1 RELU, 2 RELU6, 3 GELU_TANH, 4 SIGMOID, 5 TANH; 0 if there is none.  (Two
// activations fail the order test.)
int take_activation(hpct_op_desc& dd) {
    int act = 0;
    for (int e = 0; e < dd.n_epi && e < HPCT_MAX_EPI; ++e) {
        int code = 0;
        switch (dd.epi[e]) {
            case HPCT_EPI_RELU: code = 1; break;
            case HPCT_EPI_RELU6: code = 2; break;
            case HPCT_EPI_GELU_TANH: code = 3; break;
            case HPCT_EPI_SIGMOID: code = 4; break;
            case HPCT_EPI_TANH: code = 5; break;
            default: break;
        }
        if (code) { act = code; dd.epi[e] = HPCT_EPI_RELU; }
    }
    return act;
}

hpct_status plan_layout(const hpct_op_desc& d, hpct_plan& p);

hpct_status plan_gemm(const hpct_op_desc& d, hpct_plan& p) {
    // one activation - RELU, RELU6, GELU_TANH, SIGMOID or TANH - may stand where RELU does
    static const hpct_epilogue order[] = {HPCT_EPI_BIAS_COL, HPCT_EPI_SCALE_CONST, HPCT_EPI_RELU, HPCT_EPI_DROPOUT_HASH};
    hpct_op_desc dd = d;
    const int act = take_activation(dd);
    bool has[4];
    if (!parse_epi(dd, order, 4, has))
        return fail(HPCT_ERR_UNSUPPORTED, "GEMM anchor: epilogues must be [BIAS_COL] [SCALE_CONST] [RELU | RELU6 | GELU_TANH | SIGMOID | TANH] [DROPOUT_HASH] in that order");
    const bool has_bias = has[0], has_scale = has[1], has_relu = has[2], has_dropout = has[3];
    if (d.reduce != HPCT_RED_NONE && d.reduce != HPCT_RED_SOFTMAX_LAST && d.reduce != HPCT_RED_MEAN_LAST)
        return fail(HPCT_ERR_UNSUPPORTED, "GEMM anchor: reduction must be NONE, SOFTMAX_LAST or MEAN_LAST");
    if (d.reduce != HPCT_RED_NONE && d.reduce_before_epi) return fail(HPCT_ERR_UNSUPPORTED, "GEMM anchor: the reduction runs after the epilogues");
    const bool mean = d.reduce == HPCT_RED_MEAN_LAST;
    if (d.reduce2 != HPCT_RED_NONE && !(mean && d.reduce2 == HPCT_RED_SOFTMAX_LAST))
        return fail(HPCT_ERR_UNSUPPORTED, "GEMM anchor: the only second reduction supported is SOFTMAX_LAST after MEAN_LAST");
    const int need = 2 + (has_bias ? 1 : 0);
    if (d.n_in != need || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "GEMM chain takes %d inputs and 1 output (got %d, %d)", need, d.n_in, d.n_out);
    const hpct_tensor_desc &X = d.in[0], &W = d.in[1];
    // X[M,K] W[K,N], or a batch X[B,M,K] with W[B,K,N] (one product per b) or W[K,N] (the same W for all:
    // that is one product of the [B*M,K] matrix)
    if ((X.ndim != 2 && X.ndim != 3) || (W.ndim != 2 && W.ndim != 3) || W.ndim > X.ndim)
        return fail(HPCT_ERR_SHAPE_MISMATCH, "GEMM operands must be X[M,K], W[K,N] or X[B,M,K] with W[B,K,N] or W[K,N]");
    const int xb = X.ndim - 2, wb = W.ndim - 2;
    const int64_t B = xb ? X.shape[0] : 1;
    if (wb && W.shape[0] != B) return fail(HPCT_ERR_SHAPE_MISMATCH, "W.shape[0] = %lld does not match the batch %lld", (long long)W.shape[0], (long long)B);
    const bool fold = xb && !wb;                       // shared W: rows of all batches form one tall matrix
    const int64_t batch = (xb && wb) ? B : 1;
    const int64_t M = fold ? B * X.shape[1] : X.shape[xb], K = X.shape[xb + 1], N = W.shape[wb + 1];
    if (W.shape[wb] != K) return fail(HPCT_ERR_SHAPE_MISMATCH, "W's K extent %lld does not match X's %lld", (long long)W.shape[wb], (long long)K);
    if (has_bias) REQUIRE_SHAPE(d.in[2], "bias", N);
    if (batch > 1 && (mean || has_dropout)) return fail(HPCT_ERR_UNSUPPORTED, "batched GEMM: MEAN_LAST and DROPOUT_HASH are not supported");
    if (xb) {
        if (mean) REQUIRE_SHAPE(d.out[0], "out[0]", B, X.shape[1]);
        else REQUIRE_SHAPE(d.out[0], "out[0]", B, X.shape[1], N);
    } else {
        if (mean) REQUIRE_SHAPE(d.out[0], "out[0]", M);
        else REQUIRE_SHAPE(d.out[0], "out[0]", M, N);
    }
    // W: row-major [K,N], or the transposed storage of a linear layer's weight ([N,K] row-major seen as [K,N]
    // with strides (1, K)); with a batch the matrices follow each other (stride K*N)
    const bool wt = !contiguous(W) && W.stride[wb] == 1 && W.stride[wb + 1] == K && (!wb || W.stride[0] == K * N || B == 1);
    // X: row-major, or any other strided view (its transpose [K,M] seen as [M,K] with strides (1, M), a slice, ...), which
    // the layout kernel first copies to the workspace as a row-major matrix
    const bool x_copy = !contiguous(X);
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i]) && !(i == 1 && wt) && !(i == 0 && x_copy))
            return fail(HPCT_ERR_UNSUPPORTED, i == 1 ? "in[1]: W must be row-major [K,N] (strides N, 1) or its transpose (strides 1, K)"
                                                     : "in[%d]: only contiguous row-major layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous row-major layouts are supported");
    if (M > kI32Max || K > kI32Max || N > kI32Max || M * N > kI32Max || M * K > kI32Max || K * N > kI32Max ||
        batch * M * N > kI32Max || batch * M * K > kI32Max || batch * K * N > kI32Max || batch > 65535)
        return fail(HPCT_ERR_UNSUPPORTED, "GEMM: operand larger than 2^31-1 elements (or more than 65535 batches)");
    const bool sm = d.reduce == HPCT_RED_SOFTMAX_LAST;
    GemmParams g{};
    g.M = (int32_t)M; g.K = (int32_t)K; g.N = (int32_t)N;
    g.relu = has_relu ? act : 0; g.softmax = sm ? 1 : 0;
    g.scale = has_scale ? d.scale : 1.0f;
    g.wt = wt ? 1 : 0;
    g.batch = (int32_t)batch; g.sX = M * K; g.sW = K * N; g.sY = M * N;
    if (has_dropout) {
        if (!(d.dropout_p >= 0.f && d.dropout_p < 1.f)) return fail(HPCT_ERR_BAD_DESC, "DROPOUT_HASH: dropout_p must satisfy 0 <= p < 1");
        g.dropout = 1;
        g.drop_t = dropout_threshold(d.dropout_p);
        g.keep_scale = (float)(1.0 / (1.0 - (double)d.dropout_p));
        g.seed = d.dropout_seed;
    }
    g.mean = mean ? 1 : 0;
    g.softmax2 = d.reduce2 == HPCT_RED_SOFTMAX_LAST ? 1 : 0;
    p.kind = Kind::Gemm;
    p.u.gemm = g;
    p.slot[0] = 0; p.slot[1] = 1; p.slot[2] = has_bias ? 2 : -1; p.slot[3] = -1;
    p.shape = gemm_shape((int32_t)M, (int32_t)K, (int32_t)N, sm, mean ? 1 : 0, g.wt, g.batch);
    p.ws_bytes = gemm_workspace_bytes((int32_t)M, (int32_t)K, (int32_t)N, sm, mean ? 1 : 0, g.batch);
    if (gemm_skinny_ok((int32_t)M, (int32_t)K, (int32_t)N, sm, mean ? 1 : 0, g.dropout, g.wt, g.batch)) {
        p.u.gemm.skinny = 1;
        p.shape = gemm_skinny_shape((int32_t)M, (int32_t)K, (int32_t)N, g.wt, g.batch);
        p.ws_bytes = gemm_skinny_workspace_bytes((int32_t)M, (int32_t)K, (int32_t)N, g.wt);
    }
    p.x_copy = 0;
    if (x_copy) {
        hpct_op_desc c{};
        c.anchor = HPCT_ANCHOR_NONE; c.reduce = HPCT_RED_NONE; c.reduce2 = HPCT_RED_NONE;
        c.n_in = 1; c.in[0] = X;
        c.n_out = 1; c.out[0] = X;
        int64_t st = 1;
        for (int k = X.ndim - 1; k >= 0; --k) { c.out[0].stride[k] = st; st *= X.shape[k]; }
        hpct_plan lp{};
        const hpct_status ls = plan_layout(c, lp);
        if (ls != HPCT_OK) return ls;
        p.x_copy = 1;
        p.x_layout = lp.u.layout;
        p.x_off = (p.ws_bytes + 255) & ~(size_t)255;
        p.ws_bytes = p.x_off + (size_t)st * 4;
    }
    return HPCT_OK;
}

hpct_status plan_rows(const hpct_op_desc& d, hpct_plan& p) {
    // LAYERNORM_LAST [+GELU_TANH]  or  SOFTMAX_LAST alone
    const hpct_tensor_desc& X = d.in[0];
    if (X.ndim != 2) return fail(HPCT_ERR_SHAPE_MISMATCH, "row reductions take a 2-D input X[M,N]");
    const int64_t M = X.shape[0], N = X.shape[1];
    if (d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "row reductions produce 1 output");
    REQUIRE_SHAPE(d.out[0], "out[0]", M, N);
    if (N > kI32Max || M > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "row reduction: more than 2^31-1 rows or columns");
    if (d.reduce == HPCT_RED_SOFTMAX_LAST) {
        if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "SOFTMAX_LAST without an anchor takes no epilogues");
        if (d.n_in != 1) return fail(HPCT_ERR_BAD_DESC, "SOFTMAX_LAST takes 1 input");
        if (!contiguous(X) || !contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "only contiguous row-major layouts are supported");
        p.kind = Kind::Softmax;
        p.u.sm = SoftmaxParams{nullptr, nullptr, M, (int32_t)N};
        p.slot[0] = 0; p.slot[1] = p.slot[2] = p.slot[3] = -1;
        p.shape = softmax_shape(M, (int32_t)N);
        return HPCT_OK;
    }
    if (d.reduce == HPCT_RED_RMSNORM_LAST) {
        if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "RMSNORM_LAST takes no epilogues");
        if (d.n_in != 2 && d.n_in != 1) return fail(HPCT_ERR_BAD_DESC, "RMSNORM_LAST takes X and gamma (or X alone)");
        if (d.n_in == 2) REQUIRE_SHAPE(d.in[1], "gamma", N);
        for (int i = 0; i < d.n_in; ++i)
            if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous row-major layouts are supported", i);
        if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous row-major layouts are supported");
        if (!(d.eps >= 0.f)) return fail(HPCT_ERR_BAD_DESC, "eps must be >= 0");
        p.kind = Kind::Layernorm;
        p.u.ln = LayernormParams{nullptr, nullptr, nullptr, nullptr, M, (int32_t)N, d.eps, 0, 1};
        p.slot[0] = 0; p.slot[1] = d.n_in == 2 ? 1 : -1; p.slot[2] = -1; p.slot[3] = -1;
        p.shape = layernorm_shape(M, (int32_t)N, 1);
        return HPCT_OK;
    }
    bool gelu = false;
    if (d.n_epi == 1 && d.epi[0] == HPCT_EPI_GELU_TANH) gelu = true;
    else if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "LAYERNORM_LAST: the only epilogue supported is GELU_TANH");
    if (gelu && !d.reduce_before_epi) return fail(HPCT_ERR_UNSUPPORTED, "LAYERNORM_LAST with GELU_TANH needs reduce_before_epi = 1");
    if (d.n_in != 3 && d.n_in != 1) return fail(HPCT_ERR_BAD_DESC, "LAYERNORM_LAST takes X, gamma, beta (or X alone)");
    if (d.n_in == 3) { REQUIRE_SHAPE(d.in[1], "gamma", N); REQUIRE_SHAPE(d.in[2], "beta", N); }
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous row-major layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous row-major layouts are supported");
    if (!(d.eps >= 0.f)) return fail(HPCT_ERR_BAD_DESC, "eps must be >= 0");
    p.kind = Kind::Layernorm;
    p.u.ln = LayernormParams{nullptr, nullptr, nullptr, nullptr, M, (int32_t)N, d.eps, gelu ? 1 : 0, 0};
    p.slot[0] = 0; p.slot[1] = d.n_in == 3 ? 1 : -1; p.slot[2] = d.n_in == 3 ? 2 : -1; p.slot[3] = -1;
    p.shape = layernorm_shape(M, (int32_t)N);
    return HPCT_OK;
}

hpct_status plan_affine(const hpct_op_desc& d, hpct_plan& p) {
    static const hpct_epilogue allowed[] = {HPCT_EPI_SCALE_SHIFT_CH, HPCT_EPI_RELU, HPCT_EPI_ADD_RESIDUAL};
    bool has[3];
    if (!parse_epi(d, allowed, 3, has))
        return fail(HPCT_ERR_UNSUPPORTED, "elementwise chain: epilogues must be [SCALE_SHIFT_CH] [RELU] [ADD_RESIDUAL] in that order");
    if (d.reduce == HPCT_RED_AVGPOOL_HW && d.reduce_before_epi && d.n_epi)
        return fail(HPCT_ERR_UNSUPPORTED, "AVGPOOL_HW runs after the epilogues");
    const bool pool = d.reduce == HPCT_RED_AVGPOOL_HW;
    const int need = 1 + (has[0] ? 2 : 0) + (has[2] ? 1 : 0);
    if (d.n_in != need || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "this chain takes %d inputs and 1 output (got %d, %d)", need, d.n_in, d.n_out);
    const hpct_tensor_desc& X = d.in[0];
    if (X.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "X must be 4-D NCHW");
    const int64_t Nb = X.shape[0], C = X.shape[1], H = X.shape[2], W = X.shape[3];
    int s = 1;
    int s_scale = -1, s_shift = -1, s_res = -1;
    if (has[0]) {
        s_scale = s++; s_shift = s++;
        REQUIRE_SHAPE(d.in[s_scale], "scale", C);
        REQUIRE_SHAPE(d.in[s_shift], "shift", C);
    }
    if (has[2]) { s_res = s++; REQUIRE_SHAPE(d.in[s_res], "residual", Nb, C, H, W); }
    if (pool) REQUIRE_SHAPE(d.out[0], "out[0]", Nb, C);
    else REQUIRE_SHAPE(d.out[0], "out[0]", Nb, C, H, W);
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous NCHW layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous layouts are supported");
    if (Nb * C > kI32Max || H * W > kI32Max || C > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "more than 2^31-1 planes or plane elements");
    p.kind = Kind::Affine;
    p.u.affine = AffineParams{nullptr, nullptr, nullptr, nullptr, nullptr, Nb * C, (int32_t)C, (int32_t)(H * W),
                              has[0] ? 1 : 0, has[1] ? 1 : 0, has[2] ? 1 : 0, pool ? 1 : 0};
    p.slot[0] = 0; p.slot[1] = s_scale; p.slot[2] = s_shift; p.slot[3] = s_res;
    p.shape = affine_shape(Nb * C, (int32_t)(H * W), pool);
    return HPCT_OK;
}

// LayoutTransform: no anchor, no epilogue, no reduction, one input that is any
// strided view (stride >= 0), one contiguous output of the same shape.
hpct_status plan_layout(const hpct_op_desc& d, hpct_plan& p) {
    if (d.n_in != 1 || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "a layout transform takes 1 input and 1 output");
    const hpct_tensor_desc &I = d.in[0], &O = d.out[0];
    if (I.ndim != O.ndim) return fail(HPCT_ERR_SHAPE_MISMATCH, "layout transform: input view and output must have the same shape");
    for (int k = 0; k < I.ndim; ++k)
        if (I.shape[k] != O.shape[k]) return fail(HPCT_ERR_SHAPE_MISMATCH, "layout transform: input view and output must have the same shape");
    if (!contiguous(O)) return fail(HPCT_ERR_UNSUPPORTED, "layout transform: the output must be contiguous");
    LayoutParams q{};
    // collapse: drop extent-1 dimensions, merge neighbours that are contiguous with each other in the input
    int nd = 0;
    for (int k = 0; k < I.ndim; ++k) {
        if (I.shape[k] == 1) continue;
        if (nd > 0 && q.sin[nd - 1] == I.shape[k] * I.stride[k]) {
            q.shape[nd - 1] *= I.shape[k];
            q.sin[nd - 1] = I.stride[k];
        } else {
            q.shape[nd] = I.shape[k];
            q.sin[nd] = I.stride[k];
            ++nd;
        }
    }
    if (nd == 0) { q.shape[0] = 1; q.sin[0] = 1; nd = 1; }
    q.nd = nd;
    q.total = 1;
    for (int k = nd - 1; k >= 0; --k) { q.sout[k] = q.total; q.total *= q.shape[k]; }
    const int a = nd - 1;
    q.kind = 0;
    q.bdim = -1;
    if (q.sin[a] == 1 || q.shape[a] == 1) {
        bool vec = q.shape[a] % 4 == 0 && q.sin[a] == 1;
        for (int k = 0; k < a; ++k) vec = vec && q.sin[k] % 4 == 0;
        q.kind = vec ? 1 : 0;
    } else {
        for (int k = 0; k < a; ++k)
            if (q.sin[k] == 1) { q.bdim = k; q.kind = 2; break; }
    }
    if (q.kind == 2) {
        // work-groups of the tiled transpose must fit a 32-bit grid
        int64_t groups = ((q.shape[a] + 31) / 32) * ((q.shape[q.bdim] + 31) / 32);  // upper bound for every tile shape
        for (int k = 0; k < a; ++k)
            if (k != q.bdim) groups *= q.shape[k];
        bool fits = groups <= kI32Max;
        for (int k = 0; k < nd; ++k) fits = fits && q.shape[k] <= kI32Max - 128;   // (tile coordinates are 32-bit too)
        if (!fits) q.kind = 0, q.bdim = -1;
    }
    p.kind = Kind::Layout;
    p.u.layout = q;
    p.slot[0] = 0; p.slot[1] = p.slot[2] = p.slot[3] = -1;
    p.shape = layout_shape(q);
    return HPCT_OK;
}

// 2x2 max pooling of an NCHW tensor without an anchor.
hpct_status plan_maxpool(const hpct_op_desc& d, hpct_plan& p) {
    if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "MAXPOOL2_HW without an anchor takes no epilogues");
    if (d.n_in != 1 || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "MAXPOOL2_HW takes 1 input and 1 output");
    const hpct_tensor_desc& X = d.in[0];
    if (X.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "X must be 4-D NCHW");
    const int64_t Nb = X.shape[0], C = X.shape[1], H = X.shape[2], W = X.shape[3];
    if (H < 2 || W < 2) return fail(HPCT_ERR_SHAPE_MISMATCH, "MAXPOOL2_HW needs planes of at least 2 x 2");
    REQUIRE_SHAPE(d.out[0], "out[0]", Nb, C, H / 2, W / 2);
    if (!contiguous(X) || !contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "only contiguous NCHW layouts are supported");
    if (H > kI32Max || W > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "plane larger than 2^31-1 rows or columns");
    p.kind = Kind::MaxPool;
    p.pool_planes = Nb * C; p.pool_h = (int32_t)H; p.pool_w = (int32_t)W;
    p.slot[0] = 0; p.slot[1] = p.slot[2] = p.slot[3] = p.slot[4] = p.slot[5] = -1;
    p.shape = maxpool2_shape(Nb * C, (int32_t)H, (int32_t)W);
    return HPCT_OK;
}

// k x k max pooling with stride and padding of an NCHW tensor without an anchor.
hpct_status plan_maxpool_gen(const hpct_op_desc& d, hpct_plan& p) {
    if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "MAXPOOL_HW / AVGPOOL_WIN_HW take no epilogues");
    if (d.n_in != 1 || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "MAXPOOL_HW / AVGPOOL_WIN_HW take 1 input and 1 output");
    const hpct_tensor_desc& X = d.in[0];
    if (X.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "X must be 4-D NCHW");
    const int32_t k = d.window_hw[0], st = d.stride_hw[0], pad = d.pad_hw[0];
    if (d.window_hw[1] != k || d.stride_hw[1] != st || d.pad_hw[1] != pad)
        return fail(HPCT_ERR_UNSUPPORTED, "MAXPOOL_HW: only square windows with equal strides and padding are supported");
    if (k < 1 || k > 16) return fail(HPCT_ERR_BAD_DESC, "MAXPOOL_HW: window %d outside 1..16", k);
    if (st < 1 || st > 16) return fail(HPCT_ERR_BAD_DESC, "MAXPOOL_HW: stride %d outside 1..16", st);
    if (pad < 0 || pad >= k) return fail(HPCT_ERR_BAD_DESC, "MAXPOOL_HW: padding %d must satisfy 0 <= pad < window", pad);
    const int64_t Nb = X.shape[0], C = X.shape[1], H = X.shape[2], W = X.shape[3];
    if (H > kI32Max / 2 || W > kI32Max / 2) return fail(HPCT_ERR_UNSUPPORTED, "plane larger than 2^30 rows or columns");
    if (H + 2 * pad < k || W + 2 * pad < k) return fail(HPCT_ERR_SHAPE_MISMATCH, "MAXPOOL_HW: the window does not fit the padded plane");
    const int64_t Ho = (H + 2 * pad - k) / st + 1, Wo = (W + 2 * pad - k) / st + 1;
    REQUIRE_SHAPE(d.out[0], "out[0]", Nb, C, Ho, Wo);
    if (!contiguous(X) || !contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "only contiguous NCHW layouts are supported");
    p.kind = Kind::MaxPoolGen;
    p.pool = PoolParams{Nb * C, (int32_t)H, (int32_t)W, k, st, pad, d.reduce == HPCT_RED_AVGPOOL_WIN_HW ? 1 : 0};
    p.slot[0] = 0; p.slot[1] = p.slot[2] = p.slot[3] = p.slot[4] = p.slot[5] = -1;
    p.shape = maxpool_shape(p.pool);
    return HPCT_OK;
}

// Group normalisation of an NCHW tensor [+ ReLU] without an anchor.
hpct_status plan_groupnorm(const hpct_op_desc& d, hpct_plan& p) {
    bool relu = false;
    if (d.n_epi == 1 && d.epi[0] == HPCT_EPI_RELU) relu = true;
    else if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "GROUPNORM_NCHW: the only epilogue supported is RELU");
    if (relu && !d.reduce_before_epi) return fail(HPCT_ERR_UNSUPPORTED, "GROUPNORM_NCHW with RELU needs reduce_before_epi = 1");
    if ((d.n_in != 3 && d.n_in != 1) || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "GROUPNORM_NCHW takes X, gamma, beta (or X alone) and 1 output");
    const hpct_tensor_desc& X = d.in[0];
    if (X.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "X must be 4-D NCHW");
    const int64_t Nb = X.shape[0], C = X.shape[1], H = X.shape[2], W = X.shape[3];
    if (d.groups < 1 || C % d.groups != 0) return fail(HPCT_ERR_BAD_DESC, "GROUPNORM_NCHW: groups = %d must divide C = %lld", d.groups, (long long)C);
    if (d.n_in == 3) { REQUIRE_SHAPE(d.in[1], "gamma", C); REQUIRE_SHAPE(d.in[2], "beta", C); }
    REQUIRE_SHAPE(d.out[0], "out[0]", Nb, C, H, W);
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous layouts are supported");
    if (!(d.eps >= 0.f)) return fail(HPCT_ERR_BAD_DESC, "eps must be >= 0");
    const int64_t Cg = C / d.groups;
    if (H * W > kI32Max || Cg * H * W > kI32Max || Nb * d.groups > kI32Max)
        return fail(HPCT_ERR_UNSUPPORTED, "GROUPNORM_NCHW: more than 2^31-1 elements per group, or groups in all");
    p.kind = Kind::Groupnorm;
    p.gn = GroupnormParams{nullptr, nullptr, nullptr, nullptr, Nb, d.groups, (int32_t)Cg, (int32_t)(H * W), d.eps, relu ? 1 : 0};
    p.slot[0] = 0; p.slot[1] = d.n_in == 3 ? 1 : -1; p.slot[2] = d.n_in == 3 ? 2 : -1; p.slot[3] = p.slot[4] = p.slot[5] = -1;
    p.shape = groupnorm_shape(p.gn);
    return HPCT_OK;
}

// Elementwise chain on one or two strided views of one shape; contiguous output.
// unary step code of an epilogue inside an elementwise chain, or -1
int unary_code(hpct_epilogue e) {
    switch (e) {
        case HPCT_EPI_RELU: return kUnRelu;
        case HPCT_EPI_GELU_TANH: return kUnGelu;
        case HPCT_EPI_SCALE_CONST: return kUnScale;
        case HPCT_EPI_SQRT: return kUnSqrt;
        case HPCT_EPI_SIN: return kUnSin;
        case HPCT_EPI_COS: return kUnCos;
        case HPCT_EPI_EXP: return kUnExp;
        case HPCT_EPI_TANH: return kUnTanh;
        case HPCT_EPI_SIGMOID: return kUnSigmoid;
        case HPCT_EPI_RELU6: return kUnRelu6;
        case HPCT_EPI_ABS: return kUnAbs;
        case HPCT_EPI_NEG: return kUnNeg;
        case HPCT_EPI_SQUARE: return kUnSquare;
        case HPCT_EPI_LOG: return kUnLog;
        case HPCT_EPI_SILU: return kUnSilu;
        case HPCT_EPI_HARDSWISH: return kUnHardswish;
        default: return -1;
    }
}

int binary_code(hpct_epilogue e) {
    switch (e) {
        case HPCT_EPI_ADD_TENSOR: return kEltAdd;
        case HPCT_EPI_MUL_TENSOR: return kEltMul;
        case HPCT_EPI_SUB_TENSOR: return kEltSub;
        case HPCT_EPI_DIV_TENSOR: return kEltDiv;
        default: return -1;
    }
}

// A chain without anchor and reduction whose epilogues are [one of the *_TENSOR ops] followed by
// unary steps only.  (RELU alone on a contiguous NCHW tensor stays with the per-channel chain.)
bool is_eltwise_chain(const hpct_op_desc& d) {
    if (d.n_epi < 1) return false;
    if (binary_code(d.epi[0]) >= 0) return true;
    bool only_relu = true;
    for (int i = 0; i < d.n_epi; ++i) {
        if (unary_code(d.epi[i]) < 0) return false;
        only_relu = only_relu && d.epi[i] == HPCT_EPI_RELU;
    }
    if (d.reduce != HPCT_RED_NONE) return false;
    return !(only_relu && d.n_in >= 1 && d.in[0].ndim == 4 && contiguous(d.in[0]));
}

hpct_status plan_eltwise(const hpct_op_desc& d, hpct_plan& p) {
    const int bin = binary_code(d.epi[0]);
    const int first = bin >= 0 ? 1 : 0;
    int un[kEltwiseSteps];
    for (int i = first; i < d.n_epi; ++i) {
        un[i - first] = unary_code(d.epi[i]);
        if (un[i - first] < 0)
            return fail(HPCT_ERR_UNSUPPORTED, "elementwise chain on views: epilogues must be [ADD|MUL|SUB|DIV_TENSOR] followed by "
                        "RELU, RELU6, GELU_TANH, SCALE_CONST, SQRT, SIN, COS, EXP, TANH, SIGMOID, ABS, NEG, SQUARE, LOG, SILU or HARDSWISH steps");
    }
    if (d.reduce != HPCT_RED_NONE) return fail(HPCT_ERR_UNSUPPORTED, "elementwise chain on views: no reduction is supported after it");
    const int need = bin >= 0 ? 2 : 1;
    if (d.n_in != need || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "this elementwise chain takes %d input(s) and 1 output", need);
    const hpct_tensor_desc &A = d.in[0], &B = d.in[need - 1], &O = d.out[0];
    if (A.ndim != B.ndim || A.ndim != O.ndim) return fail(HPCT_ERR_SHAPE_MISMATCH, "elementwise chain: both views and the output must have the same shape");
    for (int k = 0; k < A.ndim; ++k)
        if (A.shape[k] != B.shape[k] || A.shape[k] != O.shape[k])
            return fail(HPCT_ERR_SHAPE_MISMATCH, "elementwise chain: both views and the output must have the same shape");
    if (!contiguous(O)) return fail(HPCT_ERR_UNSUPPORTED, "elementwise chain: the output must be contiguous");
    EltwiseParams q{};
    int nd = 0;
    for (int k = 0; k < A.ndim; ++k) {   // drop extent 1, merge neighbours that are contiguous with each other in both views
        if (A.shape[k] == 1) continue;
        if (nd > 0 && q.sa[nd - 1] == A.shape[k] * A.stride[k] && q.sb[nd - 1] == B.shape[k] * B.stride[k]) {
            q.shape[nd - 1] *= A.shape[k];
            q.sa[nd - 1] = A.stride[k];
            q.sb[nd - 1] = B.stride[k];
        } else {
            q.shape[nd] = A.shape[k]; q.sa[nd] = A.stride[k]; q.sb[nd] = B.stride[k]; ++nd;
        }
    }
    if (nd == 0) { q.shape[0] = 1; q.sa[0] = 1; q.sb[0] = 1; nd = 1; }
    q.nd = nd;
    q.total = 1;
    for (int k = 0; k < nd; ++k) q.total *= q.shape[k];
    q.op = bin >= 0 ? bin : kEltNone;
    q.n_un = d.n_epi - first;
    for (int i = 0; i < q.n_un; ++i) q.un |= (uint32_t)un[i] << (4 * i);
    q.scale = d.scale;
    bool vec = q.shape[nd - 1] % 4 == 0 && q.sa[nd - 1] == 1 && (q.sb[nd - 1] == 1 || q.sb[nd - 1] == 0);
    for (int k = 0; k + 1 < nd; ++k) vec = vec && q.sa[k] % 4 == 0 && (q.sb[k] % 4 == 0 || q.sb[nd - 1] == 0);
    q.vec = vec ? 1 : 0;
    p.kind = Kind::Eltwise;
    p.u.elt = q;
    p.slot[0] = 0; p.slot[1] = bin >= 0 ? 1 : -1; p.slot[2] = p.slot[3] = p.slot[4] = p.slot[5] = -1;
    p.shape = eltwise_shape(q);
    return HPCT_OK;
}

// Reduction over one axis of a strided view: no anchor, no epilogue; the output is the view
// without that axis, contiguous.
hpct_status plan_reduce(const hpct_op_desc& d, hpct_plan& p) {
    if (d.n_epi != 0) return fail(HPCT_ERR_UNSUPPORTED, "axis reductions take no epilogues");
    if (d.n_in != 1 || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "an axis reduction takes 1 input and 1 output");
    const hpct_tensor_desc &I = d.in[0], &O = d.out[0];
    if (d.axis < 0 || d.axis >= I.ndim) return fail(HPCT_ERR_BAD_DESC, "axis = %d outside 0..%d", d.axis, I.ndim - 1);
    // expected output shape: the input's without `axis`; a 1-D input reduces to shape [1]
    int64_t want[HPCT_MAX_DIMS];
    int nw = 0;
    for (int k = 0; k < I.ndim; ++k)
        if (k != d.axis) want[nw++] = I.shape[k];
    if (nw == 0) want[nw++] = 1;
    if (!shape_is(O, nw, want)) return fail(HPCT_ERR_SHAPE_MISMATCH, "out[0] must have the input's shape without dim %d", d.axis);
    if (!contiguous(O)) return fail(HPCT_ERR_UNSUPPORTED, "axis reduction: the output must be contiguous");
    if (I.shape[d.axis] > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "axis reduction: more than 2^31-1 elements along the axis");
    ReduceParams q{};
    q.R = (int32_t)I.shape[d.axis];
    q.sR = I.stride[d.axis];
    const bool is_max = d.reduce == HPCT_RED_ARGMAX_AXIS || d.reduce == HPCT_RED_MAX_AXIS;
    const bool is_min = d.reduce == HPCT_RED_ARGMIN_AXIS || d.reduce == HPCT_RED_MIN_AXIS;
    q.op = is_max ? 2 : (is_min ? 3 : 0);
    q.value = (d.reduce == HPCT_RED_MAX_AXIS || d.reduce == HPCT_RED_MIN_AXIS) ? 1 : 0;   // the extreme value itself, not its index
    q.mean = d.reduce == HPCT_RED_MEAN_AXIS ? 1 : 0;
    // kept dimensions: drop extent 1, merge neighbours that are contiguous with each other in the input
    int nk = 0;
    int64_t sh[HPCT_MAX_DIMS], st[HPCT_MAX_DIMS];
    for (int k = 0; k < I.ndim; ++k) {
        if (k == d.axis || I.shape[k] == 1) continue;
        if (nk > 0 && st[nk - 1] == I.shape[k] * I.stride[k]) {
            sh[nk - 1] *= I.shape[k];
            st[nk - 1] = I.stride[k];
        } else {
            sh[nk] = I.shape[k]; st[nk] = I.stride[k]; ++nk;
        }
    }
    if (nk > kReduceDims) return fail(HPCT_ERR_UNSUPPORTED, "axis reduction: more than %d kept dimensions after collapsing", kReduceDims);
    q.nk = nk;
    q.outputs = 1;
    for (int k = 0; k < nk; ++k) { q.shape[k] = sh[k]; q.stride[k] = st[k]; q.outputs *= sh[k]; }
    if (q.sR == 1 || q.R == 1) q.kind = 0;
    else if (nk > 0 && q.stride[nk - 1] == 1) q.kind = 1;
    else q.kind = 2;
    // 32-bit grids
    if (q.outputs > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "axis reduction: more than 2^31-1 outputs");
    q.split = 1;
    if (q.kind == 1) reduce_plan_cols(q);
    p.ws_bytes = reduce_workspace_bytes(q);
    p.kind = Kind::Reduce;
    p.u.red = q;
    p.slot[0] = 0; p.slot[1] = p.slot[2] = p.slot[3] = p.slot[4] = p.slot[5] = -1;
    p.shape = reduce_shape(q);
    return HPCT_OK;
}

hpct_status plan_conv(const hpct_op_desc& d, hpct_plan& p) {
    static const hpct_epilogue allowed[] = {HPCT_EPI_BIAS_COL, HPCT_EPI_SCALE_SHIFT_CH, HPCT_EPI_RELU};
    hpct_op_desc dd = d;
    const int act = take_activation(dd);
    bool has[3];
    if (!parse_epi(dd, allowed, 3, has))
        return fail(HPCT_ERR_UNSUPPORTED, "conv anchor: epilogues must be [BIAS_COL] [SCALE_SHIFT_CH] [RELU | RELU6] in that order");
    // (the other activations of the GEMM chains would cost the conv kernels about 1 % whether used or not: measured)
    if (act > 2) return fail(HPCT_ERR_UNSUPPORTED, "conv anchor: the activation must be RELU or RELU6");
    if (d.reduce != HPCT_RED_NONE && d.reduce != HPCT_RED_MAXPOOL2_HW)
        return fail(HPCT_ERR_UNSUPPORTED, "conv anchor: reduction must be NONE or MAXPOOL2_HW");
    if (d.reduce != HPCT_RED_NONE && d.reduce_before_epi) return fail(HPCT_ERR_UNSUPPORTED, "conv anchor: the pooling runs after the epilogues");
    const bool pool = d.reduce == HPCT_RED_MAXPOOL2_HW;
    const int need = 2 + (has[0] ? 1 : 0) + (has[1] ? 2 : 0);
    if (d.n_in != need || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "conv chain takes %d inputs and 1 output (got %d, %d)", need, d.n_in, d.n_out);
    const hpct_tensor_desc &I = d.in[0], &Wt = d.in[1];
    if (I.ndim != 4 || Wt.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "conv operands must be 4-D: in[N,C,H,W], wt[K,C,R,S]");
    const int64_t Nb = I.shape[0], C = I.shape[1], H = I.shape[2], W = I.shape[3];
    const int64_t K = Wt.shape[0], R = Wt.shape[2], S = Wt.shape[3];
    const int64_t groups = d.groups <= 1 ? 1 : d.groups;
    if (d.groups < 0) return fail(HPCT_ERR_BAD_DESC, "conv: groups = %d", d.groups);
    const bool depthwise = groups > 1;
    if (depthwise && !(groups == C && K == C))
        return fail(HPCT_ERR_UNSUPPORTED, "conv: only groups = 1 (dense) and groups = C = K (depthwise) are supported");
    if (Wt.shape[1] != C / groups)
        return fail(HPCT_ERR_SHAPE_MISMATCH, "wt.shape[1] = %lld does not match the input channels per group %lld", (long long)Wt.shape[1], (long long)(C / groups));
    if (depthwise && pool) return fail(HPCT_ERR_UNSUPPORTED, "conv: MAXPOOL2_HW after a depthwise conv is not supported");
    if (d.stride_hw[0] < 1 || d.stride_hw[1] < 1 || d.pad_hw[0] < 0 || d.pad_hw[1] < 0)
        return fail(HPCT_ERR_BAD_DESC, "conv: stride must be >= 1 and padding >= 0");
    // dilation 0 (a zero-initialised descriptor) means 1
    const int32_t dil_h = d.dilation_hw[0] == 0 ? 1 : d.dilation_hw[0], dil_w = d.dilation_hw[1] == 0 ? 1 : d.dilation_hw[1];
    if (dil_h < 1 || dil_w < 1) return fail(HPCT_ERR_BAD_DESC, "conv: dilation must be >= 1 (or 0 for 1)");
    const int64_t Re = (R - 1) * dil_h + 1, Se = (S - 1) * dil_w + 1;
    if (H + 2 * d.pad_hw[0] < Re || W + 2 * d.pad_hw[1] < Se) return fail(HPCT_ERR_SHAPE_MISMATCH, "conv: filter larger than the padded input");
    const int64_t Ho = (H + 2 * d.pad_hw[0] - Re) / d.stride_hw[0] + 1, Wo = (W + 2 * d.pad_hw[1] - Se) / d.stride_hw[1] + 1;
    int s = 2;
    int s_bias = -1, s_scale = -1, s_shift = -1;
    if (has[0]) { s_bias = s++; REQUIRE_SHAPE(d.in[s_bias], "bias", K); }
    if (has[1]) {
        s_scale = s++; s_shift = s++;
        REQUIRE_SHAPE(d.in[s_scale], "scale", K);
        REQUIRE_SHAPE(d.in[s_shift], "shift", K);
    }
    if (pool) {
        if (Ho < 2 || Wo < 2) return fail(HPCT_ERR_SHAPE_MISMATCH, "MAXPOOL2_HW needs a conv output of at least 2 x 2");
        REQUIRE_SHAPE(d.out[0], "out[0]", Nb, K, Ho / 2, Wo / 2);
    } else {
        REQUIRE_SHAPE(d.out[0], "out[0]", Nb, K, Ho, Wo);
    }
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous NCHW / KCRS layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous NCHW layouts are supported");
    if (Nb * C * H * W > kI32Max || Nb * K * Ho * Wo > kI32Max || K * C * R * S > kI32Max)
        return fail(HPCT_ERR_UNSUPPORTED, "conv: operand larger than 2^31-1 elements");
    const char* why = "";
    if (depthwise) {
        if (R != S || d.stride_hw[0] != d.stride_hw[1] || d.pad_hw[0] != d.pad_hw[1] || dil_h != dil_w)
            return fail(HPCT_ERR_UNSUPPORTED, "depthwise conv: filter, stride, padding and dilation must be the same in both directions");
        ConvParams q{};
        q.Nb = (int32_t)Nb; q.C = (int32_t)C; q.H = (int32_t)H; q.W = (int32_t)W; q.K = (int32_t)K; q.R = (int32_t)R; q.S = (int32_t)S;
        q.pad = d.pad_hw[0]; q.stride = d.stride_hw[0]; q.dil = dil_h; q.relu = has[2] ? act : 0;
        if (!dwconv_supported(q, &why)) return fail(HPCT_ERR_UNSUPPORTED, "depthwise conv: %s", why);
        p.kind = Kind::DwConv;
        p.u.conv = q;
        p.slot[0] = 0; p.slot[1] = 1; p.slot[2] = s_bias; p.slot[3] = s_scale; p.slot[4] = s_shift; p.slot[5] = -1;
        p.shape = dwconv_shape(q);
        return HPCT_OK;
    }
    if (!conv_supported((int32_t)C, (int32_t)H, (int32_t)W, (int32_t)K, (int32_t)R, (int32_t)S, d.stride_hw[0], d.stride_hw[1],
                        d.pad_hw[0], d.pad_hw[1], dil_h, dil_w, pool ? 1 : 0, &why))
        return fail(HPCT_ERR_UNSUPPORTED, "conv: %s", why);
    ConvParams q{};
    q.Nb = (int32_t)Nb; q.C = (int32_t)C; q.H = (int32_t)H; q.W = (int32_t)W; q.K = (int32_t)K; q.R = (int32_t)R; q.S = (int32_t)S;
    q.pad = d.pad_hw[0]; q.stride = d.stride_hw[0]; q.dil = dil_h; q.relu = has[2] ? act : 0; q.pool = pool ? 1 : 0;
    // A 1x1 filter with stride 1 and no padding acts on pixels independently: the plane is regrouped into rows of
    // 64 pixels, so that a 64-pixel tile stages exactly the pixels it computes instead of the image rows they lie in.
    if (R == 1 && q.stride == 1 && q.pad == 0 && !pool && (H * W) % 64 == 0) { q.H = (int32_t)(H * W / 64); q.W = 64; }
    q.win = conv_window_geometry(q);
    p.kind = Kind::Conv;
    p.u.conv = q;
    p.slot[0] = 0; p.slot[1] = 1; p.slot[2] = s_bias; p.slot[3] = s_scale; p.slot[4] = s_shift; p.slot[5] = -1;
    p.shape = conv_shape(p.u.conv);
    return HPCT_OK;
}

// Transposed conv = preparation of the flipped filter (and, for stride > 1, the zero-dilated input) in the
// workspace, then the stride-1 conv kernel at padding (R-1)*dilation - pad.
hpct_status plan_convt(const hpct_op_desc& d, hpct_plan& p) {
    static const hpct_epilogue allowed[] = {HPCT_EPI_BIAS_COL, HPCT_EPI_SCALE_SHIFT_CH, HPCT_EPI_RELU};
    hpct_op_desc dd = d;
    const int act = take_activation(dd);
    bool has[3];
    if (!parse_epi(dd, allowed, 3, has))
        return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: epilogues must be [BIAS_COL] [SCALE_SHIFT_CH] [RELU | RELU6] in that order");
    if (act > 2) return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: the activation must be RELU or RELU6");
    if (d.reduce != HPCT_RED_NONE) return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: no reduction is supported after it");
    if (d.groups > 1) return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: groups are not supported");
    const int need = 2 + (has[0] ? 1 : 0) + (has[1] ? 2 : 0);
    if (d.n_in != need || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "transposed conv chain takes %d inputs and 1 output (got %d, %d)", need, d.n_in, d.n_out);
    const hpct_tensor_desc &I = d.in[0], &Wt = d.in[1];
    if (I.ndim != 4 || Wt.ndim != 4) return fail(HPCT_ERR_SHAPE_MISMATCH, "transposed conv operands must be 4-D: in[N,C,H,W], wt[C,K,R,S]");
    const int64_t Nb = I.shape[0], C = I.shape[1], H = I.shape[2], W = I.shape[3];
    const int64_t K = Wt.shape[1], R = Wt.shape[2], S = Wt.shape[3];
    if (Wt.shape[0] != C) return fail(HPCT_ERR_SHAPE_MISMATCH, "wt.shape[0] = %lld does not match the input channels %lld", (long long)Wt.shape[0], (long long)C);
    if (d.stride_hw[0] < 1 || d.stride_hw[1] < 1 || d.pad_hw[0] < 0 || d.pad_hw[1] < 0)
        return fail(HPCT_ERR_BAD_DESC, "transposed conv: stride must be >= 1 and padding >= 0");
    const int32_t dil_h = d.dilation_hw[0] == 0 ? 1 : d.dilation_hw[0], dil_w = d.dilation_hw[1] == 0 ? 1 : d.dilation_hw[1];
    if (dil_h < 1 || dil_w < 1) return fail(HPCT_ERR_BAD_DESC, "transposed conv: dilation must be >= 1 (or 0 for 1)");
    if (R != S || d.stride_hw[0] != d.stride_hw[1] || d.pad_hw[0] != d.pad_hw[1] || dil_h != dil_w)
        return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: filter, stride, padding and dilation must be the same in both directions");
    const int64_t st = d.stride_hw[0], pad = d.pad_hw[0], re = (R - 1) * dil_h;
    if (pad > re) return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: padding larger than the (dilated) filter extent minus one");
    if (st > 8) return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: strides above 8 are not supported");
    const int64_t Ho = (H - 1) * st - 2 * pad + re + 1, Wo = (W - 1) * st - 2 * pad + re + 1;
    if (Ho < 1 || Wo < 1) return fail(HPCT_ERR_SHAPE_MISMATCH, "transposed conv: empty output");
    int s = 2;
    int s_bias = -1, s_scale = -1, s_shift = -1;
    if (has[0]) { s_bias = s++; REQUIRE_SHAPE(d.in[s_bias], "bias", K); }
    if (has[1]) {
        s_scale = s++; s_shift = s++;
        REQUIRE_SHAPE(d.in[s_scale], "scale", K);
        REQUIRE_SHAPE(d.in[s_shift], "shift", K);
    }
    REQUIRE_SHAPE(d.out[0], "out[0]", Nb, K, Ho, Wo);
    for (int i = 0; i < d.n_in; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous NCHW / CKRS layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous NCHW layouts are supported");
    const int64_t Hd = (H - 1) * st + 1, Wd = (W - 1) * st + 1;
    if (Nb * C * Hd * Wd > kI32Max || Nb * K * Ho * Wo > kI32Max || K * C * R * S > kI32Max)
        return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: operand larger than 2^31-1 elements");
    const char* why = "";
    if (!conv_supported((int32_t)C, (int32_t)Hd, (int32_t)Wd, (int32_t)K, (int32_t)R, (int32_t)S, 1, 1, (int32_t)(re - pad), (int32_t)(re - pad),
                        dil_h, dil_w, 0, &why))
        return fail(HPCT_ERR_UNSUPPORTED, "transposed conv: %s", why);
    ConvParams q{};
    q.Nb = (int32_t)Nb; q.C = (int32_t)C; q.H = (int32_t)Hd; q.W = (int32_t)Wd; q.K = (int32_t)K; q.R = (int32_t)R; q.S = (int32_t)S;
    q.pad = (int32_t)(re - pad); q.stride = 1; q.dil = dil_h; q.relu = has[2] ? act : 0; q.pool = 0;
    if (R == 1 && (Hd * Wd) % 64 == 0) { q.H = (int32_t)(Hd * Wd / 64); q.W = 64; }   // as in plan_conv (1x1: pad is 0 here)
    q.win = conv_window_geometry(q);
    p.kind = Kind::ConvT;
    p.u.conv = q;
    p.convt = ConvTParams{(int32_t)Nb, (int32_t)C, (int32_t)H, (int32_t)W, (int32_t)K, (int32_t)R, (int32_t)st, (int32_t)Hd, (int32_t)Wd};
    p.slot[0] = 0; p.slot[1] = 1; p.slot[2] = s_bias; p.slot[3] = s_scale; p.slot[4] = s_shift; p.slot[5] = -1;
    p.shape = conv_shape(q);
    p.ws_bytes = convt_workspace_bytes(p.convt);
    return HPCT_OK;
}

hpct_status plan_attn(const hpct_op_desc& d, hpct_plan& p) {
    static const hpct_epilogue allowed[] = {HPCT_EPI_SCALE_CONST, HPCT_EPI_CAUSAL_MASK};
    bool has[2];
    if (!parse_epi(d, allowed, 2, has))
        return fail(HPCT_ERR_UNSUPPORTED, "BGEMM_SOFTMAX_BGEMM: epilogues (on the scores) must be [SCALE_CONST] [CAUSAL_MASK] in that order");
    const float scale = has[0] ? d.scale : 1.0f;
    if (d.reduce != HPCT_RED_NONE && d.reduce != HPCT_RED_SOFTMAX_LAST)
        return fail(HPCT_ERR_UNSUPPORTED, "BGEMM_SOFTMAX_BGEMM: reduction must be NONE or SOFTMAX_LAST (the softmax is part of the anchor)");
    if (d.n_in != 3 || d.n_out != 1) return fail(HPCT_ERR_BAD_DESC, "BGEMM_SOFTMAX_BGEMM takes Q, K, V and 1 output");
    const hpct_tensor_desc &Q = d.in[0], &K = d.in[1], &V = d.in[2];
    if (Q.ndim != 3 || K.ndim != 3 || V.ndim != 3) return fail(HPCT_ERR_SHAPE_MISMATCH, "Q, K, V must be 3-D: [B,L,D]");
    const int64_t B = Q.shape[0], L = Q.shape[1], D = Q.shape[2], Lk = K.shape[1];
    REQUIRE_SHAPE(K, "K", B, Lk, D);
    REQUIRE_SHAPE(V, "V", B, Lk, D);
    REQUIRE_SHAPE(d.out[0], "out[0]", B, L, D);
    for (int i = 0; i < 3; ++i)
        if (!contiguous(d.in[i])) return fail(HPCT_ERR_UNSUPPORTED, "in[%d]: only contiguous [B,L,D] layouts are supported", i);
    if (!contiguous(d.out[0])) return fail(HPCT_ERR_UNSUPPORTED, "out[0]: only contiguous layouts are supported");
    if (B * L * D > kI32Max || B * Lk * D > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "attention: operand larger than 2^31-1 elements");
    if (Lk * D * 4 > kI32Max) return fail(HPCT_ERR_UNSUPPORTED, "attention: one batch of K / V larger than 2^31-1 bytes");
    const char* why = "";
    if (!attn_supported((int32_t)D, &why)) return fail(HPCT_ERR_UNSUPPORTED, "attention: %s", why);
    if (!(scale == scale) || scale - scale != 0.f) return fail(HPCT_ERR_BAD_DESC, "attention: scale must be finite");
    p.kind = Kind::Attn;
    p.u.attn = AttnParams{nullptr, nullptr, nullptr, nullptr, (int32_t)B, (int32_t)L, (int32_t)Lk, (int32_t)D, scale, has[1] ? 1 : 0};
    p.slot[0] = 0; p.slot[1] = 1; p.slot[2] = 2; p.slot[3] = -1;
    p.shape = attn_shape(p.u.attn);
    return HPCT_OK;
}

}  // namespace

extern "C" {

hpct_status hpct_plan_create(const hpct_op_desc* desc, hpct_plan** out) {
    clear_err();
    if (out) *out = nullptr;
    if (!desc || !out) return fail(HPCT_ERR_NULL, "hpct_plan_create: desc and out must not be NULL");
    const hpct_op_desc& d = *desc;
    if (d.n_epi < 0 || d.n_epi > HPCT_MAX_EPI) return fail(HPCT_ERR_BAD_DESC, "n_epi = %d outside 0..%d", d.n_epi, HPCT_MAX_EPI);
    if (d.n_in < 1 || d.n_in > HPCT_MAX_IN) return fail(HPCT_ERR_BAD_DESC, "n_in = %d outside 1..%d", d.n_in, HPCT_MAX_IN);
    if (d.n_out < 1 || d.n_out > HPCT_MAX_OUT) return fail(HPCT_ERR_BAD_DESC, "n_out = %d outside 1..%d", d.n_out, HPCT_MAX_OUT);
    if ((int)d.anchor < 0 || (int)d.anchor > (int)HPCT_ANCHOR_CONVT2D_NCHW) return fail(HPCT_ERR_BAD_DESC, "unknown anchor %d", (int)d.anchor);
    if ((int)d.reduce < 0 || (int)d.reduce > (int)HPCT_RED_RMSNORM_LAST) return fail(HPCT_ERR_BAD_DESC, "unknown reduction %d", (int)d.reduce);
    if ((int)d.reduce2 < 0 || (int)d.reduce2 > (int)HPCT_RED_MIN_AXIS) return fail(HPCT_ERR_BAD_DESC, "unknown second reduction %d", (int)d.reduce2);
    if (d.reduce2 != HPCT_RED_NONE && d.anchor != HPCT_ANCHOR_GEMM)
        return fail(HPCT_ERR_UNSUPPORTED, "a second reduction is supported only after a GEMM anchor with MEAN_LAST");
    for (int e = 0; e < d.n_epi; ++e)
        if ((int)d.epi[e] < 0 || (int)d.epi[e] > (int)HPCT_EPI_HARDSWISH) return fail(HPCT_ERR_BAD_DESC, "unknown epilogue %d at position %d", (int)d.epi[e], e);

    hpct_plan tmp;
    std::memset(&tmp, 0, sizeof tmp);
    tmp.n_in = d.n_in;
    tmp.n_out = d.n_out;
    int64_t cnt;
    for (int i = 0; i < d.n_in; ++i) {
        hpct_status st = check_tensor(d.in[i], "in", i, false, &cnt, &tmp.in_bytes[i]);
        if (st != HPCT_OK) return st;
    }
    for (int i = 0; i < d.n_out; ++i) {
        const bool arg = d.reduce == HPCT_RED_ARGMAX_AXIS || d.reduce == HPCT_RED_ARGMIN_AXIS;
        hpct_status st = check_tensor(d.out[i], "out", i, arg, &cnt, &tmp.out_bytes[i]);
        if (st != HPCT_OK) return st;
        for (int k = 0; k < d.out[i].ndim; ++k)
            if (d.out[i].stride[k] == 0 && d.out[i].shape[k] > 1)
                return fail(HPCT_ERR_BAD_DESC, "out[%d]: stride 0 on a dimension of extent > 1 makes output elements overlap", i);
    }

    if (d.reduce >= HPCT_RED_SUM_AXIS && d.anchor != HPCT_ANCHOR_NONE)
        return fail(HPCT_ERR_UNSUPPORTED, "axis reductions are supported only without an anchor");
    hpct_status st;
    switch (d.anchor) {
        case HPCT_ANCHOR_GEMM: st = plan_gemm(d, tmp); break;
        case HPCT_ANCHOR_CONV2D_NCHW: st = plan_conv(d, tmp); break;
        case HPCT_ANCHOR_CONVT2D_NCHW: st = plan_convt(d, tmp); break;
        case HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM: st = plan_attn(d, tmp); break;
        default:
            if (d.reduce == HPCT_RED_MEAN_LAST) return fail(HPCT_ERR_UNSUPPORTED, "MEAN_LAST is supported only after a GEMM anchor");
            if (d.reduce == HPCT_RED_MAXPOOL2_HW) { st = plan_maxpool(d, tmp); break; }
            if (d.reduce == HPCT_RED_MAXPOOL_HW || d.reduce == HPCT_RED_AVGPOOL_WIN_HW) { st = plan_maxpool_gen(d, tmp); break; }
            if (d.reduce == HPCT_RED_GROUPNORM_NCHW) { st = plan_groupnorm(d, tmp); break; }
            if (d.reduce == HPCT_RED_RMSNORM_LAST) { st = plan_rows(d, tmp); break; }
            if (is_eltwise_chain(d)) st = plan_eltwise(d, tmp);
            else if (d.reduce >= HPCT_RED_SUM_AXIS) st = plan_reduce(d, tmp);
            else if (d.reduce == HPCT_RED_LAYERNORM_LAST || d.reduce == HPCT_RED_SOFTMAX_LAST || d.reduce == HPCT_RED_RMSNORM_LAST) st = plan_rows(d, tmp);
            else if (d.reduce == HPCT_RED_NONE && d.n_epi == 0 && d.n_in >= 1 &&
                     !(d.in[0].ndim == 4 && contiguous(d.in[0]))) st = plan_layout(d, tmp);
            else st = plan_affine(d, tmp);
    }
    if (st != HPCT_OK) return st;
    hpct_plan* p = new (std::nothrow) hpct_plan(tmp);
    if (!p) return fail(HPCT_ERR_BAD_DESC, "out of host memory");
    *out = p;
    return HPCT_OK;
}

size_t hpct_plan_workspace_bytes(const hpct_plan* plan) { return plan ? plan->ws_bytes : 0; }

hpct_status hpct_plan_launch(const hpct_plan* plan, const void* const* in_ptrs, void* const* out_ptrs, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
    clear_err();
    if (!plan || !in_ptrs || !out_ptrs) return fail(HPCT_ERR_NULL, "hpct_plan_launch: plan, in_ptrs and out_ptrs must not be NULL");
    if (plan->ws_bytes) {
        if (!workspace || workspace_bytes < plan->ws_bytes)
            return fail(HPCT_ERR_WORKSPACE, "this plan needs a workspace of %zu bytes (got %zu)", plan->ws_bytes, workspace ? workspace_bytes : (size_t)0);
        if ((uintptr_t)workspace & 15) return fail(HPCT_ERR_ALIGNMENT, "workspace is not 16-byte aligned");
    }
    // layout transforms accept views that start anywhere (element alignment); their vector variant is
    // replaced by the scalar one at launch when a base is not 16-byte aligned
    const uintptr_t amask = (plan->kind == Kind::Layout || plan->kind == Kind::Reduce || plan->kind == Kind::Eltwise) ? 3 : 15;
    for (int i = 0; i < plan->n_in; ++i) {
        if (!in_ptrs[i]) return fail(HPCT_ERR_NULL, "in_ptrs[%d] is NULL", i);
        // (a strided X of a GEMM chain goes through the layout kernel first: element alignment)
        const uintptr_t m = (i == 0 && plan->kind == Kind::Gemm && plan->x_copy) ? 3 : amask;
        if ((uintptr_t)in_ptrs[i] & m) return fail(HPCT_ERR_ALIGNMENT, "in_ptrs[%d] is not %d-byte aligned", i, (int)m + 1);
    }
    for (int i = 0; i < plan->n_out; ++i) {
        if (!out_ptrs[i]) return fail(HPCT_ERR_NULL, "out_ptrs[%d] is NULL", i);
        if ((uintptr_t)out_ptrs[i] & amask) return fail(HPCT_ERR_ALIGNMENT, "out_ptrs[%d] is not %d-byte aligned", i, (int)amask + 1);
        const uintptr_t o0 = (uintptr_t)out_ptrs[i], o1 = o0 + (uintptr_t)plan->out_bytes[i];
        for (int k = 0; k < plan->n_in; ++k) {
            const uintptr_t a0 = (uintptr_t)in_ptrs[k], a1 = a0 + (uintptr_t)plan->in_bytes[k];
            if (o0 < a1 && a0 < o1) return fail(HPCT_ERR_BAD_DESC, "out_ptrs[%d] overlaps in_ptrs[%d]", i, k);
        }
    }
    if (plan->ws_bytes) {
        const uintptr_t w0 = (uintptr_t)workspace, w1 = w0 + plan->ws_bytes;
        for (int k = 0; k < plan->n_in; ++k) {
            const uintptr_t a0 = (uintptr_t)in_ptrs[k], a1 = a0 + (uintptr_t)plan->in_bytes[k];
            if (w0 < a1 && a0 < w1) return fail(HPCT_ERR_BAD_DESC, "workspace overlaps in_ptrs[%d]", k);
        }
        for (int k = 0; k < plan->n_out; ++k) {
            const uintptr_t a0 = (uintptr_t)out_ptrs[k], a1 = a0 + (uintptr_t)plan->out_bytes[k];
            if (w0 < a1 && a0 < w1) return fail(HPCT_ERR_BAD_DESC, "workspace overlaps out_ptrs[%d]", k);
        }
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    auto in = [&](int s) -> const float* { return plan->slot[s] < 0 ? nullptr : (const float*)in_ptrs[plan->slot[s]]; };
    hipError_t e = hipSuccess;
    switch (plan->kind) {
        case Kind::Gemm: {
            GemmParams q = plan->u.gemm;
            q.X = in(0); q.W = in(1); q.bias = in(2); q.Y = (float*)out_ptrs[0];
            q.ws = (float*)workspace;
            if (plan->x_copy) {   // a strided X: its row-major copy first
                LayoutParams l = plan->x_layout;
                l.in = q.X; l.out = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan->x_off);
                if (l.kind == 1 && ((uintptr_t)l.in & 15)) l.kind = 0;
                e = layout_launch(l, stream);
                if (e != hipSuccess) break;
                q.X = l.out;
            }
            e = gemm_launch(q, stream);
            break;
        }
        case Kind::Affine: {
            AffineParams q = plan->u.affine;
            q.X = in(0); q.scale = in(1); q.shift = in(2); q.R = in(3); q.out = (float*)out_ptrs[0];
            e = affine_launch(q, stream);
            break;
        }
        case Kind::Layernorm: {
            LayernormParams q = plan->u.ln;
            q.X = in(0); q.gamma = in(1); q.beta = in(2); q.Y = (float*)out_ptrs[0];
            e = layernorm_launch(q, stream);
            break;
        }
        case Kind::Softmax: {
            SoftmaxParams q = plan->u.sm;
            q.X = in(0); q.Y = (float*)out_ptrs[0];
            e = softmax_launch(q, stream);
            break;
        }
        case Kind::Conv: {
            ConvParams q = plan->u.conv;
            q.in = in(0); q.wt = in(1); q.bias = in(2); q.scale = in(3); q.shift = in(4); q.out = (float*)out_ptrs[0];
            e = conv_launch(q, stream);
            break;
        }
        case Kind::Layout: {
            LayoutParams q = plan->u.layout;
            q.in = in(0); q.out = (float*)out_ptrs[0];
            if (q.kind == 1 && (((uintptr_t)q.in | (uintptr_t)q.out) & 15)) q.kind = 0;
            e = layout_launch(q, stream);
            break;
        }
        case Kind::MaxPool:
            e = maxpool2_launch(in(0), (float*)out_ptrs[0], plan->pool_planes, plan->pool_h, plan->pool_w, stream);
            break;
        case Kind::Groupnorm: {
            GroupnormParams q = plan->gn;
            q.X = in(0); q.gamma = plan->slot[1] >= 0 ? in(1) : nullptr; q.beta = plan->slot[2] >= 0 ? in(2) : nullptr;
            q.Y = (float*)out_ptrs[0];
            e = groupnorm_launch(q, stream);
            break;
        }
        case Kind::MaxPoolGen:
            e = maxpool_launch(plan->pool, in(0), (float*)out_ptrs[0], stream);
            break;
        case Kind::ConvT: {
            const ConvTParams& t = plan->convt;
            e = convt_prep_launch(t, in(0), in(1), (float*)workspace, stream);
            if (e != hipSuccess) break;
            ConvParams q = plan->u.conv;
            q.wt = (const float*)workspace;
            q.in = t.stride > 1 ? (const float*)((const char*)workspace + convt_weights_bytes(t)) : in(0);
            q.bias = in(2); q.scale = in(3); q.shift = in(4); q.out = (float*)out_ptrs[0];
            e = conv_launch(q, stream);
            break;
        }
        case Kind::DwConv: {
            ConvParams q = plan->u.conv;
            q.in = in(0); q.wt = in(1); q.bias = in(2); q.scale = in(3); q.shift = in(4); q.out = (float*)out_ptrs[0];
            e = dwconv_launch(q, stream);
            break;
        }
        case Kind::Eltwise: {
            EltwiseParams q = plan->u.elt;
            q.a = in(0); q.b = in(1); q.out = (float*)out_ptrs[0];
            if (q.vec && (((uintptr_t)q.a | (uintptr_t)q.b | (uintptr_t)q.out) & 15)) q.vec = 0;
            e = eltwise_launch(q, stream);
            break;
        }
        case Kind::Reduce: {
            ReduceParams q = plan->u.red;
            q.in = in(0); q.out = out_ptrs[0]; q.ws = (float*)workspace;
            e = reduce_launch(q, stream);
            break;
        }
        case Kind::Attn: {
            AttnParams q = plan->u.attn;
            q.Q = in(0); q.K = in(1); q.V = in(2); q.O = (float*)out_ptrs[0];
            e = attn_launch(q, stream);
            break;
        }
    }
    if (e != hipSuccess) return fail(HPCT_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return HPCT_OK;
}

hpct_status hpct_plan_launch_noalloc(const hpct_plan* plan, const void* const* in_ptrs, void* const* out_ptrs, void* hip_stream) {
    clear_err();
    if (!plan || !in_ptrs || !out_ptrs) return fail(HPCT_ERR_NULL, "hpct_plan_launch_noalloc: plan, in_ptrs and out_ptrs must not be NULL");
    if (plan->ws_bytes > kScratchBytes)   // before any HIP call
        return fail(HPCT_ERR_WORKSPACE, "this plan needs a workspace of %zu bytes; the built-in scratch of hpct_plan_launch_noalloc holds %zu",
                    plan->ws_bytes, kScratchBytes);
    void* ws = nullptr;
    if (plan->ws_bytes) {
        int dev = -1;
        const hipError_t e = scratch_address(&ws, &dev);
        if (e != hipSuccess) return fail(HPCT_ERR_HIP, "cannot locate the built-in scratch on device %d: %s", dev, hipGetErrorString(e));
    }
    // every workspace-using kernel sequence writes what it later reads, so nothing has to be cleared
    return hpct_plan_launch(plan, in_ptrs, out_ptrs, ws, plan->ws_bytes, hip_stream);
}

void hpct_plan_destroy(hpct_plan* plan) { delete plan; }

const char* hpct_plan_kernel_name(const hpct_plan* plan) { return plan ? plan->shape.kernel : ""; }

hpct_status hpct_plan_launch_shape(const hpct_plan* plan, uint32_t grid[3], uint32_t block[3], uint32_t* lds_bytes) {
    clear_err();
    if (!plan) return fail(HPCT_ERR_NULL, "hpct_plan_launch_shape: plan must not be NULL");
    for (int i = 0; i < 3; ++i) {
        if (grid) grid[i] = plan->shape.grid[i];
        if (block) block[i] = plan->shape.block[i];
    }
    if (lds_bytes) *lds_bytes = plan->shape.lds_bytes;
    return HPCT_OK;
}

const char* hpct_last_error(void) { return g_err; }

const char* hpct_version(void) { return "hpct 0.2 (gfx950)"; }

size_t hpct_sizeof_tensor_desc(void) { return sizeof(hpct_tensor_desc); }
size_t hpct_sizeof_op_desc(void) { return sizeof(hpct_op_desc); }

}  // extern "C"
