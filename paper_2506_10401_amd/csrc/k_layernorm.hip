// Layer normalisation over the last dimension with an optional tanh-form GELU,
// and a plain row softmax (Reduction and Elementwise classes of the paper's
// Table 1).  Memory-bound: each row is read from HBM once with 128-bit loads,
// held in registers for the two reduction passes and the epilogue, and written
// once.  The kernels are templated on the row operation: layernorm, layernorm +
// GELU, or softmax (max, then sum of exponentials, both from registers).
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kMaxVec = 16;  // float4 per thread held in registers
constexpr int kLn = 0, kLnGelu = 1, kSoftmax = 2, kRms = 3;  // row operations (kRms: x / sqrt(mean x^2 + eps), no mean)

// The row operation on the VPT vectors a thread holds (vector i is element j = t + i*TPR of nv;
// vectors with j >= nv do not exist).  Leaves the row's result in v; NW waves share `slots`.
template <int OPK, int VPT, int TPR, int NW>
__device__ __forceinline__ void row_op(float4v* v, int t, int nv, int N, float eps, float* slots) {
    if constexpr (OPK == kSoftmax) {
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < VPT; ++i)
            if (t + i * TPR < nv) m = fmaxf(m, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
        m = block_reduce<OpMax, NW>(m, slots);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            float4v e = (v[i] - m) * kLog2e;
            e.x = fast_exp2(e.x); e.y = fast_exp2(e.y); e.z = fast_exp2(e.z); e.w = fast_exp2(e.w);
            if (t + i * TPR >= nv) e = float4v{0.f, 0.f, 0.f, 0.f};
            v[i] = e;
            s += (e.x + e.y) + (e.z + e.w);
        }
        const float inv = 1.0f / block_reduce<OpSum, NW>(s, slots);
#pragma unroll
        for (int i = 0; i < VPT; ++i) v[i] = v[i] * inv;
    } else if constexpr (OPK == kRms) {
        float q = 0.f;   // (vectors beyond the row were loaded as zeros)
#pragma unroll
        for (int i = 0; i < VPT; ++i) q += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
        const float ms = block_reduce<OpSum, NW>(q, slots) * (1.0f / (float)N);
        const float rstd = fast_rsq(ms + eps);
#pragma unroll
        for (int i = 0; i < VPT; ++i) v[i] = v[i] * rstd;
    } else {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < VPT; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        const float inv_n = 1.0f / (float)N;
        const float mu = block_reduce<OpSum, NW>(s, slots) * inv_n;
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            float4v d = v[i] - mu;
            if (t + i * TPR >= nv) d = float4v{0.f, 0.f, 0.f, 0.f};
            v[i] = d;
            q += (d.x * d.x + d.y * d.y) + (d.z * d.z + d.w * d.w);
        }
        const float var = block_reduce<OpSum, NW>(q, slots) * inv_n;
        const float rstd = fast_rsq(var + eps);
#pragma unroll
        for (int i = 0; i < VPT; ++i) v[i] = v[i] * rstd;
    }
}

// scale / shift / GELU of a normalised vector (layernorm only)
template <int OPK>
__device__ __forceinline__ float4v ln_out(float4v o, float4v g, float4v b) {
    if constexpr (OPK == kSoftmax) return o;
    o = o * g + b;
    if (OPK == kLnGelu) { o.x = gelu_tanh(o.x); o.y = gelu_tanh(o.y); o.z = gelu_tanh(o.z); o.w = gelu_tanh(o.w); }
    return o;
}

// One row per group of TPR threads (TPR = 64: a wave per row, four rows per
// work-group, no LDS; TPR = 256: a work-group per row, LDS cross-wave combine).
// Thread t of the group owns vectors t, t+TPR, ... (< N/4), so consecutive
// lanes read consecutive 16-byte words.
template <int TPR, int VPT, int OPK>
__global__ __launch_bounds__(256) void rows_vec(const float* __restrict__ X, const float* __restrict__ gamma,
                                                const float* __restrict__ beta, float* __restrict__ Y,
                                                int64_t rows, int N, float eps) {
    constexpr int RPB = 256 / TPR;
    constexpr int NW = TPR / kWave;
    __shared__ float slots[16];
    const int t = threadIdx.x % TPR;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
    const bool live = row < rows;
    const int nv = N >> 2;
    const float* x = X + (live ? row : 0) * (int64_t)N;

    float4v v[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int j = t + i * TPR;
        v[i] = (live && j < nv) ? load4_nt(x + 4 * j) : float4v{0.f, 0.f, 0.f, 0.f};
    }
    row_op<OPK, VPT, TPR, NW>(v, t, nv, N, eps, slots);
    if (!live) return;
    float* y = Y + row * (int64_t)N;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int j = t + i * TPR;
        if (j < nv) {
            float4v g = (OPK != kSoftmax && gamma) ? load4(gamma + 4 * j) : float4v{1.f, 1.f, 1.f, 1.f};
            float4v b = (OPK != kSoftmax && beta) ? load4(beta + 4 * j) : float4v{0.f, 0.f, 0.f, 0.f};
            store4_nt(y + 4 * j, ln_out<OPK>(v[i], g, b));
        }
    }
}

// Rows of 2048..4096 elements (VPT <= 4): a fixed grid of two work-groups per
// CU walks the rows with stride gridDim.x.  gamma and beta stay in registers
// for the whole kernel and the next row's loads are issued before the current
// row is reduced, so HBM reads never wait for the reductions.
constexpr int kPersistGrid = 768;  // 3 x 256 CUs (8192 x 4096: 512 -> 45.4 us, 768 -> 44.8, 1024 -> 46.6)

template <int VPT, int OPK>
__global__ __launch_bounds__(256) void rows_persist(const float* __restrict__ X, const float* __restrict__ gamma,
                                                    const float* __restrict__ beta, float* __restrict__ Y,
                                                    int64_t rows, int N, float eps) {
    __shared__ float slots[16];
    const int t = threadIdx.x;
    const int nv = N >> 2;
    float4v g[VPT], b[VPT], v[VPT], nx[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int j = t + i * 256;
        g[i] = (OPK != kSoftmax && gamma && j < nv) ? load4(gamma + 4 * j) : float4v{1.f, 1.f, 1.f, 1.f};
        b[i] = (OPK != kSoftmax && beta && j < nv) ? load4(beta + 4 * j) : float4v{0.f, 0.f, 0.f, 0.f};
    }
    auto load_row = [&](int64_t row, float4v* dst) {
        const float* x = X + row * (int64_t)N;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int j = t + i * 256;
            dst[i] = j < nv ? load4_nt(x + 4 * j) : float4v{0.f, 0.f, 0.f, 0.f};
        }
    };
    int64_t row = blockIdx.x;
    if (row >= rows) return;
    load_row(row, v);
    for (; row < rows; row += gridDim.x) {
        const int64_t nrow = row + gridDim.x;
        if (nrow < rows) load_row(nrow, nx);
        row_op<OPK, VPT, 256, 4>(v, t, nv, N, eps, slots);
        float* y = Y + row * (int64_t)N;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int j = t + i * 256;
            if (j < nv) store4_nt(y + 4 * j, ln_out<OPK>(v[i], g[i], b[i]));
        }
#pragma unroll
        for (int i = 0; i < VPT; ++i) v[i] = nx[i];
    }
}

// Any N: a work-group per row, three strided passes over the row (the second
// and third are served by the caches for rows of moderate length).
template <bool GELU, bool RMS>
__global__ __launch_bounds__(256) void layernorm_rows_any(const float* __restrict__ X, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float* __restrict__ Y,
                                                          int64_t rows, int N, float eps) {
    __shared__ float slots[16];
    const int64_t row = blockIdx.x;
    const float* x = X + row * (int64_t)N;
    float s = 0.f;
    if (!RMS) for (int j = threadIdx.x; j < N; j += 256) s += x[j];
    const float mu = RMS ? 0.f : block_reduce<OpSum, 4>(s, slots) / (float)N;
    float q = 0.f;
    for (int j = threadIdx.x; j < N; j += 256) { float d = x[j] - mu; q += d * d; }
    const float var = block_reduce<OpSum, 4>(q, slots) / (float)N;
    const float rstd = fast_rsq(var + eps);
    float* y = Y + row * (int64_t)N;
    for (int j = threadIdx.x; j < N; j += 256) {
        float o = (x[j] - mu) * rstd * (gamma ? gamma[j] : 1.f) + (beta ? beta[j] : 0.f);
        y[j] = GELU ? gelu_tanh(o) : o;
    }
}

// Row softmax, a work-group per row, any N.  X and Y may be the same buffer: a thread
// reads and writes only its own elements (no __restrict__ here for that reason).
__global__ __launch_bounds__(256) void softmax_rows_any(const float* X, float* Y, int64_t rows, int N) {
    __shared__ float slots[16];
    const int64_t row = blockIdx.x;
    const float* x = X + row * (int64_t)N;
    float m = -INFINITY;
    for (int j = threadIdx.x; j < N; j += 256) m = fmaxf(m, x[j]);
    m = block_reduce<OpMax, 4>(m, slots);
    float s = 0.f;
    for (int j = threadIdx.x; j < N; j += 256) s += fast_exp2((x[j] - m) * kLog2e);
    s = block_reduce<OpSum, 4>(s, slots);
    const float inv = 1.0f / s;
    float* y = Y + row * (int64_t)N;
    for (int j = threadIdx.x; j < N; j += 256) y[j] = fast_exp2((x[j] - m) * kLog2e) * inv;
}

// In-place row softmax for rows of up to 1024 elements, N % 4 == 0 (the second launch behind a small GEMM): a wave
// per row, the row read once into registers, no LDS and no barrier.  The three-pass kernel above walks the row three
// times with a dependent round trip to the cache each (3.5 us on a [64,256] matrix against 2.4 us here, the launch floor).
template <int VPT>
__global__ __launch_bounds__(256) void softmax_rows_inplace(float* Y, int64_t rows, int N) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;   // wave-uniform
    float* y = Y + row * (int64_t)N;
    const int nv = N >> 2;
    float4v v[VPT];
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int j = lane + 64 * u;
        v[u] = j < nv ? load4(y + 4 * j) : float4v{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        m = fmaxf(m, fmaxf(fmaxf(v[u].x, v[u].y), fmaxf(v[u].z, v[u].w)));
    }
    m = wave_reduce<OpMax>(m);
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {   // exp2(-inf) = 0: slots past the row add nothing
        v[u].x = fast_exp2((v[u].x - m) * kLog2e); v[u].y = fast_exp2((v[u].y - m) * kLog2e);
        v[u].z = fast_exp2((v[u].z - m) * kLog2e); v[u].w = fast_exp2((v[u].w - m) * kLog2e);
        s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    const float inv = 1.0f / wave_reduce<OpSum>(s);
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int j = lane + 64 * u;
        if (j < nv) store4(y + 4 * j, v[u] * inv);
    }
}

struct LnPick { int tpr; int vpt; };  // tpr = 0: the any-N kernel

LnPick pick(int32_t N) {
    if (N % 4 != 0) return {0, 0};
    const int nv = N / 4;
    if (nv <= 64 * 4) {  // a wave per row up to N = 1024
        int vpt = (nv + 63) / 64;
        return {64, vpt <= 1 ? 1 : (vpt <= 2 ? 2 : 4)};
    }
    if (nv <= 256 * kMaxVec) {
        int vpt = (nv + 255) / 256;
        return {256, vpt <= 2 ? 2 : (vpt <= 4 ? 4 : (vpt <= 8 ? 8 : 16))};
    }
    return {0, 0};
}

template <int VPT, int OPK>
hipError_t launch_persist(const LayernormParams& p, hipStream_t stream) {
    dim3 grid((unsigned)(p.rows < kPersistGrid ? p.rows : kPersistGrid)), block(256);
    hipLaunchKernelGGL((rows_persist<VPT, OPK>), grid, block, 0, stream, p.X, p.gamma, p.beta, p.Y, p.rows, p.N, p.eps);
    return hipGetLastError();
}

template <int TPR, int VPT, int OPK>
hipError_t launch_vec(const LayernormParams& p, hipStream_t stream) {
    constexpr int RPB = 256 / TPR;
    dim3 grid((unsigned)((p.rows + RPB - 1) / RPB)), block(256);
    hipLaunchKernelGGL((rows_vec<TPR, VPT, OPK>), grid, block, 0, stream, p.X, p.gamma, p.beta, p.Y, p.rows, p.N, p.eps);
    return hipGetLastError();
}

// the register-resident kernels for N % 4 == 0 and N <= 16384; false: the caller takes its any-N kernel
template <int OPK>
bool launch_rows(const LayernormParams& p, hipStream_t stream, hipError_t* e) {
    const LnPick k = pick(p.N);
    if (k.tpr == 64) {
        switch (k.vpt) {
            case 1: *e = launch_vec<64, 1, OPK>(p, stream); break;
            case 2: *e = launch_vec<64, 2, OPK>(p, stream); break;
            default: *e = launch_vec<64, 4, OPK>(p, stream);
        }
        return true;
    }
    if (k.tpr == 256) {
        switch (k.vpt) {
            case 2: *e = launch_persist<2, OPK>(p, stream); break;
            case 4: *e = launch_persist<4, OPK>(p, stream); break;
            case 8: *e = launch_vec<256, 8, OPK>(p, stream); break;
            default: *e = launch_vec<256, 16, OPK>(p, stream);
        }
        return true;
    }
    return false;
}

void rows_shape(int64_t rows, int32_t N, LaunchShape& s, const char* const names[4]) {
    const LnPick k = pick(N);
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.grid[1] = s.grid[2] = 1;
    s.lds_bytes = 64;
    if (k.tpr == 0) { s.grid[0] = (uint32_t)rows; s.kernel = names[0]; }
    else if (k.tpr == 64) { s.grid[0] = (uint32_t)((rows + 3) / 4); s.kernel = names[1]; }
    else if (k.vpt <= 4) {
        s.grid[0] = (uint32_t)(rows < kPersistGrid ? rows : kPersistGrid);
        s.kernel = names[2];
    } else { s.grid[0] = (uint32_t)rows; s.kernel = names[3]; }
}

}  // namespace

LaunchShape layernorm_shape(int64_t rows, int32_t N, int32_t rms) {
    static const char* const names[4] = {"layernorm_rows_any", "layernorm_rows_vec<wave-per-row>", "layernorm_rows_persist",
                                         "layernorm_rows_vec<group-per-row>"};
    static const char* const rnames[4] = {"rmsnorm_rows_any", "rmsnorm_rows_vec<wave-per-row>", "rmsnorm_rows_persist",
                                          "rmsnorm_rows_vec<group-per-row>"};
    LaunchShape s{};
    rows_shape(rows, N, s, rms ? rnames : names);
    return s;
}

hipError_t layernorm_launch(const LayernormParams& p, hipStream_t stream) {
    hipError_t e = hipSuccess;
    if (p.rms ? launch_rows<kRms>(p, stream, &e) : (p.gelu ? launch_rows<kLnGelu>(p, stream, &e) : launch_rows<kLn>(p, stream, &e))) return e;
    dim3 grid((unsigned)p.rows), block(256);
    if (p.rms)
        hipLaunchKernelGGL((layernorm_rows_any<false, true>), grid, block, 0, stream, p.X, p.gamma, p.beta, p.Y, p.rows, p.N, p.eps);
    else if (p.gelu)
        hipLaunchKernelGGL((layernorm_rows_any<true, false>), grid, block, 0, stream, p.X, p.gamma, p.beta, p.Y, p.rows, p.N, p.eps);
    else
        hipLaunchKernelGGL((layernorm_rows_any<false, false>), grid, block, 0, stream, p.X, p.gamma, p.beta, p.Y, p.rows, p.N, p.eps);
    return hipGetLastError();
}

LaunchShape softmax_shape(int64_t rows, int32_t N) {
    static const char* const names[4] = {"softmax_rows_any", "softmax_rows_vec<wave-per-row>", "softmax_rows_persist",
                                         "softmax_rows_vec<group-per-row>"};
    LaunchShape s{};
    rows_shape(rows, N, s, names);
    return s;
}

// X and Y may be the same buffer (every kernel reads a row completely before it writes it, or
// touches only a thread's own elements).
hipError_t softmax_launch(const SoftmaxParams& p, hipStream_t stream) {
    hipError_t e = hipSuccess;
    if (p.X != p.Y) {   // the register-resident kernels declare X and Y __restrict__
        const LayernormParams q{p.X, nullptr, nullptr, p.Y, p.rows, p.N, 0.f, 0, 0};
        if (launch_rows<kSoftmax>(q, stream, &e)) return e;
    }
    if (p.X == p.Y && p.N % 4 == 0 && p.N <= 1024 && (p.rows + 3) / 4 <= 0x7fffffff) {
        const dim3 grid((unsigned)((p.rows + 3) / 4));
        const int vpt = (p.N / 4 + 63) / 64;
        if (vpt <= 1) hipLaunchKernelGGL(softmax_rows_inplace<1>, grid, dim3(256), 0, stream, p.Y, p.rows, p.N);
        else if (vpt <= 2) hipLaunchKernelGGL(softmax_rows_inplace<2>, grid, dim3(256), 0, stream, p.Y, p.rows, p.N);
        else hipLaunchKernelGGL(softmax_rows_inplace<4>, grid, dim3(256), 0, stream, p.Y, p.rows, p.N);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(softmax_rows_any, dim3((unsigned)p.rows), dim3(256), 0, stream, p.X, p.Y, p.rows, p.N);
    return hipGetLastError();
}

}  // namespace hpct
