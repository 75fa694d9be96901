// Elementwise chains on strided views (Table 1 of the paper: Elementwise "add,
// sub, mul, div, sqrt, sin, cos, relu and etc."): v = a, or a (+, *, -, /) b for
// two views of one shape (broadcasting = a stride of 0), then up to eight unary
// steps in list order; contiguous output.  Memory-bound; one thread per output
// vector or element, the linear output index decoded into the input offsets.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

// BIN: kEltAdd .. kEltDiv, kEltNone (one operand)
template <int BIN>
__device__ __forceinline__ float combine(float x, float y) {
    return BIN == kEltAdd ? x + y : BIN == kEltMul ? x * y : BIN == kEltSub ? x - y : BIN == kEltDiv ? x / y : x;
}

// One unary step on the E values of a thread.  The step code is uniform over the grid, so the
// switch costs a scalar branch; sqrt and the division above are the correctly rounded ones, the
// transcendental functions the full-range library routines.
template <int E>
__device__ __forceinline__ void unary_step(float (&v)[E], int code, float scale) {
    switch (code) {
        case kUnRelu:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = fmaxf(v[i], 0.f);
            break;
        case kUnGelu:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = gelu_tanh(v[i]);
            break;
        case kUnScale:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] *= scale;
            break;
        case kUnSqrt:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = sqrtf(v[i]);
            break;
        case kUnSin:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = sinf(v[i]);
            break;
        case kUnCos:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = cosf(v[i]);
            break;
        case kUnExp:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = expf(v[i]);
            break;
        case kUnTanh:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = tanhf(v[i]);
            break;
        case kUnSigmoid:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = 1.f / (1.f + expf(-v[i]));
            break;
        case kUnRelu6:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = fminf(fmaxf(v[i], 0.f), 6.f);
            break;
        case kUnAbs:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = fabsf(v[i]);
            break;
        case kUnNeg:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = -v[i];
            break;
        case kUnSquare:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = v[i] * v[i];
            break;
        case kUnLog:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = logf(v[i]);
            break;
        case kUnSilu:
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = v[i] / (1.f + expf(-v[i]));
            break;
        default:  // kUnHardswish
#pragma unroll
            for (int i = 0; i < E; ++i) v[i] = v[i] * fminf(fmaxf(v[i] + 3.f, 0.f), 6.f) * (1.f / 6.f);
            break;
    }
}

// Vectors (VEC) or elements a thread has in flight per pass.  A thread that moves one 16-byte
// vector per operand lives about as long as the memory latency, and the bytes in flight of a full
// chip of such waves are too few for the HBM rate; two independent loads per operand make up for it
// ([8192,4096] + bias row, ReLU: 1 -> 51.6 us, 2 -> 45.3, 4 -> 47.2, 8 -> 49.3).
constexpr int kEltU = 2;

// VEC: the last dimension is contiguous in a (stride 1), contiguous or broadcast in b (stride 1 or 0),
// its extent, every other stride and the bases are multiples of 4 elements.
// IDX: int32_t when the element count fits (32-bit divisions in the index decode), else int64_t.
template <int BIN, bool VEC, typename IDX>
__global__ __launch_bounds__(256) void eltwise_map(EltwiseParams p) {
    constexpr int E = VEC ? 4 : 1;
    const int64_t total = p.total / E;
    const int last = p.nd - 1;
    const bool b_scalar = BIN != kEltNone && p.sb[last] == 0;
    for (int64_t base = (int64_t)blockIdx.x * (256 * kEltU) + threadIdx.x; base < total; base += (int64_t)gridDim.x * (256 * kEltU)) {
        float v[kEltU][E];
        int64_t oa[kEltU], ob[kEltU];
#pragma unroll
        for (int u = 0; u < kEltU; ++u) {
            const int64_t g = base + u * 256;
            IDX rem = (IDX)((g < total ? g : total - 1) * E);   // past the end: the last vector again, not stored
            oa[u] = 0; ob[u] = 0;
#pragma unroll
            for (int d = kEltwiseDims - 1; d >= 0; --d) {
                if (d < p.nd) {
                    const IDX n = (IDX)p.shape[d];
                    const IDX q = rem / n;
                    const IDX i = rem - q * n;
                    oa[u] += (int64_t)i * p.sa[d];
                    if (BIN != kEltNone) ob[u] += (int64_t)i * p.sb[d];
                    rem = q;
                }
            }
        }
        if (VEC) {
            float4v x[kEltU], y[kEltU];
#pragma unroll
            for (int u = 0; u < kEltU; ++u) x[u] = load4_nt(p.a + oa[u]);
            if (BIN != kEltNone) {
                if (b_scalar) {
#pragma unroll
                    for (int u = 0; u < kEltU; ++u) { const float s = p.b[ob[u]]; y[u] = float4v{s, s, s, s}; }
                } else {
#pragma unroll
                    for (int u = 0; u < kEltU; ++u) y[u] = load4_nt(p.b + ob[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < kEltU; ++u) {
                if (BIN == kEltNone) y[u] = x[u];
                v[u][0] = combine<BIN>(x[u].x, y[u].x); v[u][E > 1 ? 1 : 0] = combine<BIN>(x[u].y, y[u].y);
                v[u][E > 2 ? 2 : 0] = combine<BIN>(x[u].z, y[u].z); v[u][E > 3 ? 3 : 0] = combine<BIN>(x[u].w, y[u].w);
            }
        } else {
            float x[kEltU], y[kEltU];
#pragma unroll
            for (int u = 0; u < kEltU; ++u) { x[u] = p.a[oa[u]]; y[u] = BIN != kEltNone ? p.b[ob[u]] : 0.f; }
#pragma unroll
            for (int u = 0; u < kEltU; ++u) v[u][0] = combine<BIN>(x[u], y[u]);
        }
        uint32_t steps = p.un;   // walked by shifting: no memory access per step
        for (int k = 0; k < p.n_un; ++k, steps >>= 4) {
            const int code = (int)(steps & 15u);
#pragma unroll
            for (int u = 0; u < kEltU; ++u) unary_step<E>(v[u], code, p.scale);
        }
#pragma unroll
        for (int u = 0; u < kEltU; ++u) {
            const int64_t g = base + u * 256;
            if (g < total) {
                if (VEC) store4_nt(p.out + g * 4, float4v{v[u][0], v[u][E > 1 ? 1 : 0], v[u][E > 2 ? 2 : 0], v[u][E > 3 ? 3 : 0]});
                else p.out[g] = v[u][0];
            }
        }
    }
}

unsigned grid_for(int64_t work) {
    const int64_t g = (work + 256 * kEltU - 1) / (256 * kEltU);
    return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

template <int BIN>
void launch_bin(const EltwiseParams& p, dim3 grid, hipStream_t stream) {
    const bool i32 = p.total <= 0x7fffffff;
    if (p.vec) {
        if (i32) hipLaunchKernelGGL((eltwise_map<BIN, true, int32_t>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((eltwise_map<BIN, true, int64_t>), grid, dim3(256), 0, stream, p);
    } else {
        if (i32) hipLaunchKernelGGL((eltwise_map<BIN, false, int32_t>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((eltwise_map<BIN, false, int64_t>), grid, dim3(256), 0, stream, p);
    }
}

}  // namespace

LaunchShape eltwise_shape(const EltwiseParams& p) {
    LaunchShape s{};
    s.grid[0] = grid_for(p.total / (p.vec ? 4 : 1)); s.grid[1] = s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    if (p.op == kEltNone) s.kernel = p.vec ? "eltwise_unary<vec4>" : "eltwise_unary<scalar>";
    else s.kernel = p.vec ? "eltwise_binary<vec4>" : "eltwise_binary<scalar>";
    return s;
}

hipError_t eltwise_launch(const EltwiseParams& p, hipStream_t stream) {
    const dim3 grid(grid_for(p.total / (p.vec ? 4 : 1)));
    switch (p.op) {
        case kEltAdd: launch_bin<kEltAdd>(p, grid, stream); break;
        case kEltMul: launch_bin<kEltMul>(p, grid, stream); break;
        case kEltSub: launch_bin<kEltSub>(p, grid, stream); break;
        case kEltDiv: launch_bin<kEltDiv>(p, grid, stream); break;
        default: launch_bin<kEltNone>(p, grid, stream); break;
    }
    return hipGetLastError();
}

}  // namespace hpct
