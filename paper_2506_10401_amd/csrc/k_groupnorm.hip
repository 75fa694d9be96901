// Group normalisation of an NCHW tensor with an optional ReLU (Reduction and Elementwise classes of the
// paper's Table 1; the "norm" of the activation-and-norm fusions its Section 5.1 describes as Level-2
// tasks).  The C channels form G groups of C/G neighbours; image n and group g share one mean and one
// variance over their (C/G) H W elements, which are contiguous in NCHW: a row of a [N G, (C/G) H W] matrix.
// G = C is instance normalisation, G = 1 layer normalisation over C, H and W.  gamma / beta act per channel.
//
// A work-group per row.  Rows of up to 32768 elements are read once and held in registers for the mean, the
// variance (two passes, as in the layer normalisation kernels) and the output - by 256 threads up to 8192
// elements, by 1024 beyond (a 56 x 56 layer with 8 channels per group has rows of 25088: 29.1 -> 13 us against
// three passes over the row); still longer rows are walked three times, the second and third time out of the caches.
// 128-bit access when H W is a multiple of 4 (a vector then lies inside one channel).
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;
constexpr int kRegVecs = 8;   // vectors per thread that the register variant holds

template <bool RELU>
__device__ __forceinline__ float4v gn_out(float4v v, float mean, float inv, float ga, float be) {
    float4v y = (v - mean) * (inv * ga) + be;
    if (RELU) { y.x = fmaxf(y.x, 0.f); y.y = fmaxf(y.y, 0.f); y.z = fmaxf(y.z, 0.f); y.w = fmaxf(y.w, 0.f); }
    return y;
}

template <bool REG, bool RELU, int NT>
__global__ __launch_bounds__(NT) void groupnorm_rows(const float* __restrict__ X, const float* __restrict__ gamma,
                                                           const float* __restrict__ beta, float* __restrict__ Y,
                                                           int G, int Cg, int HW, float eps) {
    __shared__ float slots[NT / kWave];
    const int64_t row = blockIdx.x;
    const int g = (int)(row % G);
    const int L = Cg * HW, nv = L >> 2;
    const float* x = X + row * (int64_t)L;
    float* y = Y + row * (int64_t)L;
    const int tid = threadIdx.x;
    float4v v[REG ? kRegVecs : 1];
    float s = 0.f;
    if (REG) {
#pragma unroll
        for (int u = 0; u < kRegVecs; ++u) {
            const int j = tid + u * NT;
            v[u] = j < nv ? load4(x + 4 * j) : float4v{0.f, 0.f, 0.f, 0.f};
            s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
        }
    } else {
        for (int j = tid; j < nv; j += NT) {
            const float4v t = load4(x + 4 * j);
            s += (t.x + t.y) + (t.z + t.w);
        }
    }
    const float mean = block_reduce<OpSum, NT / kWave>(s, slots) / (float)L;
    float q = 0.f;
    if (REG) {
#pragma unroll
        for (int u = 0; u < kRegVecs; ++u) {
            if (tid + u * NT < nv) {
                const float4v d = v[u] - mean;
                q += (d.x * d.x + d.y * d.y) + (d.z * d.z + d.w * d.w);
            }
        }
    } else {
        for (int j = tid; j < nv; j += NT) {
            const float4v d = load4(x + 4 * j) - mean;
            q += (d.x * d.x + d.y * d.y) + (d.z * d.z + d.w * d.w);
        }
    }
    const float var = block_reduce<OpSum, NT / kWave>(q, slots) / (float)L;
    const float inv = 1.0f / sqrtf(var + eps);
    if (REG) {
#pragma unroll
        for (int u = 0; u < kRegVecs; ++u) {
            const int j = tid + u * NT;
            if (j < nv) {
                const int c = g * Cg + (4 * j) / HW;
                store4_nt(y + 4 * j, gn_out<RELU>(v[u], mean, inv, gamma ? gamma[c] : 1.f, beta ? beta[c] : 0.f));
            }
        }
    } else {
        for (int j = tid; j < nv; j += NT) {
            const int c = g * Cg + (4 * j) / HW;
            store4_nt(y + 4 * j, gn_out<RELU>(load4(x + 4 * j), mean, inv, gamma ? gamma[c] : 1.f, beta ? beta[c] : 0.f));
        }
    }
}

// Any H W: an element per thread and step, three passes.
template <bool RELU>
__global__ __launch_bounds__(kThreads) void groupnorm_rows_any(const float* __restrict__ X, const float* __restrict__ gamma,
                                                               const float* __restrict__ beta, float* __restrict__ Y,
                                                               int G, int Cg, int HW, float eps) {
    __shared__ float slots[kThreads / kWave];
    const int64_t row = blockIdx.x;
    const int g = (int)(row % G);
    const int L = Cg * HW;
    const float* x = X + row * (int64_t)L;
    float* y = Y + row * (int64_t)L;
    float s = 0.f;
    for (int i = threadIdx.x; i < L; i += kThreads) s += x[i];
    const float mean = block_reduce<OpSum, kThreads / kWave>(s, slots) / (float)L;
    float q = 0.f;
    for (int i = threadIdx.x; i < L; i += kThreads) { const float d = x[i] - mean; q += d * d; }
    const float var = block_reduce<OpSum, kThreads / kWave>(q, slots) / (float)L;
    const float inv = 1.0f / sqrtf(var + eps);
    for (int i = threadIdx.x; i < L; i += kThreads) {
        const int c = g * Cg + i / HW;
        float t = (x[i] - mean) * (inv * (gamma ? gamma[c] : 1.f)) + (beta ? beta[c] : 0.f);
        if (RELU) t = fmaxf(t, 0.f);
        y[i] = t;
    }
}

}  // namespace

constexpr int kBigThreads = 1024;

LaunchShape groupnorm_shape(const GroupnormParams& p) {
    LaunchShape s{};
    s.grid[0] = (uint32_t)(p.Nb * p.G); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (kThreads / kWave) * 4;
    const int64_t L = (int64_t)p.Cg * p.HW;
    if (p.HW % 4) s.kernel = "groupnorm_rows_any";
    else if (L <= kThreads * 4 * kRegVecs) s.kernel = "groupnorm_rows<registers>";
    else if (L <= kBigThreads * 4 * kRegVecs) { s.kernel = "groupnorm_rows<registers,1024>"; s.block[0] = kBigThreads; s.lds_bytes = (kBigThreads / kWave) * 4; }
    else s.kernel = "groupnorm_rows<three passes>";
    return s;
}

hipError_t groupnorm_launch(const GroupnormParams& p, hipStream_t stream) {
    const dim3 grid((unsigned)(p.Nb * p.G));
    const int64_t L = (int64_t)p.Cg * p.HW;
    const bool vec = p.HW % 4 == 0 && ((((uintptr_t)p.X) | ((uintptr_t)p.Y)) & 15) == 0;
#define HPCT_GN(K, NT) hipLaunchKernelGGL(K, grid, dim3(NT), 0, stream, p.X, p.gamma, p.beta, p.Y, p.G, p.Cg, p.HW, p.eps)
    if (!vec) { if (p.relu) HPCT_GN(groupnorm_rows_any<true>, kThreads); else HPCT_GN(groupnorm_rows_any<false>, kThreads); }
    else if (L <= kThreads * 4 * kRegVecs) {
        if (p.relu) HPCT_GN((groupnorm_rows<true, true, kThreads>), kThreads); else HPCT_GN((groupnorm_rows<true, false, kThreads>), kThreads);
    } else if (L <= kBigThreads * 4 * kRegVecs) {
        if (p.relu) HPCT_GN((groupnorm_rows<true, true, kBigThreads>), kBigThreads); else HPCT_GN((groupnorm_rows<true, false, kBigThreads>), kBigThreads);
    } else {
        if (p.relu) HPCT_GN((groupnorm_rows<false, true, kThreads>), kThreads); else HPCT_GN((groupnorm_rows<false, false, kThreads>), kThreads);
    }
#undef HPCT_GN
    return hipGetLastError();
}

}  // namespace hpct
