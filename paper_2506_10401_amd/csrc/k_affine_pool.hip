// Per-channel affine, ReLU and residual add over the planes of an NCHW tensor
// (Elementwise class of the paper's Table 1), followed either by a global
// average pool over each H*W plane (Reduction class, "mean") or by a plain
// store of the full tensor.  Memory-bound: both inputs are read once with
// 128-bit loads; with the pool the intermediate never leaves registers.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;  // threads per plane
constexpr int kUnroll = 4;    // independent 16-byte loads per input in flight per thread

template <bool AFF, bool RELU, bool RES>
__device__ __forceinline__ float4v chain(float4v x, float4v r, float sc, float sh) {
    float4v t = x;
    if (AFF) t = t * sc + sh;
    if (RELU) { t.x = fmaxf(t.x, 0.f); t.y = fmaxf(t.y, 0.f); t.z = fmaxf(t.z, 0.f); t.w = fmaxf(t.w, 0.f); }
    if (RES) t = t + r;
    return t;
}

// One work-group per plane p = n*C + c.  HW % 4 == 0, so every plane starts on
// a 16-byte boundary.  Thread t takes vectors t, t+kThreads, ...; kUnroll of them
// are loaded before any is used (a [56,56] plane is one such batch).  At 50 MB a
// launch lasts a few memory latencies, so what a wave does before its first
// vector load counts: the first batch is issued straight after the kernel
// arguments arrive, and only then are the channel's scale and shift fetched
// (a scalar load that depends on p % C) - in the other order every wave waits
// for that second round trip before it requests anything (measured 9.36 -> 9.16 us
// at [32,64,56,56]).  Slots past the end of the plane re-read its last vector
// (no branch between the loads) and are left out of the sum.  The plane sum is
// accumulated per thread in a fixed order, reduced over the wave on DPP and over
// the waves through LDS, so the result does not vary from run to run.
template <bool AFF, bool RELU, bool RES, bool POOL>
__global__ __launch_bounds__(kThreads) void affine_planes_vec(const float* __restrict__ X, const float* __restrict__ scale,
                                                         const float* __restrict__ shift, const float* __restrict__ R,
                                                         float* __restrict__ out, int C, int HW) {
    __shared__ float slots[kThreads / kWave];
    __builtin_assume(HW >= 4);   // (the launcher's precondition) no early exit in front of the argument loads: one scalar load fetches them all
    const unsigned p = blockIdx.x;
    const unsigned nv = (unsigned)HW >> 2;
    const size_t plane = (size_t)p * (unsigned)HW;
    const float* x = X + plane;
    const float* r = RES ? R + plane : nullptr;
    float4v xv[kUnroll], rv[kUnroll];
    auto issue = [&](unsigned base) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            unsigned j = base + u * kThreads + threadIdx.x;
            j = j < nv ? j : nv - 1;
            xv[u] = load4_nt(x + 4 * j);
            if (RES) rv[u] = load4_nt(r + 4 * j);
        }
    };
    issue(0);
    __builtin_amdgcn_sched_barrier(0);   // nothing below is moved above the first batch of loads
    const unsigned c = p % (unsigned)C;
    const float sc = AFF ? scale[c] : 1.f, sh = AFF ? shift[c] : 0.f;
    float* o = POOL ? nullptr : out + plane;
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    for (unsigned base = 0; base < nv; base += kThreads * kUnroll) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const unsigned j = base + u * kThreads + threadIdx.x;
            const float4v t = chain<AFF, RELU, RES>(xv[u], rv[u], sc, sh);
            if (j < nv) {
                if (POOL) acc = acc + t; else store4_nt(o + 4 * j, t);
            }
        }
        if (base + kThreads * kUnroll < nv) issue(base + kThreads * kUnroll);
    }
    if (POOL) {
        const float w = wave_reduce<OpSum>((acc.x + acc.y) + (acc.z + acc.w));
        if ((threadIdx.x & (kWave - 1)) == 0) slots[threadIdx.x / kWave] = w;
        __syncthreads();
        if (threadIdx.x == 0) {
            float s = slots[0];
#pragma unroll
            for (int i = 1; i < kThreads / kWave; ++i) s += slots[i];
            out[p] = s / (float)HW;
        }
    }
}

// Any HW (planes need not be 16-byte aligned): one element per thread per step.
template <bool POOL>
__global__ __launch_bounds__(256) void affine_planes_any(const float* __restrict__ X, const float* __restrict__ scale,
                                                         const float* __restrict__ shift, const float* __restrict__ R,
                                                         float* __restrict__ out, int C, int HW, int aff, int relu,
                                                         int res) {
    __shared__ float slots[16];
    const int64_t p = blockIdx.x;
    const int c = (int)(p % C);
    const float sc = aff ? scale[c] : 1.f, sh = aff ? shift[c] : 0.f;
    const float* x = X + p * (int64_t)HW;
    float acc = 0.f;
    for (int j = threadIdx.x; j < HW; j += 256) {
        float t = x[j];
        if (aff) t = t * sc + sh;
        if (relu) t = fmaxf(t, 0.f);
        if (res) t += R[p * (int64_t)HW + j];
        if (POOL) acc += t; else out[p * (int64_t)HW + j] = t;
    }
    if (POOL) {
        float s = block_reduce<OpSum, 4>(acc, slots);
        if (threadIdx.x == 0) out[p] = s / (float)HW;
    }
}

// 2x2 / stride-2 max pooling of NCHW planes (the pooling of a VGG block as an operator of its own).
// VEC (W % 4 == 0): a thread reads one 128-bit vector from each of the two input rows and writes two
// outputs; otherwise a thread per output.  Odd trailing rows / columns are dropped.
template <bool VEC>
__global__ __launch_bounds__(256) void maxpool2_planes(const float* __restrict__ X, float* __restrict__ out, int64_t planes,
                                                       int H, int W) {
    const int Hp = H >> 1, Wp = W >> 1;
    constexpr int E = VEC ? 2 : 1;            // outputs per thread
    const int wq = VEC ? W >> 2 : Wp;         // threads per output row
    const int64_t total = planes * Hp * wq;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int xq = (int)(t % wq);
        const int64_t r = t / wq;
        const int y = (int)(r % Hp);
        const int64_t pl = r / Hp;
        const float* src = X + (pl * H + 2 * y) * (int64_t)W + xq * 2 * E;
        float* dst = out + (pl * Hp + y) * (int64_t)Wp + xq * E;
        if (VEC) {
            const float4v a = load4_nt(src), b = load4_nt(src + W);
            const float m0 = fmaxf(fmaxf(a.x, a.y), fmaxf(b.x, b.y)), m1 = fmaxf(fmaxf(a.z, a.w), fmaxf(b.z, b.w));
            *reinterpret_cast<float2v*>(dst) = float2v{m0, m1};
        } else {
            dst[0] = fmaxf(fmaxf(src[0], src[1]), fmaxf(src[W], src[W + 1]));
        }
    }
}

template <bool AFF, bool RELU, bool RES>
hipError_t launch_vec(const AffineParams& p, hipStream_t stream) {
    dim3 grid((unsigned)p.planes), block(kThreads);
    if (p.pool)
        hipLaunchKernelGGL((affine_planes_vec<AFF, RELU, RES, true>), grid, block, 0, stream, p.X, p.scale, p.shift, p.R,
                           p.out, p.C, p.HW);
    else
        hipLaunchKernelGGL((affine_planes_vec<AFF, RELU, RES, false>), grid, block, 0, stream, p.X, p.scale, p.shift, p.R,
                           p.out, p.C, p.HW);
    return hipGetLastError();
}

}  // namespace

LaunchShape affine_shape(int64_t planes, int32_t HW, int32_t pool) {
    LaunchShape s{};
    s.grid[0] = (uint32_t)planes; s.grid[1] = s.grid[2] = 1;
    s.block[0] = HW % 4 == 0 ? kThreads : 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = HW % 4 == 0 ? (kThreads / kWave) * 4 : 64;
    if (HW % 4 == 0) s.kernel = pool ? "affine_planes_vec<pool>" : "affine_planes_vec<store>";
    else s.kernel = pool ? "affine_planes_any<pool>" : "affine_planes_any<store>";
    return s;
}

LaunchShape maxpool2_shape(int64_t planes, int32_t H, int32_t W) {
    LaunchShape s{};
    const bool vec = W % 4 == 0;
    const int64_t threads = planes * (H / 2) * (vec ? W / 4 : W / 2);
    const int64_t g = (threads + 255) / 256;
    s.grid[0] = (uint32_t)(g < 1 ? 1 : (g > 131072 ? 131072 : g)); s.grid[1] = s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    s.kernel = vec ? "maxpool2_planes<vec4>" : "maxpool2_planes<scalar>";
    return s;
}

hipError_t maxpool2_launch(const float* X, float* out, int64_t planes, int32_t H, int32_t W, hipStream_t stream) {
    const LaunchShape s = maxpool2_shape(planes, H, W);
    // 64-bit output vectors need an even pooled width, i.e. W % 4 == 0, and 8-byte aligned rows: both hold with W % 4 == 0
    if (W % 4 == 0) hipLaunchKernelGGL(maxpool2_planes<true>, dim3(s.grid[0]), dim3(256), 0, stream, X, out, planes, H, W);
    else hipLaunchKernelGGL(maxpool2_planes<false>, dim3(s.grid[0]), dim3(256), 0, stream, X, out, planes, H, W);
    return hipGetLastError();
}

hipError_t affine_launch(const AffineParams& p, hipStream_t stream) {
    if (p.HW % 4 == 0) {
        const int key = (p.has_affine ? 4 : 0) | (p.relu ? 2 : 0) | (p.has_residual ? 1 : 0);
        switch (key) {
            case 0: return launch_vec<false, false, false>(p, stream);
            case 1: return launch_vec<false, false, true>(p, stream);
            case 2: return launch_vec<false, true, false>(p, stream);
            case 3: return launch_vec<false, true, true>(p, stream);
            case 4: return launch_vec<true, false, false>(p, stream);
            case 5: return launch_vec<true, false, true>(p, stream);
            case 6: return launch_vec<true, true, false>(p, stream);
            default: return launch_vec<true, true, true>(p, stream);
        }
    }
    dim3 grid((unsigned)p.planes), block(256);
    if (p.pool)
        hipLaunchKernelGGL(affine_planes_any<true>, grid, block, 0, stream, p.X, p.scale, p.shift, p.R, p.out, p.C, p.HW,
                           p.has_affine, p.relu, p.has_residual);
    else
        hipLaunchKernelGGL(affine_planes_any<false>, grid, block, 0, stream, p.X, p.scale, p.shift, p.R, p.out, p.C, p.HW,
                           p.has_affine, p.relu, p.has_residual);
    return hipGetLastError();
}

}  // namespace hpct
