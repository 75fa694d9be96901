// GEMM anchor with bias / ReLU epilogues held in registers and an optional row
// softmax fused behind it (Table 1 of the paper: ComputeIntensive "matmul",
// Elementwise "add, relu", Reduction "softmax"; the fused Matmul ... Softmax
// chain of its Section 5.3).
//
// A work-group of four waves owns 16 rows x BN columns of the output, so with
// N <= BN a row's softmax never leaves the work-group.  The contraction runs on
// v_mfma_f32_16x16x4_f32: each wave accumulates BN/64 16x16 blocks.  X and W
// tiles of 32 k-values are staged through LDS, double buffered: the global
// loads of tile t+1 are in flight while tile t is multiplied.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int BM = 16;
constexpr int BK = 32;
constexpr int XS_LD = BK + 4;  // padded row of the X tile: conflict-free 128-bit fragment reads

// k-permutation inside a group of 16 k-values: lane quarter q = lane/16 reads
// k = 4q..4q+3 of the A row with one 128-bit LDS read; MFMA step t (t = 0..3)
// therefore contracts k = {t, 4+t, 8+t, 12+t}.  The B fragment of step t is
// W[4q + t][col], so both operands agree and the sum over k is complete after
// the four steps.
template <int BN, bool VEC>
__global__ __launch_bounds__(256) void gemm_rows16(const float* __restrict__ X, const float* __restrict__ W,
                                                   const float* __restrict__ bias, float* __restrict__ Y, int M, int K,
                                                   int N, int relu, int softmax) {
    constexpr int NB = BN / 64;        // 16-column blocks per wave
    constexpr int WS_LD = BN + 4;      // 4*WS_LD % 64 == 16: the four lane quarters hit distinct banks
    constexpr int WV = BK * BN / 4 / 256;  // float4 of the W tile per thread
    __shared__ float Xs[2][BM * XS_LD];
    __shared__ float Ws[2][BK * WS_LD];
    __shared__ float red[4][BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, l16 = lane & 15;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;

    // global -> register staging of one k-tile
    float4v xg = {0.f, 0.f, 0.f, 0.f};
    float4v wg[WV];
    const int xr = tid >> 3, xc = (tid & 7) * 4;  // threads 0..127: X tile row / k offset
    auto fetch = [&](int k0) {
        if (tid < 128) {
            const int m = m0 + xr, k = k0 + xc;
            xg = float4v{0.f, 0.f, 0.f, 0.f};
            if (m < M) {
                const float* src = X + (int64_t)m * K + k;
                if (VEC && k + 3 < K) xg = load4(src);
                else {
                    if (k < K) xg.x = src[0];
                    if (k + 1 < K) xg.y = src[1];
                    if (k + 2 < K) xg.z = src[2];
                    if (k + 3 < K) xg.w = src[3];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < WV; ++i) {
            const int v = tid + i * 256;
            const int kr = v / (BN / 4), c = (v % (BN / 4)) * 4;
            const int k = k0 + kr, n = n0 + c;
            float4v t = {0.f, 0.f, 0.f, 0.f};
            if (k < K) {
                const float* src = W + (int64_t)k * N + n;
                if (VEC && n + 3 < N) t = load4(src);
                else {
                    if (n < N) t.x = src[0];
                    if (n + 1 < N) t.y = src[1];
                    if (n + 2 < N) t.z = src[2];
                    if (n + 3 < N) t.w = src[3];
                }
            }
            wg[i] = t;
        }
    };
    auto stash = [&](int buf) {
        if (tid < 128) *reinterpret_cast<float4v*>(&Xs[buf][xr * XS_LD + xc]) = xg;
#pragma unroll
        for (int i = 0; i < WV; ++i) {
            const int v = tid + i * 256;
            const int kr = v / (BN / 4), c = (v % (BN / 4)) * 4;
            *reinterpret_cast<float4v*>(&Ws[buf][kr * WS_LD + c]) = wg[i];
        }
    };

    float4v acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = float4v{0.f, 0.f, 0.f, 0.f};

    const int nt = (K + BK - 1) / BK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int t = 0; t < nt; ++t) {
        const int cur = t & 1;
        if (t + 1 < nt) fetch((t + 1) * BK);
#pragma unroll
        for (int g = 0; g < BK / 16; ++g) {
            const float4v a = *reinterpret_cast<const float4v*>(&Xs[cur][l16 * XS_LD + g * 16 + q * 4]);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float* wrow = &Ws[cur][(g * 16 + q * 4 + s) * WS_LD + wave * (BN / 4) + l16];
#pragma unroll
                for (int b = 0; b < NB; ++b) acc[b] = mfma_16x16x4(a[s], wrow[b * 16], acc[b]);
            }
        }
        if (t + 1 < nt) stash(cur ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds rows 4q..4q+3 (register r) of column col(b) per block
    float bv[NB];
    bool cok[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int n = n0 + wave * (BN / 4) + b * 16 + l16;
        cok[b] = n < N;
        bv[b] = (bias && cok[b]) ? bias[n] : 0.f;
        acc[b] = acc[b] + bv[b];
        if (relu) {
            acc[b].x = fmaxf(acc[b].x, 0.f); acc[b].y = fmaxf(acc[b].y, 0.f);
            acc[b].z = fmaxf(acc[b].z, 0.f); acc[b].w = fmaxf(acc[b].w, 0.f);
        }
    }
    if (softmax) {
        // row max over the 16 lanes of a DPP row, the NB blocks and the four waves
        float4v mx = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (cok[b]) { mx.x = fmaxf(mx.x, acc[b].x); mx.y = fmaxf(mx.y, acc[b].y); mx.z = fmaxf(mx.z, acc[b].z); mx.w = fmaxf(mx.w, acc[b].w); }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v = mx[r];
            v = fmaxf(v, dpp_mov<0xB1>(v)); v = fmaxf(v, dpp_mov<0x4E>(v));
            v = fmaxf(v, dpp_mov<0x141>(v)); v = fmaxf(v, dpp_mov<0x140>(v));
            mx[r] = v;
        }
        if (l16 == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][q * 4 + r] = mx[r];
        }
        __syncthreads();
        float4v sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = q * 4 + r;
            const float m = fmaxf(fmaxf(red[0][row], red[1][row]), fmaxf(red[2][row], red[3][row]));
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float e = cok[b] ? fast_exp2((acc[b][r] - m) * kLog2e) : 0.f;
                acc[b][r] = e;
                sum[r] += e;
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v = sum[r];
            v += dpp_mov<0xB1>(v); v += dpp_mov<0x4E>(v); v += dpp_mov<0x141>(v); v += dpp_mov<0x140>(v);
            sum[r] = v;
        }
        if (l16 == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][q * 4 + r] = sum[r];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = q * 4 + r;
            const float inv = 1.0f / ((red[0][row] + red[1][row]) + (red[2][row] + red[3][row]));
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b][r] *= inv;
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = m0 + q * 4 + r;
        if (m < M) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
                if (cok[b]) Y[(int64_t)m * N + n0 + wave * (BN / 4) + b * 16 + l16] = acc[b][r];
        }
    }
}

int pick_bn(int32_t N) { return N <= 64 ? 64 : (N <= 128 ? 128 : 256); }

template <int BN>
hipError_t launch_bn(const GemmParams& p, hipStream_t stream) {
    dim3 grid((unsigned)((p.M + BM - 1) / BM), (unsigned)((p.N + BN - 1) / BN)), block(256);
    const bool vec = (p.K % 4 == 0) && (p.N % 4 == 0);
    if (vec)
        hipLaunchKernelGGL((gemm_rows16<BN, true>), grid, block, 0, stream, p.X, p.W, p.bias, p.Y, p.M, p.K, p.N, p.relu, p.softmax);
    else
        hipLaunchKernelGGL((gemm_rows16<BN, false>), grid, block, 0, stream, p.X, p.W, p.bias, p.Y, p.M, p.K, p.N, p.relu, p.softmax);
    return hipGetLastError();
}

}  // namespace

LaunchShape gemm_shape(int32_t M, int32_t, int32_t N, int32_t) {
    const int bn = pick_bn(N);
    LaunchShape s{};
    s.grid[0] = (uint32_t)((M + BM - 1) / BM); s.grid[1] = (uint32_t)((N + bn - 1) / bn); s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)(2 * BM * XS_LD * 4 + 2 * BK * (bn + 4) * 4 + 4 * BM * 4);
    s.kernel = bn == 64 ? "gemm_rows16<64>" : (bn == 128 ? "gemm_rows16<128>" : "gemm_rows16<256>");
    return s;
}

hipError_t gemm_launch(const GemmParams& p, hipStream_t stream) {
    switch (pick_bn(p.N)) {
        case 64: return launch_bn<64>(p, stream);
        case 128: return launch_bn<128>(p, stream);
        default: return launch_bn<256>(p, stream);
    }
}

}  // namespace hpct
