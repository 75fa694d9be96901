// Products with one very small dimension (Table 1 of the paper: ComputeIntensive "matmul", here the
// matrix-vector products and tall-skinny shapes among them): Y[M,N] = X[M,K] W[K,N] with N <= 8, or with
// M <= 8 and W stored transposed ([N,K] row-major, a linear layer's weight applied to a few rows).  Such a
// product reads its large operand once and does 2 flop per 4 bytes of it per small column: it is bound by
// HBM, the matrix cores have nothing to add, and the tiled kernel's one-chunk pipeline keeps far too few
// bytes in flight for it (256 x 131072 times a vector: 1.8 ms, 74 GB/s).
//
// gemm_skinny streams the rows of the large operand A[R,K] like the row reductions do: TPR threads (a wave, or
// a work-group for few long rows) walk a row with four independent 128-bit loads in flight each, multiply every
// quad of k with the NS small columns - from S[K,NS] row-major (4 NS contiguous floats per quad of k) or from
// S[NS,K] (a 128-bit load per column) - and keep NS partial sums; a DPP wave reduction, for a work-group per row
// an LDS combine, in a fixed order.  Output element (r, j) goes to out[r * ldr + j * ldj], so the same kernel
// serves Y = X W (A = X, r = m) and Y^T = W^T-rows times X-rows (A = W^T, r = n, the few rows of X as S).
// Epilogue: bias, constant, activation.
//
// gemm_skinny_cols: M <= 8 under a row-major W[K,N], whose rows run along n.  A thread owns four columns, a wave one
// 1 KB piece of a row of W per load (four rows in flight), the few values of X it multiplies them with are uniform
// per wave; K is cut into slices over the work-groups, the four waves of a group take every fourth row of a slice
// and combine through LDS, the slices' partial results go to the workspace and the split-K finishing kernel of
// the tiled GEMM adds them in slice order and applies the epilogue.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;
constexpr int kU = 4;   // 128-bit loads of the large operand in flight per thread

struct SkinnyParams {
    const float* A; const float* S; const float* bias; float* out;
    int64_t R; int32_t K; int64_t ldr, ldj; int32_t bias_on_r; float scale; int32_t act;
    int64_t sA, sS, sO;   // batch strides (elements); blockIdx.y is the batch index
};

template <int NS, bool BT, int TPR>
__global__ __launch_bounds__(kThreads) void gemm_skinny(SkinnyParams p) {
    __shared__ float slots[NS][kThreads / kWave];
    constexpr int RPG = kThreads / TPR;   // rows per work-group
    const int t = threadIdx.x % TPR;
    const int64_t r = (int64_t)blockIdx.x * RPG + threadIdx.x / TPR;
    const bool live = r < p.R;             // (uniform per wave; a dead wave still takes part in the barriers of TPR = 256)
    const float* __restrict__ a = p.A + blockIdx.y * p.sA + (live ? r : 0) * (int64_t)p.K;
    const float* __restrict__ s = p.S + blockIdx.y * p.sS;
    const int nq = p.K >> 2;               // quads of k
    float acc[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[j] = 0.f;
    for (int base = 0; base < nq; base += TPR * kU) {
        float4v x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int q = base + u * TPR + t;
            x[u] = (live && q < nq) ? load4_nt(a + 4 * q) : float4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int q = base + u * TPR + t;
            if (q < nq) {
                if (BT) {
#pragma unroll
                    for (int j = 0; j < NS; ++j) {
                        const float4v w = load4(s + (int64_t)j * p.K + 4 * q);
                        acc[j] += (x[u].x * w.x + x[u].y * w.y) + (x[u].z * w.z + x[u].w * w.w);
                    }
                } else {
                    float w[4 * NS];   // rows 4 q .. 4 q + 3 of S[K, NS]: w[i * NS + j] = S[4 q + i][j]
#pragma unroll
                    for (int v = 0; v < NS; ++v) {
                        const float4v f = load4(s + (int64_t)q * (4 * NS) + 4 * v);
                        w[4 * v] = f.x; w[4 * v + 1] = f.y; w[4 * v + 2] = f.z; w[4 * v + 3] = f.w;
                    }
#pragma unroll
                    for (int j = 0; j < NS; ++j)
                        acc[j] += (x[u].x * w[j] + x[u].y * w[NS + j]) + (x[u].z * w[2 * NS + j] + x[u].w * w[3 * NS + j]);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[j] = wave_reduce<OpSum>(acc[j]);
    if (TPR > kWave) {
        const int wave = threadIdx.x / kWave;
        if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
            for (int j = 0; j < NS; ++j) slots[j][wave] = acc[j];
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            float v = slots[j][0];
#pragma unroll
            for (int w = 1; w < kThreads / kWave; ++w) v += slots[j][w];
            acc[j] = v;
        }
    }
    if (live && t == 0) {
        float* __restrict__ o = p.out + blockIdx.y * p.sO + r * p.ldr;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            float v = acc[j];
            if (p.bias) v += p.bias[p.bias_on_r ? r : j];
            v *= p.scale;
            if (p.act) v = activate(v, p.act);
            o[j * p.ldj] = v;
        }
    }
}

template <int MS>
__global__ __launch_bounds__(kThreads) void gemm_skinny_cols(const float* __restrict__ X, const float* __restrict__ W,
                                                             float* __restrict__ part, int M, int K, int N, int kslice) {
    __shared__ float4v comb[3][MS][64];
    const int lane = threadIdx.x & 63;
    const int kl = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // this wave takes rows kl, kl + 4, ... of the slice
    const int n4 = (blockIdx.x * 64 + lane) * 4;                          // first of this thread's four columns
    const bool col_ok = n4 < N;                                           // N % 4 == 0
    const int k_lo = blockIdx.y * kslice;
    const int k_hi = k_lo + kslice < K ? k_lo + kslice : K;
    float4v acc[MS];
#pragma unroll
    for (int m = 0; m < MS; ++m) acc[m] = float4v{0.f, 0.f, 0.f, 0.f};
    for (int k0 = k_lo + kl; k0 < k_hi; k0 += 4 * kU) {
        float4v w[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int k = k0 + 4 * u;
            w[u] = (col_ok && k < k_hi) ? load4_nt(W + (int64_t)k * N + n4) : float4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int k = k0 + 4 * u;
            if (k < k_hi) {   // uniform per wave
#pragma unroll
                for (int m = 0; m < MS; ++m) acc[m] = acc[m] + w[u] * X[(int64_t)m * K + k];
            }
        }
    }
    if (kl > 0) {
#pragma unroll
        for (int m = 0; m < MS; ++m) comb[kl - 1][m][lane] = acc[m];
    }
    __syncthreads();
    if (kl == 0 && col_ok) {
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            const float4v v = ((acc[m] + comb[0][m][lane]) + comb[1][m][lane]) + comb[2][m][lane];
            store4(part + ((int64_t)blockIdx.y * M + m) * N + n4, v);
        }
    }
}

// K slices of the column-streaming kernel: about 1024 work-groups, at least 64 rows of W per slice, at most 64 slices
int cols_slices(int32_t K, int32_t N) {
    const int64_t blocks = (N / 4 + 63) / 64;
    int64_t s = (1024 + blocks - 1) / blocks;
    if (s > K / 64) s = K / 64;
    if (s > 64) s = 64;
    return (int)(s < 1 ? 1 : s);
}

template <int NS>
void launch_ns(const SkinnyParams& p, bool bt, bool group, int batch, hipStream_t stream) {
    const int rpg = group ? 1 : kThreads / kWave;
    const dim3 grid((unsigned)((p.R + rpg - 1) / rpg), (unsigned)batch), block(kThreads);
    if (bt) {
        if (group) hipLaunchKernelGGL((gemm_skinny<NS, true, kThreads>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((gemm_skinny<NS, true, kWave>), grid, block, 0, stream, p);
    } else {
        if (group) hipLaunchKernelGGL((gemm_skinny<NS, false, kThreads>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((gemm_skinny<NS, false, kWave>), grid, block, 0, stream, p);
    }
}

// which operand is streamed: 1 = X (N small), 2 = the transposed W (M small), 3 = a row-major W along its rows
// (M small), 0 = neither
int skinny_mode(int32_t M, int32_t K, int32_t N, int32_t wt) {
    if ((K & 3) || K < 256) return 0;
    if (N <= 8 && (int64_t)M * K >= (int64_t)1 << 20) return 1;
    if (M <= 8 && wt && (int64_t)N * K >= (int64_t)1 << 20) return 2;
    if (M <= 8 && !wt && (N & 3) == 0 && (int64_t)N * K >= (int64_t)1 << 20) return 3;
    return 0;
}
// a work-group per row when a wave per row would leave the chip short of waves, or for long rows
bool skinny_group(int64_t R, int32_t K) { return K >= 16384 || (R < 4096 && K >= 2048); }

}  // namespace

// No softmax, row mean or dropout behind it; K a multiple of 4 and at least 256; a large operand of at least 4 MB;
// N <= 8 (any W layout), or M <= 8 with a transposed W.
bool gemm_skinny_ok(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t dropout, int32_t wt, int32_t batch) {
    if (softmax || mean || dropout) return false;
    const int mode = skinny_mode(M, K, N, wt);
    return mode != 0 && !(mode == 3 && batch > 1);   // (the column kernel's workspace holds one product)
}

size_t gemm_skinny_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t wt) {
    return skinny_mode(M, K, N, wt) == 3 ? (size_t)cols_slices(K, N) * (size_t)M * (size_t)N * 4 : 0;
}

LaunchShape gemm_skinny_shape(int32_t M, int32_t K, int32_t N, int32_t wt, int32_t batch) {
    const int mode = skinny_mode(M, K, N, wt);
    if (mode == 3) {
        LaunchShape s{};
        s.grid[0] = (uint32_t)((N / 4 + 63) / 64); s.grid[1] = (uint32_t)cols_slices(K, N); s.grid[2] = 1;
        s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
        s.lds_bytes = (uint32_t)(3 * M * 64 * 16);
        s.kernel = "gemm_skinny_cols";
        return s;
    }
    const int64_t R = mode == 1 ? M : N;
    const bool group = skinny_group(R, K);
    LaunchShape s{};
    s.grid[0] = (uint32_t)(group ? R : (R + 3) / 4); s.grid[1] = (uint32_t)batch; s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)((mode == 1 ? N : M) * (kThreads / kWave) * 4);
    s.kernel = mode == 1 ? (wt ? "gemm_skinny<rows of X,wt>" : "gemm_skinny<rows of X>") : "gemm_skinny<rows of W>";
    return s;
}

hipError_t gemm_skinny_launch(const GemmParams& g, hipStream_t stream) {
    const int mode = skinny_mode(g.M, g.K, g.N, g.wt);
    if (mode == 3) {
        const int slices = cols_slices(g.K, g.N);
        const int kslice = (((g.K + slices - 1) / slices) + 3) & ~3;
        const dim3 grid((unsigned)((g.N / 4 + 63) / 64), (unsigned)slices), block(kThreads);
#define HPCT_COLS(MS) hipLaunchKernelGGL(gemm_skinny_cols<MS>, grid, block, 0, stream, g.X, g.W, g.ws, g.M, g.K, g.N, kslice)
        switch (g.M) {
            case 1: HPCT_COLS(1); break;
            case 2: HPCT_COLS(2); break;
            case 3: HPCT_COLS(3); break;
            case 4: HPCT_COLS(4); break;
            case 5: HPCT_COLS(5); break;
            case 6: HPCT_COLS(6); break;
            case 7: HPCT_COLS(7); break;
            default: HPCT_COLS(8); break;
        }
#undef HPCT_COLS
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        GemmParams f = g;
        f.ksplit = slices;
        return gemm_split_finish_launch(f, stream);
    }
    SkinnyParams p{};
    p.K = g.K; p.bias = g.bias; p.out = g.Y; p.scale = g.scale; p.act = g.relu;
    p.sO = g.sY;
    int ns;
    bool bt;
    if (mode == 1) {   // rows of X times the few columns of W
        p.A = g.X; p.S = g.W; p.R = g.M; p.ldr = g.N; p.ldj = 1; p.bias_on_r = 0; p.sA = g.sX; p.sS = g.sW;
        ns = g.N; bt = g.wt != 0;
    } else {           // rows of the transposed W times the few rows of X: Y^T
        p.A = g.W; p.S = g.X; p.R = g.N; p.ldr = 1; p.ldj = g.N; p.bias_on_r = 1; p.sA = g.sW; p.sS = g.sX;
        ns = g.M; bt = true;
    }
    const bool group = skinny_group(p.R, g.K);
    const int batch = g.batch < 1 ? 1 : g.batch;
    switch (ns) {
        case 1: launch_ns<1>(p, bt, group, batch, stream); break;
        case 2: launch_ns<2>(p, bt, group, batch, stream); break;
        case 3: launch_ns<3>(p, bt, group, batch, stream); break;
        case 4: launch_ns<4>(p, bt, group, batch, stream); break;
        case 5: launch_ns<5>(p, bt, group, batch, stream); break;
        case 6: launch_ns<6>(p, bt, group, batch, stream); break;
        case 7: launch_ns<7>(p, bt, group, batch, stream); break;
        default: launch_ns<8>(p, bt, group, batch, stream); break;
    }
    return hipGetLastError();
}

}  // namespace hpct
