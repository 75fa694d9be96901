// GEMM with a short K (Table 1 of the paper: ComputeIntensive "matmul", here the shapes whose inner
// dimension is a few dozen: products of a tall and a wide matrix, batches of Q K^T with a small head
// dimension).  Per output element such a product does 2 K flop for 4 bytes written, so below K of
// about 40 it is bound by the stores and just above by the matrix cores; staging operands in LDS,
// which pays when every staged value is used for a long K loop, only adds barriers and latency here.
//
// gemm_direct: no LDS, no barrier.  A wave owns 32 rows x 128 columns of the output as four
// accumulators of v_mfma_f32_32x32x2_f32 and loads its operands from global memory (they are small and
// stay in L2) straight into the MFMA layout:
//   * the MFMA contracts two k per instruction, one from each half-wave h.  The wave walks K in chunks
//     of 32 and gives half-wave h the k range [16 h, 16 h + 16) of the chunk, so MFMA s of a chunk
//     contracts k = s and k = 16 + s: lane (l, h) needs X[row l][16 h .. 16 h + 15] - four 128-bit
//     loads along its row - as A operands;
//   * accumulator j holds the columns 4 l + j, l = 0..31, of the wave's 128, so one 128-bit load of
//     W[k][4 l .. 4 l + 3] is the B operand of all four accumulators for that k (16 loads per chunk),
//     and at the end a lane holds four neighbouring columns of each of its rows: the output goes out as
//     128-bit stores, 512 contiguous bytes per half-wave, without any exchange.
// Rows, columns and k outside the operands are raw buffer loads at an offset beyond the descriptor's
// size: zeros, no branches.  The four waves of a work-group take four row blocks of the same 128
// columns, so their B loads meet in the CU's vector cache.
//
// Measured against the tiled kernel (plain / this): 64 x (512 x 64 x 512) 32.0 / 26.2 us, 8192 x 64 x 8192
// 112 / 92-101, 16384 x 32 x 16384 313 / 299.  Timing-only copies of this kernel at K = 32 take 196 us without
// the stores and 202 us without the MFMAs (the stores alone would take 155, the MFMAs alone 119): supplying
// the operands from L2 costs as much as writing the output.  Two things that did not help: a transposed W
// read along its rows (four loads per column and lane; 40 us against the tiled kernel's 32 for the batch
// above, so a transposed W stays with the tiled kernel), and persistent work-groups that issue the next
// tile's loads ahead of the current tile's stores (31.5 us against 26.2).
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;
constexpr int kXcds = 8;
constexpr int DM = 128, DN = 128;   // a work-group's tile: four waves of 32 x 128
constexpr int DK = 32;              // k per chunk

template <bool ACT>
__global__ __launch_bounds__(kThreads) void gemm_direct(GemmParams p, int tiles_n, int items) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int M = p.M, K = p.K, N = p.N;

    // a contiguous range of tiles goes to the same L2 domain; inside it runs of 8 tile rows, column-major
    // (tile rows of all the matrices of a batch one after the other)
    int item;
    {
        const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        const int q = items / kXcds, r = items % kXcds;
        item = x * q + (x < r ? x : r) + j;
    }
    const int tiles_m = items / tiles_n;
    const int run = item / (8 * tiles_n), in_run = item - run * 8 * tiles_n;
    const int rows = tiles_m - run * 8 < 8 ? tiles_m - run * 8 : 8;
    const int tmv = run * 8 + in_run % rows, tn = in_run / rows;
    const int tiles_m1 = (M + DM - 1) / DM;
    const int bz = tmv / tiles_m1, tm = tmv - bz * tiles_m1;
    const int m0 = tm * DM + wave * 32, n0 = tn * DN;
    if (m0 >= M) return;   // the whole wave (uniform); there are no barriers in this kernel

    const float* __restrict__ X = p.X + bz * p.sX;
    const float* __restrict__ W = p.W + bz * p.sW;
    float* __restrict__ Y = p.Y + bz * p.sY;
    constexpr unsigned kOob = 0x80000000u;
    constexpr int kWord3 = 0x00020000;
    const bool row_ok = m0 + l32 < M;
    const bool col_ok = n0 + 4 * l32 < N;   // N % 4 == 0: the lane's four columns are inside or outside together

    // byte offsets of this lane's loads inside a chunk (the chunk offset rides in the descriptor and the scalar operand)
    unsigned a_off[4], b_off[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_off[i] = row_ok ? (unsigned)((l32 * K + 16 * h + 4 * i) * 4) : kOob;
#pragma unroll
    for (int s = 0; s < 16; ++s) b_off[s] = col_ok ? (unsigned)(((16 * h + s) * N + 4 * l32) * 4) : kOob;   // k = 16 h + s
    const int rows_here = M - m0 < 32 ? M - m0 : 32;   // rows of X this wave may touch

    float16v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    for (int k0 = 0; k0 < K; k0 += DK) {
        const bool tail = k0 + DK > K;   // uniform; K % 4 == 0: a quad of k is inside or outside as a whole
        // both descriptors end where their operand ends (seen from this chunk's base), so an offset that is wrong
        // for any reason reads 0 instead of a neighbour: rows of X beyond the wave's, k beyond K, columns beyond W
        const __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(X) + (int64_t)m0 * K + k0, 0,
                                                                              ((rows_here - 1) * K + (K - k0)) * 4, kWord3);
        const __amdgpu_buffer_rsrc_t b_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W) + (int64_t)k0 * N + n0, 0,
                                                                              (int)(((int64_t)(K - k0) * N - n0) * 4), kWord3);
        float4v a[4], b[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned v = a_off[i];
            if (tail && k0 + 16 * h + 4 * i >= K) v = kOob;
            a[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(a_rs, (int)v, 0, 0));
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            unsigned v = b_off[s];
            if (tail && k0 + 16 * h + s >= K) v = kOob;
            b[s] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(b_rs, (int)v, 0, 0));
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {   // k = k0 + 16 h + s
            const float av = a[s >> 2][s & 3];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = mfma_32x32x2(av, b[s][j], acc[j]);
        }
    }

    // ---- epilogue: register r of accumulator j is row 8 (r / 4) + 4 h + r % 4, column 4 l + j
    float4v bv = {0.f, 0.f, 0.f, 0.f};
    if (p.bias && col_ok) bv = load4(p.bias + n0 + 4 * l32);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + 8 * (r >> 2) + 4 * h + (r & 3);
        float4v v = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
        v = (v + bv) * p.scale;
        if (ACT) { v.x = activate(v.x, p.relu); v.y = activate(v.y, p.relu); v.z = activate(v.z, p.relu); v.w = activate(v.w, p.relu); }
        else if (p.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
        if (p.dropout) {
            const uint64_t off = (uint64_t)row * (uint64_t)N + (uint64_t)(n0 + 4 * l32) + p.seed;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = dropout_u(off + j) < p.drop_t ? 0.f : v[j] * p.keep_scale;
        }
        if (row < M && col_ok) store4_nt(Y + (int64_t)row * N + n0 + 4 * l32, v);   // non-temporal: 16384 x 32 x 16384 310 -> 276 us
    }
}

}  // namespace

// Short K, a row-major W, whole 128-bit vectors on every side, matrices that fill their tiles and enough
// tiles to fill the chip, and offsets that fit the 31 bits of a buffer load.  The row means are fused
// only in the tiled kernel.
bool gemm_direct_ok(int32_t M, int32_t K, int32_t N, int32_t mean, int32_t wt, int32_t batch) {
    if (mean || wt || K > 64 || (K & 3) || (N & 3) || N > (1 << 22)) return false;
    const int64_t tm = (M + DM - 1) / DM, tn = (N + DN - 1) / DN;
    if ((int64_t)M * N * 10 < tm * DM * tn * DN * 6) return false;   // matrices much smaller than a tile: mostly idle lanes
    return tm * tn * batch >= 256;
}

LaunchShape gemm_direct_shape(int32_t M, int32_t N, int32_t batch) {
    LaunchShape s{};
    s.grid[0] = (uint32_t)(((M + DM - 1) / DM) * ((N + DN - 1) / DN) * batch); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    s.kernel = "gemm_direct";
    return s;
}

hipError_t gemm_direct_launch(const GemmParams& p, hipStream_t stream) {
    const int tiles_m = (p.M + DM - 1) / DM * p.batch, tiles_n = (p.N + DN - 1) / DN;
    const int items = tiles_m * tiles_n;
    if (p.relu > 1) hipLaunchKernelGGL(gemm_direct<true>, dim3(items), dim3(kThreads), 0, stream, p, tiles_n, items);   // an activation other than ReLU
    else hipLaunchKernelGGL(gemm_direct<false>, dim3(items), dim3(kThreads), 0, stream, p, tiles_n, items);
    return hipGetLastError();
}

}  // namespace hpct
