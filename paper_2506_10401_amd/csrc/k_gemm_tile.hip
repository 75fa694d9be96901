// Tiled GEMM for outputs large enough to fill the chip, with the epilogues of
// the fused Matmul chains in registers (Table 1 of the paper: ComputeIntensive
// "matmul", Elementwise "add, relu", Reduction "mean, softmax"; the
// [Matmul, Dropout, Mean, Softmax] group of its Section 5.3), and the two small
// kernels that finish a mean over the columns and a softmax over the rows.
//
// gemm_tile: a work-group of four waves owns a 128 x 128 output tile, a wave
// 64 x 64 of it as 2 x 2 accumulators of v_mfma_f32_32x32x2_f32 (64 x 64 tiles,
// one accumulator per wave, when 128-tiles would be too few to fill the chip).  K is walked
// in chunks of 16 through a double-buffered LDS stage: the global loads of
// chunk t+1 are issued before the MFMAs of chunk t and written to the other
// buffer after them, one barrier per chunk.
//
// Fragment layout.  In a 32x32x2 MFMA lane l supplies A[l%32][l/32] and
// B[l/32][l%32].  Lane half h = l/32 reads k = 8t+4h .. 8t+4h+3 of its A row
// with one 128-bit LDS read; MFMA e (0..3) of that group therefore contracts
// k = {8t+e, 8t+4+e} and its B fragment is the 32-bit read Bs[8t+4h+e][col].
// Row strides: A rows are 20 words apart (16 lanes x 4 words of a 128-bit read
// cover all 64 banks), B rows tile + 8 words (the two lane halves, 4 rows apart,
// land on disjoint bank halves).
//
// Epilogue.  Register r of accumulator (i, j) is output row
// 64 wm + 32 i + 8 (r/4) + 4 h + r%4, column 64 wn + 32 j + l%32.  Bias, ReLU
// and the hash dropout act on it in place; the result is either stored or, for
// a mean over the last dimension, summed over the tile's columns in a fixed
// order and written as one partial per (column tile, row) for the finishing
// kernel, so results do not depend on scheduling.
#include <type_traits>
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int BK = 16;
constexpr int LDA = 20;
constexpr int kThreads = 256;
constexpr int kXcds = 8;

// T = tile edge, 128 or 64: a wave owns (T/2) x (T/2) as WB x WB accumulators, WB = T/64.
// 128: three work-groups per CU (one wave of each per SIMD), up to 168 registers per lane, 64 of them
// accumulators (a budget of 128 for four groups spills once the chunk loop keeps its LDS pointers and
// buffer offsets in registers: 4096 x 1024 x 4096 106 TFLOP/s against 130 with three groups).
// 64: for outputs with too few 128-tiles to fill the chip; 16 accumulator registers.
// BT: W is stored transposed ([N,K] row-major, the layout of a linear layer's weight).  Its tile is
// then staged and read exactly like the A tile (rows = output columns, 128-bit reads along k):
// the MFMA's A and B operands have mirror-image lane layouts.
template <int T, bool VEC, bool BT, bool ACT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 8))) void gemm_tile(GemmParams p, int tiles_n, int items) {
    constexpr int TM = T, TN = T, WB = T / 64, LDB = T + 8;
    // one LDS block: the two stages of the A and B tiles, and after the chunk loop the waves' output strips
    constexpr int kAs = TM * LDA, kBs = BT ? TN * LDA : BK * LDB;
    constexpr int QW = TN / 2, EXP = QW + 8;   // a wave's quadrant is QW columns wide; pitch of its output strip
    constexpr int kSmem = 2 * kAs + 2 * kBs > 4 * 32 * EXP ? 2 * kAs + 2 * kBs : 4 * 32 * EXP;
    __shared__ __attribute__((aligned(16))) float smem[kSmem];
    float (*As)[kAs] = reinterpret_cast<float (*)[kAs]>(smem);
    float (*Bs)[kBs] = reinterpret_cast<float (*)[kBs]>(smem + 2 * kAs);
    __shared__ float rs[2][TM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int M = p.M, K = p.K, N = p.N;

    // a contiguous range of items goes to the same L2 domain (and runs there at the same time)
    int item;
    {
        const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        const int q = items / kXcds, r = items % kXcds;
        item = x * q + (x < r ? x : r) + j;
    }
    // grouped order: runs of 8 tile rows, column-major inside a run, so such a range covers a compact
    // block of tiles (8 rows x n columns) and shares both its A rows and its B columns in L2
    const int tiles = items / p.ksplit;
    const int ks = item / tiles;          // K slice (0 without split-K); a slice's tiles are neighbours
    item -= ks * tiles;
    const int tiles_m = tiles / tiles_n;  // tile rows of all the matrices of a batch, one after the other
    const int run = item / (8 * tiles_n), in_run = item - run * 8 * tiles_n;
    const int rows = tiles_m - run * 8 < 8 ? tiles_m - run * 8 : 8;
    const int tmv = run * 8 + in_run % rows, tn = in_run / rows;
    const int tiles_m1 = (M + TM - 1) / TM;          // tile rows of one matrix
    const int bz = tmv / tiles_m1, tm = tmv - bz * tiles_m1;
    const int m0 = tm * TM, n0 = tn * TN;
    // this work-group's slice of K (split-K: the slices' partial products go to the workspace and
    // split_k_finish adds them in slice order and applies the epilogue)
    const int kc = p.ksplit > 1 ? (((K + p.ksplit - 1) / p.ksplit + BK - 1) / BK) * BK : K;
    const int k_lo = ks * kc;
    const int k_hi = k_lo + kc < K ? k_lo + kc : K;

    // staging coordinates: A rows ar (+64) at k offset ak; B rows bk (+ BSTEP) at column offset bn
    constexpr int BSTEP = kThreads / (TN / 4);   // B rows covered by one pass of the work-group
    const int ar = tid >> 2, ak = (tid & 3) * 4;
    const int bk = tid / (TN / 4), bn = (tid % (TN / 4)) * 4;
    const float* __restrict__ X = p.X + bz * p.sX;
    const float* __restrict__ W = p.W + bz * p.sW;
    float* __restrict__ Yb = p.Y + bz * p.sY;

    float4v ra[WB], rb[WB];
    // VEC: raw buffer loads.  A lane's byte offset inside its tile's rows is worked out once; a lane outside
    // the matrix (row >= M, column >= N) gets an offset beyond the descriptor's size, for which the hardware
    // returns 0 without touching memory, so the chunk loop has no address arithmetic, select or zero fill on
    // the vector ALU (which does not overlap the MFMAs) and the chunk offset rides in the scalar operand.
    // Only the last chunk of a K slice can be partial; that case is a scalar branch.
    constexpr unsigned kOob = 0x80000000u;
    constexpr int kWord3 = 0x00020000;   // descriptor word 3 for plain 32-bit data
    unsigned a_voff[WB], b_voff[WB];
    __amdgpu_buffer_rsrc_t a_rs, b_rs;
    if (VEC) {
        a_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(X) + (int64_t)m0 * K, 0, 0x7fffffff, kWord3);
        if (BT) b_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W) + (int64_t)n0 * K, 0, 0x7fffffff, kWord3);
#pragma unroll
        for (int i = 0; i < WB; ++i) {
            a_voff[i] = m0 + ar + 64 * i < M ? (unsigned)(((ar + 64 * i) * K + ak) * 4) : kOob;
            if (BT) b_voff[i] = n0 + ar + 64 * i < N ? (unsigned)(((ar + 64 * i) * K + ak) * 4) : kOob;
            else b_voff[i] = n0 + bn < N ? (unsigned)(((bk + BSTEP * i) * N + bn) * 4) : kOob;
        }
    }
    auto fetch = [&](int k0) {
        if constexpr (VEC) {
            const bool tail = k0 + BK > k_hi;   // uniform
            if (!BT) b_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W) + (int64_t)k0 * N + n0, 0, 0x7fffffff, kWord3);
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                unsigned va = a_voff[i], vb = b_voff[i];
                if (tail) {
                    if (k0 + ak >= k_hi) va = kOob;
                    if (BT ? k0 + ak >= k_hi : k0 + bk + BSTEP * i >= k_hi) vb = kOob;
                }
                ra[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(a_rs, (int)va, k0 * 4, 0));
                rb[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(b_rs, (int)vb, BT ? k0 * 4 : 0, 0));
            }
        } else {
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                const int m = m0 + ar + 64 * i, k = k0 + ak;
                const float* src = X + (int64_t)m * K + k;
#pragma unroll
                for (int e = 0; e < 4; ++e) ra[i][e] = *((m < M && k + e < k_hi) ? src + e : X);
                if (BT) {
                    const int n = n0 + ar + 64 * i;
                    const float* wsrc = W + (int64_t)n * K + k;
#pragma unroll
                    for (int e = 0; e < 4; ++e) rb[i][e] = *((n < N && k + e < k_hi) ? wsrc + e : W);
                } else {
                    const int kk = k0 + bk + BSTEP * i, n = n0 + bn;
                    const float* wsrc = W + (int64_t)kk * N + n;
#pragma unroll
                    for (int e = 0; e < 4; ++e) rb[i][e] = *((kk < k_hi && n + e < N) ? wsrc + e : W);
                }
            }
        }
    };
    // write the chunk to LDS stage `buf` (scalar path: zero what lies outside the operands first)
    auto stash = [&](int k0, auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
#pragma unroll
        for (int i = 0; i < WB; ++i) {
            if constexpr (!VEC) {
                const int m = m0 + ar + 64 * i, k = k0 + ak;
                const int kk = k0 + bk + BSTEP * i, n = n0 + bn;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (!(m < M && k + e < k_hi)) ra[i][e] = 0.f;
                    if (BT ? !(n0 + ar + 64 * i < N && k + e < k_hi) : !(kk < k_hi && n + e < N)) rb[i][e] = 0.f;
                }
            }
            *reinterpret_cast<float4v*>(&As[buf][(ar + 64 * i) * LDA + ak]) = ra[i];
            if (BT) *reinterpret_cast<float4v*>(&Bs[buf][(ar + 64 * i) * LDA + ak]) = rb[i];
            else *reinterpret_cast<float4v*>(&Bs[buf][(bk + BSTEP * i) * LDB + bn]) = rb[i];
        }
    };

    float16v acc[WB][WB];
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto compute = [&](auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;   // compile-time: fragment reads are lane base + immediate
        // waves inside their MFMA block win the issue arbitration over waves that are staging
        __builtin_amdgcn_s_setprio(1);
        const float* a_base = &As[buf][(wm * (TM / 2) + l32) * LDA + 4 * h];
        const float* b_base = BT ? &Bs[buf][(wn * (TN / 2) + l32) * LDA + 4 * h] : &Bs[buf][(4 * h) * LDB + wn * (TN / 2) + l32];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float4v a[WB];
#pragma unroll
            for (int i = 0; i < WB; ++i) a[i] = *reinterpret_cast<const float4v*>(a_base + i * 32 * LDA + 8 * t);
            float4v bt[WB];
            if (BT) {
#pragma unroll
                for (int j = 0; j < WB; ++j) bt[j] = *reinterpret_cast<const float4v*>(b_base + j * 32 * LDA + 8 * t);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float b[WB];
#pragma unroll
                for (int j = 0; j < WB; ++j) b[j] = BT ? bt[j][e] : b_base[(8 * t + e) * LDB + j * 32];
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int j = 0; j < WB; ++j) acc[i][j] = mfma_32x32x2(a[i][e], b[j], acc[i][j]);
            }
        }
        __builtin_amdgcn_s_setprio(0);
    };

    const int nk = (k_hi - k_lo + BK - 1) / BK;
    constexpr std::integral_constant<int, 0> buf0{};
    constexpr std::integral_constant<int, 1> buf1{};
    auto step = [&](int k_next, auto cur_tag, auto next_tag) {
        fetch(k_next);
        __builtin_amdgcn_sched_barrier(0);  // the next chunk's loads are in flight before the MFMAs start
        compute(cur_tag);
        stash(k_next, next_tag);
        __syncthreads();
    };
    fetch(k_lo);
    stash(k_lo, buf0);
    __syncthreads();
    int t = 0;   // chunk t is in stage 0 here; two chunks per trip keep the stage index a compile-time constant
    for (; t + 2 < nk; t += 2) {
        step(k_lo + (t + 1) * BK, buf0, buf1);
        step(k_lo + (t + 2) * BK, buf1, buf0);
    }
    if (t + 1 < nk) {
        step(k_lo + (t + 1) * BK, buf0, buf1);
        compute(buf1);
    } else {
        compute(buf0);
    }

    if (p.ksplit > 1) {  // uniform over the grid: raw partial products of this K slice
        float* __restrict__ part = p.ws + (int64_t)ks * M * N;
#pragma unroll
        for (int j = 0; j < WB; ++j) {
            const int col = n0 + wn * (TN / 2) + j * 32 + l32;
#pragma unroll
            for (int i = 0; i < WB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wm * (TM / 2) + i * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (col < N && row < M) part[(int64_t)row * N + col] = acc[i][j][r];
                }
        }
        return;
    }

    // ---- epilogue in registers
    const float* __restrict__ bias = p.bias;
    if constexpr (VEC) {
        if (!p.mean && (N & 3) == 0) {  // uniform over the grid (a transposed W is read as vectors whatever N is)
            // An accumulator holds four consecutive rows of one column, so storing it directly writes 128-byte
            // pieces with 32-bit stores.  Instead each wave passes 32 rows of its quadrant at a time through a
            // strip of LDS of its own (the tiles' stages are free now) and writes them as 128-bit vectors along
            // the rows: four times fewer store instructions, which is what bounds products with a short K.
            // Pitch QW + 8: the two half-waves' rows (4 apart) fall on opposite halves of the 64 banks.
            constexpr int LPR = QW / 4, RPI = 64 / LPR;   // lanes per strip row, rows per store instruction
            __syncthreads();   // every wave has read the last chunk's stage
            float* ex = smem + wave * (32 * EXP);
            const int colw = n0 + wn * QW;
            const int rr = lane / LPR, c4 = (lane % LPR) * 4;
            float bv[WB];
#pragma unroll
            for (int j = 0; j < WB; ++j) bv[j] = (bias && colw + j * 32 + l32 < N) ? bias[colw + j * 32 + l32] : 0.f;
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                const int rowq = m0 + wm * (TM / 2) + i * 32;
#pragma unroll
                for (int j = 0; j < WB; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int lr = 8 * (r >> 2) + 4 * h + (r & 3);
                        float v = (acc[i][j][r] + bv[j]) * p.scale;
                        if (p.relu) v = ACT ? activate(v, p.relu) : fmaxf(v, 0.f);
                        if (p.dropout) {
                            const uint64_t off = (uint64_t)(rowq + lr) * (uint64_t)N + (uint64_t)(colw + j * 32 + l32);
                            v = dropout_u(off + p.seed) < p.drop_t ? 0.f : v * p.keep_scale;
                        }
                        ex[lr * EXP + j * 32 + l32] = v;
                    }
                // LDS operations of one wave execute in order; the fences only keep the compiler from moving them
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 32 / RPI; ++it) {
                    const int lr = it * RPI + rr;
                    const float4v v = *reinterpret_cast<const float4v*>(&ex[lr * EXP + c4]);
                    if (rowq + lr < M && colw + c4 < N)   // N % 4 == 0: a vector is inside or outside as a whole
                        *reinterpret_cast<float4v*>(&Yb[(int64_t)(rowq + lr) * N + colw + c4]) = v;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
            return;
        }
    }
    float rsum[WB][16];
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) rsum[i][r] = 0.f;
#pragma unroll
    for (int j = 0; j < WB; ++j) {
        const int col = n0 + wn * (TN / 2) + j * 32 + l32;
        const bool cok = col < N;
        const float bv = (bias && cok) ? bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < WB; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * (TM / 2) + i * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                float v = (acc[i][j][r] + bv) * p.scale;
                if (p.relu) v = ACT ? activate(v, p.relu) : fmaxf(v, 0.f);
                if (p.dropout) {
                    const uint64_t off = (uint64_t)row * (uint64_t)N + (uint64_t)col;
                    v = dropout_u(off + p.seed) < p.drop_t ? 0.f : v * p.keep_scale;
                }
                if (p.mean) {
                    rsum[i][r] += cok ? v : 0.f;
                } else if (cok && row < M) {
                    Yb[(int64_t)row * N + col] = v;
                }
            }
        }
    }
    if (p.mean) {  // uniform over the grid
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = rsum[i][r];  // over the 32 lanes of this half: four DPP steps inside each 16-lane row, then the two rows
                v += dpp_mov<0xB1>(v); v += dpp_mov<0x4E>(v); v += dpp_mov<0x141>(v); v += dpp_mov<0x140>(v);
                v += __shfl_xor(v, 16, 64);
                if (l32 == 0) rs[wn][wm * (TM / 2) + i * 32 + 8 * (r >> 2) + 4 * h + (r & 3)] = v;
            }
        __syncthreads();
        if (tid < TM && m0 + tid < M) p.ws[(int64_t)tn * M + m0 + tid] = rs[0][tid] + rs[1][tid];
    }
}

// Y = epilogue(sum_s ws[s]): the K slices' partial products added in slice order, then bias, ReLU
// and the hash dropout as in the tile kernel's own epilogue.  A thread per four columns when N % 4 == 0.
template <bool VEC>
__global__ __launch_bounds__(256) void split_k_finish(GemmParams p) {
    constexpr int E = VEC ? 4 : 1;
    const int64_t total = (int64_t)p.M * p.N / E, plane = (int64_t)p.M * p.N;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        const int64_t idx = v * E;
        float x[E];
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = 0.f;
        for (int s = 0; s < p.ksplit; ++s) {
            if (VEC) {
                const float4v t = load4_nt(p.ws + s * plane + idx);
                x[0] += t.x; x[1 % E] += t.y; x[2 % E] += t.z; x[3 % E] += t.w;
            } else {
                x[0] += p.ws[s * plane + idx];
            }
        }
        const int row = (int)(idx / p.N), col = (int)(idx - (int64_t)row * p.N);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float y = (x[e] + (p.bias ? p.bias[col + e] : 0.f)) * p.scale;
            if (p.relu) y = activate(y, p.relu);
            if (p.dropout) y = dropout_u((uint64_t)idx + (uint64_t)e + p.seed) < p.drop_t ? 0.f : y * p.keep_scale;
            x[e] = y;
        }
        if (VEC) store4_nt(p.Y + idx, float4v{x[0], x[1 % E], x[2 % E], x[3 % E]});
        else p.Y[idx] = x[0];
    }
}

// out[m] = (1/N) sum_t ws[t][m], the partial row sums added in tile order.  A thread per row;
// the T loads of a row are independent, so they are all in flight together.
__global__ __launch_bounds__(256) void rows_mean(const float* __restrict__ ws, float* __restrict__ out, int M, int T, float inv_n) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= M) return;
    float s = 0.f;
    int t = 0;
    for (; t + 8 <= T; t += 8) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = ws[(int64_t)(t + u) * M + m];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += x[u];
    }
    for (; t < T; ++t) s += ws[(int64_t)t * M + m];
    out[m] = s * inv_n;
}

// Both steps in one work-group, for small M * T (one launch less): out[m] = mean, then softmax in place.
constexpr int kFinThreads = 1024;
__device__ __forceinline__ void softmax_in_place(float* __restrict__ v, int M, float* slots) {
    const int tid = threadIdx.x;
    float mx = -INFINITY;
    for (int m = tid; m < M; m += kFinThreads) mx = fmaxf(mx, v[m]);
    mx = block_reduce<OpMax, kFinThreads / kWave>(mx, slots);
    float sum = 0.f;
    for (int m = tid; m < M; m += kFinThreads) {
        const float e = fast_exp2((v[m] - mx) * kLog2e);
        v[m] = e;
        sum += e;
    }
    sum = block_reduce<OpSum, kFinThreads / kWave>(sum, slots);
    const float inv = 1.0f / sum;
    for (int m = tid; m < M; m += kFinThreads) v[m] *= inv;
}

__global__ __launch_bounds__(kFinThreads) void rows_mean_softmax(const float* __restrict__ ws, float* __restrict__ out, int M,
                                                                int T, float inv_n, int softmax) {
    __shared__ float slots[kFinThreads / kWave];
    for (int m = threadIdx.x; m < M; m += kFinThreads) {
        float s = 0.f;
        for (int t = 0; t < T; ++t) s += ws[(int64_t)t * M + m];
        out[m] = s * inv_n;
    }
    if (softmax) softmax_in_place(out, M, slots);   // uniform; every thread reads back only what it wrote
}

// v = softmax(v) over a vector of M values, in place.  One work-group; every
// thread owns the elements tid, tid + 1024, ... in all three passes.
__global__ __launch_bounds__(kFinThreads) void vector_softmax(float* __restrict__ v, int M) {
    __shared__ float slots[kFinThreads / kWave];
    softmax_in_place(v, M, slots);
}

}  // namespace

// K slices for outputs whose 64 x 64 tiles alone cannot fill the chip: enough slices for about two
// work-groups per CU, each at least 256 deep, at most 8.  Not with the fused row sums.
int32_t gemm_ksplit(int32_t M, int32_t K, int32_t N, int32_t mean, int32_t batch) {
    if (mean || batch > 1) return 1;
    const int64_t tiles64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
    if (tiles64 >= 512) return 1;
    int64_t s = (512 + tiles64 - 1) / tiles64;
    if (s > K / 256) s = K / 256;
    if (s > 8) s = 8;
    return s < 2 ? 1 : (int32_t)s;
}

// 128 x 128 tiles when there are at least two per CU and they spread evenly over the 256 CUs
// (the busiest CU within 15 % of the average); otherwise 64 x 64 tiles, four times as many.
// Measured at K = 1024: 2048^2 85 -> 96 TFLOP/s, 2560^2 84 -> 92, 1536^2 47 -> 66 with the small tiles.
int gemm_tile_edge(int32_t M, int32_t N, int32_t batch = 1) {
    const int64_t tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128) * batch;
    const int64_t per_cu = (tiles + 255) / 256;
    return (tiles >= 512 && tiles * 100 >= per_cu * 256 * 85) ? 128 : 64;
}

LaunchShape gemm_tile_shape(int32_t M, int32_t N, int32_t ksplit, int32_t wt, int32_t batch) {
    const int t = gemm_tile_edge(M, N, batch);
    LaunchShape s{};
    s.grid[0] = (uint32_t)(((M + t - 1) / t) * ((N + t - 1) / t) * ksplit * batch); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    const int stages = 2 * t * LDA + 2 * (wt ? t * LDA : BK * (t + 8)), strips = 4 * 32 * (t / 2 + 8);
    s.lds_bytes = (uint32_t)(((stages > strips ? stages : strips) + 2 * t) * 4);
    if (wt) s.kernel = t == 128 ? "gemm_tile128<wt>" : (ksplit > 1 ? "gemm_tile64<wt,split-k>" : "gemm_tile64<wt>");
    else s.kernel = t == 128 ? "gemm_tile128" : (ksplit > 1 ? "gemm_tile64<split-k>" : "gemm_tile64");
    return s;
}

int32_t gemm_tile_col_tiles(int32_t M, int32_t N, int32_t batch) { const int t = gemm_tile_edge(M, N, batch); return (N + t - 1) / t; }

template <int T>
hipError_t launch_tile(const GemmParams& p, hipStream_t stream) {
    const int tiles_m = (p.M + T - 1) / T * p.batch, tiles_n = (p.N + T - 1) / T;
    const int items = tiles_m * tiles_n * p.ksplit;
    // (the vector instances address a tile's rows with 31-bit byte offsets)
    const bool fits = p.K <= (1 << 21) && p.N <= (1 << 24);
    // ACT: an activation other than ReLU (its code costs the plain instances 2-3 % when it is merely present)
    const bool act = p.relu > 1;
#define HPCT_TILE(V, B) do { \
        if (act) hipLaunchKernelGGL((gemm_tile<T, V, B, true>), dim3(items), dim3(kThreads), 0, stream, p, tiles_n, items); \
        else hipLaunchKernelGGL((gemm_tile<T, V, B, false>), dim3(items), dim3(kThreads), 0, stream, p, tiles_n, items); } while (0)
    if (p.wt) {   // both operands are read along k
        if (p.K % 4 == 0 && fits) HPCT_TILE(true, true); else HPCT_TILE(false, true);
    } else {
        if ((p.K % 4 == 0) && (p.N % 4 == 0) && fits) HPCT_TILE(true, false); else HPCT_TILE(false, false);
    }
#undef HPCT_TILE
    return hipGetLastError();
}

hipError_t gemm_tile_launch(const GemmParams& p, hipStream_t stream) {
    hipError_t e = gemm_tile_edge(p.M, p.N, p.batch) == 128 ? launch_tile<128>(p, stream) : launch_tile<64>(p, stream);
    if (e != hipSuccess || p.ksplit <= 1) return e;
    return gemm_split_finish_launch(p, stream);
}

// Y = epilogue(sum over the p.ksplit slices of p.ws[slice][M][N]) (also behind the column-streaming kernel of k_gemm_skinny.hip)
hipError_t gemm_split_finish_launch(const GemmParams& p, hipStream_t stream) {
    const bool vec = p.N % 4 == 0;
    const int64_t work = (int64_t)p.M * p.N / (vec ? 4 : 1);
    const unsigned grid = (unsigned)((work + 255) / 256 < 4096 ? (work + 255) / 256 : 4096);
    if (vec) hipLaunchKernelGGL((split_k_finish<true>), dim3(grid), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((split_k_finish<false>), dim3(grid), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t rows_finish_launch(const float* ws, float* out, int32_t M, int32_t T, int32_t N, int32_t softmax, hipStream_t stream) {
    if ((int64_t)M * T <= 16384) {  // a few loads per thread: one work-group does both steps
        hipLaunchKernelGGL(rows_mean_softmax, dim3(1), dim3(kFinThreads), 0, stream, ws, out, M, T, 1.0f / (float)N, softmax);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(rows_mean, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, stream, ws, out, M, T, 1.0f / (float)N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !softmax) return e;
    hipLaunchKernelGGL(vector_softmax, dim3(1), dim3(kFinThreads), 0, stream, out, M);
    return hipGetLastError();
}

}  // namespace hpct
