// GEMM anchor with bias / ReLU epilogues held in registers and an optional row
// softmax fused behind it (Table 1 of the paper: ComputeIntensive "matmul",
// Elementwise "add, relu", Reduction "softmax"; the fused Matmul ... Softmax
// chain of its Section 5.3).
//
// A work-group owns 16 rows x BN <= 256 columns of the output, so with N <= BN
// a row's softmax never leaves the work-group.  It has BN/64 column groups x 4
// k-groups of waves: a wave multiplies its 16 x 64 output slab over a quarter
// of K on v_mfma_f32_16x16x4_f32, with both operands loaded from global memory
// straight into the MFMA register layout (no LDS staging, no barrier in the
// k-loop, all loads of a 64-k step in flight at once).  The four k-groups'
// partial sums are combined through LDS in a fixed order.  This shape is chosen
// for small M, where only a handful of work-groups exist and the kernel is
// bound by the latency of its load -> MFMA chain rather than by throughput.
//
// Register layout.  In a 16x16x4 MFMA lane l supplies A[l%16][l/16] and
// B[l/16][l%16].  Lane quarter q = l/16 reads k = 4q..4q+3 of its A row with
// one 128-bit load; step s (0..3) of a 16-k group therefore contracts
// k = {s, 4+s, 8+s, 12+s} and its B fragment is W[4q+s][col].  The four 16x16
// blocks of a wave are interleaved in columns: block b, lane column j is output
// column 4j+b, so one 128-bit load of W[k][4j..4j+3] feeds all four blocks and
// a lane ends up with four consecutive output columns per row.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int BM = 16;
constexpr int KG = 4;   // k-groups of waves
// up to this many 16-row blocks the kernel whose waves share K (plus a softmax launch) beats this one: measured at
// K = N = 256 with the softmax, 16-row kernel -> K-sharing kernel: M = 64 10.6 -> 5.3 us, 1024 11.3 -> 7.0, 2048 12.0 -> 10.3,
// 4096 12.2 -> 17.5; at K = 1024, M = 64 30 -> 8.4
constexpr int kKsplit16MaxRowBlocks = 128;

// EXT: the instance that also carries the hash dropout and the row-sum output (kept out of the
// plain instance, whose 128-register budget at 1024 threads it would overflow)
// BT: W stored transposed ([N,K] row-major).  A lane's four B values of a 16-k group for one output
// column are then 16 contiguous bytes of that column's row; loading them lane by lane would make
// neighbouring lanes read different rows (a quarter of the load rate, 27 us instead of 9 for
// 64 x 256 x 256).  Instead a quad of lanes reads 64 contiguous bytes of one row and the wave
// turns the 16 rows x 16 k block round through a private LDS strip (rows 20 words apart: the
// 128-bit reads of 16 lanes cover all 64 banks).  A lane then owns columns l16, l16 + 16,
// l16 + 32, l16 + 48 of its wave's 64 instead of four neighbours.
template <int BN, bool VEC, bool EXT, bool BT>
__global__ __launch_bounds__(BN * 4) void gemm_rows16(GemmParams p) {
    const float* __restrict__ X = p.X + blockIdx.z * p.sX;   // blockIdx.z: the matrix of a batch
    const float* __restrict__ W = p.W + blockIdx.z * p.sW;
    const float* __restrict__ bias = p.bias;
    float* __restrict__ Y = p.Y + blockIdx.z * p.sY;
    const int M = p.M, K = p.K, N = p.N, relu = p.relu, softmax = p.softmax;
    constexpr int NG = BN / 64;  // column groups of waves
    __shared__ __attribute__((aligned(16))) float part[(KG - 1) * NG * 16 * 64];
    __shared__ float red[NG][BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, l16 = lane & 15;
    const int ng = wave % NG, kg = wave / NG;
    const int m0 = blockIdx.x * BM;
    const int cb = blockIdx.y * BN + ng * 64;              // first column of this wave
    const int ncol = cb + 4 * l16;                         // first of this lane's four columns (row-major W)
    const int mrow = m0 + l16;                             // A row this lane loads
    auto colb = [&](int b) { return BT ? cb + l16 + 16 * b : ncol + b; };   // output column of block b in this lane
    float* const strip = part + wave * (16 * 20);          // BT: this wave's 16 x 16 exchange strip (part is free until the k-loop ends)

    // this wave's slice of K: a multiple of 16 per group
    const int ks = ((K + KG - 1) / KG + 15) & ~15;
    const int kbeg = kg * ks;
    const int kend = kbeg + ks < K ? kbeg + ks : K;

    float4v acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[b] = float4v{0.f, 0.f, 0.f, 0.f};

    // Loads are branch-free: a predicate picks between the real address and the
    // tensor base (always readable) and the value is zeroed after every load of
    // the step has been issued, so all 20 loads are in flight together.  With
    // VEC (K % 4 == 0 and N % 4 == 0; kend is then a multiple of 4) a 4-vector
    // is entirely inside or entirely outside.
    constexpr int G = VEC ? (((EXT || BT) && BN == 256) ? 2 : 4) : 1;  // 16-k groups loaded together (fewer where registers are short)
    for (int k0 = kbeg; k0 < kend; k0 += 16 * G) {
        float4v a[G], w[G][4];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int k = k0 + 16 * g + 4 * q;
            const float* src = X + (int64_t)mrow * K + k;
            if (VEC) {
                a[g] = load4((mrow < M && k < kend) ? src : X);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) a[g][e] = *((mrow < M && k + e < kend) ? src + e : X);
            }
            if (BT) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {   // row (= output column) cb + 16 b + lane / 4, k = kt .. kt + 3
                    const int wr = cb + 16 * b + (lane >> 2), kt = k0 + 16 * g + 4 * (lane & 3);
                    const float* wsrc = W + (int64_t)wr * K + kt;
                    if (VEC) {
                        w[g][b] = load4((wr < N && kt < kend) ? wsrc : W);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) w[g][b][e] = *((wr < N && kt + e < kend) ? wsrc + e : W);
                    }
                }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const float* wsrc = W + (int64_t)(k + s) * N + ncol;
                    if (VEC) {
                        w[g][s] = load4((k + s < kend && ncol < N) ? wsrc : W);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) w[g][s][e] = *((k + s < kend && ncol + e < N) ? wsrc + e : W);
                    }
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // every load of the step is issued before anything uses one
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int k = k0 + 16 * g + 4 * q;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (!(mrow < M && k + e < kend)) a[g][e] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // BT: w[g][s] is still row cb + 16 s + lane / 4 at k = kt + e
                    const bool ok = BT ? (cb + 16 * s + (lane >> 2) < N && k0 + 16 * g + 4 * (lane & 3) + e < kend)
                                       : (k + s < kend && ncol + e < N);
                    if (!ok) w[g][s][e] = 0.f;
                }
        }
        if (BT) {   // turn each 16-row x 16-k block round: afterwards w[g][s][b] = W(k0 + 16 g + 4 q + s, column colb(b))
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float4v t[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    // LDS operations of one wave execute in order; the fences only keep the compiler from moving them
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    *reinterpret_cast<float4v*>(strip + (lane >> 2) * 20 + 4 * (lane & 3)) = w[g][b];
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    t[b] = *reinterpret_cast<const float4v*>(strip + l16 * 20 + 4 * q);
                }
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) w[g][s2] = float4v{t[0][s2], t[1][s2], t[2][s2], t[3][s2]};
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = mfma_16x16x4(a[g][s], w[g][s][b], acc[b]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- combine the k-groups: groups 1..3 publish, group 0 adds them in order
    if (BT) __syncthreads();   // the exchange strips share `part`: every wave has left its k-loop
    if (kg > 0) {
        float* dst = part + ((kg - 1) * NG + ng) * 16 * 64 + lane;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[(b * 4 + r) * 64] = acc[b][r];
    }
    __syncthreads();
    const bool lead = kg == 0;
    if (lead) {
#pragma unroll
        for (int g2 = 0; g2 < KG - 1; ++g2) {
            const float* src = part + (g2 * NG + ng) * 16 * 64 + lane;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[b][r] += src[(b * 4 + r) * 64];
        }
    }

    // ---- epilogue (lead waves): lane holds rows 4q..4q+3 (register r) of columns ncol..ncol+3 (block b)
    bool cok[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) cok[b] = colb(b) < N;
    if (lead) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float bv = (bias && cok[b]) ? bias[colb(b)] : 0.f;
            acc[b] = (acc[b] + bv) * p.scale;
            if (EXT && relu > 1) {   // (the further activations live in the EXT instances only: their code costs the plain ones 9 %)
                acc[b].x = activate(acc[b].x, relu); acc[b].y = activate(acc[b].y, relu);
                acc[b].z = activate(acc[b].z, relu); acc[b].w = activate(acc[b].w, relu);
            } else if (relu) {
                acc[b].x = fmaxf(acc[b].x, 0.f); acc[b].y = fmaxf(acc[b].y, 0.f);
                acc[b].z = fmaxf(acc[b].z, 0.f); acc[b].w = fmaxf(acc[b].w, 0.f);
            }
            if (EXT && p.dropout) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint64_t off = (uint64_t)(m0 + q * 4 + r) * (uint64_t)N + (uint64_t)colb(b);
                    acc[b][r] = dropout_u(off + p.seed) < p.drop_t ? 0.f : acc[b][r] * p.keep_scale;
                }
            }
        }
    }
    if (EXT && p.mean) {  // uniform over the grid: one partial row sum per (column tile, row), finished by another kernel
        if (lead) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = 0.f;
#pragma unroll
                for (int b = 0; b < 4; ++b) v += cok[b] ? acc[b][r] : 0.f;
                v += dpp_mov<0xB1>(v); v += dpp_mov<0x4E>(v); v += dpp_mov<0x141>(v); v += dpp_mov<0x140>(v);
                if (l16 == 0) red[ng][q * 4 + r] = v;
            }
        }
        __syncthreads();
        if (tid < BM && m0 + tid < M) {
            float t = red[0][tid];
#pragma unroll
            for (int g2 = 1; g2 < NG; ++g2) t += red[g2][tid];
            p.ws[(int64_t)blockIdx.y * M + m0 + tid] = t;
        }
        return;
    }
    if (softmax) {  // uniform over the work-group: every wave reaches the barriers
        float4v mx = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (lead) {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (cok[b]) { mx.x = fmaxf(mx.x, acc[b].x); mx.y = fmaxf(mx.y, acc[b].y); mx.z = fmaxf(mx.z, acc[b].z); mx.w = fmaxf(mx.w, acc[b].w); }
#pragma unroll
            for (int r = 0; r < 4; ++r) {  // over the 16 lanes that share a row
                float v = mx[r];
                v = fmaxf(v, dpp_mov<0xB1>(v)); v = fmaxf(v, dpp_mov<0x4E>(v));
                v = fmaxf(v, dpp_mov<0x141>(v)); v = fmaxf(v, dpp_mov<0x140>(v));
                mx[r] = v;
            }
            if (l16 == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) red[ng][q * 4 + r] = mx[r];
            }
        }
        __syncthreads();
        float4v sum = {0.f, 0.f, 0.f, 0.f};
        if (lead) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = q * 4 + r;
                float m = red[0][row];
#pragma unroll
                for (int g2 = 1; g2 < NG; ++g2) m = fmaxf(m, red[g2][row]);
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float e = cok[b] ? fast_exp2((acc[b][r] - m) * kLog2e) : 0.f;
                    acc[b][r] = e;
                    sum[r] += e;
                }
            }
        }
        __syncthreads();
        if (lead) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = sum[r];
                v += dpp_mov<0xB1>(v); v += dpp_mov<0x4E>(v); v += dpp_mov<0x141>(v); v += dpp_mov<0x140>(v);
                sum[r] = v;
            }
            if (l16 == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) red[ng][q * 4 + r] = sum[r];
            }
        }
        __syncthreads();
        if (lead) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = q * 4 + r;
                float t = red[0][row];
#pragma unroll
                for (int g2 = 1; g2 < NG; ++g2) t += red[g2][row];
                const float inv = 1.0f / t;
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b][r] *= inv;
            }
        }
    }
    if (lead) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + q * 4 + r;
            if (m < M) {
                float* dst = Y + (int64_t)m * N;
                if (!BT && VEC && cok[3]) store4(dst + ncol, float4v{acc[0][r], acc[1][r], acc[2][r], acc[3][r]});
                else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (cok[b]) dst[colb(b)] = acc[b][r];
                }
            }
        }
    }
}


// ---- small outputs: the contraction split over the waves of a work-group ----------------------------
// With few output rows the 16-row kernel above has only a handful of work-groups, each of which pulls
// all of W through one compute unit's vector-memory path - measured at 64 x 256 x 256: 5.3 of its 8 us
// pass before the last wave has issued its loads.  Here a work-group owns 16 rows x 32 columns and its
// 16 waves split K between them (wave w takes the 16-k groups w, w + 16, ...), so 64 x 256 x 256 runs
// on 32 compute units that each load 48 KB, and a wave's whole share is one step of loads.  Each wave
// multiplies two 16 x 16 blocks (block b, lane column j = output column 2j + b: one 64-bit load of W
// feeds both), the 16 partial tiles are added through LDS in wave order (fixed: bit-identical from run
// to run) by the first 512 threads, which apply the epilogue and store along the rows.  A row softmax
// cannot stay in the work-group any more; it follows as the in-place row kernel (a second launch).
// Cross-group exchange through global memory inside one launch was measured instead and is far
// slower: the release / acquire fences it needs write back and invalidate the whole L2 (15 - 35 us).
// The column block is the fast grid index: the row blocks that share a slice of W are neighbours in
// dispatch order modulo 8, i.e. they land on one XCD and that slice crosses into its L2 once.
constexpr int KS_CT = 32;            // columns per work-group
constexpr int KS_RS = KS_CT + 8;     // LDS row stride of a partial tile: the two lane halves of a 64-bit store hit disjoint banks

// The hot arguments are plain leading parameters (13 dwords), so that they arrive preloaded in scalar registers with the
// wave (build flag -amdgpu-kernarg-preload-count) and the first loads need no argument fetch; the dropout parameters,
// used only in the epilogue, stay in memory.
struct KsplitTail { int32_t dropout; uint32_t drop_t; float keep_scale; uint64_t seed; int32_t shared_w; };

template <bool VEC>
__global__ __launch_bounds__(1024) void gemm_ksplit16(const float* __restrict__ X0, const float* __restrict__ W0,
                                                      const float* __restrict__ bias, float* __restrict__ Y0, int M, int K, int N,
                                                      int act, float scale, KsplitTail tail) {
    // blockIdx.z: the matrix of a batch (contiguous matrices; one W for all when shared_w)
    const float* __restrict__ X = X0 + (int64_t)blockIdx.z * M * K;
    const float* __restrict__ W = W0 + (tail.shared_w ? 0 : (int64_t)blockIdx.z * K * N);
    float* __restrict__ Y = Y0 + (int64_t)blockIdx.z * M * N;
    __shared__ __attribute__((aligned(16))) float part[16][16 * KS_RS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, l16 = lane & 15;
    const int c0 = blockIdx.x * KS_CT, m0 = blockIdx.y * BM;
    const int mrow = m0 + l16, ncol = c0 + 2 * l16;
    const int groups = (K + 15) >> 4;

    float4v acc[2] = {float4v{0.f, 0.f, 0.f, 0.f}, float4v{0.f, 0.f, 0.f, 0.f}};
    // element offsets fit 32 bits (the plan refuses operands of 2^31 elements or more)
    const int arow = mrow * K, wcol = ncol;
    const bool rok = mrow < M, cok0 = ncol < N, cok1 = ncol + 1 < N;
    for (int g0 = wave; g0 < groups; g0 += 32) {   // two 16-k groups of this wave per trip, all their loads issued first
        const bool two = g0 + 16 < groups;         // wave-uniform
        float4v a[2];
        float2v w[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u == 1 && !two) break;
            const int k = 16 * (g0 + 16 * u) + 4 * q;
            const float* asrc = X + arow + k;
            if (VEC) {
                a[u] = load4((rok && k < K) ? asrc : X);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) a[u][e] = *((rok && k + e < K) ? asrc + e : X);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float* wsrc = W + (k + s) * N + wcol;
                if (VEC) {
                    w[u][s] = *reinterpret_cast<const float2v*>((k + s < K && cok0) ? wsrc : W);
                } else {
                    w[u][s][0] = *((k + s < K && cok0) ? wsrc : W);
                    w[u][s][1] = *((k + s < K && cok1) ? wsrc + 1 : W);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u == 1 && !two) break;
            const int k = 16 * (g0 + 16 * u) + 4 * q;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (!(rok && k + e < K)) a[u][e] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (!(k + s < K && cok0)) w[u][s][0] = 0.f;
                if (!(k + s < K && cok1)) w[u][s][1] = 0.f;
            }
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[b] = mfma_16x16x4(a[u][s], w[u][s][b], acc[b]);
        }
    }
    // lane holds rows 4q .. 4q+3 (register r) of columns 2 l16 + b
#pragma unroll
    for (int r = 0; r < 4; ++r)
        *reinterpret_cast<float2v*>(&part[wave][(4 * q + r) * KS_RS + 2 * l16]) = float2v{acc[0][r], acc[1][r]};
    __syncthreads();
    if (tid < BM * KS_CT) {
        const int row = tid / KS_CT, col = tid % KS_CT;
        float v = part[0][row * KS_RS + col];
#pragma unroll
        for (int g = 1; g < 16; ++g) v += part[g][row * KS_RS + col];
        const int m = m0 + row, c = c0 + col;
        if (m < M && c < N) {
            v = (v + (bias ? bias[c] : 0.f)) * scale;
            v = activate(v, act);
            if (tail.dropout) {
                const uint64_t off = (uint64_t)m * (uint64_t)N + (uint64_t)c;
                v = dropout_u(off + tail.seed) < tail.drop_t ? 0.f : v * tail.keep_scale;
            }
            Y[(int64_t)m * N + c] = v;
        }
    }
}

int pick_bn(int32_t N) { return N <= 64 ? 64 : (N <= 128 ? 128 : 256); }

template <int BN>
hipError_t launch_bn(const GemmParams& p, hipStream_t stream) {
    dim3 grid((unsigned)((p.M + BM - 1) / BM), (unsigned)((p.N + BN - 1) / BN), (unsigned)p.batch), block(BN * 4);
    const bool vec = (p.K % 4 == 0) && (p.N % 4 == 0);
    const bool ext = p.dropout || p.mean || p.relu > 1;
    if (p.wt) {
        if (vec && ext) hipLaunchKernelGGL((gemm_rows16<BN, true, true, true>), grid, block, 0, stream, p);
        else if (vec) hipLaunchKernelGGL((gemm_rows16<BN, true, false, true>), grid, block, 0, stream, p);
        else if (ext) hipLaunchKernelGGL((gemm_rows16<BN, false, true, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((gemm_rows16<BN, false, false, true>), grid, block, 0, stream, p);
    } else {
        if (vec && ext) hipLaunchKernelGGL((gemm_rows16<BN, true, true, false>), grid, block, 0, stream, p);
        else if (vec) hipLaunchKernelGGL((gemm_rows16<BN, true, false, false>), grid, block, 0, stream, p);
        else if (ext) hipLaunchKernelGGL((gemm_rows16<BN, false, true, false>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((gemm_rows16<BN, false, false, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace

// The tiled kernel takes over once its tiles give every XCD work - 32 tiles of 128 x 128, or fewer
// if K is long enough to be split into slices that make up for it; below that the 16-row kernel's
// many small work-groups finish sooner.  The fused row softmax exists only in the 16-row kernel.
bool gemm_use_tile(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t batch) {
    if (softmax && N <= kGemmSoftmaxMaxN) return false;   // fused: the row fits one work-group
    if ((int64_t)((M + 127) / 128) * ((N + 127) / 128) * batch >= 32) return true;
    const int64_t tiles64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
    return tiles64 * gemm_ksplit(M, K, N, mean, batch) >= 128 && gemm_ksplit(M, K, N, mean, batch) > 1;
}

// Few row blocks and a K worth splitting: the kernel whose waves share K (threshold: see kKsplit16MaxRowBlocks).
bool gemm_use_ksplit16(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t wt, int32_t batch) {
    if (mean || wt || K < 64) return false;
    if (gemm_use_tile(M, K, N, softmax, mean, batch)) return false;
    return (int64_t)((M + BM - 1) / BM) * batch <= kKsplit16MaxRowBlocks;
}

int32_t gemm_col_tiles(int32_t M, int32_t K, int32_t N) {
    return gemm_use_tile(M, K, N, 0, 1) ? gemm_tile_col_tiles(M, N) : (N + pick_bn(N) - 1) / pick_bn(N);
}

size_t gemm_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t batch) {
    if (mean) return (size_t)gemm_col_tiles(M, K, N) * (size_t)M * 4;
    if (!gemm_use_tile(M, K, N, softmax, 0, batch)) return 0;
    const int32_t s = gemm_ksplit(M, K, N, 0, batch);
    return s > 1 ? (size_t)s * (size_t)M * (size_t)N * 4 : 0;
}

LaunchShape gemm_shape(int32_t M, int32_t K, int32_t N, int32_t softmax, int32_t mean, int32_t wt, int32_t batch) {
    if (gemm_use_tile(M, K, N, softmax, mean, batch) && gemm_direct_ok(M, K, N, mean, wt, batch)) return gemm_direct_shape(M, N, batch);
    if (gemm_use_tile(M, K, N, softmax, mean, batch)) return gemm_tile_shape(M, N, gemm_ksplit(M, K, N, mean, batch), wt, batch);
    if (gemm_use_ksplit16(M, K, N, softmax, mean, wt, batch)) {
        LaunchShape s{};
        s.grid[0] = (uint32_t)((N + KS_CT - 1) / KS_CT); s.grid[1] = (uint32_t)((M + BM - 1) / BM); s.grid[2] = (uint32_t)batch;
        s.block[0] = 1024; s.block[1] = s.block[2] = 1;
        s.lds_bytes = (uint32_t)(16 * 16 * KS_RS * 4);
        s.kernel = "gemm_ksplit16<32>";
        return s;
    }
    const int bn = pick_bn(N);
    LaunchShape s{};
    s.grid[0] = (uint32_t)((M + BM - 1) / BM); s.grid[1] = (uint32_t)((N + bn - 1) / bn); s.grid[2] = (uint32_t)batch;
    s.block[0] = (uint32_t)(bn * 4); s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)(((KG - 1) * (bn / 64) * 16 * 64 + (bn / 64) * BM) * 4);
    if (wt) s.kernel = bn == 64 ? "gemm_rows16<64,wt>" : (bn == 128 ? "gemm_rows16<128,wt>" : "gemm_rows16<256,wt>");
    else s.kernel = bn == 64 ? "gemm_rows16<64>" : (bn == 128 ? "gemm_rows16<128>" : "gemm_rows16<256>");
    return s;
}

hipError_t gemm_launch(const GemmParams& p0, hipStream_t stream) {
    GemmParams p = p0;
    // rows wider than one work-group: the GEMM stores its epilogue's result, a second kernel takes
    // the row softmax of it in place
    if (p.batch < 1) p.batch = 1;
    const bool ks16 = !p.skinny && gemm_use_ksplit16(p.M, p.K, p.N, p0.softmax, p.mean, p.wt, p.batch);
    const bool split_softmax = p.softmax && (p.N > kGemmSoftmaxMaxN || ks16);
    if (split_softmax) p.softmax = 0;
    hipError_t e;
    p.ksplit = 1;
    if (p.skinny) return gemm_skinny_launch(p, stream);
    if (ks16) {
        dim3 grid((unsigned)((p.N + KS_CT - 1) / KS_CT), (unsigned)((p.M + BM - 1) / BM), (unsigned)p.batch);
        const KsplitTail tail{p.dropout, p.drop_t, p.keep_scale, p.seed, p.sW == 0 ? 1 : 0};
        if (p.K % 4 == 0 && p.N % 2 == 0)
            hipLaunchKernelGGL(gemm_ksplit16<true>, grid, dim3(1024), 0, stream, p.X, p.W, p.bias, p.Y, p.M, p.K, p.N, p.relu, p.scale, tail);
        else
            hipLaunchKernelGGL(gemm_ksplit16<false>, grid, dim3(1024), 0, stream, p.X, p.W, p.bias, p.Y, p.M, p.K, p.N, p.relu, p.scale, tail);
        e = hipGetLastError();
        if (e == hipSuccess && split_softmax) return softmax_launch(SoftmaxParams{p.Y, p.Y, (int64_t)p.M * p.batch, p.N}, stream);
        return e;
    }
    if (gemm_use_tile(p.M, p.K, p.N, p0.softmax, p.mean, p.batch)) {
        p.ksplit = gemm_ksplit(p.M, p.K, p.N, p.mean, p.batch);
        e = gemm_direct_ok(p.M, p.K, p.N, p.mean, p.wt, p.batch) ? gemm_direct_launch(p, stream) : gemm_tile_launch(p, stream);
    }
    else switch (pick_bn(p.N)) {
        case 64: e = launch_bn<64>(p, stream); break;
        case 128: e = launch_bn<128>(p, stream); break;
        default: e = launch_bn<256>(p, stream);
    }
    if (e == hipSuccess && split_softmax) return softmax_launch(SoftmaxParams{p.Y, p.Y, (int64_t)p.M * p.batch, p.N}, stream);   // sY = M N: the batch is one tall matrix
    if (e != hipSuccess || !p.mean) return e;
    return rows_finish_launch(p.ws, p.Y, p.M, gemm_col_tiles(p.M, p.K, p.N), p.N, p.softmax2, stream);
}

}  // namespace hpct
