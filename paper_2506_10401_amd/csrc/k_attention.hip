// Batched GEMM - softmax - GEMM, O = softmax_j(scale * Q K^T) V, head dim 32, 64 or 128
// (Table 1 of the paper: ComputeIntensive "matmul", Reduction "softmax").  The
// score matrix is never materialised: K/V are streamed in blocks of 64 keys
// through LDS (double buffered) and the softmax is evaluated online (running
// max m, running sum l, rescaled accumulator).
//
// Both contractions run transposed on v_mfma_f32_32x32x2_f32 so that a lane
// owns one query:
//     S^T[key, query] = sum_d K[key, d] Q[query, d]      A = K block, B = Q^T
//     O^T[d,   query] = sum_key V[key, d] P^T[key, query] A = V^T,    B = P^T
// In the 32x32 accumulator layout lane l holds column (query) l%32 and rows
// (keys) 8*(r/4) + 4*(l/32) + r%4, r = 0..15.  That is exactly the B-operand
// layout of a 2-deep MFMA step if step r contracts keys {8*(r/4)+r%4,
// 8*(r/4)+4+r%4}: the probabilities feed the second contraction straight from
// the accumulator registers, with the V fragment rows permuted to match.
// Row max needs one exchange between the two lane halves per key block; row
// sums stay per-half until the end.
//
// A wave owns 32 queries.  A work-group has NQW query waves x KS key groups:
// with KS = 2 the two key groups take alternate 32-key halves of every staged
// block for the same queries and merge their (m, l, O) states through LDS at
// the end, which puts two waves on every SIMD.  NQW = 4 (128 queries, eight
// waves) measured faster than two 64-query groups per CU, which stage every
// K/V block twice.
//
// CAUSAL: query i sees keys j <= i.  A work-group stops at the key block that
// holds its last query's diagonal; a wave skips (both contractions) every
// 32-key sub-block that lies wholly above its 32 queries' diagonal and masks
// inside the sub-blocks the diagonal crosses.  The work of a query block grows
// with its position, so the causal instance is PAIRed: a work-group of 64
// queries x 4 key groups (128-key staged blocks) handles query block i and then
// block n-1-i of the same batch, which gives every work-group the same number of
// key blocks to walk.
#include <type_traits>
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int QW = 32;        // queries per wave
constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 8.0f;  // log2 headroom of a probability before the softmax reference is moved
constexpr int kXcds = 8;      // work-groups are dealt round-robin to this many L2 domains

__device__ __forceinline__ float xchg_half(float v) {  // value held by lane ^ 32
    return __shfl_xor(v, 32, 64);
}

template <int D, int KS, int NQW, bool CAUSAL, bool PAIR>
__global__ __launch_bounds__(64 * NQW * KS) void attn_fwd(const float* __restrict__ Q, const float* __restrict__ K,
                                                         const float* __restrict__ V, float* __restrict__ O, int Lq,
                                                         int Lk, float scale_log2e) {
    constexpr int KLD = D + 4;                  // K row stride in LDS: conflict-free 128-bit fragment reads
    constexpr int VLD = D + 8;                  // V row stride: rows 4 apart land 32 banks apart
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int MROWS = 16 * DB + 2;          // rows of 64 floats one wave publishes for the merge
    constexpr int NT = 64 * NQW * KS;
    constexpr int QT = NQW * QW;                // queries per work-group (and pass)
    constexpr int KB = KS == 4 ? 128 : 64;      // keys per staged block
    constexpr int SUB = KB / 32 / KS;           // 32-key sub-blocks per wave per staged block
    constexpr int LD4 = KB * D / 4 / NT;        // float4 per thread per matrix per block
    static_assert(KB * D / 4 % NT == 0, "staging loop must divide evenly");
    static_assert((size_t)(2 * KB * (KLD + VLD)) >= (size_t)(KS - 1) * NQW * MROWS * 64, "merge area must fit in the stage buffers");
    extern __shared__ __align__(16) float lds[];
    float* const Ks = lds;                      // [2][KB*KLD]
    float* const Vs = lds + 2 * KB * KLD;       // [2][KB*VLD]

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: everything derived from it (key sub-block, masks' conditions) is then uniform for
    // the compiler too, so the rare tail / diagonal masking is a scalar branch instead of 32 selects per block
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int qwave = wave % NQW, kgrp = wave / NQW;
    // work item = (batch, query block); consecutive items share a batch's K/V and
    // are dealt to the same L2 domain, so each K/V block is fetched from HBM once
    const int nqb = (Lq + QT - 1) / QT;
    const int per_batch = PAIR ? (nqb + 1) / 2 : nqb;   // work items per batch
    int item;
    {
        const int items = gridDim.x;
        const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        const int qq = items / kXcds, r = items % kXcds;
        item = x * qq + (x < r ? x : r) + j;
    }
    const int b = item / per_batch;
    const int qb0 = item % per_batch;
    const float* Kb = K + (int64_t)b * Lk * D;
    const float* Vb = V + (int64_t)b * Lk * D;
    const int npass = (PAIR && nqb - 1 - qb0 != qb0) ? 2 : 1;
    // staging constants of this thread: float4 i of a block is key v / (D/4), dims 4 (v % (D/4)) .., v = tid + i NT
    const __amdgpu_buffer_rsrc_t k_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Kb), 0, Lk * D * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Vb), 0, Lk * D * 4, 0x00020000);
    unsigned kv_off[LD4];
    float* ks_ptr[LD4];
    float* vs_ptr[LD4];
#pragma unroll
    for (int i = 0; i < LD4; ++i) {
        const int v = tid + i * NT;
        const int kr = v / (D / 4), d = (v % (D / 4)) * 4;
        kv_off[i] = (unsigned)((kr * D + d) * 4);
        ks_ptr[i] = Ks + kr * KLD + d;
        vs_ptr[i] = Vs + kr * VLD + d;
    }
  for (int pass = 0; pass < npass; ++pass) {
    const int qb = pass == 0 ? qb0 : nqb - 1 - qb0;
    const int q0 = qb * QT + qwave * QW;

    // Q fragment, pre-multiplied by scale*log2(e): lane (query l32, half) holds
    // Q[q][8c + 4*half + t] in qf[c][t].
    float4v qf[D / 8];
    {
        const int q = q0 + l32;
        const float* src = Q + ((int64_t)b * Lq + (q < Lq ? q : 0)) * D + 4 * half;
#pragma unroll
        for (int c = 0; c < D / 8; ++c) {
            float4v t = load4(src + 8 * c);
            qf[c] = (q < Lq) ? t * scale_log2e : float4v{0.f, 0.f, 0.f, 0.f};
        }
    }

    // K/V staging through raw buffer loads: a thread's byte offsets inside a block are constants, the block
    // offset rides in the scalar operand, and only the last block can reach past Lk - then (a scalar branch)
    // lanes past the end get an offset beyond the descriptor's size, for which the hardware returns 0.  No
    // address arithmetic, select or zero fill per block on the vector ALU, which does not overlap the MFMAs.
    float4v kreg[LD4], vreg[LD4];
    auto fetch = [&](int key0) {
        if (key0 + KB <= Lk) {   // uniform; a branch of its own, so that whole blocks pay no compare / select per load
#pragma unroll
            for (int i = 0; i < LD4; ++i) {
                kreg[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(k_rs, (int)kv_off[i], key0 * D * 4, 0));
                vreg[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(v_rs, (int)kv_off[i], key0 * D * 4, 0));
            }
        } else {
#pragma unroll
            for (int i = 0; i < LD4; ++i) {
                const unsigned off = key0 + (tid + i * NT) / (D / 4) >= Lk ? 0x80000000u : kv_off[i];
                kreg[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(k_rs, (int)off, key0 * D * 4, 0));
                vreg[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(v_rs, (int)off, key0 * D * 4, 0));
            }
        }
    };
    auto stash = [&](auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
#pragma unroll
        for (int i = 0; i < LD4; ++i) {
            *reinterpret_cast<float4v*>(ks_ptr[i] + buf * KB * KLD) = kreg[i];
            *reinterpret_cast<float4v*>(vs_ptr[i] + buf * KB * VLD) = vreg[i];
        }
    };

    float16v o[DB];  // O^T rows d = 32*db .. 32*db+31, column = this lane's query
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m = kNegBig;   // softmax reference (log2 domain), same in both lane halves; within kSlack of the running max
    float lsum = 0.f;    // running sum over this lane half's keys only

    int nblocks = (Lk + KB - 1) / KB;
    if (CAUSAL) {  // same for every wave of the group: the block of the group's last query
        const int q_last = qb * QT + QT - 1 < Lq ? qb * QT + QT - 1 : Lq - 1;
        const int nb = q_last / KB + 1;
        nblocks = nb < nblocks ? nb : nblocks;
    }
    unsigned vrow[2][SUB][4];   // byte offset in LDS of V row (sub-block's first key + 4 half + 8 g), column l32, per stage
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int u = 0; u < SUB; ++u)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                vrow[b2][u][g4] = (unsigned)(2 * KB * KLD + b2 * KB * VLD + ((kgrp * SUB + u) * 32 + 4 * half + 8 * g4) * VLD + l32) * 4u;
                asm volatile("" : "+v"(vrow[b2][u][g4]));
            }
    auto block = [&](int t, auto cur_tag, auto next_tag) {   // stage index compile-time: fragment reads are base + immediate
        constexpr int cur = decltype(cur_tag)::value;
        if (t + 1 < nblocks) fetch((t + 1) * KB);
        const float* Kc = Ks + cur * KB * KLD;
        const float* Vc = Vs + cur * KB * VLD;
        // ---- scores of this wave's sub-blocks: S^T = K Q^T -------------------
        float16v s[SUB];
        bool skip[SUB];   // wave-uniform: the sub-block lies above the diagonal of all 32 queries
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[u][i] = CAUSAL ? -INFINITY : 0.f;
            const int kb = (kgrp * SUB + u) * 32;
            skip[u] = CAUSAL && t * KB + kb > q0 + QW - 1;
            if (skip[u]) continue;
            if (CAUSAL) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[u][i] = 0.f;
            }
            const float* krow = Kc + (kb + l32) * KLD + 4 * half;
#pragma unroll
            for (int c = 0; c < D / 8; ++c) {
                const float4v kf = *reinterpret_cast<const float4v*>(krow + 8 * c);
#pragma unroll
                for (int j = 0; j < 4; ++j) s[u] = mfma_32x32x2(kf[j], qf[c][j], s[u]);
            }
        }
        // ---- mask keys past the end, block max ---------------------------------
        float bm = kNegBig;
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            const int kb = t * KB + (kgrp * SUB + u) * 32;
            if (kb + 32 > Lk) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kb + 8 * (r >> 2) + 4 * half + (r & 3) >= Lk) s[u][r] = -INFINITY;
            }
            if (CAUSAL && !skip[u] && kb + 31 > q0) {  // the diagonal crosses this sub-block
                const int q = q0 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kb + 8 * (r >> 2) + 4 * half + (r & 3) > q) s[u][r] = -INFINITY;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) bm = fmaxf(bm, s[u][r]);
        }
        bm = fmaxf(bm, xchg_half(bm));
        // The softmax reference m is moved only when a block exceeds it by more
        // than kSlack (always at the first block, where m = kNegBig): probabilities
        // stay below 2^kSlack, the result does not depend on the reference, and
        // the 32-register accumulator rescale almost never runs.
        if (__any(bm > m + kSlack)) {  // wave-uniform
            const float m_new = fmaxf(m, bm);
            const float alpha = fast_exp2(m - m_new);
            m = m_new;
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        }
        float ps = 0.f;
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(s[u][r] - m);
                s[u][r] = p;
                ps += p;
            }
        }
        lsum += ps;
        // The next block goes to the other LDS stage here, between the two contractions: every reader of that stage
        // passed the barrier that ended the previous block, the loads were issued a whole contraction ago, and the LDS
        // writes then run under the second contraction's MFMAs instead of between its end and the barrier
        // (16 x 2048 x 64: 138.1 -> 136.1 us).
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < nblocks) stash(next_tag);
        __builtin_amdgcn_sched_barrier(0);
        // ---- O^T += V^T P^T ---------------------------------------------------------
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            if (skip[u]) continue;
            // one byte offset per group of four fragment rows, kept opaque: the compiler would otherwise re-derive each
            // group's address from one base with a vector add in front of its reads, inside the MFMA block (paired LDS
            // reads only take 8-bit offsets)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float* vr = reinterpret_cast<const float*>(reinterpret_cast<const char*>(lds) + vrow[cur][u][r >> 2]) + (r & 3) * VLD;
#pragma unroll
                for (int db = 0; db < DB; ++db) o[db] = mfma_32x32x2(vr[32 * db], s[u][r], o[db]);
            }
        }
        __syncthreads();
    };
    constexpr std::integral_constant<int, 0> buf0{};
    constexpr std::integral_constant<int, 1> buf1{};
    fetch(0);
    stash(buf0);
    __syncthreads();
    for (int t = 0; t < nblocks; t += 2) {
        block(t, buf0, buf1);
        if (t + 1 < nblocks) block(t + 1, buf1, buf0);
    }

    // ---- combine the two lane halves' sums, merge wave groups, normalise, store
    lsum += xchg_half(lsum);
    if (KS > 1) {
        // groups 1.. publish (o, m, l) as [kgrp-1][qwave][MROWS][64]; the loop's last
        // barrier has retired every read of the stage buffers
        if (kgrp > 0) {
            float* mg = lds + ((kgrp - 1) * NQW + qwave) * MROWS * 64;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) mg[(16 * db + i) * 64 + lane] = o[db][i];
            mg[16 * DB * 64 + lane] = m;
            mg[(16 * DB + 1) * 64 + lane] = lsum;
        }
        __syncthreads();
        if (kgrp == 0) {
#pragma unroll
            for (int g = 1; g < KS; ++g) {   // in group order
                const float* mg = lds + ((g - 1) * NQW + qwave) * MROWS * 64;
                const float m2 = mg[16 * DB * 64 + lane], l2 = mg[(16 * DB + 1) * 64 + lane];
                const float mm = fmaxf(m, m2);
                const float a1 = fast_exp2(m - mm), a2 = fast_exp2(m2 - mm);
                m = mm;
                lsum = lsum * a1 + l2 * a2;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[db][i] = o[db][i] * a1 + mg[(16 * db + i) * 64 + lane] * a2;
            }
        }
    }
    const int q = q0 + l32;
    if (kgrp == 0 && q < Lq) {
        const float inv = 1.0f / lsum;
        float* dst = O + ((int64_t)b * Lq + q) * D + 4 * half;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                store4(dst + 32 * db + 8 * g, float4v{o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv});
    }
    if (pass + 1 < npass) __syncthreads();   // the merge area is the next pass's stage buffer
  }
}

// plain: 128 queries x 2 key groups, 64-key blocks.  causal: paired 64-query blocks; 4 key groups
// and 128-key blocks up to head dim 64, 2 key groups and 64-key blocks at head dim 128 (128-key
// blocks would not fit in LDS there): four waves per CU, but every work-group walks the same
// number of key blocks (16 x 2048 x 128: 65 -> 92 TFLOP/s against the unpaired plain shape).
template <int D, bool CAUSAL> struct AttnCfg {
    static constexpr bool PAIR = CAUSAL;
    static constexpr int KS = (PAIR && D <= 64) ? 4 : 2;
    static constexpr int NQW = PAIR ? 2 : 4;
    static constexpr int QT = NQW * QW;
    static constexpr int KB = KS == 4 ? 128 : 64;
    static constexpr size_t LDS = (size_t)(2 * KB * (D + 4) + 2 * KB * (D + 8)) * 4;
    static constexpr int NT = 64 * NQW * KS;
    static_assert(LDS <= 160 * 1024, "stage buffers exceed the LDS of a CU");
};

template <int D, bool CAUSAL>
unsigned attn_items(const AttnParams& p) {
    using C = AttnCfg<D, CAUSAL>;
    const int nqb = (p.Lq + C::QT - 1) / C::QT;
    return (unsigned)((C::PAIR ? (nqb + 1) / 2 : nqb) * p.B);
}

template <int D, bool CAUSAL>
hipError_t launch_attn(const AttnParams& p, hipStream_t stream) {
    using C = AttnCfg<D, CAUSAL>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd<D, C::KS, C::NQW, CAUSAL, C::PAIR>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((attn_fwd<D, C::KS, C::NQW, CAUSAL, C::PAIR>), dim3(attn_items<D, CAUSAL>(p)), dim3(C::NT), C::LDS, stream,
                       p.Q, p.K, p.V, p.O, p.Lq, p.Lk, p.scale * kLog2e);
    return hipGetLastError();
}

template <int D>
void shape_d(const AttnParams& p, LaunchShape& s) {
    s.grid[0] = p.causal ? attn_items<D, true>(p) : attn_items<D, false>(p);
    s.block[0] = p.causal ? AttnCfg<D, true>::NT : AttnCfg<D, false>::NT;
    s.lds_bytes = (uint32_t)(p.causal ? AttnCfg<D, true>::LDS : AttnCfg<D, false>::LDS);
}

}  // namespace

bool attn_supported(int32_t d, const char** why) {
    if (d != 32 && d != 64 && d != 128) { *why = "head dimension must be 32, 64 or 128"; return false; }
    return true;
}

LaunchShape attn_shape(const AttnParams& p) {
    LaunchShape s{};
    s.grid[1] = s.grid[2] = 1; s.block[1] = s.block[2] = 1;
    static const char* const names[3][2] = {{"attn_fwd_d32<ks2>", "attn_fwd_d32<ks4,causal,paired>"},
                                            {"attn_fwd_d64<ks2>", "attn_fwd_d64<ks4,causal,paired>"},
                                            {"attn_fwd_d128<ks2>", "attn_fwd_d128<ks2,causal,paired>"}};
    switch (p.D) {
        case 32: shape_d<32>(p, s); s.kernel = names[0][p.causal ? 1 : 0]; break;
        case 64: shape_d<64>(p, s); s.kernel = names[1][p.causal ? 1 : 0]; break;
        default: shape_d<128>(p, s); s.kernel = names[2][p.causal ? 1 : 0];
    }
    return s;
}

hipError_t attn_launch(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 32: return p.causal ? launch_attn<32, true>(p, stream) : launch_attn<32, false>(p, stream);
        case 64: return p.causal ? launch_attn<64, true>(p, stream) : launch_attn<64, false>(p, stream);
        default: return p.causal ? launch_attn<128, true>(p, stream) : launch_attn<128, false>(p, stream);
    }
}

}  // namespace hpct
