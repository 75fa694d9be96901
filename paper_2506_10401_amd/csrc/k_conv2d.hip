// NCHW conv2d (cross-correlation, zero padding, square filter 1/3/5/7, stride
// and dilation up to 4) with its epilogue held in registers - bias, per-channel scale/shift
// (a folded batch-norm), ReLU and optionally the 2x2 max pooling that closes a
// VGG block: the convolution of the paper's VGG-16 case study (Section 5.3;
// Table 1 "conv"; "Conv2d BN" of Section 5.2).  Implicit GEMM on
// v_mfma_f32_32x32x2_f32:
//
//     D[k_out, pixel] = sum_{c,kh,kw} wt[k_out, c, kh, kw] * in[c, h-P+kh, w-P+kw]
//
// Rows of D are output channels (A operand = weights), columns are output
// pixels (B operand = input patches), so a lane owns one pixel and an
// accumulator register is stored as 32 consecutive pixels = 128 contiguous
// bytes of the NCHW output.
//
// A work-group of four waves owns KT = 64 output channels x TP = 64
// consecutive output pixels of one image; a wave owns KT/2 channels x 32 pixels.
// Channels are processed CC at a time.  Per chunk the LDS holds
//   * the input rows the tile touches, with their zero halo, per channel, and
//   * for every output channel its CC*R*S weights in memory order (a plain
//     copy of a contiguous piece of the KCRS tensor, row stride padded against
//     bank conflicts).
// Both are double buffered: the global loads of chunk t+1 are issued before the
// MFMAs of chunk t and written to the other buffer after them (window geometry: ahead of the last
// fragment group).  Vector-ALU
// instructions do not overlap MFMAs, so the chunk loop is kept almost free of
// them: raw buffer loads with per-slot offsets worked out once (the zero halo is
// an out-of-range offset), two chunks per trip so the LDS stage is a compile-time
// constant, one precomputed LDS pointer per fragment row.
//
// Contraction order: within a chunk, lane half 0 multiplies channels
// 0..CC/2-1 and lane half 1 channels CC/2..CC-1, so MFMA step s contracts
// (channel s/TAPS, tap s%TAPS) of both halves.  The A fragment is then a run of
// consecutive floats of the weight row (vector LDS reads) and the B fragment of
// every step is an LDS read at lane base + a constant.
//
// Window geometry (WIN; always with POOL, and without it for images wider than 64, whose whole
// rows would cost too much LDS): the 64 pixels of a tile are 8 output rows x 8 output columns
// (each 32-pixel block is 4 rows x 8 columns, lane = 8*row + column), the LDS
// holds the window of the input those need instead of whole rows, and the
// epilogue takes the 2x2 maximum entirely in registers: the vertical partner
// is 8 lanes away inside a 16-lane DPP row, the horizontal one the neighbouring
// lane; one lane in four stores.  8 divides the 224/112/56 extents of VGG maps.
#include <type_traits>
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int TP = 64;   // output pixels per work-group
constexpr int kXcds = 8; // work-groups are dealt round-robin to this many L2 domains

struct ConvGeom {
    int Nb, C, H, W, K, P;
    int St;        // stride
    int Dl;        // dilation
    int Ho, Wo, HoWo;
    int Hp, Wp;    // pooled output size (POOL)
    int ctiles;    // 8-column tiles per 8-row band (window geometry)
    int tiles_per_img, tiles;
    int rows_max;  // input rows staged per tile
    int lpad;      // left pad of an LDS row so that iw = 0 lands on a 16-byte boundary
    int ldw;       // LDS row stride (floats, multiple of 4)
    int ch_ld;     // LDS channel stride (floats)
};

template <int R, int CC, int KT> struct Cfg {
    static constexpr int TAPS = R * R;
    static constexpr int FPR = CC * TAPS;        // weight floats per output channel per chunk
    static constexpr int HALF = FPR / 2;         // MFMA steps per chunk
    static constexpr int VW = HALF % 4 == 0 ? 4 : 2;  // A-fragment vector width (floats)
    // LDS row stride of the weight stage.  128-bit fragment reads: FPR + 4 (16 lanes cover all 64 banks).
    // 64-bit fragment reads: FPR + 2, an odd number of 8-byte words, so 32 lanes cover all 64 banks.
    static constexpr int WLD = FPR + (VW == 4 ? 4 : 2);
    static constexpr int NV4 = KT * FPR / 4;     // float4 of weights per chunk
    static constexpr int WPT = (NV4 + 255) / 256;
    static constexpr int W_STAGE = KT * WLD;     // floats
};

struct ConvEpi {
    const float* bias;   // [K] or null
    const float* scale;  // [K] or null
    const float* shift;  // [K] or null
    int relu;            // 0 none, 1 relu, 2 relu6
};

// MODE 0 (general): every element is loaded with its own bounds test, chunk by chunk.
// MODE 1..4 (pipelined): C % CC == 0, dilation 1, and the image width is a multiple
// of the input vector width IV, so input rows are staged with aligned IV-wide loads that lie
// entirely inside or outside the image; IPT such slots per thread go through registers, software
// pipelined against the MFMAs.  1: IV 4, IPT 2;  2: IV 4, IPT 4;  3: IV 2, IPT 4;  4: IV 1, IPT 4.
template <int IV> struct VecOf;
template <> struct VecOf<4> { typedef float4v type; };
template <> struct VecOf<2> { typedef float2v type; };
template <> struct VecOf<1> { typedef float type; };
// Raw buffer loads for the pipelined staging: the hardware compares a lane's byte offset with the
// descriptor's size and returns 0 for a lane beyond it without touching memory.  A slot in the
// zero padding (or a weight row past K) is given the offset 2^31, larger than any tensor the
// pipelined modes accept, so the halo costs no branch, no select and no zero fill, and the
// channel-chunk offset rides in the scalar offset operand.
constexpr unsigned kBufOob = 0x80000000u;
constexpr int kBufWord3 = 0x00020000;   // descriptor word 3 for plain 32-bit data
template <int IV>
__device__ __forceinline__ typename VecOf<IV>::type buffer_load(__amdgpu_buffer_rsrc_t rs, unsigned voff, int soff) {
    if constexpr (IV == 4) return __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, soff, 0));
    else if constexpr (IV == 2) return __builtin_bit_cast(float2v, __builtin_amdgcn_raw_buffer_load_b64(rs, (int)voff, soff, 0));
    else return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)voff, soff, 0));
}
constexpr int mode_iv(int mode) { return mode <= 2 ? 4 : (mode == 3 ? 2 : 1); }
constexpr int mode_ipt(int mode) { return mode == 1 ? 2 : 4; }

template <int R, int CC, int KT, int MODE, bool POOL, bool WIN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MODE != 0 ? 5 : 4, MODE != 0 ? 5 : 8))) void conv2d_nchw_mfma(const float* __restrict__ in, const float* __restrict__ wt,
                                                        ConvEpi epi, float* __restrict__ out, ConvGeom g) {
    using cfg = Cfg<R, CC, KT>;
    constexpr bool FAST = MODE != 0;
    constexpr int IV = mode_iv(MODE), IN_PER_T = mode_ipt(MODE);
    typedef typename VecOf<IV>::type ivec;
    constexpr int KB = KT / 64;  // 32-channel accumulator blocks per wave
    constexpr int TAPS = cfg::TAPS, FPR = cfg::FPR, HALF = cfg::HALF, WLD = cfg::WLD, VW = cfg::VW;
    constexpr int WPT = cfg::WPT;
    extern __shared__ __align__(16) float lds[];
    const int in_stage = CC * g.ch_ld;  // floats
    constexpr int NBUF = FAST ? 2 : 1;  // the general variant stages one chunk at a time
    // weight stages first: their offsets are compile-time, so A-fragment reads need no address arithmetic
    auto wS = [&](int buf) { return lds + buf * cfg::W_STAGE; };
    auto inS = [&](int buf) { return lds + NBUF * cfg::W_STAGE + buf * in_stage; };
    float* const mulS = lds + NBUF * in_stage + NBUF * cfg::W_STAGE;  // KT floats: per-channel factor
    float* const addS = mulS + KT;                              // KT floats: per-channel addend
    float* const dumpS = addS + KT;                             // 4 floats nobody reads

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: what depends on it alone costs no vector ALU
    const int half = lane >> 5, l32 = lane & 31;

    // work item = (pixel tile, channel block); consecutive items (same tile, then
    // the next tile of the same image, sharing halo rows) go to the same L2 domain
    const int kblocks = (g.K + KT - 1) / KT;
    int item;
    {
        const int items = g.tiles * kblocks;
        const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        const int q = items / kXcds, r = items % kXcds;
        item = x * q + (x < r ? x : r) + j;
    }
    const int tile = item / kblocks;
    const int n = tile / g.tiles_per_img;
    const int tin = tile % g.tiles_per_img;
    static_assert(WIN || !POOL, "pooling needs the window geometry");
    const int p0 = WIN ? 0 : tin * TP;
    const int k0 = (item % kblocks) * KT;
    const int h_lo = WIN ? 8 * (tin / g.ctiles) : p0 / g.Wo;  // first output row of the tile
    const int w_lo = WIN ? 8 * (tin % g.ctiles) : 0;          // first output column of the tile (window geometry)
    const int ih0 = h_lo * g.St - g.P;  // first staged input row
    const int iw0 = w_lo * g.St;        // input column the staged window is anchored at (window geometry)
    const int HW = g.H * g.W;
    const int ldw4 = g.ldw >> 2;
    const int slots = CC * g.rows_max * ldw4;  // float4 slots of one input stage: slot -> (c, row, x4)

    auto slot_geom = [&](int s, int& goff, int& loff, int& c, int& mask) {
        c = s / (g.rows_max * ldw4);
        const int rem = s - c * (g.rows_max * ldw4);
        const int row = rem / ldw4, x4 = (rem - row * ldw4) * 4;
        const int ih = ih0 + row, iw = iw0 + x4 - g.P - g.lpad;
        loff = c * g.ch_ld + rem * 4;
        goff = ((n * g.C + c) * g.H + ih) * g.W + iw;
        mask = 0;
        if (ih >= 0 && ih < g.H) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (iw + j >= 0 && iw + j < g.W) mask |= 1 << j;
        }
    };

    // ---- pipelined staging: geometry worked out once, loads through registers ------
    ivec ireg[IN_PER_T];
    float4v wreg[WPT];
    unsigned s_goff[IN_PER_T], w_goff[WPT];   // byte offsets inside image n / the weight tensor, or kBufOob
    int s_loff[IN_PER_T], w_loff[WPT];        // LDS word offsets, -1: nothing to write
    // Where slot i goes in either stage.  Row geometry: slots with nothing to stage point at four spare words
    // and the writes carry no predicate (-2 % of the kernel's time); window geometry: three slots in four are
    // empty, whole waves skip their write under the predicate, which is cheaper there (+2.5 % without it).
    constexpr bool PRED = WIN;
    float* s_lptr[2][IN_PER_T];
    float* w_lptr[2][WPT];
    __amdgpu_buffer_rsrc_t in_rs, wt_rs;
    if (FAST) {
        in_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(in) + (int64_t)n * g.C * HW, 0, g.C * HW * 4, kBufWord3);
        wt_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(wt), 0, g.K * g.C * TAPS * 4, kBufWord3);
        const int ldwv = g.ldw / IV;                         // IV-wide slots per staged row
        const int vslots = CC * g.rows_max * ldwv;           // slot -> (c, row, x)
#pragma unroll
        for (int i = 0; i < IN_PER_T; ++i) {
            const int s = tid + i * 256;
            s_goff[i] = kBufOob; s_loff[i] = -1;
            if (s < vslots) {
                const int c = s / (g.rows_max * ldwv);
                const int rem = s - c * (g.rows_max * ldwv);
                const int row = rem / ldwv, x = (rem - row * ldwv) * IV;
                const int ih = ih0 + row, iw = iw0 + x - g.P - g.lpad;   // a multiple of IV, like W: all in or all out
                s_loff[i] = c * g.ch_ld + row * g.ldw + x;
                if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) s_goff[i] = (unsigned)(((c * g.H + ih) * g.W + iw) * 4);
            }
        }
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int v = tid + i * 256;
            const int k = v / (FPR / 4), f4 = v % (FPR / 4);
            const bool live = v < cfg::NV4 && k0 + k < g.K;   // rows past K are not staged: their accumulator rows are never stored
            w_goff[i] = live ? (unsigned)((((k0 + k) * g.C) * TAPS + 4 * f4) * 4) : kBufOob;
            w_loff[i] = live ? k * WLD + 4 * f4 : -1;
        }
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < IN_PER_T; ++i) s_lptr[b][i] = s_loff[i] >= 0 ? inS(b) + s_loff[i] : dumpS;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < WPT; ++i) w_lptr[b][i] = w_loff[i] >= 0 ? wS(b) + w_loff[i] : dumpS;
    }
    auto fetch = [&](int c0) {
#pragma unroll
        for (int i = 0; i < IN_PER_T; ++i)
            ireg[i] = buffer_load<IV>(in_rs, s_goff[i], c0 * HW * 4);
#pragma unroll
        for (int i = 0; i < WPT; ++i) wreg[i] = buffer_load<4>(wt_rs, w_goff[i], c0 * TAPS * 4);
    };
    auto stash = [&](auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
#pragma unroll
        for (int i = 0; i < IN_PER_T; ++i)
            if (!PRED || s_loff[i] >= 0) *reinterpret_cast<ivec*>(s_lptr[buf][i]) = ireg[i];
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            if (PRED && w_loff[i] < 0) continue;
            float* const dst = PRED ? wS(buf) + w_loff[i] : w_lptr[buf][i];
            if (WLD % 4 == 0) {
                *reinterpret_cast<float4v*>(dst) = wreg[i];
            } else {  // rows are only 8-byte aligned
                *reinterpret_cast<float2v*>(dst) = float2v{wreg[i].x, wreg[i].y};
                *reinterpret_cast<float2v*>(dst + 2) = float2v{wreg[i].z, wreg[i].w};
            }
        }
    };
    // ---- general staging: every element with its own bounds test; four slots (input) or eight
    // elements (weights) are loaded before any is written, so their latencies overlap -----------
    auto copy_chunk = [&](int buf, int c0) {
        float* const ib = inS(buf);
        float* const wb = wS(buf);
        const bool rows_aligned = (g.W & 3) == 0;
        for (int s0 = tid; s0 < slots; s0 += 256 * 4) {
            float4v v[4];
            int loff[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u * 256;
                v[u] = float4v{0.f, 0.f, 0.f, 0.f};
                loff[u] = -1;
                if (s < slots) {
                    int goff, c, mask;
                    slot_geom(s, goff, loff[u], c, mask);
                    if (c0 + c < g.C) {
                        const float* src = in + goff + c0 * HW;
                        if (mask == 15 && rows_aligned) {   // wholly inside, and rows keep 16-byte alignment
                            v[u] = load4(src);
                        } else {
                            if (mask & 1) v[u].x = src[0];
                            if (mask & 2) v[u].y = src[1];
                            if (mask & 4) v[u].z = src[2];
                            if (mask & 8) v[u].w = src[3];
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (loff[u] >= 0) *reinterpret_cast<float4v*>(ib + loff[u]) = v[u];
        }
        for (int e0 = tid; e0 < KT * FPR; e0 += 256 * 8) {
            float w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * 256;
                const int k = e / FPR, f = e - k * FPR;
                const int c = c0 + f / TAPS;
                w[u] = (e < KT * FPR && k0 + k < g.K && c < g.C) ? wt[((int64_t)(k0 + k) * g.C + c0) * TAPS + f] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * 256;
                if (e < KT * FPR) { const int k = e / FPR; wb[k * WLD + (e - k * FPR)] = w[u]; }
            }
        }
    };

    // ---- per-lane fragment addresses -------------------------------------------
    const int kb0 = (wave & 1) * (KT / 2);  // this wave's output channels inside the tile
    const int pb = (wave >> 1) * 32;  // this wave's 32 pixels inside the tile
    int p = p0 + pb + l32;
    bool p_ok;
    int oh, ow;
    if (WIN) {  // pixel block = 4 rows x 8 columns; the staged window covers the whole tile
        oh = h_lo + 4 * (wave >> 1) + (l32 >> 3); ow = w_lo + (l32 & 7);
        p_ok = oh < g.Ho && ow < g.Wo;   // (only the un-pooled store uses it)
        p = oh * g.Wo + ow;
    } else {
        p_ok = p < g.HoWo;
        if (!p_ok) p = g.HoWo - 1;    // clamp: reads stay inside the staged rows, the store is masked
        oh = p / g.Wo; ow = p - oh * g.Wo;
    }
    // input element of (chunk channel c, tap kh,kw): c*ch_ld + ((oh-h_lo)*St+kh*Dl)*ldw + (ow-w_lo)*St + kw*Dl + lpad
    const int b_base = half * (CC / 2) * g.ch_ld + (oh - h_lo) * g.St * g.ldw + (ow - w_lo) * g.St + g.lpad;
    const int a_base = (kb0 + l32) * WLD + half * HALF;

    float16v acc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[kb][i] = 0.f;

    // the pipelined variant is built for dilation 1 only, so that its tap offsets stay compile-time
    // immediates of the LDS reads (a run-time dilation costs 4.5 % there); dilated convs take the general one
    const int dl = FAST ? 1 : g.Dl;
    // B-fragment rows: one LDS pointer per (stage, chunk channel of this lane half, filter row), worked out
    // once, so that inside the chunk loop a fragment read is pointer + immediate (kw) and costs no vector ALU
    // instruction (with run-time pitches every (c, kh) pair was an add per chunk, not overlapped with the MFMAs)
    // (kept as byte offsets the compiler cannot relate to each other: it would otherwise keep one pointer per row
    // and re-derive the second stage's with a vector add in front of every read, inside the MFMA block)
    unsigned brow[NBUF][CC / 2][R];
    unsigned arow[NBUF];
    auto lds_at = [&](unsigned bytes) { return reinterpret_cast<const float*>(reinterpret_cast<const char*>(lds) + bytes); };
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
#pragma unroll
        for (int c = 0; c < CC / 2; ++c)
#pragma unroll
            for (int kh = 0; kh < R; ++kh) {
                brow[b][c][kh] = (unsigned)(NBUF * cfg::W_STAGE + b * in_stage + b_base + c * g.ch_ld + kh * dl * g.ldw) * 4u;
                asm volatile("" : "+v"(brow[b][c][kh]));
            }
        arow[b] = (unsigned)(b * cfg::W_STAGE + a_base) * 4u;
        asm volatile("" : "+v"(arow[b]));
    }
    // `stash_next` writes the next chunk to the other LDS stage, whose readers all passed the previous barrier.  In the
    // window geometry it runs ahead of the chunk's last fragment group, so its predicated LDS writes and the wait for
    // their loads lie inside the MFMA block instead of between its end and the barrier (pooled 3x3 block 125.7 ->
    // 122.7 us); in the row geometry, where that measured 0.3 % slower, and with a single group it runs after the block.
    auto compute = [&](auto cur_tag, auto&& stash_next) {
        constexpr int cur = decltype(cur_tag)::value;
        constexpr int NG = HALF / VW;
        constexpr bool EARLY = WIN && NG > 1;
        // waves inside their MFMA block win the issue arbitration over waves that are staging
        __builtin_amdgcn_s_setprio(1);
        const float* aW = lds_at(arow[cur]);
#pragma unroll
        for (int j = 0; j < NG; ++j) {
            if (EARLY && j == NG - 1) {
                __builtin_amdgcn_sched_barrier(0);
                stash_next();
                __builtin_amdgcn_sched_barrier(0);
            }
            float a[KB][VW];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                if (VW == 4) {
                    const float4v t = *reinterpret_cast<const float4v*>(aW + kb * 32 * WLD + VW * j);
#pragma unroll
                    for (int e = 0; e < VW; ++e) a[kb][e] = t[e];
                } else {
                    const float2v t = *reinterpret_cast<const float2v*>(aW + kb * 32 * WLD + VW * j);
#pragma unroll
                    for (int e = 0; e < VW; ++e) a[kb][e] = t[e];
                }
            }
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int s = VW * j + e;  // MFMA step inside the chunk
                const int c = s / TAPS, tap = s % TAPS;
                const float b = lds_at(brow[cur][c][tap / R])[(tap % R) * dl];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) acc[kb] = mfma_32x32x2(a[kb][e], b, acc[kb]);
            }
        }
        __builtin_amdgcn_s_setprio(0);
        if (!EARLY) {
            __builtin_amdgcn_sched_barrier(0);
            stash_next();
        }
    };
    constexpr std::integral_constant<int, 0> buf0{};
    constexpr std::integral_constant<int, NBUF - 1> buf1{};   // (the general variant has one stage)

    if (tid < KT) {  // v = (acc + bias) * scale + shift = acc * mul + add; visible after the first barrier
        const bool ok = k0 + tid < g.K;
        const float mul = (epi.scale && ok) ? epi.scale[k0 + tid] : 1.f;
        const float b = (epi.bias && ok) ? epi.bias[k0 + tid] : 0.f;
        const float sh = (epi.shift && ok) ? epi.shift[k0 + tid] : 0.f;
        mulS[tid] = mul;
        addS[tid] = b * mul + sh;
    }

    const int nchunks = (g.C + CC - 1) / CC;
    if (FAST) {
        // software pipeline over channel chunks; the last chunk is peeled so the
        // loop body has no conditional loads
        // (two chunks per trip, so that the stage index is a compile-time constant everywhere)
        auto step = [&](int next_c0, auto cur_tag, auto next_tag) {
            fetch(next_c0);
            __builtin_amdgcn_sched_barrier(0);  // keep the global loads ahead of the MFMAs they overlap with
            compute(cur_tag, [&] { stash(next_tag); });
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        };
        fetch(0);
        stash(buf0);
        __syncthreads();
        int t = 0;   // chunk t is in stage 0 here
        for (; t + 2 < nchunks; t += 2) {
            step((t + 1) * CC, buf0, buf1);
            step((t + 2) * CC, buf1, buf0);
        }
        if (t + 1 < nchunks) {
            step((t + 1) * CC, buf0, buf1);
            compute(buf1, [] {});
        } else {
            compute(buf0, [] {});
        }
    } else {
        for (int t = 0; t < nchunks; ++t) {
            copy_chunk(0, t * CC);
            __syncthreads();
            compute(buf0, [] {});
            __syncthreads();
        }
    }

    // ---- epilogue: register r of lane holds channel 8*(r/4) + 4*half + r%4 of the block.
    // Vector-ALU instructions of one wave hold up the MFMAs of the others, so per register there is a multiply-add,
    // the clamp and the store: the four channels of a register group are consecutive, so their factors come as
    // 128-bit LDS reads issued together; a register's address is a scalar base (image, channel) plus one per-lane
    // 32-bit offset worked out once; the activation is a template value behind a scalar switch.
    auto finish = [&](auto relu_tag) {
        constexpr int RELU = decltype(relu_tag)::value;
        auto act = [](float v) {
            if (RELU) v = fmaxf(v, 0.f);
            if (RELU == 2) v = fminf(v, 6.f);
            return v;
        };
        const int plane = POOL ? g.Hp * g.Wp : g.HoWo;   // elements of one output channel
        // this lane's byte offset inside the 8-channel group of a register quartet (the host admits planes below 2^27 elements)
        unsigned loff;
        bool st_ok;
        if (POOL) {
            // lane = 8*row + column inside the block: the vertical partner of a window is lane ^ 8
            // (a rotation by 8 inside the 16-lane DPP row), the horizontal one lane ^ 1
            const int rp = oh >> 1, px = ow >> 1;
            st_ok = (lane & 9) == 0 && rp < g.Hp && px < g.Wp;
            loff = (unsigned)(4 * half * plane + rp * g.Wp + px) * 4u;
        } else {
            st_ok = p_ok;
            loff = (unsigned)(4 * half * plane + p) * 4u;
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int kl0 = kb0 + kb * 32;   // scalar
            float4v mul[4], add[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                mul[q] = *reinterpret_cast<const float4v*>(mulS + kl0 + 8 * q + 4 * half);
                add[q] = *reinterpret_cast<const float4v*>(addS + kl0 + 8 * q + 4 * half);
            }
            float* const ob = out + ((int64_t)n * g.K + k0 + kl0) * plane;   // scalar
            const bool whole = k0 + kl0 + 32 <= g.K;                         // scalar: all 32 channels of the block exist
            float v[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                v[r] = act(acc[kb][r] * mul[r >> 2][r & 3] + add[r >> 2][r & 3]);
                if (POOL) {
                    v[r] = fmaxf(v[r], dpp_mov<0x128>(v[r]));  // row_ror:8
                    v[r] = fmaxf(v[r], dpp_mov<0xB1>(v[r]));   // quad_perm [1,0,3,2]
                }
            }
            // Channel of half 0 inside the block: kr = 8 * (r / 4) + r % 4.  Raw buffer stores: the descriptor covers the
            // channels of this block that exist, a lane with nothing to store carries an offset beyond it and the
            // hardware drops its store, so there is no predicate; a register's channel offset is a scalar operand.
            // (The scalar operand takes no part in the range check: it is used only where all 32 channels exist.)
            const int left = g.K - (k0 + kl0);   // scalar
            if (plane < (1 << 24)) {   // 32 channels x plane x 4 bytes stay below 2^31, the offset of a lane with nothing to store
                const int chans = left >= 32 ? 32 : (left > 0 ? left : 0);
                const int bytes = __builtin_amdgcn_readfirstlane(chans * plane * 4);   // (scalar already; keeps the descriptor in scalar registers)
                __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(ob, 0, bytes, kBufWord3);
                const unsigned voff = st_ok ? loff : kBufOob;
                if (whole) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v[r]), rs, (int)voff, (8 * (r >> 2) + (r & 3)) * plane * 4, 0);
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v[r]), rs,
                                                              (int)(st_ok ? loff + (unsigned)((8 * (r >> 2) + (r & 3)) * plane * 4) : kBufOob), 0, 0);
                }
            } else if (st_ok) {   // planes too large for a 32-bit descriptor
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kr = 8 * (r >> 2) + (r & 3);
                    if (kr + 4 * half < left) *reinterpret_cast<float*>(reinterpret_cast<char*>(ob + (int64_t)kr * plane) + loff) = v[r];
                }
            }
        }
    };
    if (epi.relu == 0) finish(std::integral_constant<int, 0>{});
    else if (epi.relu == 1) finish(std::integral_constant<int, 1>{});
    else finish(std::integral_constant<int, 2>{});
}

// input channels per LDS chunk: 4 (x 9 taps = 18 MFMA steps per chunk for 3x3); a 1x1 filter has one
// tap per channel, so it takes 16 channels per chunk (except in the window geometry, whose bank
// layout is worked out for 4)
constexpr int cc_of(int R, bool win) { return (R == 1 && !win) ? 16 : 4; }

// iv: vector width of the input staging (the left pad of an LDS row makes image column 0 land on
// a multiple of it)
ConvGeom geom(const ConvParams& p, int iv = 4) {
    ConvGeom g{};
    g.Nb = p.Nb; g.C = p.C; g.H = p.H; g.W = p.W; g.K = p.K; g.P = p.pad; g.St = p.stride; g.Dl = p.dil;
    const int re = (p.R - 1) * p.dil + 1;   // rows / columns the dilated filter spans
    g.Ho = (p.H + 2 * p.pad - re) / p.stride + 1;
    g.Wo = (p.W + 2 * p.pad - re) / p.stride + 1;
    g.HoWo = g.Ho * g.Wo;
    g.lpad = (iv - p.pad % iv) % iv;
    if (p.win) {
        g.Hp = g.Ho / 2; g.Wp = g.Wo / 2;
        const int rows = p.pool ? 2 * g.Hp : g.Ho, cols = p.pool ? 2 * g.Wp : g.Wo;   // pooling drops an odd last row / column
        g.ctiles = (cols + 7) / 8;
        g.tiles_per_img = ((rows + 7) / 8) * g.ctiles;
        g.rows_max = 7 * p.stride + re;                                    // eight output rows
        g.ldw = (7 * p.stride + re + g.lpad + 3) & ~3;                     // eight output columns
    } else {
        g.tiles_per_img = (g.HoWo + TP - 1) / TP;
        // a run of TP consecutive pixels touches at most (TP-1)/Wo + 2 output rows; exactly TP/Wo when
        // rows divide a tile (tiles then start at row starts)
        int out_rows = TP % g.Wo == 0 ? TP / g.Wo : (TP - 1) / g.Wo + 2;
        if (out_rows > g.Ho) out_rows = g.Ho;
        g.rows_max = (out_rows - 1) * p.stride + re;
        g.ldw = (p.W + 2 * p.pad + g.lpad + 3) & ~3;
    }
    g.tiles = p.Nb * g.tiles_per_img;
    // The two lane halves read the same pixel pattern of channels CC/2 apart in one LDS access.
    // CC = 4: a channel stride of 16 (mod 32) words puts the halves' 32-word runs on complementary
    // bank halves; in the pooled geometry a half covers words 0-7 of four 16-word rows, and a channel
    // stride of 4 (mod 32) moves the other half onto words 8-15.  CC = 16 (halves 8 channels apart):
    // 4 (mod 8) gives the same 32-bank shift.
    const int cc = cc_of(p.R, p.win != 0);
    const int mod = cc == 16 ? 8 : 32, want = cc == 16 ? 4 : (p.win ? 4 : 16);
    g.ch_ld = g.rows_max * g.ldw;
    g.ch_ld += ((want - g.ch_ld % mod) + mod) % mod;
    return g;
}

template <int R, int CC, int KT>
size_t lds_bytes(const ConvGeom& g, bool fast) {
    const int nbuf = fast ? 2 : 1;
    return (size_t)(nbuf * CC * g.ch_ld + nbuf * Cfg<R, CC, KT>::W_STAGE + 2 * KT + 4) * 4;
}

// Output channels per work-group.  With 4 input channels per chunk, 64 keeps a work-group near
// 30 KB of LDS (five per CU hide each other's staging and barriers) and makes the work items small
// enough to balance over 256 CUs.
constexpr int kKT = 64;

// Staging mode and the geometry that goes with it.
int pick_mode(const ConvParams& p, ConvGeom* g_out) {
    const int cc = cc_of(p.R, p.win != 0);
    // (the pipelined modes address one image and the weight tensor with 31-bit byte offsets)
    const bool fits = (int64_t)p.C * p.H * p.W * 4 < (int64_t)1 << 31 && (int64_t)p.K * p.C * p.R * p.R * 4 < (int64_t)1 << 31;
    if ((p.R == 1 || p.R == 3) && p.dil == 1 && p.C % cc == 0 && fits) {
        for (int iv = 4; iv >= 1; iv >>= 1) {
            if (p.W % iv) continue;
            const ConvGeom g = geom(p, iv);
            const int slots = cc * g.rows_max * (g.ldw / iv);
            if (slots > 256 * 4) break;   // narrower vectors only need more slots
            *g_out = g;
            return iv == 4 ? (slots <= 256 * 2 ? 1 : 2) : (iv == 2 ? 3 : 4);
        }
    }
    *g_out = geom(p, 4);
    return 0;
}

int conv_items(const ConvParams& p, const ConvGeom& g) { return g.tiles * ((p.K + kKT - 1) / kKT); }

template <int R, int MODE, bool POOL, bool WIN>
hipError_t launch_conv(const ConvParams& p, const ConvGeom& g, hipStream_t stream) {
    constexpr int CC = cc_of(R, WIN);
    const size_t lds = lds_bytes<R, CC, kKT>(g, MODE != 0);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv2d_nchw_mfma<R, CC, kKT, MODE, POOL, WIN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)conv_items(p, g)), block(256);
    const ConvEpi epi{p.bias, p.scale, p.shift, p.relu};
    hipLaunchKernelGGL((conv2d_nchw_mfma<R, CC, kKT, MODE, POOL, WIN>), grid, block, lds, stream, p.in, p.wt, epi, p.out, g);
    return hipGetLastError();
}

template <int R, bool POOL, bool WIN>
hipError_t launch_mode(const ConvParams& p, const ConvGeom& g, int mode, hipStream_t stream) {
    if constexpr (R == 1 || R == 3) {
        switch (mode) {
            case 1: return launch_conv<R, 1, POOL, WIN>(p, g, stream);
            case 2: return launch_conv<R, 2, POOL, WIN>(p, g, stream);
            case 3: return launch_conv<R, 3, POOL, WIN>(p, g, stream);
            case 4: return launch_conv<R, 4, POOL, WIN>(p, g, stream);
            default: break;
        }
    }
    return launch_conv<R, 0, POOL, WIN>(p, g, stream);
}

template <int R>
hipError_t launch_pool(const ConvParams& p, const ConvGeom& g, int mode, hipStream_t stream) {
    if (p.pool) return launch_mode<R, true, true>(p, g, mode, stream);
    return p.win ? launch_mode<R, false, true>(p, g, mode, stream) : launch_mode<R, false, false>(p, g, mode, stream);
}

size_t lds_any(const ConvParams& p) {
    ConvGeom g;
    const bool fast = pick_mode(p, &g) != 0;
    switch (p.R) {
        case 1: return p.win ? lds_bytes<1, cc_of(1, true), kKT>(g, fast) : lds_bytes<1, cc_of(1, false), kKT>(g, fast);
        case 3: return lds_bytes<3, cc_of(3, false), kKT>(g, fast);
        case 5: return lds_bytes<5, cc_of(5, false), kKT>(g, fast);
        default: return lds_bytes<7, cc_of(7, false), kKT>(g, fast);
    }
}

}  // namespace

// Window geometry: always with pooling; without it for filters larger than 1x1 on images wider
// than 64, where staging whole input rows costs LDS (and occupancy) for nothing: 224-wide 64 -> 64
// channels 88 -> 116 TFLOP/s, 112-wide 115 -> 122; at 56 the two geometries take the same time.
// Below that width the rows stay unless only the window geometry can be staged by the pipelined
// variant (odd widths of 47 .. 63 have too many scalar slots per row tile: 55-wide 128 -> 64
// channels 53 -> 91 TFLOP/s, 63-wide 52 -> 101; at 45, where both can, rows are faster, 102 vs 75).
// (A 1x1 filter keeps rows: its 16-channel chunks need the row layout.)
int32_t conv_window_geometry(const ConvParams& p0) {
    if (p0.pool) return 1;
    if (p0.R == 1) return 0;
    if (p0.W > 64) return 1;
    ConvParams p = p0;
    ConvGeom g;
    p.win = 0;
    if (pick_mode(p, &g) != 0) return 0;
    p.win = 1;
    return pick_mode(p, &g) != 0 ? 1 : 0;
}

bool conv_supported(int32_t C, int32_t H, int32_t W, int32_t K, int32_t R, int32_t S, int32_t stride_h, int32_t stride_w,
                    int32_t pad_h, int32_t pad_w, int32_t dil_h, int32_t dil_w, int32_t pool, const char** why) {
    if (dil_h != dil_w) { *why = "the dilation must be the same in both directions"; return false; }
    if (dil_h < 1 || dil_h > 4) { *why = "dilations outside 1..4 are not supported"; return false; }
    if (stride_h != stride_w) { *why = "the stride must be the same in both directions"; return false; }
    if (stride_h > 4) { *why = "strides above 4 are not supported"; return false; }
    if (R != S || (R != 1 && R != 3 && R != 5 && R != 7)) { *why = "only square 1x1, 3x3, 5x5 and 7x7 filters are supported"; return false; }
    if (pad_h != pad_w) { *why = "padding must be the same in both directions"; return false; }
    if (pad_h > (R - 1) * dil_h) { *why = "padding larger than the (dilated) filter extent minus one"; return false; }
    {   // the epilogue addresses a lane's element inside a group of 8 output channels with a 32-bit byte offset
        const int re = (R - 1) * dil_h + 1;
        const int64_t Ho = (H + 2 * pad_h - re) / stride_h + 1, Wo = (W + 2 * pad_w - re) / stride_w + 1;
        if (Ho * Wo > ((int64_t)1 << 27)) { *why = "more than 2^27 output pixels per channel"; return false; }
    }
    ConvParams p{};
    p.C = C; p.H = H; p.W = W; p.K = K; p.R = R; p.S = S; p.pad = pad_h; p.Nb = 1; p.stride = stride_h; p.dil = dil_h; p.pool = pool; p.win = conv_window_geometry(p);
    if (lds_any(p) > 160 * 1024) { *why = "the input of one 64-pixel tile does not fit in LDS (image too wide)"; return false; }
    return true;
}

LaunchShape conv_shape(const ConvParams& p) {
    if (conv1x1_stream_ok(p)) return conv1x1_shape(p);
    if (conv_fewc_ok(p)) return conv_fewc_shape(p);
    ConvGeom g;
    const int mode = pick_mode(p, &g);
    LaunchShape s{};
    s.grid[0] = (uint32_t)conv_items(p, g); s.grid[1] = 1; s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)lds_any(p);
    static const char* const names[4][3][2] = {
        {{"conv2d_nchw_mfma<1x1,general>", "conv2d_nchw_mfma<1x1,pipelined>"},
         {"conv2d_nchw_mfma<1x1,general,maxpool2>", "conv2d_nchw_mfma<1x1,pipelined,maxpool2>"},
         {"conv2d_nchw_mfma<1x1,general,window>", "conv2d_nchw_mfma<1x1,pipelined,window>"}},
        {{"conv2d_nchw_mfma<3x3,general>", "conv2d_nchw_mfma<3x3,pipelined>"},
         {"conv2d_nchw_mfma<3x3,general,maxpool2>", "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"},
         {"conv2d_nchw_mfma<3x3,general,window>", "conv2d_nchw_mfma<3x3,pipelined,window>"}},
        {{"conv2d_nchw_mfma<5x5,general>", "conv2d_nchw_mfma<5x5,general>"},
         {"conv2d_nchw_mfma<5x5,general,maxpool2>", "conv2d_nchw_mfma<5x5,general,maxpool2>"},
         {"conv2d_nchw_mfma<5x5,general,window>", "conv2d_nchw_mfma<5x5,general,window>"}},
        {{"conv2d_nchw_mfma<7x7,general>", "conv2d_nchw_mfma<7x7,general>"},
         {"conv2d_nchw_mfma<7x7,general,maxpool2>", "conv2d_nchw_mfma<7x7,general,maxpool2>"},
         {"conv2d_nchw_mfma<7x7,general,window>", "conv2d_nchw_mfma<7x7,general,window>"}}};
    s.kernel = names[p.R / 2][p.pool ? 1 : (p.win ? 2 : 0)][mode != 0 ? 1 : 0];
    return s;
}

hipError_t conv_launch(const ConvParams& p, hipStream_t stream) {
    if (conv1x1_stream_ok(p)) return conv1x1_launch(p, stream);
    if (conv_fewc_ok(p)) return conv_fewc_launch(p, stream);
    ConvGeom g;
    const int mode = pick_mode(p, &g);
    switch (p.R) {
        case 1: return launch_pool<1>(p, g, mode, stream);
        case 3: return launch_pool<3>(p, g, mode, stream);
        case 5: return launch_pool<5>(p, g, mode, stream);
        default: return launch_pool<7>(p, g, mode, stream);
    }
}

}  // namespace hpct
