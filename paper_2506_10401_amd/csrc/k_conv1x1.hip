// 1x1 convolution, stride 1, no padding (the pointwise layers of ResNet / MobileNetV2
// blocks; Table 1 "conv", the "1x1 filters" of the conv anchor) as a weight-stationary
// streaming kernel: out[n][k][p] = act((sum_c wt[k][c] in[n][c][p] + bias[k]) scale[k] + shift[k]).
//
// Per image this is a GEMM [K x C] [C x HW] whose second operand is used by one output
// tile only once all K outputs of a pixel are made together, so the input needs no
// staging at all.  A work-group keeps KT <= 128 output channels' weights in LDS (rows
// C + 4 words apart: conflict-free 128-bit fragment reads) for its whole life; each of
// its four waves walks 32-pixel blocks of the flattened (n, p) axis on its own, loads
// the block's input straight from global memory into the MFMA B-operand layout (a lane
// half reads 32 consecutive pixels of one channel: 128 contiguous bytes) through raw
// buffer loads whose channel offset rides in the scalar operand, and stores 128-byte
// pieces of the output planes.  Used for few input channels (see conv1x1_stream_ok),
// where the tile kernel's 64-pixel tiles spend their time in prologues.
//
// Fragment layout (v_mfma_f32_32x32x2_f32): lane l supplies A[l%32][l/32] and
// B[l/32][l%32].  Lane half h reads channels 8t + 4h .. 8t + 4h + 3 of its weight row
// with one 128-bit LDS read; MFMA e of that group contracts channels {8t + e, 8t + 4 + e}
// and its B value is in[n][8t + 4h + e][p].
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kPwThreads = 256;

struct PwGeom {
    int C, K, HW;
    int64_t total;   // Nb * HW pixels
    int nblk;        // 32-pixel blocks
    int kt_tiles;    // KT-channel slices of K
    int Cp;          // C rounded up to whole chunks: the weight rows are zero beyond C, loads beyond C return 0
    int lda;         // LDS pitch of a weight row: Cp + 4
};

struct PwEpi {
    const float* bias;
    const float* scale;
    const float* shift;
    int relu;        // 0 none, 1 relu, 2 relu6
};

// KB: 32-channel accumulator blocks per wave (KT = 32 KB output channels per work-group).
// CH: input channels per chunk, 64 or 32: the loads of a chunk (CH/2 registers per lane) are in flight
// together, two chunks at a time; C is padded to whole chunks with zeros so that the loop has no branches.
template <int KB, int CH>
__global__ __launch_bounds__(kPwThreads) void conv1x1_stream(const float* __restrict__ in, const float* __restrict__ wt,
                                                             PwEpi epi, float* __restrict__ out, PwGeom g) {
    constexpr int KT = 32 * KB;
    extern __shared__ __align__(16) float lds[];
    float* const Ws = lds;                       // [KT][lda]
    float* const mulS = lds + KT * g.lda;        // [KT]
    float* const addS = mulS + KT;               // [KT]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int kt = blockIdx.x % g.kt_tiles, wg = blockIdx.x / g.kt_tiles, nwg = gridDim.x / g.kt_tiles;
    const int k0 = kt * KT;

    // ---- weights of this slice, once
    const int c4n = g.C >> 2;
    for (int i = tid; i < KT * c4n; i += kPwThreads) {
        const int row = i / c4n, c4 = i - row * c4n;
        float4v v = {0.f, 0.f, 0.f, 0.f};
        if (k0 + row < g.K) v = load4(wt + (int64_t)(k0 + row) * g.C + 4 * c4);
        *reinterpret_cast<float4v*>(Ws + row * g.lda + 4 * c4) = v;
    }
    const int p4n = (g.Cp - g.C) >> 2;   // zero columns C .. Cp
    for (int i = tid; i < KT * p4n; i += kPwThreads) {
        const int row = i / p4n, c4 = i - row * p4n;
        *reinterpret_cast<float4v*>(Ws + row * g.lda + g.C + 4 * c4) = float4v{0.f, 0.f, 0.f, 0.f};
    }
    if (tid < KT) {   // v = (acc + bias) * scale + shift = acc * mul + add
        const bool ok = k0 + tid < g.K;
        const float mul = (epi.scale && ok) ? epi.scale[k0 + tid] : 1.f;
        const float b = (epi.bias && ok) ? epi.bias[k0 + tid] : 0.f;
        const float sh = (epi.shift && ok) ? epi.shift[k0 + tid] : 0.f;
        mulS[tid] = mul;
        addS[tid] = b * mul + sh;
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t in_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(in), 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rs = __builtin_amdgcn_make_buffer_rsrc(out, 0, 0x7fffffff, 0x00020000);
    const int hw4 = g.HW * 4;                                 // bytes between channels
    const float* a_row = Ws + l32 * g.lda + 4 * half;         // + kb * 32 * lda + channel

    // A wave's work is the sequence of (block, 64-channel chunk) pairs of its blocks; the loads of the next pair
    // are issued before the MFMAs of the current one, so a wave keeps two chunks (16 KB) in flight.
    const int bstep = nwg * 4;
    auto lane_off = [&](int blk, int ch_per_img, int k_first) -> unsigned {   // byte offset of this lane's pixel, channel k_first + 4 half
        const int64_t pix = (int64_t)blk * 32 + l32;
        if (pix >= g.total) return 0x80000000u;   // past the end: loads return 0, stores are dropped
        const int n = (int)(pix / g.HW), p = (int)(pix - (int64_t)n * g.HW);
        return (unsigned)((((int64_t)n * ch_per_img + k_first + 4 * half) * g.HW + p) * 4);
    };
    auto fetch = [&](float (&b)[CH / 8][4], unsigned voff, int c0) {
#pragma unroll
        for (int t = 0; t < CH / 8; ++t) {
            const unsigned vo = c0 + 8 * t < g.C ? voff : 0x80000000u;   // (uniform) channels past C: nothing is read
#pragma unroll
            for (int e = 0; e < 4; ++e)
                b[t][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(in_rs, (int)vo, (c0 + 8 * t + e) * hw4, 0));
        }
    };
    float16v acc[KB];
    auto zero_acc = [&]() {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[kb][i] = 0.f;
    };
    auto compute = [&](const float (&b)[CH / 8][4], int c0) {
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int t = 0; t < CH / 8; ++t) {
            float4v a[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) a[kb] = *reinterpret_cast<const float4v*>(a_row + kb * 32 * g.lda + c0 + 8 * t);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) acc[kb] = mfma_32x32x2(a[kb][e], b[t][e], acc[kb]);
        }
        __builtin_amdgcn_s_setprio(0);
    };
    // register r of block kb is channel k0 + 32 kb + 8 (r/4) + 4 half + r%4, pixel l32; buffer stores with one
    // lane offset and the channel's plane offset in the scalar operand
    auto finish = [&](int blk) {
        const unsigned ooff = lane_off(blk, g.K, k0);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ku = kb * 32 + 8 * (r >> 2) + (r & 3);      // uniform part of the channel index
                const int kl = ku + 4 * half;
                float v = acc[kb][r] * mulS[kl] + addS[kl];
                if (epi.relu) v = fmaxf(v, 0.f);
                if (epi.relu == 2) v = fminf(v, 6.f);
                // a channel past K (only in the last slice): that lane half's offset is moved out of range
                const unsigned oo = (k0 + ku + 4 < g.K || k0 + kl < g.K) ? ooff : 0x80000000u;
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), out_rs, (int)oo, ku * hw4, 0);
            }
    };

    int blk = wg * 4 + wave, c0 = 0;          // current pair
    if (blk >= g.nblk) return;
    float b0[CH / 8][4], b1[CH / 8][4];
    unsigned voff = lane_off(blk, g.C, 0);
    fetch(b0, voff, 0);
    zero_acc();
    // one trip handles two pairs so that the two register sets alternate without copies
    auto advance = [&](int& nblk_, int& nc0, unsigned& nvoff) {   // the pair after (blk, c0); false when there is none
        nblk_ = blk; nc0 = c0 + CH; nvoff = voff;
        if (nc0 >= g.C) { nblk_ = blk + bstep; nc0 = 0; if (nblk_ >= g.nblk) return false; nvoff = lane_off(nblk_, g.C, 0); }
        return true;
    };
    for (;;) {
        int nb, nc; unsigned nv;
        bool more = advance(nb, nc, nv);
        if (more) fetch(b1, nv, nc);
        compute(b0, c0);
        if (!more || nb != blk) { finish(blk); zero_acc(); }
        if (!more) break;
        blk = nb; c0 = nc; voff = nv;
        more = advance(nb, nc, nv);
        if (more) fetch(b0, nv, nc);
        compute(b1, c0);
        if (!more || nb != blk) { finish(blk); zero_acc(); }
        if (!more) break;
        blk = nb; c0 = nc; voff = nv;
    }
}

int pw_ch(int C) { return C % 64 == 0 ? 64 : 32; }
int pw_cp(int C) { const int ch = pw_ch(C); return (C + ch - 1) / ch * ch; }

int pw_kt(int C, int K) {   // output channels per work-group: as many as fit next to 64 KB of weights, at most 128
    int kt = 128;
    while (kt > 32 && ((size_t)kt * (pw_cp(C) + 4) * 4 > 64 * 1024 || kt / 2 >= K)) kt >>= 1;
    return kt;
}

PwGeom pw_geom(const ConvParams& p, int kt) {
    PwGeom g{};
    g.C = p.C; g.K = p.K; g.HW = p.H * p.W;
    g.total = (int64_t)p.Nb * g.HW;
    g.nblk = (int)((g.total + 31) / 32);
    g.kt_tiles = (p.K + kt - 1) / kt;
    g.Cp = pw_cp(p.C);
    g.lda = g.Cp + 4;
    return g;
}

size_t pw_lds(int C, int kt) { return ((size_t)kt * (pw_cp(C) + 4) + 2 * kt) * 4; }

unsigned pw_grid(const PwGeom& g) {   // about four blocks per wave (the weights are staged once per work-group), 256 .. 1024 groups
    int64_t wgs = (g.nblk + 15) / 16;
    if (wgs < 256) wgs = 256;
    if (wgs > 1024) wgs = 1024;
    if (wgs > (g.nblk + 3) / 4) wgs = (g.nblk + 3) / 4;
    return (unsigned)(wgs * g.kt_tiles);
}

}  // namespace

// Stride 1, no padding, no pooling, C a multiple of 8 and at most 96; the input and the output addressed with
// 31-bit byte offsets.  Measured against the tile kernel on [32,C,56,56] (rotating buffers): 64 -> 256 52 vs 62 us,
// 96 -> 24 17.6 vs 20.7, 24 -> 144 29 vs 36, 64 -> 64 equal; with more input channels (256 -> 64 47 vs 44 us,
// 512 -> 128 59 vs 43) a work-group's share of the pixels no longer pays for staging its weights, and the tile
// kernel, which streams them chunk by chunk, is the better one.
bool conv1x1_stream_ok(const ConvParams& p) {
    if (p.R != 1 || p.S != 1 || p.stride != 1 || p.pad != 0 || p.pool) return false;
    if (p.C % 8 != 0 || p.C > 96) return false;
    const int64_t in_b = (int64_t)p.Nb * p.C * p.H * p.W * 4, out_b = (int64_t)p.Nb * p.K * p.H * p.W * 4;
    return in_b < ((int64_t)1 << 31) && out_b < ((int64_t)1 << 31);
}

LaunchShape conv1x1_shape(const ConvParams& p) {
    const int kt = pw_kt(p.C, p.K);
    const PwGeom g = pw_geom(p, kt);
    LaunchShape s{};
    s.grid[0] = pw_grid(g); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kPwThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)pw_lds(p.C, kt);
    s.kernel = kt == 32 ? "conv1x1_stream<32>" : (kt == 64 ? "conv1x1_stream<64>" : "conv1x1_stream<128>");
    return s;
}

template <int KB, int CH>
hipError_t pw_launch(const ConvParams& p, const PwGeom& g, hipStream_t stream) {
    const size_t lds = pw_lds(p.C, 32 * KB);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv1x1_stream<KB, CH>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const PwEpi epi{p.bias, p.scale, p.shift, p.relu};
    hipLaunchKernelGGL((conv1x1_stream<KB, CH>), dim3(pw_grid(g)), dim3(kPwThreads), lds, stream, p.in, p.wt, epi, p.out, g);
    return hipGetLastError();
}

template <int KB>
hipError_t pw_launch_ch(const ConvParams& p, const PwGeom& g, hipStream_t stream) {
    return pw_ch(p.C) == 64 ? pw_launch<KB, 64>(p, g, stream) : pw_launch<KB, 32>(p, g, stream);
}

hipError_t conv1x1_launch(const ConvParams& p, hipStream_t stream) {
    const int kt = pw_kt(p.C, p.K);
    const PwGeom g = pw_geom(p, kt);
    switch (kt) {
        case 32: return pw_launch_ch<1>(p, g, stream);
        case 64: return pw_launch_ch<2>(p, g, stream);
        default: return pw_launch_ch<4>(p, g, stream);
    }
}

}  // namespace hpct
