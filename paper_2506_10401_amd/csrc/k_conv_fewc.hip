// 3 x 3 convolution of an image with very few channels (the first layer of the VGG-16 that Section 5.3
// of the paper uses, of ResNets and MobileNets: C = 3, or 1 for grey images) with the conv epilogue in
// registers: bias, per-channel scale/shift, ReLU or ReLU6.
//
// With C <= 4 the contraction is only 9 C <= 36 deep while every output element is written once: the
// layer is bound by its stores (32 x 3 x 224 x 224 -> 64 channels: 411 MB out for 19 MB in) and a
// work-group that stages a tile in LDS spends its life on latencies.  conv3x3_fewc has no LDS and no
// barrier.  A wave owns 32 output channels x 128 pixels of one image row as four accumulators of
// v_mfma_f32_32x32x2_f32, channels as the MFMA's rows (A operand = weights, held in registers for all the
// wave's rows), pixels as its columns:
//   * accumulator j holds the pixels 4 l + j, l = 0..31, so a lane needs the inputs of four neighbouring
//     pixels per tap: for a tap (c, dy) one aligned 128-bit load q = in[c][y + dy][4 l .. 4 l + 3] and the
//     two single values left and right of it give all three dx of that tap - {left, q.x, q.y, q.z}, q,
//     {q.y, q.z, q.w, right} - as B operands of the four accumulators;
//   * an MFMA contracts two k, one per half-wave: half-wave h takes the taps 2 i + h of the 3 C taps
//     (c, dy), i = 0 .. ceil(3 C / 2) - 1 (for odd 3 C the last one of h = 1 is a zero weight), and
//     step (dx, i) contracts them at that dx;
//   * rows above and below the image, quads beyond its right edge and the values left of column 0 and
//     right of column W - 1 are buffer loads at an offset beyond the descriptor's size: zeros, so the
//     padding has no special case; every other load is inside the image by construction (W % 4 == 0);
//   * at the end a lane holds four neighbouring pixels of each of its 16 channels: 128-bit stores, 512
//     contiguous bytes per half-wave.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;
constexpr int kSeg = 128;      // pixels of a wave's row segment
constexpr int kRowsPerWave = 4;   // 1: 134 us, 2: 126, 4: 122, 8: 131 for 32 x 3 x 224 x 224 -> 64 channels

// ST = 2 (a MobileNet's first convolution, 3 x 3 / stride 2 / pad 1): the lane's four output pixels 4 l + j read the
// input columns 8 l - 1 .. 8 l + 7 of a tap - two aligned quads and the value left of them - output j at dx taking
// x[2 j + dx]; input row 2 y + dy - 1.
template <int C, int ST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 8))) void conv3x3_fewc(ConvParams p, int Ho, int Wo, int nseg, int kblocks, int ybands, int rows, int64_t items) {
    constexpr int T = 3 * C;             // taps (c, dy)
    constexpr int NI = (T + 1) / 2;      // taps per half-wave
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t item = (int64_t)blockIdx.x * (kThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= items) return;   // the whole wave; there are no barriers in this kernel
    // item = ((n * ybands + yb) * nseg + seg) * kblocks + kb: neighbouring waves share their pixels
    const int kb = (int)(item % kblocks);
    int64_t t = item / kblocks;
    const int seg = (int)(t % nseg); t /= nseg;
    const int yb = (int)(t % ybands);
    const int n = (int)(t / ybands);
    const int H = p.H, W = p.W, K = p.K;
    const int oxq = seg * kSeg + 4 * l32;   // first of this lane's four output pixels
    const int xq = oxq * ST;                // the input column under it

    // A operand: weights of channel kb * 32 + l32 at this half-wave's taps, all three dx, times the channel's
    // scale: (acc + bias) * scale + shift = sum (w * scale) x + (bias * scale + shift)
    float wv[3][NI];
    int rel[NI], dyv[NI];   // byte offset of the tap's plane and row relative to (c = 0, input row ST y); its dy
    {
        const float* wch = p.wt + (int64_t)(kb * 32 + l32) * (C * 9);
        const float sc = p.scale ? p.scale[kb * 32 + l32] : 1.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int tap = 2 * i + h;
            const bool ok = tap < T;
            const int c = ok ? tap / 3 : 0, dyi = ok ? tap % 3 : 0;
#pragma unroll
            for (int dxi = 0; dxi < 3; ++dxi) wv[dxi][i] = ok ? wch[(c * 3 + dyi) * 3 + dxi] * sc : 0.f;
            rel[i] = ok ? ((c * H + dyi - 1) * W) * 4 : -1;   // -1: no tap, nothing is loaded
            dyv[i] = dyi - 1;
        }
    }
    // the constant term of this lane's 16 channels: the accumulators start from it
    float add[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ch = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        add[r] = (p.bias ? p.bias[ch] : 0.f) * (p.scale ? p.scale[ch] : 1.f) + (p.shift ? p.shift[ch] : 0.f);
    }
    // output: the 32 channel planes of this block; a lane's address is its own part plus a scalar per register
    const __amdgpu_buffer_rsrc_t os = __builtin_amdgcn_make_buffer_rsrc(
        p.out + ((int64_t)n * K + kb * 32) * Ho * Wo, 0, 32 * Ho * Wo * 4, 0x00020000);
    constexpr unsigned kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.in) + (int64_t)n * C * H * W, 0, C * H * W * 4, 0x00020000);
    bool q_ok[ST];                                  // W % 4 == 0: an input quad is inside or outside as a whole
#pragma unroll
    for (int q = 0; q < ST; ++q) q_ok[q] = xq + 4 * q < W;
    const bool l_ok = xq >= 1 && xq - 1 < W;        // the value left of them
    const bool r_ok = xq + 4 < W;                   // the value right of them (stride 1 only)
    const bool o_ok = oxq < Wo;                     // Wo % 4 == 0

#pragma unroll 1
    for (int yy = 0; yy < rows; ++yy) {
        const int y = yb * rows + yy;
        if (y >= Ho) break;   // uniform
        float4v q[NI][ST];
        float lf[NI], rt[NI];
        const int rowoff = (ST * y * W + xq) * 4;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bool row_ok = rel[i] != -1 && (unsigned)(ST * y + dyv[i]) < (unsigned)H;
            const unsigned o = (unsigned)(rel[i] + rowoff);
#pragma unroll
            for (int k = 0; k < ST; ++k)
                q[i][k] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)((row_ok && q_ok[k]) ? o + 16 * k : kOob), 0, 0));
            lf[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)((row_ok && l_ok) ? o - 4 : kOob), 0, 0));
            if (ST == 1) rt[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)((row_ok && r_ok) ? o + 16 : kOob), 0, 0));
            else rt[i] = 0.f;
        }
        float16v acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = add[r];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            float x[4 * ST + 2];   // x[0] = the column left of the lane's first, then its quads, then (stride 1) the one right of them
            x[0] = lf[i];
#pragma unroll
            for (int k = 0; k < ST; ++k) { x[1 + 4 * k] = q[i][k].x; x[2 + 4 * k] = q[i][k].y; x[3 + 4 * k] = q[i][k].z; x[4 + 4 * k] = q[i][k].w; }
            x[4 * ST + 1] = rt[i];
#pragma unroll
            for (int dxi = 0; dxi < 3; ++dxi)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma_32x32x2(wv[dxi][i], x[ST * j + dxi], acc[j]);
        }
        // register r of accumulator j: channel 8 (r / 4) + 4 h + r % 4 of the block, pixel 4 l + j of the segment
        const unsigned ov = o_ok ? (unsigned)(((4 * h) * Ho * Wo + y * Wo + oxq) * 4) : kOob;   // (a store beyond the descriptor is dropped)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float4v v = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            if (p.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
            if (p.relu == 2) { v.x = fminf(v.x, 6.f); v.y = fminf(v.y, 6.f); v.z = fminf(v.z, 6.f); v.w = fminf(v.w, 6.f); }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned, v), os, (int)ov,
                                                   ((8 * (r >> 2) + (r & 3)) * Ho * Wo) * 4, 2);   // aux 2: non-temporal, the output is not read again here (122 -> 110 us)
        }
    }
}

// 7 x 7, stride 2, pad 3 on at most 3 channels (a ResNet's first convolution): the same scheme.  A lane's four
// output pixels 4 l + j read the input columns 8 l - 3 .. 8 l + 9 of a tap row (c, dy): four aligned quads
// x[0..15] = columns 8 l - 4 .. 8 l + 11, of which output j at tap dx takes x[2 j + dx + 1]; a quad is inside
// or outside the row as a whole (W % 4 == 0), so the zero padding is again the out-of-range buffer load.
// Half-wave h takes the tap rows 2 i + h of the 7 C, and the seven dx of a tap row are seven MFMA steps.
// The weights of the wave's 32 channels stay in registers (77 per lane for C = 3).
constexpr int kRows7 = 2;   // output rows per wave

template <int C>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 8))) void conv7x7s2_fewc(ConvParams p, int Ho, int Wo, int nseg, int kblocks, int ybands, int rows, int64_t items) {
    constexpr int T = 7 * C;             // tap rows (c, dy)
    constexpr int NI = (T + 1) / 2;      // tap rows per half-wave
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t item = (int64_t)blockIdx.x * (kThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= items) return;   // the whole wave; there are no barriers in this kernel
    const int kb = (int)(item % kblocks);
    int64_t t = item / kblocks;
    const int seg = (int)(t % nseg); t /= nseg;
    const int yb = (int)(t % ybands);
    const int n = (int)(t / ybands);
    const int H = p.H, W = p.W, K = p.K;
    const int oxq = seg * kSeg + 4 * l32;    // first of this lane's four output pixels
    const int xin = 2 * oxq - 4;             // input column of x[0]

    float wv[NI][7];
    int rel[NI], dyv[NI];   // byte offset of the tap row's plane relative to (c = 0, input row 2 y); its dy - 3
    {
        const float* wch = p.wt + (int64_t)(kb * 32 + l32) * (C * 49);
        const float sc = p.scale ? p.scale[kb * 32 + l32] : 1.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int tap = 2 * i + h;
            const bool ok = tap < T;
            const int c = ok ? tap / 7 : 0, dyi = ok ? tap % 7 : 0;
#pragma unroll
            for (int dx = 0; dx < 7; ++dx) wv[i][dx] = ok ? wch[(c * 7 + dyi) * 7 + dx] * sc : 0.f;
            rel[i] = ok ? ((c * H + dyi - 3) * W) * 4 : -1;   // -1: no tap row, nothing is loaded
            dyv[i] = dyi - 3;
        }
    }
    float add[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ch = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        add[r] = (p.bias ? p.bias[ch] : 0.f) * (p.scale ? p.scale[ch] : 1.f) + (p.shift ? p.shift[ch] : 0.f);
    }
    const __amdgpu_buffer_rsrc_t os = __builtin_amdgcn_make_buffer_rsrc(
        p.out + ((int64_t)n * K + kb * 32) * Ho * Wo, 0, 32 * Ho * Wo * 4, 0x00020000);
    constexpr unsigned kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.in) + (int64_t)n * C * H * W, 0, C * H * W * 4, 0x00020000);
    bool q_ok[4];   // W % 4 == 0 and xin % 4 == 0: each quad is inside or outside the row as a whole
#pragma unroll
    for (int q = 0; q < 4; ++q) q_ok[q] = xin + 4 * q >= 0 && xin + 4 * q < W;
    const bool o_ok = oxq < Wo;   // Wo % 4 == 0

#pragma unroll 1
    for (int yy = 0; yy < rows; ++yy) {
        const int y = yb * rows + yy;
        if (y >= Ho) break;   // uniform
        float16v acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = add[r];
        const int rowoff = (2 * y * W + xin) * 4;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bool row_ok = rel[i] != -1 && (unsigned)(2 * y + dyv[i]) < (unsigned)H;
            const unsigned o = (unsigned)(rel[i] + rowoff);
            float x[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4v v = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)((row_ok && q_ok[q]) ? o + 16 * q : kOob), 0, 0));
                x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int dx = 0; dx < 7; ++dx)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma_32x32x2(wv[i][dx], x[2 * j + dx + 1], acc[j]);
        }
        const unsigned ov = o_ok ? (unsigned)(((4 * h) * Ho * Wo + y * Wo + oxq) * 4) : kOob;   // (a store beyond the descriptor is dropped)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float4v v = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            if (p.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
            if (p.relu == 2) { v.x = fminf(v.x, 6.f); v.y = fminf(v.y, 6.f); v.z = fminf(v.z, 6.f); v.w = fminf(v.w, 6.f); }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned, v), os, (int)ov,
                                                   ((8 * (r >> 2) + (r & 3)) * Ho * Wo) * 4, 2);   // non-temporal
        }
    }
}

struct FewcGeom { int Ho, Wo, nseg, kblocks, ybands, rows; int64_t items; };
bool is7(const ConvParams& p) { return p.R == 7; }
FewcGeom fewc_geom(const ConvParams& p) {
    FewcGeom g{};
    g.Ho = (p.H - 1) / p.stride + 1;   // both kernels: pad = (R - 1) / 2
    g.Wo = (p.W - 1) / p.stride + 1;
    g.nseg = (g.Wo + kSeg - 1) / kSeg;
    g.kblocks = p.K / 32;
    // output rows per wave (the weights are loaded once per wave): as many as leave about four waves per SIMD
    int rows = is7(p) ? kRows7 : kRowsPerWave;
    while (rows > 1 && (int64_t)p.Nb * ((g.Ho + rows - 1) / rows) * g.nseg * g.kblocks < 4096) rows >>= 1;
    g.rows = rows;
    g.ybands = (g.Ho + rows - 1) / rows;
    g.items = (int64_t)p.Nb * g.ybands * g.nseg * g.kblocks;
    return g;
}

}  // namespace

// No dilation, no pooling; output channels in blocks of 32; rows of whole quads on both sides that fill at least three
// quarters of their 128-pixel segments; an image and a block of 32 output planes within 31-bit byte offsets; and either
// 3 x 3 / stride 1 or 2 / pad 1 on at most 4 input channels or 7 x 7 / stride 2 / pad 3 on at most 3.
bool conv_fewc_ok(const ConvParams& p) {
    if (p.R != p.S || p.dil != 1 || p.pool || (p.K & 31) || (p.W & 3) || p.C < 1) return false;
    const bool k3 = p.R == 3 && (p.stride == 1 || p.stride == 2) && p.pad == 1 && p.C <= 4;
    const bool k7 = p.R == 7 && p.stride == 2 && p.pad == 3 && p.C <= 3;
    if (!k3 && !k7) return false;
    const int Ho = (p.H - 1) / p.stride + 1, Wo = (p.W - 1) / p.stride + 1;
    if (Wo & 3) return false;
    if ((int64_t)p.C * p.H * p.W * 4 >= (int64_t)1 << 31 || (int64_t)32 * Ho * Wo * 4 >= (int64_t)1 << 31) return false;
    const int nseg = (Wo + kSeg - 1) / kSeg;
    return Wo * 4 >= nseg * kSeg * 3;
}

LaunchShape conv_fewc_shape(const ConvParams& p) {
    const FewcGeom g = fewc_geom(p);
    LaunchShape s{};
    s.grid[0] = (uint32_t)((g.items + kThreads / 64 - 1) / (kThreads / 64)); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    s.kernel = is7(p) ? "conv7x7s2_fewc" : (p.stride == 2 ? "conv3x3_fewc<stride2>" : "conv3x3_fewc");
    return s;
}

hipError_t conv_fewc_launch(const ConvParams& p, hipStream_t stream) {
    const FewcGeom g = fewc_geom(p);
    const dim3 grid((unsigned)((g.items + kThreads / 64 - 1) / (kThreads / 64))), block(kThreads);
    if (is7(p)) {
        switch (p.C) {
            case 1: hipLaunchKernelGGL(conv7x7s2_fewc<1>, grid, block, 0, stream, p, g.Ho, g.Wo, g.nseg, g.kblocks, g.ybands, g.rows, g.items); break;
            case 2: hipLaunchKernelGGL(conv7x7s2_fewc<2>, grid, block, 0, stream, p, g.Ho, g.Wo, g.nseg, g.kblocks, g.ybands, g.rows, g.items); break;
            default: hipLaunchKernelGGL(conv7x7s2_fewc<3>, grid, block, 0, stream, p, g.Ho, g.Wo, g.nseg, g.kblocks, g.ybands, g.rows, g.items); break;
        }
        return hipGetLastError();
    }
#define HPCT_FEWC(CC) do { \
        if (p.stride == 2) hipLaunchKernelGGL((conv3x3_fewc<CC, 2>), grid, block, 0, stream, p, g.Ho, g.Wo, g.nseg, g.kblocks, g.ybands, g.rows, g.items); \
        else hipLaunchKernelGGL((conv3x3_fewc<CC, 1>), grid, block, 0, stream, p, g.Ho, g.Wo, g.nseg, g.kblocks, g.ybands, g.rows, g.items); } while (0)
    switch (p.C) {
        case 1: HPCT_FEWC(1); break;
        case 2: HPCT_FEWC(2); break;
        case 3: HPCT_FEWC(3); break;
        default: HPCT_FEWC(4); break;
    }
#undef HPCT_FEWC
    return hipGetLastError();
}

}  // namespace hpct
