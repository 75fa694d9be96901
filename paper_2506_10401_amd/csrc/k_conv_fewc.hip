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

template <int C>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 8))) void conv3x3_fewc(ConvParams p, int nseg, int kblocks, int ybands, int64_t items) {
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
    const int x0 = seg * kSeg, xq = x0 + 4 * l32;   // first of this lane's four pixels

    // A operand: weights of channel kb * 32 + l32 at this half-wave's taps, all three dx, times the channel's
    // scale: (acc + bias) * scale + shift = sum (w * scale) x + (bias * scale + shift)
    float wv[3][NI];
    int rel[NI], dyv[NI];   // byte offset of the tap's plane and row relative to (c = 0, row y); its dy
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
        p.out + ((int64_t)n * K + kb * 32) * H * W, 0, 32 * H * W * 4, 0x00020000);
    constexpr unsigned kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.in) + (int64_t)n * C * H * W, 0, C * H * W * 4, 0x00020000);
    const bool q_ok = xq < W;                       // W % 4 == 0: the quad is inside or outside as a whole
    const bool l_ok = xq >= 1 && xq - 1 < W;        // the value left of it
    const bool r_ok = xq + 4 < W;                   // the value right of it

#pragma unroll 1
    for (int yy = 0; yy < kRowsPerWave; ++yy) {
        const int y = yb * kRowsPerWave + yy;
        if (y >= H) break;   // uniform
        float4v q[NI];
        float lf[NI], rt[NI];
        const int rowoff = (y * W + xq) * 4;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bool row_ok = rel[i] != -1 && (unsigned)(y + dyv[i]) < (unsigned)H;
            const unsigned o = (unsigned)(rel[i] + rowoff);
            q[i] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)((row_ok && q_ok) ? o : kOob), 0, 0));
            lf[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)((row_ok && l_ok) ? o - 4 : kOob), 0, 0));
            rt[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)((row_ok && r_ok) ? o + 16 : kOob), 0, 0));
        }
        float16v acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = add[r];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const float x[6] = {lf[i], q[i].x, q[i].y, q[i].z, q[i].w, rt[i]};
#pragma unroll
            for (int dxi = 0; dxi < 3; ++dxi)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma_32x32x2(wv[dxi][i], x[j + dxi], acc[j]);
        }
        // register r of accumulator j: channel 8 (r / 4) + 4 h + r % 4 of the block, pixel 4 l + j of the segment
        const unsigned ov = q_ok ? (unsigned)(((4 * h) * H * W + y * W + xq) * 4) : kOob;   // (a store beyond the descriptor is dropped)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float4v v = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            if (p.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
            if (p.relu == 2) { v.x = fminf(v.x, 6.f); v.y = fminf(v.y, 6.f); v.z = fminf(v.z, 6.f); v.w = fminf(v.w, 6.f); }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned, v), os, (int)ov,
                                                   ((8 * (r >> 2) + (r & 3)) * H * W) * 4, 0);
        }
    }
}

struct FewcGeom { int nseg, kblocks, ybands; int64_t items; };
FewcGeom fewc_geom(const ConvParams& p) {
    FewcGeom g{};
    g.nseg = (p.W + kSeg - 1) / kSeg;
    g.kblocks = p.K / 32;
    g.ybands = (p.H + kRowsPerWave - 1) / kRowsPerWave;
    g.items = (int64_t)p.Nb * g.ybands * g.nseg * g.kblocks;
    return g;
}

}  // namespace

// 3 x 3, stride 1, pad 1, no dilation, no pooling; at most 4 input channels; output channels in blocks of 32; rows of
// whole quads that fill at least three quarters of their 128-pixel segments; an image within 31-bit byte offsets.
bool conv_fewc_ok(const ConvParams& p) {
    if (p.R != 3 || p.S != 3 || p.stride != 1 || p.pad != 1 || p.dil != 1 || p.pool) return false;
    if (p.C < 1 || p.C > 4 || (p.K & 31) || (p.W & 3)) return false;
    if ((int64_t)p.C * p.H * p.W * 4 >= (int64_t)1 << 31 || (int64_t)32 * p.H * p.W * 4 >= (int64_t)1 << 31) return false;
    const int nseg = (p.W + kSeg - 1) / kSeg;
    return p.W * 4 >= nseg * kSeg * 3;
}

LaunchShape conv_fewc_shape(const ConvParams& p) {
    const FewcGeom g = fewc_geom(p);
    LaunchShape s{};
    s.grid[0] = (uint32_t)((g.items + kThreads / 64 - 1) / (kThreads / 64)); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    s.kernel = "conv3x3_fewc";
    return s;
}

hipError_t conv_fewc_launch(const ConvParams& p, hipStream_t stream) {
    const FewcGeom g = fewc_geom(p);
    const dim3 grid((unsigned)((g.items + kThreads / 64 - 1) / (kThreads / 64))), block(kThreads);
    switch (p.C) {
        case 1: hipLaunchKernelGGL(conv3x3_fewc<1>, grid, block, 0, stream, p, g.nseg, g.kblocks, g.ybands, g.items); break;
        case 2: hipLaunchKernelGGL(conv3x3_fewc<2>, grid, block, 0, stream, p, g.nseg, g.kblocks, g.ybands, g.items); break;
        case 3: hipLaunchKernelGGL(conv3x3_fewc<3>, grid, block, 0, stream, p, g.nseg, g.kblocks, g.ybands, g.items); break;
        default: hipLaunchKernelGGL(conv3x3_fewc<4>, grid, block, 0, stream, p, g.nseg, g.kblocks, g.ybands, g.items); break;
    }
    return hipGetLastError();
}

}  // namespace hpct
