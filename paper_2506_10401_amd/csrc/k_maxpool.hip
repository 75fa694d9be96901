// Max and average pooling of NCHW planes with a k x k window, a stride and padding (Reduction class of the
// paper's Table 1; the pooling layers of the networks that its Section 5.1 names as Level-3 tasks, e.g. the
// 3 x 3 / stride 2 / pad 1 pooling behind a ResNet's first convolution).  Max: padding never wins, the maximum
// is taken over the window's positions inside the image; exact.  Average (AVG instances): positions outside
// the image count as zeros and the divisor is always k * k.  Memory-bound.
//
// maxpool3x3_rows: 3 x 3, pad 1, stride 1 or 2, whole quads on both sides - the stencil scheme of the
// depthwise 3 x 3 kernel with max in place of multiply-add.  A wave owns 56 output columns x 16 output rows
// of a plane; each of its four 16-lane rows takes 4 of those rows; lanes 1..14 own four output columns each
// (the ST input quads under them), lanes 0 and 15 only load the quads beside the segment; the input column
// left of a lane's first (and, at stride 1, right of its last) comes from the neighbouring lane by a DPP row
// shift.  Rows and quads outside the image are not read (buffer-load offset beyond the descriptor) and are
// replaced by -inf.  No LDS, no barrier.
// maxpool_any: every other window / stride / padding, an output per thread.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;
constexpr int kSeg = 56;     // output columns of a wave's segment: 14 computing lanes
constexpr int kCH = 2;       // output rows per lane (4: 27.6 us at [32,64,112,112] / 2, 2: 26.8)

struct PoolRowsGeom { int H, W, Ho, Wo, nseg, bands; int64_t items; };

template <int ST, bool AVG>
__global__ __launch_bounds__(kThreads) void maxpool3x3_rows(const float* __restrict__ in, float* __restrict__ out, PoolRowsGeom g) {
    constexpr int NQ = ST, NR = (kCH - 1) * ST + 3;   // input quads per lane and row; input rows per lane
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * (kThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= g.items) return;   // the whole wave; there are no barriers in this kernel
    const int seg = (int)(item % g.nseg);
    const int64_t t = item / g.nseg;
    const int band = (int)(t % g.bands);
    const int64_t plane = t / g.bands;
    const int dr = lane >> 4, cq = lane & 15;
    const int ox0 = seg * kSeg + 4 * (cq - 1);              // first of this lane's four output columns
    const int xi0 = ox0 * ST;                               // the input column under it
    const bool comp = cq >= 1 && cq <= 14 && ox0 < g.Wo;    // Wo % 4 == 0: a quad is inside or outside as a whole
    const int rr = (band * 4 + dr) * kCH;                   // first output row of this lane
    constexpr unsigned kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(in) + plane * (int64_t)g.H * g.W, 0, g.H * g.W * 4, 0x00020000);

    float4v v[NR][NQ];
    bool ok[NR][NQ];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int y = rr * ST + j - 1;
        const bool row_ok = y >= 0 && y < g.H;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {   // W % 4 == 0: an input quad is inside or outside as a whole
            const int xq = xi0 + 4 * q;
            ok[j][q] = row_ok && xq >= 0 && xq < g.W;
            const unsigned off = ok[j][q] ? (unsigned)((y * g.W + xq) * 4) : kOob;
            v[j][q] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0));
        }
    }
    float x[NR][4 * NQ + 2];   // x[j][1 + e] = input column xi0 + e of row j; x[j][0] the column left of them
#pragma unroll
    for (int j = 0; j < NR; ++j) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            if (!AVG && !ok[j][q]) v[j][q] = float4v{-INFINITY, -INFINITY, -INFINITY, -INFINITY};   // (AVG: the zeros the load returned)
            x[j][1 + 4 * q] = v[j][q].x; x[j][2 + 4 * q] = v[j][q].y; x[j][3 + 4 * q] = v[j][q].z; x[j][4 + 4 * q] = v[j][q].w;
        }
        x[j][0] = dpp_mov<0x111>(v[j][NQ - 1].w);       // row_shr:1 - the last column of the lane to the left
        x[j][4 * NQ + 1] = dpp_mov<0x101>(v[j][0].x);   // row_shl:1 - the first column of the lane to the right (stride 1 only)
    }
    float* __restrict__ po = out + plane * (int64_t)g.Ho * g.Wo + ox0;
#pragma unroll
    for (int i = 0; i < kCH; ++i) {
        float m[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = AVG ? 0.f : -INFINITY;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int j = 0; j < 4; ++j) m[j] = AVG ? m[j] + x[i * ST + kh][j * ST + kw] : fmaxf(m[j], x[i * ST + kh][j * ST + kw]);
        if (AVG) {
#pragma unroll
            for (int j = 0; j < 4; ++j) m[j] *= (1.f / 9.f);
        }
        if (comp && rr + i < g.Ho) store4_nt(po + (int64_t)(rr + i) * g.Wo, float4v{m[0], m[1], m[2], m[3]});
    }
}

template <bool AVG>
__global__ __launch_bounds__(kThreads) void maxpool_any(const float* __restrict__ in, float* __restrict__ out, int64_t planes,
                                                        int H, int W, int Ho, int Wo, int k, int s, int p) {
    const int64_t total = planes * Ho * Wo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int ox = (int)(o % Wo);
        const int64_t t = o / Wo;
        const int oy = (int)(t % Ho);
        const int64_t plane = t / Ho;
        const float* src = in + plane * (int64_t)H * W;
        float m = AVG ? 0.f : -INFINITY;
        for (int dy = 0; dy < k; ++dy) {
            const int iy = oy * s - p + dy;
            if (iy < 0 || iy >= H) continue;
            for (int dx = 0; dx < k; ++dx) {
                const int ix = ox * s - p + dx;
                if (ix >= 0 && ix < W) m = AVG ? m + src[(int64_t)iy * W + ix] : fmaxf(m, src[(int64_t)iy * W + ix]);
            }
        }
        out[o] = AVG ? m / (float)(k * k) : m;
    }
}

// The register variant: 3 x 3, pad 1, stride 1 or 2, whole quads on both sides, at least three computing lanes per
// segment (narrow maps leave lanes idle and still stream 2 - 5 times faster than the one-output-per-thread kernel:
// [32,256,28,28] 49 -> 11 us), a plane within the 32-bit byte offsets of a buffer descriptor.
bool rows_ok(const PoolParams& p) {
    if (p.k != 3 || p.pad != 1 || (p.stride != 1 && p.stride != 2) || (p.W & 3)) return false;
    if ((int64_t)p.H * p.W * 4 >= (int64_t)1 << 31) return false;
    const int Wo = (p.W - 1) / p.stride + 1;
    if (Wo & 3) return false;
    const int nseg = (Wo + kSeg - 1) / kSeg;
    return Wo >= nseg * 12;
}

PoolRowsGeom rows_geom(const PoolParams& p) {
    PoolRowsGeom g{};
    g.H = p.H; g.W = p.W;
    g.Ho = (p.H - 1) / p.stride + 1; g.Wo = (p.W - 1) / p.stride + 1;
    g.nseg = (g.Wo + kSeg - 1) / kSeg;
    g.bands = (g.Ho + 4 * kCH - 1) / (4 * kCH);
    g.items = p.planes * g.bands * g.nseg;
    return g;
}

unsigned any_grid(const PoolParams& p) {
    const int Ho = (p.H + 2 * p.pad - p.k) / p.stride + 1, Wo = (p.W + 2 * p.pad - p.k) / p.stride + 1;
    const int64_t g = (p.planes * Ho * Wo + kThreads - 1) / kThreads;
    return (unsigned)(g < 1 ? 1 : (g > 262144 ? 262144 : g));
}

}  // namespace

LaunchShape maxpool_shape(const PoolParams& p) {
    if (!p.avg && p.k == 2 && p.stride == 2 && p.pad == 0) return maxpool2_shape(p.planes, p.H, p.W);
    LaunchShape s{};
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.grid[1] = s.grid[2] = 1;
    s.lds_bytes = 0;
    if (rows_ok(p)) {
        const PoolRowsGeom g = rows_geom(p);
        s.grid[0] = (uint32_t)((g.items + kThreads / 64 - 1) / (kThreads / 64));
        s.kernel = p.avg ? (p.stride == 2 ? "avgpool3x3_rows<stride2>" : "avgpool3x3_rows")
                         : (p.stride == 2 ? "maxpool3x3_rows<stride2>" : "maxpool3x3_rows");
    } else {
        s.grid[0] = any_grid(p);
        s.kernel = p.avg ? "avgpool_any" : "maxpool_any";
    }
    return s;
}

hipError_t maxpool_launch(const PoolParams& p, const float* in, float* out, hipStream_t stream) {
    if (!p.avg && p.k == 2 && p.stride == 2 && p.pad == 0) return maxpool2_launch(in, out, p.planes, p.H, p.W, stream);
    if (rows_ok(p)) {
        const PoolRowsGeom g = rows_geom(p);
        const dim3 grid((unsigned)((g.items + kThreads / 64 - 1) / (kThreads / 64))), block(kThreads);
        if (p.avg) {
            if (p.stride == 2) hipLaunchKernelGGL((maxpool3x3_rows<2, true>), grid, block, 0, stream, in, out, g);
            else hipLaunchKernelGGL((maxpool3x3_rows<1, true>), grid, block, 0, stream, in, out, g);
        } else {
            if (p.stride == 2) hipLaunchKernelGGL((maxpool3x3_rows<2, false>), grid, block, 0, stream, in, out, g);
            else hipLaunchKernelGGL((maxpool3x3_rows<1, false>), grid, block, 0, stream, in, out, g);
        }
    } else {
        const int Ho = (p.H + 2 * p.pad - p.k) / p.stride + 1, Wo = (p.W + 2 * p.pad - p.k) / p.stride + 1;
        if (p.avg) hipLaunchKernelGGL(maxpool_any<true>, dim3(any_grid(p)), dim3(kThreads), 0, stream, in, out, p.planes, p.H, p.W, Ho, Wo, p.k, p.stride, p.pad);
        else hipLaunchKernelGGL(maxpool_any<false>, dim3(any_grid(p)), dim3(kThreads), 0, stream, in, out, p.planes, p.H, p.W, Ho, Wo, p.k, p.stride, p.pad);
    }
    return hipGetLastError();
}

}  // namespace hpct
