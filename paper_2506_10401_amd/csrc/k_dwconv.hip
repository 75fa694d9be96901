// Depthwise NCHW convolution (groups = C = K: every channel is filtered by its own
// R x R filter; the depthwise layers of the MobileNetV2 blocks that Section 5.2 of
// the paper names among its Level-3 models) with the conv epilogue in registers:
// bias, per-channel scale/shift, ReLU or ReLU6.
//
// 2 R^2 flop per 8 bytes moved: memory-bound, a stencil.  A work-group owns a band
// of output rows of one (n, c) plane: the input rows the band needs are staged in
// LDS once (zero padding written as zeros), the channel's R^2 weights sit in
// registers, and a thread produces four neighbouring outputs of a row per step from
// whole 128-bit LDS reads and stores them as one 128-bit vector.  Planes too small to
// occupy a work-group (14 x 14, 7 x 7) are packed several to a work-group.
//
// The commonest cases - 3 x 3, stride 1 or 2, pad 1, output rows of a multiple of 4 columns that
// fill most of a 16-lane row - do not go through LDS at all (dwconv3x3_rows): a lane owns four
// output columns of a few rows, the input rows under them are 128-bit vectors in registers and
// the columns it lacks come from the neighbouring lanes by DPP row shifts.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kDwThreads = 256;

struct DwGeom {
    int C, H, W, Ho, Wo, St, P, Dl;
    int BH;        // output rows per band
    int bands;     // bands per plane
    int in_rows;   // staged input rows of a band: (BH-1)*St + (R-1)*Dl + 1
    int ldw;       // LDS row pitch (floats), a multiple of 4; LDS column x holds image column x - P
    int pp;        // planes per work-group (small planes; then bands = 1)
    int64_t planes;
};

template <int R, bool MULTI>
__global__ __launch_bounds__(kDwThreads) void dwconv_planes(const float* __restrict__ in, const float* __restrict__ wt,
                                                            const float* __restrict__ bias, const float* __restrict__ scale,
                                                            const float* __restrict__ shift, float* __restrict__ out,
                                                            DwGeom g, int relu) {
    extern __shared__ __align__(16) float rows[];
    const int tid = threadIdx.x;
    const int64_t plane0 = MULTI ? (int64_t)blockIdx.x * g.pp : blockIdx.x / g.bands;   // plane = n*C + c
    const int band = MULTI ? 0 : blockIdx.x - (int)plane0 * g.bands;
    const int np = MULTI ? (int)(g.planes - plane0 < g.pp ? g.planes - plane0 : g.pp) : 1;
    const int oh0 = band * g.BH;
    const int bh = g.Ho - oh0 < g.BH ? g.Ho - oh0 : g.BH;     // output rows of this band
    const int ih0 = oh0 * g.St - g.P;                         // first staged input row
    const int nrows = (bh - 1) * g.St + (R - 1) * g.Dl + 1;
    const int tile = g.in_rows * g.ldw;                       // floats per staged plane

    // ---- stage.  LDS column x (a multiple of 4 per slot) holds image column x - P, so that a thread's
    // fragment reads below start on 16-byte boundaries; the global side of a slot is then an unaligned
    // 128-bit load, which the memory system takes, with a per-element test at the two row ends.
    const int ldw4 = g.ldw >> 2;
    const int per_plane = nrows * ldw4;
    for (int s = tid; s < np * per_plane; s += kDwThreads) {
        const int pl = MULTI ? s / per_plane : 0;
        const int rem = s - pl * per_plane;
        const int r = rem / ldw4, x = (rem - r * ldw4) * 4;
        const int ih = ih0 + r, iw = x - g.P;
        float4v v = {0.f, 0.f, 0.f, 0.f};
        if (ih >= 0 && ih < g.H) {
            const float* p = in + ((plane0 + pl) * g.H + ih) * (int64_t)g.W + iw;
            if (iw >= 0 && iw + 3 < g.W) {
                v = float4v{p[0], p[1], p[2], p[3]};          // (the compiler merges these into one 128-bit load)
            } else {
                if (iw >= 0 && iw < g.W) v.x = p[0];
                if (iw + 1 >= 0 && iw + 1 < g.W) v.y = p[1];
                if (iw + 2 >= 0 && iw + 2 < g.W) v.z = p[2];
                if (iw + 3 >= 0 && iw + 3 < g.W) v.w = p[3];
            }
        }
        *reinterpret_cast<float4v*>(rows + pl * tile + r * g.ldw + x) = v;
    }
    float w[R * R];
    float mul = 1.f, add = 0.f;
    auto load_channel = [&](int c) {
#pragma unroll
        for (int i = 0; i < R * R; ++i) w[i] = wt[c * R * R + i];
        mul = scale ? scale[c] : 1.f;
        add = (bias ? bias[c] : 0.f) * mul + (shift ? shift[c] : 0.f);   // (acc + bias) * scale + shift
    };
    if (!MULTI) load_channel((int)(plane0 % g.C));   // uniform over the work-group
    __syncthreads();

    // ---- compute: task = (plane of the group, output row of the band, four output columns)
    const int cols4 = (g.Wo + 3) >> 2;
    const bool vec_out = (g.Wo & 3) == 0;
    const int per_plane_t = bh * cols4;
    for (int t = tid; t < np * per_plane_t; t += kDwThreads) {
        const int pl = MULTI ? t / per_plane_t : 0;
        const int rem = t - pl * per_plane_t;
        const int ohl = rem / cols4, ow = (rem - ohl * cols4) * 4;
        if (MULTI) load_channel((int)((plane0 + pl) % g.C));
        const float* base = rows + pl * tile + ohl * g.St * g.ldw + ow * g.St;   // 16-byte aligned
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kh = 0; kh < R; ++kh) {
            const float* rp = base + kh * g.Dl * g.ldw;
            if (g.St == 1 && g.Dl == 1) {   // uniform: the 4 + R - 1 inputs of the row as whole 128-bit reads
                constexpr int NV = (4 + R - 1 + 3) / 4;
                float x[NV * 4];
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    const float4v t4 = *reinterpret_cast<const float4v*>(rp + 4 * q);
                    x[4 * q] = t4.x; x[4 * q + 1] = t4.y; x[4 * q + 2] = t4.z; x[4 * q + 3] = t4.w;
                }
#pragma unroll
                for (int kw = 0; kw < R; ++kw)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] += x[j + kw] * w[kh * R + kw];
            } else if (g.St == 2 && g.Dl == 1) {
                constexpr int NV = (7 + R - 1 + 3) / 4;
                float x[NV * 4];
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    const float4v t4 = *reinterpret_cast<const float4v*>(rp + 4 * q);
                    x[4 * q] = t4.x; x[4 * q + 1] = t4.y; x[4 * q + 2] = t4.z; x[4 * q + 3] = t4.w;
                }
#pragma unroll
                for (int kw = 0; kw < R; ++kw)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] += x[2 * j + kw] * w[kh * R + kw];
            } else {
#pragma unroll
                for (int kw = 0; kw < R; ++kw)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] += rp[j * g.St + kw * g.Dl] * w[kh * R + kw];
            }
        }
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = acc[j] * mul + add;
            if (relu) v[j] = fmaxf(v[j], 0.f);
            if (relu == 2) v[j] = fminf(v[j], 6.f);
        }
        float* o = out + ((plane0 + pl) * g.Ho + oh0 + ohl) * (int64_t)g.Wo + ow;
        if (vec_out) {
            store4_nt(o, float4v{v[0], v[1], v[2], v[3]});
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (ow + j < g.Wo) o[j] = v[j];
        }
    }
}

// ---- 3 x 3, stride 1 or 2, pad 1, without LDS
// A wave owns a segment of 56 output columns of 4 * CH output rows of one plane.  Each of its four 16-lane rows
// takes CH of those rows; inside it lanes 1..14 own four output columns each - the ST input quads under them, ST =
// stride - lanes 0 and 15 load the quads left and right of the segment and compute nothing (beyond the image
// border they read zeros, like every row above or below the image: offsets past the buffer descriptor's size).
// So a shift by one lane inside the 16-lane row (DPP, no LDS) brings the input column left of a lane's first and,
// at stride 1, the one right of its last, and the zero padding needs no special case.
// A lane issues the loads of all the (CH - 1) ST + 3 input rows of its CH output rows together.
constexpr int kDwSeg = 56;           // output columns of a segment: 14 computing lanes
struct DwRowsGeom { int C, H, W, Ho, Wo, nseg, bands; int64_t items; };

template <int ST, int CH>
__global__ __launch_bounds__(kDwThreads) void dwconv3x3_rows(const float* __restrict__ in, const float* __restrict__ wt,
                                                             const float* __restrict__ bias, const float* __restrict__ scale,
                                                             const float* __restrict__ shift, float* __restrict__ out,
                                                             DwRowsGeom g, int relu) {
    constexpr int NQ = ST, NR = (CH - 1) * ST + 3;   // input quads per lane and row; input rows per lane
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * (kDwThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= g.items) return;   // the whole wave; there are no barriers in this kernel
    const int seg = (int)(item % g.nseg);
    const int64_t t = item / g.nseg;
    const int band = (int)(t % g.bands);
    const int64_t plane = t / g.bands;
    const int c = (int)(plane % g.C);
    float w[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) w[i] = wt[c * 9 + i];
    const float mul = scale ? scale[c] : 1.f;
    const float add = (bias ? bias[c] : 0.f) * mul + (shift ? shift[c] : 0.f);   // (acc + bias) * scale + shift

    const int dr = lane >> 4, cq = lane & 15;
    const int ox0 = seg * kDwSeg + 4 * (cq - 1);                // first of this lane's four output columns
    const int xi0 = ox0 * ST;                                   // the input column under it
    const bool comp = cq >= 1 && cq <= 14 && ox0 < g.Wo;        // Wo % 4 == 0: a quad is inside or outside as a whole
    const int rr = (band * 4 + dr) * CH;                        // first output row of this lane
    constexpr unsigned kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(in) + plane * (int64_t)g.H * g.W, 0, g.H * g.W * 4, 0x00020000);

    float4v v[NR][NQ];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int y = rr * ST + j - 1;
        const bool row_ok = y >= 0 && y < g.H;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {   // W % 4 == 0: an input quad is inside or outside as a whole
            const int xq = xi0 + 4 * q;
            const unsigned off = (row_ok && xq >= 0 && xq < g.W) ? (unsigned)((y * g.W + xq) * 4) : kOob;
            v[j][q] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0));
        }
    }
    float x[NR][4 * NQ + 2];   // x[j][1 + e] = input column xi0 + e of row j; x[j][0] the column left of them
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        x[j][0] = dpp_mov<0x111>(v[j][NQ - 1].w);   // row_shr:1 - the last column of the lane to the left
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            x[j][1 + 4 * q] = v[j][q].x; x[j][2 + 4 * q] = v[j][q].y; x[j][3 + 4 * q] = v[j][q].z; x[j][4 + 4 * q] = v[j][q].w;
        }
        x[j][4 * NQ + 1] = dpp_mov<0x101>(v[j][0].x);   // row_shl:1 - the first column of the lane to the right (stride 1 only)
    }
    float* __restrict__ po = out + plane * (int64_t)g.Ho * g.Wo + ox0;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] += x[i * ST + kh][j * ST + kw] * w[kh * 3 + kw];
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = acc[j] * mul + add;
            if (relu) o[j] = fmaxf(o[j], 0.f);
            if (relu == 2) o[j] = fminf(o[j], 6.f);
        }
        if (comp && rr + i < g.Ho) store4_nt(po + (int64_t)(rr + i) * g.Wo, float4v{o[0], o[1], o[2], o[3]});
    }
}

// Output rows per lane.  Many short waves stream better than fewer long ones (stride 1, 56 x 56 planes, 32 x 144 of
// them: 4 rows 21.0 us, 7 rows 21.6, 14 rows 25.0; 64 x 144: 38.3 / 38.3 / 42.3), although a lane then loads 6 rows
// for 4.
constexpr int kDwRowsCH = 4, kDwRowsCH2 = 4;   // at stride 1, at stride 2

// The register variant: 3 x 3, stride 1 or 2, dilation 1, pad 1, whole quads on both sides (W % 4 == 0 and
// Wo % 4 == 0), at least three quarters of the lanes computing (Wo = 56: 14 of 16; Wo = 28 would be 7 of 16 and
// stays with the LDS variant), a plane within the 32-bit byte offsets of a buffer descriptor.
bool dw_rows_ok(const ConvParams& p) {
    if (p.R != 3 || (p.stride != 1 && p.stride != 2) || p.dil != 1 || p.pad != 1 || (p.W & 3)) return false;
    if ((int64_t)p.H * p.W * 4 >= (int64_t)1 << 31) return false;
    const int Wo = (p.W - 1) / p.stride + 1;
    if (Wo & 3) return false;
    const int nseg = (Wo + kDwSeg - 1) / kDwSeg;
    return Wo >= nseg * 16 * 3;
}

DwRowsGeom dw_rows_geom(const ConvParams& p) {
    DwRowsGeom g{};
    g.C = p.C; g.H = p.H; g.W = p.W;
    g.Ho = (p.H - 1) / p.stride + 1; g.Wo = (p.W - 1) / p.stride + 1;
    g.nseg = (g.Wo + kDwSeg - 1) / kDwSeg;
    const int ch = p.stride == 2 ? kDwRowsCH2 : kDwRowsCH;
    g.bands = (g.Ho + 4 * ch - 1) / (4 * ch);
    g.items = (int64_t)p.Nb * p.C * g.bands * g.nseg;
    return g;
}

DwGeom dw_geom(const ConvParams& p) {
    DwGeom g{};
    g.C = p.C; g.H = p.H; g.W = p.W; g.St = p.stride; g.P = p.pad; g.Dl = p.dil;
    const int re = (p.R - 1) * p.dil + 1;
    g.Ho = (p.H + 2 * p.pad - re) / p.stride + 1;
    g.Wo = (p.W + 2 * p.pad - re) / p.stride + 1;
    g.planes = (int64_t)p.Nb * p.C;
    const int cols4 = (g.Wo + 3) / 4;
    // LDS columns the compute loop can touch: the last task of a row reads whole 128-bit vectors from its
    // first input on (4 + R - 1 inputs at stride 1, 7 + R - 1 at stride 2, rounded up to a multiple of 4)
    int span = 3 * p.stride + re;
    if (p.dil == 1 && p.stride <= 2) span = (span + 3) & ~3;
    const int need = (cols4 - 1) * 4 * p.stride + span;
    const int have = p.W + 2 * p.pad;
    g.ldw = ((need > have ? need : have) + 3) & ~3;
    // whole planes while they are small; otherwise bands of at most 16 KB of LDS, and enough
    // work-groups to fill the chip
    int bh = g.Ho;
    auto lds_of = [&](int b) { return (size_t)((b - 1) * p.stride + re) * g.ldw * 4; };
    while (bh > 1 && (lds_of(bh) > 16 * 1024 || (g.planes * ((g.Ho + bh - 1) / bh) < 1024 && bh > 8))) bh = (bh + 1) / 2;
    g.BH = bh;
    g.bands = (g.Ho + bh - 1) / bh;
    g.in_rows = (bh - 1) * p.stride + re;
    // small planes: several per work-group, about one task per thread, at most 16 KB of LDS
    g.pp = 1;
    if (g.bands == 1) {
        const int tasks = g.Ho * cols4;
        int pp = kDwThreads / tasks;
        const int fit = (int)(16 * 1024 / ((size_t)g.in_rows * g.ldw * 4));
        if (pp > fit) pp = fit;
        if (pp > 1) g.pp = pp;
    }
    return g;
}

size_t dw_lds(const DwGeom& g) { return (size_t)g.pp * g.in_rows * g.ldw * 4; }
unsigned dw_grid(const DwGeom& g) { return (unsigned)(g.pp > 1 ? (g.planes + g.pp - 1) / g.pp : g.planes * g.bands); }

}  // namespace

bool dwconv_supported(const ConvParams& p, const char** why) {
    if (p.R != 1 && p.R != 3 && p.R != 5 && p.R != 7) { *why = "only square 1x1, 3x3, 5x5 and 7x7 filters are supported"; return false; }
    if (p.stride > 4 || p.dil > 4) { *why = "strides and dilations above 4 are not supported"; return false; }
    if (p.pad > (p.R - 1) * p.dil) { *why = "padding larger than the (dilated) filter extent minus one"; return false; }
    if (dw_rows_ok(p)) return true;   // no LDS
    const DwGeom g = dw_geom(p);
    if (dw_lds(g) > 64 * 1024) { *why = "one band of input rows does not fit in LDS (image too wide)"; return false; }
    return true;
}

LaunchShape dwconv_shape(const ConvParams& p) {
    LaunchShape s{};
    if (dw_rows_ok(p)) {
        const DwRowsGeom r = dw_rows_geom(p);
        s.grid[0] = (uint32_t)((r.items + kDwThreads / 64 - 1) / (kDwThreads / 64)); s.grid[1] = s.grid[2] = 1;
        s.block[0] = kDwThreads; s.block[1] = s.block[2] = 1;
        s.lds_bytes = 0;
        s.kernel = p.stride == 2 ? "dwconv3x3_rows<stride2>" : "dwconv3x3_rows";
        return s;
    }
    const DwGeom g = dw_geom(p);
    s.grid[0] = dw_grid(g); s.grid[1] = s.grid[2] = 1;
    s.block[0] = kDwThreads; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)dw_lds(g);
    static const char* const names[4] = {"dwconv_planes<1x1>", "dwconv_planes<3x3>", "dwconv_planes<5x5>", "dwconv_planes<7x7>"};
    s.kernel = names[p.R / 2];
    return s;
}

template <int R>
void dw_launch_r(const ConvParams& p, const DwGeom& g, hipStream_t stream) {
    const dim3 grid(dw_grid(g)), block(kDwThreads);
    const size_t lds = dw_lds(g);
    if (g.pp > 1) hipLaunchKernelGGL((dwconv_planes<R, true>), grid, block, lds, stream, p.in, p.wt, p.bias, p.scale, p.shift, p.out, g, p.relu);
    else hipLaunchKernelGGL((dwconv_planes<R, false>), grid, block, lds, stream, p.in, p.wt, p.bias, p.scale, p.shift, p.out, g, p.relu);
}

hipError_t dwconv_launch(const ConvParams& p, hipStream_t stream) {
    if (dw_rows_ok(p)) {
        const DwRowsGeom r = dw_rows_geom(p);
        const dim3 grid((unsigned)((r.items + kDwThreads / 64 - 1) / (kDwThreads / 64))), block(kDwThreads);
        if (p.stride == 2) hipLaunchKernelGGL((dwconv3x3_rows<2, kDwRowsCH2>), grid, block, 0, stream, p.in, p.wt, p.bias, p.scale, p.shift, p.out, r, p.relu);
        else hipLaunchKernelGGL((dwconv3x3_rows<1, kDwRowsCH>), grid, block, 0, stream, p.in, p.wt, p.bias, p.scale, p.shift, p.out, r, p.relu);
        return hipGetLastError();
    }
    const DwGeom g = dw_geom(p);
    switch (p.R) {
        case 1: dw_launch_r<1>(p, g, stream); break;
        case 3: dw_launch_r<3>(p, g, stream); break;
        case 5: dw_launch_r<5>(p, g, stream); break;
        default: dw_launch_r<7>(p, g, stream); break;
    }
    return hipGetLastError();
}

}  // namespace hpct
