// NCHW conv2d (cross-correlation, zero padding, stride 1, 1x1 or 3x3 filter)
// with the bias / ReLU epilogue held in registers: the convolution of the
// paper's VGG-16 case study (Section 5.3; Table 1 "conv").  Implicit GEMM on
// v_mfma_f32_32x32x2_f32:
//
//     D[k_out, pixel] = sum_{c,kh,kw} wt[k_out, c, kh, kw] * in[c, h-P+kh, w-P+kw]
//
// Rows of D are output channels (A operand = weights), columns are output
// pixels (B operand = input patches), so a lane owns one pixel and an
// accumulator register is stored as 32 consecutive pixels = 128 contiguous
// bytes of the NCHW output.
//
// A work-group of four waves owns KT = 128 output channels x TP = 64
// consecutive output pixels of one image.  Channels are processed CC at a time:
// the input rows the tile touches (with their zero halo) and the CC*R*S weight
// columns are staged in LDS, double buffered, with the global loads of chunk
// t+1 in flight while chunk t is multiplied.  One MFMA contracts two channels
// (lane half 0 / 1 = channel 2cp / 2cp+1) at the same filter tap, so the B
// fragment of every tap is a plain LDS read at lane base + constant.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int KT = 128;  // output channels per work-group
constexpr int TP = 64;   // output pixels per work-group
constexpr int CC = 8;    // input channels per LDS chunk (multiple of 4)

struct ConvGeom {
    int Nb, C, H, W, K, P;
    int Ho, Wo, HoWo;
    int tiles_per_img;
    int rows_max;  // input rows staged per tile
    int lpad;      // left pad of an LDS row so that iw = 0 lands on a 16-byte boundary
    int ldw;       // LDS row stride (floats, multiple of 4)
    int ch_ld;     // LDS channel stride (floats)
};

template <int R>
__host__ __device__ constexpr int wt_chunk_floats() {
    // per channel: R*R taps for KT output channels, taps grouped by four
    return R == 3 ? CC * (2 * KT * 4 + KT) : CC * KT;
}

// LDS weight layout for 3x3, per chunk channel c:
//   [c][g=0,1][k_out][4]  taps 4g..4g+3        (128-bit fragment reads)
//   [c][k_out]            tap 8, after the two groups
// for 1x1: [c][k_out].
// VEC: W % 4 == 0, C % CC == 0 and K % KT == 0 (aligned vector loads, no channel tails).
// WIDE: more float4 input slots per chunk than the register-staged 3 per thread.
template <int R, bool VEC, bool WIDE>
__global__ __launch_bounds__(256) void conv2d_nchw_mfma(const float* __restrict__ in, const float* __restrict__ wt,
                                                        const float* __restrict__ bias, float* __restrict__ out,
                                                        ConvGeom g, int relu) {
    constexpr int TAPS = R * R;
    constexpr int WCH = wt_chunk_floats<R>();
    extern __shared__ __align__(16) float lds[];
    const int in_chunk = CC * g.ch_ld;  // floats
    auto inS = [&](int buf) { return lds + buf * in_chunk; };
    auto wS = [&](int buf) { return lds + 2 * in_chunk + buf * WCH; };
    float* const biasS = lds + 2 * in_chunk + 2 * WCH;  // KT floats

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;

    const int tile = blockIdx.x;
    const int n = tile / g.tiles_per_img;
    const int p0 = (tile % g.tiles_per_img) * TP;
    const int k0 = blockIdx.y * KT;
    const int h_lo = p0 / g.Wo;                // first output row of the tile
    const int ih0 = h_lo - g.P;                // first staged input row

    // ---- staging: global -> registers -> LDS ---------------------------------
    // input: CC x rows_max x ldw floats as float4 slots, slot s -> (c, row, x4).
    // The slot geometry does not depend on the chunk, so it is worked out once:
    // global offset for the chunk starting at channel 0, LDS offset, chunk-local
    // channel and a 4-bit mask of the elements that lie inside the image.
    const int ldw4 = g.ldw >> 2;
    const int slots = CC * g.rows_max * ldw4;
    const int HW = g.H * g.W;
    constexpr int IN_PER_T = 3;  // slots staged through registers per thread
    float4v ireg[IN_PER_T];
    int s_goff[IN_PER_T], s_loff[IN_PER_T], s_c[IN_PER_T], s_mask[IN_PER_T];
    auto slot_geom = [&](int s, int& goff, int& loff, int& c, int& mask) {
        c = s / (g.rows_max * ldw4);
        const int rem = s - c * (g.rows_max * ldw4);
        const int row = rem / ldw4, x4 = (rem - row * ldw4) * 4;
        const int ih = ih0 + row, iw = x4 - g.P - g.lpad;
        loff = c * g.ch_ld + rem * 4;
        goff = ((n * g.C + c) * g.H + ih) * g.W + iw;
        mask = 0;
        if (ih >= 0 && ih < g.H) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (iw + j >= 0 && iw + j < g.W) mask |= 1 << j;
        }
    };
#pragma unroll
    for (int i = 0; i < IN_PER_T; ++i) {
        const int s = tid + i * 256;
        if (s < slots) slot_geom(s, s_goff[i], s_loff[i], s_c[i], s_mask[i]);
        else { s_goff[i] = 0; s_loff[i] = -1; s_c[i] = 0; s_mask[i] = 0; }
    }
    auto load_slot = [&](int goff, int c, int mask, int c0) -> float4v {
        float4v v = {0.f, 0.f, 0.f, 0.f};
        if (VEC) {  // W % 4 == 0: a slot lies entirely inside or entirely outside a row; C % CC == 0
            if (mask == 15) v = load4(in + goff + c0 * HW);
        } else if (c0 + c < g.C) {
            const float* src = in + goff + c0 * HW;
            {
                if (mask & 1) v.x = src[0];
                if (mask & 2) v.y = src[1];
                if (mask & 4) v.z = src[2];
                if (mask & 8) v.w = src[3];
            }
        }
        return v;
    };
    // weights: thread (wk = tid % 128, wpart = tid / 128) takes CC/2 channels x TAPS
    // contiguous floats of output channel k0 + wk
    constexpr int WF = (CC / 2) * TAPS;      // floats per thread
    constexpr int WV = WF % 4 == 0 ? 4 : 2;  // widest aligned vector (CC/2 even channels -> 8-byte aligned)
    float wreg[WF];
    const int wk = tid & 127, wpart = tid >> 7;
    const float* const wsrc0 = wt + ((int64_t)(k0 + wk) * g.C + wpart * (CC / 2)) * TAPS;

    auto fetch = [&](int c0) {
#pragma unroll
        for (int i = 0; i < IN_PER_T; ++i) ireg[i] = load_slot(s_goff[i], s_c[i], s_mask[i], c0);
        const float* wsrc = wsrc0 + c0 * TAPS;
        if (VEC) {  // K % KT == 0 and C % CC == 0: no tails
            if (WV == 4) {
#pragma unroll
                for (int i = 0; i < WF / 4; ++i) {
                    const float4v t = load4(wsrc + 4 * i);
                    wreg[4 * i] = t.x; wreg[4 * i + 1] = t.y; wreg[4 * i + 2] = t.z; wreg[4 * i + 3] = t.w;
                }
            } else {
#pragma unroll
                for (int i = 0; i < WF / 2; ++i) {
                    const float2v t = *reinterpret_cast<const float2v*>(wsrc + 2 * i);
                    wreg[2 * i] = t.x; wreg[2 * i + 1] = t.y;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < WF; ++i) {
                const int c = c0 + wpart * (CC / 2) + i / TAPS;
                wreg[i] = (k0 + wk < g.K && c < g.C) ? wsrc[i] : 0.f;
            }
        }
    };
    auto stash = [&](int buf, int c0) {
        float* const ib = inS(buf);
#pragma unroll
        for (int i = 0; i < IN_PER_T; ++i)
            if (s_loff[i] >= 0) *reinterpret_cast<float4v*>(ib + s_loff[i]) = ireg[i];
        // wide images: slots beyond the register-staged ones are copied directly
        if (WIDE) {
            for (int s = tid + IN_PER_T * 256; s < slots; s += 256) {
                int goff, loff, c, mask;
                slot_geom(s, goff, loff, c, mask);
                *reinterpret_cast<float4v*>(ib + loff) = load_slot(goff, c, mask, c0);
            }
        }
        float* w = wS(buf);
#pragma unroll
        for (int cc = 0; cc < CC / 2; ++cc) {
            const int c = wpart * (CC / 2) + cc;
            if (R == 3) {
                float* base = w + c * (2 * KT * 4 + KT);
                *reinterpret_cast<float4v*>(base + wk * 4) =
                    float4v{wreg[cc * 9 + 0], wreg[cc * 9 + 1], wreg[cc * 9 + 2], wreg[cc * 9 + 3]};
                *reinterpret_cast<float4v*>(base + KT * 4 + wk * 4) =
                    float4v{wreg[cc * 9 + 4], wreg[cc * 9 + 5], wreg[cc * 9 + 6], wreg[cc * 9 + 7]};
                base[2 * KT * 4 + wk] = wreg[cc * 9 + 8];
            } else {
                w[c * KT + wk] = wreg[cc];
            }
        }
    };

    // ---- per-lane fragment addresses -------------------------------------------
    const int kb0 = (wave & 1) * 64;       // this wave's 64 output channels inside the tile
    const int pb = (wave >> 1) * 32;       // this wave's 32 pixels inside the tile
    int p = p0 + pb + l32;
    const bool p_ok = p < g.HoWo;
    if (!p_ok) p = g.HoWo - 1;             // clamp: reads stay inside the staged rows, store is masked
    const int oh = p / g.Wo, ow = p - oh * g.Wo;
    // input element of tap (kh, kw), chunk channel c: c*ch_ld + (oh-h_lo+kh)*ldw + ow + kw + lpad
    const int b_base = half * g.ch_ld + (oh - h_lo) * g.ldw + ow + g.lpad;

    float16v acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; }

    auto compute = [&](int cur) {
        const float* bI = inS(cur) + b_base;
        const float* aW = wS(cur);
#pragma unroll
        for (int cp = 0; cp < CC / 2; ++cp) {
            const int c = 2 * cp + half;  // this lane half's channel
            float a[2][TAPS];
            if (R == 3) {
                const float* base = aW + c * (2 * KT * 4 + KT);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const int kk = kb0 + kb * 32 + l32;
                    const float4v lo = *reinterpret_cast<const float4v*>(base + kk * 4);
                    const float4v hi = *reinterpret_cast<const float4v*>(base + KT * 4 + kk * 4);
                    a[kb][0] = lo.x; a[kb][1] = lo.y; a[kb][2] = lo.z; a[kb][3] = lo.w;
                    a[kb][4] = hi.x; a[kb][5] = hi.y; a[kb][6] = hi.z; a[kb][7] = hi.w;
                    a[kb][8] = base[2 * KT * 4 + kk];
                }
            } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) a[kb][0] = aW[c * KT + kb0 + kb * 32 + l32];
            }
            const float* bc = bI + 2 * cp * g.ch_ld;
#pragma unroll
            for (int kh = 0; kh < R; ++kh) {
#pragma unroll
                for (int kw = 0; kw < R; ++kw) {
                    const float b = bc[kh * g.ldw + kw];
                    acc[0] = mfma_32x32x2(a[0][kh * R + kw], b, acc[0]);
                    acc[1] = mfma_32x32x2(a[1][kh * R + kw], b, acc[1]);
                }
            }
        }
    };

    if (tid < KT) biasS[tid] = (bias && k0 + tid < g.K) ? bias[k0 + tid] : 0.f;  // visible after the first barrier

    // software pipeline over channel chunks; the last chunk is peeled so the
    // loop body has no conditional loads
    const int nchunks = (g.C + CC - 1) / CC;
    fetch(0);
    stash(0, 0);
    __syncthreads();
    for (int t = 0; t + 1 < nchunks; ++t) {
        fetch((t + 1) * CC);
        __builtin_amdgcn_sched_barrier(0);  // keep the global loads ahead of the MFMAs they overlap with
        compute(t & 1);
        __builtin_amdgcn_sched_barrier(0);
        stash((t + 1) & 1, (t + 1) * CC);
        __syncthreads();
    }
    compute((nchunks - 1) & 1);

    // ---- epilogue: register r of lane holds channel 8*(r/4) + 4*half + r%4 of the block
    if (p_ok) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kl = kb0 + kb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                const int k = k0 + kl;
                if (k < g.K) {
                    float v = acc[kb][r] + biasS[kl];
                    if (relu) v = fmaxf(v, 0.f);
                    out[((int64_t)n * g.K + k) * g.HoWo + p] = v;
                }
            }
        }
    }
}

ConvGeom geom(const ConvParams& p) {
    ConvGeom g{};
    g.Nb = p.Nb; g.C = p.C; g.H = p.H; g.W = p.W; g.K = p.K; g.P = p.pad;
    g.Ho = p.H + 2 * p.pad - p.R + 1;
    g.Wo = p.W + 2 * p.pad - p.S + 1;
    g.HoWo = g.Ho * g.Wo;
    g.tiles_per_img = (g.HoWo + TP - 1) / TP;
    // a run of TP consecutive pixels touches at most (TP-1)/Wo + 2 output rows
    int out_rows = (TP - 1) / g.Wo + 2;
    if (out_rows > g.Ho) out_rows = g.Ho;
    g.rows_max = out_rows + p.R - 1;
    g.lpad = (4 - p.pad % 4) % 4;
    g.ldw = (p.W + 2 * p.pad + g.lpad + 3) & ~3;
    g.ch_ld = g.rows_max * g.ldw;
    return g;
}

size_t lds_bytes(const ConvGeom& g, int R) {
    const int w = R == 3 ? wt_chunk_floats<3>() : wt_chunk_floats<1>();
    return (size_t)(2 * CC * g.ch_ld + 2 * w + KT) * 4;
}

}  // namespace

bool conv_supported(int32_t C, int32_t H, int32_t W, int32_t K, int32_t R, int32_t S, int32_t stride_h, int32_t stride_w,
                    int32_t pad_h, int32_t pad_w, const char** why) {
    (void)C; (void)K;
    if (stride_h != 1 || stride_w != 1) { *why = "only stride 1 is supported"; return false; }
    if (R != S || (R != 1 && R != 3)) { *why = "only 1x1 and 3x3 filters are supported"; return false; }
    if (pad_h != pad_w) { *why = "padding must be the same in both directions"; return false; }
    if (pad_h > R - 1) { *why = "padding larger than the filter extent minus one"; return false; }
    ConvParams p{};
    p.C = C; p.H = H; p.W = W; p.K = K; p.R = R; p.S = S; p.pad = pad_h; p.Nb = 1;
    const ConvGeom g = geom(p);
    if (lds_bytes(g, R) > 160 * 1024) { *why = "the input rows of one 64-pixel tile do not fit in LDS (image too wide)"; return false; }
    return true;
}

LaunchShape conv_shape(const ConvParams& p) {
    const ConvGeom g = geom(p);
    LaunchShape s{};
    s.grid[0] = (uint32_t)(p.Nb * g.tiles_per_img); s.grid[1] = (uint32_t)((p.K + KT - 1) / KT); s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = (uint32_t)lds_bytes(g, p.R);
    s.kernel = p.R == 3 ? "conv2d_nchw_mfma<3x3>" : "conv2d_nchw_mfma<1x1>";
    return s;
}

template <int R, bool VEC, bool WIDE>
static hipError_t launch_conv(const ConvParams& p, const ConvGeom& g, hipStream_t stream) {
    const size_t lds = lds_bytes(g, R);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv2d_nchw_mfma<R, VEC, WIDE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)(p.Nb * g.tiles_per_img), (unsigned)((p.K + KT - 1) / KT)), block(256);
    hipLaunchKernelGGL((conv2d_nchw_mfma<R, VEC, WIDE>), grid, block, lds, stream, p.in, p.wt, p.bias, p.out, g, p.relu);
    return hipGetLastError();
}

hipError_t conv_launch(const ConvParams& p, hipStream_t stream) {
    const ConvGeom g = geom(p);
    const bool vec = (p.W % 4 == 0) && (p.C % CC == 0) && (p.K % KT == 0);
    const bool wide = CC * g.rows_max * (g.ldw / 4) > 3 * 256;
    if (p.R == 3) {
        if (vec) return wide ? launch_conv<3, true, true>(p, g, stream) : launch_conv<3, true, false>(p, g, stream);
        return wide ? launch_conv<3, false, true>(p, g, stream) : launch_conv<3, false, false>(p, g, stream);
    }
    if (vec) return wide ? launch_conv<1, true, true>(p, g, stream) : launch_conv<1, true, false>(p, g, stream);
    return wide ? launch_conv<1, false, true>(p, g, stream) : launch_conv<1, false, false>(p, g, stream);
}

}  // namespace hpct
