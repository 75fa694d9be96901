// Transposed convolution ("Conv-Trans", a Level-2 operator named in Section 5.2 of
// the paper) through the conv kernels: scattering in[n][c][ih][iw] through
// wt[c][k][kh][kw] to out[ih*s - P + kh*d][iw*s - P + kw*d] is the stride-1
// cross-correlation of the zero-dilated input (s - 1 zeros between neighbours) with
// the filter flipped in both directions and its channel axes swapped, at padding
// (R - 1) d - P.  This file prepares those two operands in the caller's workspace:
//     wt2[k][c][kh][kw] = wt[c][k][R-1-kh][S-1-kw]
//     xd[n][c][hd][wd]  = in[n][c][hd/s][wd/s] if s divides hd and wd, else 0   (s > 1 only)
// one grid-stride kernel for both; the conv kernel then runs on them unchanged.
// At stride s the conv multiplies s^2 - 1 zeros for every input element; a
// decomposition into s^2 smaller convolutions would avoid that.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

__global__ __launch_bounds__(256) void convt_prep(const float* __restrict__ in, const float* __restrict__ wt,
                                                  float* __restrict__ xd, float* __restrict__ wt2, ConvTParams p) {
    const int64_t n_w = (int64_t)p.K * p.C * p.R * p.R;
    const int64_t n_x = p.stride > 1 ? (int64_t)p.Nb * p.C * p.Hd * p.Wd : 0;
    const int taps = p.R * p.R;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_w + n_x; i += (int64_t)gridDim.x * 256) {
        if (i < n_w) {
            const int tap = (int)(i % taps);
            const int64_t kc = i / taps;
            const int c = (int)(kc % p.C), k = (int)(kc / p.C);
            wt2[i] = wt[((int64_t)c * p.K + k) * taps + (taps - 1 - tap)];   // both flips = reversing the R*S taps
        } else {
            const int64_t j = i - n_w;
            const int wd = (int)(j % p.Wd);
            const int64_t r = j / p.Wd;
            const int hd = (int)(r % p.Hd);
            const int64_t plane = r / p.Hd;
            float v = 0.f;
            if (hd % p.stride == 0 && wd % p.stride == 0)
                v = in[(plane * p.H + hd / p.stride) * p.W + wd / p.stride];
            xd[j] = v;
        }
    }
}

}  // namespace

size_t convt_weights_bytes(const ConvTParams& p) { return (((size_t)p.K * p.C * p.R * p.R * 4) + 255) & ~(size_t)255; }

size_t convt_workspace_bytes(const ConvTParams& p) {
    return convt_weights_bytes(p) + (p.stride > 1 ? (size_t)p.Nb * p.C * p.Hd * p.Wd * 4 : 0);
}

hipError_t convt_prep_launch(const ConvTParams& p, const float* in, const float* wt, float* workspace, hipStream_t stream) {
    float* wt2 = workspace;
    float* xd = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + convt_weights_bytes(p));
    const int64_t work = (int64_t)p.K * p.C * p.R * p.R + (p.stride > 1 ? (int64_t)p.Nb * p.C * p.Hd * p.Wd : 0);
    int64_t grid = (work + 255) / 256;
    if (grid > 16384) grid = 16384;
    hipLaunchKernelGGL(convt_prep, dim3((unsigned)grid), dim3(256), 0, stream, in, wt, xd, wt2, p);
    return hipGetLastError();
}

}  // namespace hpct
