// LayoutTransform operators (Table 1 of the paper: "reshape, transpose"):
// out = contiguous copy of a strided view of the input.  Memory-bound; values
// are moved as 32-bit patterns, so results are bit-exact.
//
// The plan layer collapses the view to at most kLayoutDims dimensions and picks
//   * layout_transpose: some dimension b other than the last has input stride 1
//     (NCHW <-> NHWC, matrix transpose).  A work-group moves a tile (32 x 32 up to
//     128 x 128) of the (last dim a, dim b) plane through LDS: it reads along b
//     and writes along a, so both sides are coalesced; the tile's row stride is
//     odd so the transposed LDS reads spread over the banks.
//   * layout_rows: every other view (inner dimension already contiguous, a
//     strided slice, a broadcast).  One thread per output vector or element;
//     the linear output index is decoded into the input offset.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {


// ---- rows: out[lin] = in[offset(lin)]; VEC: the last dimension is contiguous in
// the input too, its extent, every other input stride and both bases are
// multiples of 4, so 4 consecutive outputs are 4 consecutive inputs.
template <bool VEC>
__global__ __launch_bounds__(256) void layout_rows(const float* __restrict__ in, float* __restrict__ out, LayoutParams p) {
    constexpr int E = VEC ? 4 : 1;
    const int64_t total = p.total / E;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        int64_t rem = v * E, off = 0;
#pragma unroll
        for (int d = kLayoutDims - 1; d >= 0; --d) {
            if (d < p.nd) {
                const int64_t q = rem / p.shape[d];
                off += (rem - q * p.shape[d]) * p.sin[d];
                rem = q;
            }
        }
        if (VEC) store4_nt(out + v * 4, load4_nt(in + off));
        else out[v] = in[off];
    }
}

// ---- transpose: dimension nd-1 (= a, output stride 1, input stride sa) against
// dimension p.bdim (= b, input stride 1, output stride sb); the other
// dimensions are batch.  One work-group per (batch, a-tile, b-tile) moves a
// TA x TB tile: 128-bit global reads along b, scalar LDS writes, scalar LDS reads
// of the transposed positions, 128-bit global writes along a.  Tiles are visited
// diagonally (b-tile index offset by the a-tile index), so work-groups that run
// together touch different columns on the read side and on the write side:
// with power-of-two row pitches a straight sweep would keep hitting the same
// memory channels.
// VEC: sa, sb, the batch strides and both bases are multiples of 4 elements.
// Work-group decode in 32-bit arithmetic from scalar arguments (tile counts and
// extents are computed on the host): the decode precedes the first load of every
// work-group, so its length is part of a short kernel's run time.
struct TransposeBatch {
    int32_t n;                         // batch dimensions, innermost first
    uint32_t shape[kLayoutDims - 2];
    int64_t sin[kLayoutDims - 2];
    int64_t sout[kLayoutDims - 2];
};

template <int TA, int TB, bool VEC>
__global__ __launch_bounds__(256) void layout_transpose(const float* __restrict__ in, float* __restrict__ out, uint32_t La, uint32_t Lb,
                                                        uint32_t ta, uint32_t tb, int64_t sa, int64_t sb, TransposeBatch bt) {
    __shared__ float tile[TA][TB + 1];
    uint32_t w = blockIdx.x;
    const uint32_t x = w % tb; w /= tb;
    const uint32_t y = w % ta; w /= ta;
    const uint32_t b0 = ((x + y) % tb) * TB, a0 = y * TA;
    int64_t in_off = 0, out_off = 0;
#pragma unroll
    for (int d = 0; d < kLayoutDims - 2; ++d) {
        if (d < bt.n) {
            const uint32_t q = w / bt.shape[d];
            const uint32_t i = w - q * bt.shape[d];
            in_off += i * bt.sin[d];
            out_off += i * bt.sout[d];
            w = q;
        }
    }
    constexpr int RPP1 = 256 / (TB / 4);  // a-rows per read pass
    constexpr int RPP2 = 256 / (TA / 4);  // b-rows per write pass
    const int r1 = threadIdx.x / (TB / 4), c1 = (threadIdx.x % (TB / 4)) * 4;
    const int r2 = threadIdx.x / (TA / 4), c2 = (threadIdx.x % (TA / 4)) * 4;
    if (VEC && a0 + TA <= La && b0 + TB <= Lb) {
        // interior tile (uniform per work-group): no bounds tests, so every load of the tile is issued at once
        const float* src = in + in_off + (int64_t)(a0 + r1) * sa + b0 + c1;
        float4v v[TA / RPP1];
#pragma unroll
        for (int i = 0; i < TA / RPP1; ++i) v[i] = load4_nt(src + (int64_t)(RPP1 * i) * sa);
#pragma unroll
        for (int i = 0; i < TA / RPP1; ++i) {
            const int ar = r1 + RPP1 * i;
            tile[ar][c1] = v[i].x; tile[ar][c1 + 1] = v[i].y; tile[ar][c1 + 2] = v[i].z; tile[ar][c1 + 3] = v[i].w;
        }
        __syncthreads();
        float* dst = out + out_off + (int64_t)(b0 + r2) * sb + a0 + c2;
#pragma unroll
        for (int i = 0; i < TB / RPP2; ++i) {
            const int br = r2 + RPP2 * i;
            store4_nt(dst + (int64_t)(RPP2 * i) * sb, float4v{tile[c2][br], tile[c2 + 1][br], tile[c2 + 2][br], tile[c2 + 3][br]});
        }
        return;
    }
    // edge tile or unaligned view: element loads from clamped coordinates, without
    // branches, so they are all in flight together (a load behind a bounds branch
    // would expose one memory latency per pass); positions outside the view hold
    // copies of edge elements and are never written out
    {
        float v[TA / RPP1][4];
#pragma unroll
        for (int i = 0; i < TA / RPP1; ++i) {
            const uint32_t a = a0 + r1 + RPP1 * i;
            const float* row = in + in_off + (int64_t)(a < La ? a : La - 1) * sa;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t b = b0 + c1 + j;
                v[i][j] = row[b < Lb ? b : Lb - 1];
            }
        }
#pragma unroll
        for (int i = 0; i < TA / RPP1; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) tile[r1 + RPP1 * i][c1 + j] = v[i][j];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TB / RPP2; ++i) {  // write rows of b, contiguous along a
        const int br = r2 + RPP2 * i;
        const uint32_t b = b0 + br, a = a0 + c2;
        if (b < Lb) {
            float* dst = out + out_off + (int64_t)b * sb + a;
            if (VEC && a + 3 < La) {
                store4_nt(dst, float4v{tile[c2][br], tile[c2 + 1][br], tile[c2 + 2][br], tile[c2 + 3][br]});
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (a + j < La) dst[j] = tile[c2 + j][br];
            }
        }
    }
}

// tile edges by problem size: the wide edges (longer contiguous runs) only
// where they divide the extent, because an edge tile takes the slower
// element-wise path and a short kernel waits for its slowest work-group;
// otherwise 32 x 32 tiles (128-byte runs, one load per thread), which measured
// 4 % faster than 64 x 64 on the [32,64,56,56] NCHW <-> NHWC pair
void pick_tile(const LayoutParams& p, int& TA, int& TB) {
    const int64_t La = p.shape[p.nd - 1], Lb = p.shape[p.bdim];
    TB = Lb % 128 == 0 ? 128 : 32;
    TA = TB == 32 ? 32 : (La % 128 == 0 ? 128 : 64);
}

template <int TA, int TB>
void launch_transpose(const LayoutParams& p, dim3 grid, bool vec, hipStream_t stream) {
    const int a_dim = p.nd - 1, b_dim = p.bdim;
    const uint32_t La = (uint32_t)p.shape[a_dim], Lb = (uint32_t)p.shape[b_dim];
    const uint32_t ta = (La + TA - 1) / TA, tb = (Lb + TB - 1) / TB;
    TransposeBatch bt{};
    for (int d = p.nd - 1; d >= 0; --d) {
        if (d == a_dim || d == b_dim) continue;
        bt.shape[bt.n] = (uint32_t)p.shape[d];
        bt.sin[bt.n] = p.sin[d];
        bt.sout[bt.n] = p.sout[d];
        ++bt.n;
    }
    if (vec) hipLaunchKernelGGL((layout_transpose<TA, TB, true>), grid, dim3(256), 0, stream, p.in, p.out, La, Lb, ta, tb, p.sin[a_dim], p.sout[b_dim], bt);
    else hipLaunchKernelGGL((layout_transpose<TA, TB, false>), grid, dim3(256), 0, stream, p.in, p.out, La, Lb, ta, tb, p.sin[a_dim], p.sout[b_dim], bt);
}

}  // namespace

LaunchShape layout_shape(const LayoutParams& p) {
    LaunchShape s{};
    s.grid[1] = s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    if (p.kind == 2) {
        int TA, TB;
        pick_tile(p, TA, TB);
        const int64_t ta = (p.shape[p.nd - 1] + TA - 1) / TA, tb = (p.shape[p.bdim] + TB - 1) / TB;
        int64_t batch = 1;
        for (int d = 0; d < p.nd - 1; ++d)
            if (d != p.bdim) batch *= p.shape[d];
        s.grid[0] = (uint32_t)(batch * ta * tb);
        s.lds_bytes = (uint32_t)(TA * (TB + 1) * 4);
        s.kernel = TA == 128 ? "layout_transpose<128x128>" : (TB == 128 ? "layout_transpose<64x128>" : "layout_transpose<32x32>");
    } else {
        const int64_t units = p.total / (p.kind == 1 ? 4 : 1);
        int64_t blocks = (units + 255) / 256;
        if (blocks > 256 * 64) blocks = 256 * 64;  // grid-stride beyond 64 groups per CU
        s.grid[0] = (uint32_t)(blocks < 1 ? 1 : blocks);
        s.lds_bytes = 0;
        s.kernel = p.kind == 1 ? "layout_rows<vec4>" : "layout_rows<scalar>";
    }
    return s;
}

hipError_t layout_launch(const LayoutParams& p, hipStream_t stream) {
    const LaunchShape s = layout_shape(p);
    dim3 grid(s.grid[0]), block(256);
    if (p.kind == 2) {
        bool vec = ((((uintptr_t)p.in | (uintptr_t)p.out) & 15) == 0) && p.sout[p.bdim] % 4 == 0;
        for (int d = 0; d < p.nd; ++d)
            if (d != p.bdim) vec = vec && p.sin[d] % 4 == 0 && (d == p.nd - 1 || p.sout[d] % 4 == 0);
        int TA, TB;
        pick_tile(p, TA, TB);
        // the kernel decodes its work-group index and tile coordinates in 32 bits
        int64_t groups = 1;
        for (int d = 0; d < p.nd; ++d) {
            if (p.shape[d] > (int64_t)INT32_MAX - 128) return hipErrorInvalidValue;
            groups *= d == p.nd - 1 ? (p.shape[d] + TA - 1) / TA : d == p.bdim ? (p.shape[d] + TB - 1) / TB : p.shape[d];
            if (groups > INT32_MAX) return hipErrorInvalidValue;
        }
        if (TA == 128) launch_transpose<128, 128>(p, grid, vec, stream);
        else if (TB == 128) launch_transpose<64, 128>(p, grid, vec, stream);
        else launch_transpose<32, 32>(p, grid, vec, stream);
    }
    else if (p.kind == 1) hipLaunchKernelGGL(layout_rows<true>, grid, block, 0, stream, p.in, p.out, p);
    else hipLaunchKernelGGL(layout_rows<false>, grid, block, 0, stream, p.in, p.out, p);
    return hipGetLastError();
}

}  // namespace hpct
