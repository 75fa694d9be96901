// Elementwise operators on two strided views of the same shape (Table 1 of the
// paper: Elementwise "add, mul, relu"): out = [relu](a op b), contiguous output,
// broadcasting expressed as a stride of 0.  Memory-bound; one thread per output
// vector or element, the linear output index decoded into the two input offsets.
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

template <int OP>
__device__ __forceinline__ float apply(float x, float y, int relu) {
    const float v = OP == 0 ? x + y : x * y;
    return relu ? fmaxf(v, 0.f) : v;
}

// VEC: the last dimension is contiguous in a (stride 1), contiguous or broadcast in b (stride 1 or 0),
// its extent, every other stride and the bases are multiples of 4 elements.
template <int OP, bool VEC>
__global__ __launch_bounds__(256) void eltwise_binary(EltwiseParams p) {
    constexpr int E = VEC ? 4 : 1;
    const int64_t total = p.total / E;
    const int last = p.nd - 1;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        int64_t rem = v * E, oa = 0, ob = 0;
#pragma unroll
        for (int d = kEltwiseDims - 1; d >= 0; --d) {
            if (d < p.nd) {
                const int64_t q = rem / p.shape[d];
                const int64_t i = rem - q * p.shape[d];
                oa += i * p.sa[d];
                ob += i * p.sb[d];
                rem = q;
            }
        }
        if (VEC) {
            const float4v x = load4_nt(p.a + oa);
            float4v y;
            if (p.sb[last] == 0) { const float s = p.b[ob]; y = float4v{s, s, s, s}; }
            else y = load4_nt(p.b + ob);
            store4_nt(p.out + v * 4, float4v{apply<OP>(x.x, y.x, p.relu), apply<OP>(x.y, y.y, p.relu),
                                             apply<OP>(x.z, y.z, p.relu), apply<OP>(x.w, y.w, p.relu)});
        } else {
            p.out[v] = apply<OP>(p.a[oa], p.b[ob], p.relu);
        }
    }
}

unsigned grid_for(int64_t work) {
    const int64_t g = (work + 255) / 256;
    return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

}  // namespace

LaunchShape eltwise_shape(const EltwiseParams& p) {
    LaunchShape s{};
    s.grid[0] = grid_for(p.total / (p.vec ? 4 : 1)); s.grid[1] = s.grid[2] = 1;
    s.block[0] = 256; s.block[1] = s.block[2] = 1;
    s.lds_bytes = 0;
    s.kernel = p.vec ? "eltwise_binary<vec4>" : "eltwise_binary<scalar>";
    return s;
}

hipError_t eltwise_launch(const EltwiseParams& p, hipStream_t stream) {
    const dim3 grid(grid_for(p.total / (p.vec ? 4 : 1))), block(256);
    if (p.op == 0) {
        if (p.vec) hipLaunchKernelGGL((eltwise_binary<0, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((eltwise_binary<0, false>), grid, block, 0, stream, p);
    } else {
        if (p.vec) hipLaunchKernelGGL((eltwise_binary<1, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((eltwise_binary<1, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hpct
