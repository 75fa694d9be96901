// Device primitives for gfx950 (CDNA4, wave64): cross-lane reductions on DPP,
// a fixed-order cross-wave combine through LDS, 128-bit global access, fast
// transcendental wrappers and the fp32 MFMA intrinsics.
#pragma once
#include <hip/hip_runtime.h>

namespace hpct {

typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- DPP lane movement -----------------------------------------------------
// dpp_ctrl encodings: quad_perm = 8-bit selector, row_mirror = 0x140,
// row_half_mirror = 0x141.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ float readlane_f(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };

// Reduction over the 64 lanes of a wave.  Four DPP steps leave every lane of a
// 16-lane row with that row's result; the four rows are then read into scalar
// registers and combined in a fixed order, so the result is wave-uniform and
// bit-identical from run to run.
template <class Op>
__device__ __forceinline__ float wave_reduce(float v) {
    Op op;
    v = op(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
    v = op(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
    v = op(v, dpp_mov<0x141>(v));  // row_half_mirror
    v = op(v, dpp_mov<0x140>(v));  // row_mirror
    float r0 = readlane_f(v, 0), r1 = readlane_f(v, 16), r2 = readlane_f(v, 32), r3 = readlane_f(v, 48);
    return op(op(r0, r1), op(r2, r3));
}

// Reduction over a work-group of NWAVES waves.  `slots` is LDS with room for
// NWAVES floats; the call contains one barrier before the read and one after,
// so the same slots can be reused by the next call.
template <class Op, int NWAVES>
__device__ __forceinline__ float block_reduce(float v, float* slots) {
    Op op;
    float w = wave_reduce<Op>(v);
    if constexpr (NWAVES == 1) return w;
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) slots[wave] = w;
    __syncthreads();
    float r = slots[0];
#pragma unroll
    for (int i = 1; i < NWAVES; ++i) r = op(r, slots[i]);
    __syncthreads();
    return r;
}

// ---- 128-bit global access ---------------------------------------------------
__device__ __forceinline__ float4v load4(const float* p) { return *reinterpret_cast<const float4v*>(p); }
__device__ __forceinline__ void store4(float* p, float4v v) { *reinterpret_cast<float4v*>(p) = v; }
// Streaming store: the data is not read again by this kernel.
__device__ __forceinline__ void store4_nt(float* p, float4v v) {
    __builtin_nontemporal_store(v, reinterpret_cast<float4v*>(p));
}
__device__ __forceinline__ float4v load4_nt(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const float4v*>(p));
}

// ---- fast transcendentals (hardware v_exp_f32 / v_rcp_f32 / v_rsq_f32) -------
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_rsq(float x) { return __builtin_amdgcn_rsqf(x); }
constexpr float kLog2e = 1.4426950408889634f;

// tanh-form GELU written as y * sigmoid(2u), u = sqrt(2/pi) (y + 0.044715 y^3):
// 0.5 (1 + tanh u) = 1 / (1 + exp(-2u)).  No cancellation; one exp2, one rcp.
__device__ __forceinline__ float gelu_tanh(float y) {
    const float c0 = -2.0f * 0.7978845608028654f * kLog2e;
    const float c1 = c0 * 0.044715f;
    float t = y * (c0 + c1 * y * y);  // = -2u * log2(e)
    return y * fast_rcp(1.0f + fast_exp2(t));
}

// The activation at the end of a contraction kernel's epilogue (GemmParams::relu): 0 none, 1 ReLU, 2 ReLU6,
// 3 tanh-form GELU, 4 logistic, 5 tanh - the same formulas as the elementwise kernels.  The code is uniform.
__device__ __forceinline__ float activate(float v, int act) {
    switch (act) {
        case 0: return v;
        case 1: return fmaxf(v, 0.f);
        case 2: return fminf(fmaxf(v, 0.f), 6.f);
        case 3: return gelu_tanh(v);
        case 4: return 1.f / (1.f + expf(-v));
        default: return tanhf(v);
    }
}

// ---- hash dropout (Section 5.3 case study of the paper) -------------------------
// rand as the integer u = h % 1000 for h = offset + seed:
// h ^= h >> 17; h ^= h << 31; h ^= h >> 8, all in 64 bits.
__device__ __forceinline__ uint32_t dropout_u(uint64_t h) {
    h ^= h >> 17;
    h ^= h << 31;
    h ^= h >> 8;
    // h % 1000 from 32-bit pieces: 2^32 = 296 (mod 1000), so h = hi * 2^32 + lo is congruent to
    // (hi % 1000) * 296 + lo % 1000, which is below 2^32; three 32-bit remainders by a constant
    // instead of a 64-bit division
    const uint32_t hi = (uint32_t)(h >> 32), lo = (uint32_t)h;
    return ((hi % 1000u) * 296u + lo % 1000u) % 1000u;
}

// ---- fp32 MFMA ----------------------------------------------------------------
// D(32x32) += A(32x2) B(2x32).  Lane l supplies A[l%32][l/32] and B[l/32][l%32];
// register r of lane l holds D[8*(r/4) + 4*(l/32) + r%4][l%32].
__device__ __forceinline__ float16v mfma_32x32x2(float a, float b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
// D(16x16) += A(16x4) B(4x16).  Lane l supplies A[l%16][l/16] and B[l/16][l%16];
// register r of lane l holds D[4*(l/16) + r][l%16].
__device__ __forceinline__ float4v mfma_16x16x4(float a, float b, float4v c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

}  // namespace hpct
