// Reduction operators over one axis of a strided view (Table 1 of the paper:
// Reduction "sum, mean", and the arg-reductions): sum, mean, argmax, argmin.
// Memory-bound: every input element is read once.  The plan layer removes the
// reduced axis (extent R, input stride sR), collapses the kept dimensions and
// picks one of three kernels by where the contiguous direction of the input lies:
//
//   reduce_rows   sR == 1: the reduced axis is contiguous.  A wave (or, for few
//                 and long rows, a work-group) owns one output; its lanes stride
//                 over the row with 128-bit loads and combine with DPP.
//   reduce_cols   the innermost kept dimension is contiguous in the input: threads
//                 lie along it (coalesced loads and stores), the 256 threads of a
//                 work-group are TC column threads x TR row groups, each row group
//                 walks every TR-th element of the reduced axis, and the groups'
//                 partial results are combined through LDS in group order.
//   reduce_gather anything else: a thread per output walks the reduced axis.
//
// All combinations run in a fixed order, so results are bit-identical from run
// to run.  Arg-reductions compare fp32 values exactly and resolve ties towards
// the lowest index, whatever the order partial results are combined in.
#include <type_traits>
#include "kernels.hpp"
#include "prim.hpp"

namespace hpct {
namespace {

constexpr int kThreads = 256;

// Running result of a reduction: a sum, or the best value with its index.
template <int OP> struct Acc;
template <> struct Acc<0> {  // sum / mean
    float s = 0.f;
    __device__ __forceinline__ void take(float x, int) { s += x; }
    __device__ __forceinline__ void merge(const Acc& o) { s += o.s; }
};
template <bool MAX> struct ArgAcc {
    float v = MAX ? -INFINITY : INFINITY;
    int i = 0x7fffffff;
    // elements arrive in increasing index order: a strict comparison keeps the first of equals
    __device__ __forceinline__ void take(float x, int idx) {
        if (MAX ? x > v : x < v) { v = x; i = idx; }
        else if (i == 0x7fffffff) { v = x; i = idx; }   // first element (also when it is +-inf)
    }
    __device__ __forceinline__ void merge(const ArgAcc& o) {
        const bool better = MAX ? o.v > v : o.v < v;
        if (better || (o.v == v && o.i < i)) { v = o.v; i = o.i; }
    }
};
template <> struct Acc<2> : ArgAcc<true> {};
template <> struct Acc<3> : ArgAcc<false> {};

template <int CTRL, int OP>
__device__ __forceinline__ Acc<OP> dpp_acc(const Acc<OP>& a) {
    Acc<OP> o;
    if constexpr (OP == 0) {
        o.s = dpp_mov<CTRL>(a.s);
    } else {
        o.v = dpp_mov<CTRL>(a.v);
        o.i = __builtin_bit_cast(int, dpp_mov<CTRL>(__builtin_bit_cast(float, a.i)));
    }
    return o;
}

template <int OP>
__device__ __forceinline__ Acc<OP> lane_acc(const Acc<OP>& a, int lane) {
    Acc<OP> o;
    if constexpr (OP == 0) {
        o.s = readlane_f(a.s, lane);
    } else {
        o.v = readlane_f(a.v, lane);
        o.i = __builtin_amdgcn_readlane(a.i, lane);
    }
    return o;
}

// all 64 lanes -> wave-uniform result, fixed order
template <int OP>
__device__ __forceinline__ Acc<OP> wave_combine(Acc<OP> a) {
    a.merge(dpp_acc<0xB1, OP>(a));
    a.merge(dpp_acc<0x4E, OP>(a));
    a.merge(dpp_acc<0x141, OP>(a));
    a.merge(dpp_acc<0x140, OP>(a));
    Acc<OP> r = lane_acc<OP>(a, 0);
    r.merge(lane_acc<OP>(a, 16));
    r.merge(lane_acc<OP>(a, 32));
    r.merge(lane_acc<OP>(a, 48));
    return r;
}

template <int OP>
__device__ __forceinline__ void emit(const ReduceParams& p, int64_t o, const Acc<OP>& a) {
    if constexpr (OP == 0) {
        reinterpret_cast<float*>(p.out)[o] = p.mean ? a.s / (float)p.R : a.s;
    } else if (p.value) {
        reinterpret_cast<float*>(p.out)[o] = a.v;
    } else {
        reinterpret_cast<int32_t*>(p.out)[o] = a.i;
    }
}

// input offset of output element o (row-major over the kept dimensions)
__device__ __forceinline__ int64_t kept_offset(const ReduceParams& p, int64_t o) {
    int64_t off = 0;
#pragma unroll
    for (int d = kReduceDims - 1; d >= 0; --d) {
        if (d < p.nk) {
            const int64_t q = o / p.shape[d];
            off += (o - q * p.shape[d]) * p.stride[d];
            o = q;
        }
    }
    return off;
}

// ---- reduced axis contiguous.  WPO = waves per output: 1 (a wave per output) or
// 4 (a work-group per output).  VEC: R, every kept stride and the base are multiples of 4.
template <int OP, bool VEC, int WPO>
__global__ __launch_bounds__(kThreads) void reduce_rows(ReduceParams p) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t o = WPO == 1 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    const bool live = o < p.outputs;   // wave-uniform
    Acc<OP> a;
    if (live) {
        const float* row = p.in + kept_offset(p, o);
        const int R = p.R;
        constexpr int E = VEC ? 4 : 1;
        const int step = 64 * E * WPO;
        int i = (wave * (WPO == 1 ? 0 : 64) + lane) * E;
        if (VEC) {   // four, then two independent 128-bit loads in flight per lane
            auto batch = [&](auto tag) {
                constexpr int U = decltype(tag)::value;
                for (; i + (U - 1) * step < R; i += U * step) {
                    float4v x[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) x[u] = load4_nt(row + i + u * step);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int j = i + u * step;
                        a.take(x[u].x, j); a.take(x[u].y, j + 1); a.take(x[u].z, j + 2); a.take(x[u].w, j + 3);
                    }
                }
            };
            batch(std::integral_constant<int, 4>{});
            batch(std::integral_constant<int, 2>{});
        }
        for (; i < R; i += step) {
            if (VEC) {
                const float4v x = load4_nt(row + i);
                a.take(x.x, i); a.take(x.y, i + 1); a.take(x.z, i + 2); a.take(x.w, i + 3);
            } else {
                a.take(row[(int64_t)i * p.sR], i);
            }
        }
        a = wave_combine<OP>(a);
    }
    if (WPO == 1) {
        if (live && lane == 0) emit<OP>(p, o, a);
    } else {
        if (lane == 0) {
            if constexpr (OP == 0) sv[wave] = a.s; else { sv[wave] = a.v; si[wave] = a.i; }
        }
        __syncthreads();
        if (threadIdx.x == 0 && live) {
            Acc<OP> r;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                Acc<OP> t;
                if constexpr (OP == 0) t.s = sv[w]; else { t.v = sv[w]; t.i = si[w]; }
                if (w == 0) r = t; else r.merge(t);
            }
            emit<OP>(p, o, r);
        }
    }
}

// ---- innermost kept dimension contiguous (extent Lc): TC column threads x TR row
// groups, V columns per thread.  blockIdx.x = (strip of TC*V columns, index over the
// other kept dimensions, chunk of the reduced axis).  With p.split > 1 the reduced
// axis is cut into p.split chunks handled by different work-groups (few outputs
// cannot fill the chip otherwise); each writes its partial result to the workspace
// and reduce_finish merges the chunks in order.
constexpr int kColsUnroll = 8;  // elements of the reduced axis in flight per thread

template <int OP, int V>
__global__ __launch_bounds__(kThreads) void reduce_cols(ReduceParams p, int tc_log2, int strips) {
    __shared__ float sv[kThreads * V];
    __shared__ int si[OP == 0 ? 1 : kThreads * V];
    const int TC = 1 << tc_log2, TR = kThreads >> tc_log2;
    const int ct = threadIdx.x & (TC - 1), rg = threadIdx.x >> tc_log2;
    // every extent and the grid fit 32 bits (the plan refuses more than 2^31-1 outputs): 32-bit divisions, a few
    // instructions each where the 64-bit ones are a routine of their own in front of the first load
    const unsigned Lc = (unsigned)p.shape[p.nk - 1];
    unsigned b = blockIdx.x;
    // work-groups are dealt to the 8 XCDs in turn; with the plain numbering an XCD sees every 8th strip only, i.e.
    // always the same few of its L2 channels.  Renumbered so that an XCD walks neighbouring strips (8192 x 4096 over
    // axis 0 on 256-column strips: 30.2 -> 24.2 us)
    if ((gridDim.x & 7) == 0) b = (b & 7) * (gridDim.x >> 3) + (b >> 3);
    const unsigned strip = b % (unsigned)strips; b /= (unsigned)strips;
    const int chunk_id = (int)(b % (unsigned)p.split);
    const unsigned rest0 = b / (unsigned)p.split;
    const int64_t c = (int64_t)(strip * TC + ct) * V;
    // offset of the other kept dimensions
    unsigned rest = rest0;
    int64_t off = 0;
#pragma unroll
    for (int d = kReduceDims - 2; d >= 0; --d) {
        if (d < p.nk - 1) {
            const unsigned ext = (unsigned)p.shape[d];
            const unsigned q = rest / ext;
            off += (int64_t)(rest - q * ext) * p.stride[d];
            rest = q;
        }
    }
    // this work-group's piece of the reduced axis
    const int chunk = (p.R + p.split - 1) / p.split;
    const int r_lo = chunk_id * chunk;
    const int r_hi = r_lo + chunk < p.R ? r_lo + chunk : p.R;
    Acc<OP> a[V];
    if (c < Lc) {
        const float* src = p.in + off + c;
        const int64_t sR = p.sR;
        constexpr int U = kColsUnroll;
        int r = r_lo + rg;
        for (; r + (U - 1) * TR < r_hi; r += U * TR) {   // U loads in flight
            float x[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float* q = src + (int64_t)(r + u * TR) * sR;
                if constexpr (V == 4) {
                    const float4v t = load4_nt(q);
                    x[u][0] = t.x; x[u][1] = t.y; x[u][2] = t.z; x[u][3] = t.w;
                } else {
                    x[u][0] = __builtin_nontemporal_load(q);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < V; ++v) a[v].take(x[u][v], r + u * TR);
        }
        if (r < r_hi) {   // last, partial pass: rows past the end re-read the first row of the piece and are not taken
            float x[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int rr = r + u * TR;
                const float* q = src + (int64_t)(rr < r_hi ? rr : r_lo) * sR;
                if constexpr (V == 4) {
                    const float4v t = load4_nt(q);
                    x[u][0] = t.x; x[u][1] = t.y; x[u][2] = t.z; x[u][3] = t.w;
                } else {
                    x[u][0] = __builtin_nontemporal_load(q);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int rr = r + u * TR;
                if (rr < r_hi) {
#pragma unroll
                    for (int v = 0; v < V; ++v) a[v].take(x[u][v], rr);
                }
            }
        }
    }
    // row groups 1.. publish, group 0 merges them in order
    if (rg > 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int slot = (rg * TC + ct) * V + v;
            if constexpr (OP == 0) sv[slot] = a[v].s; else { sv[slot] = a[v].v; si[slot] = a[v].i; }
        }
    }
    __syncthreads();
    if (rg == 0 && c < Lc) {
        for (int g = 1; g < TR; ++g) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int slot = (g * TC + ct) * V + v;
                Acc<OP> t;
                if constexpr (OP == 0) t.s = sv[slot]; else { t.v = sv[slot]; t.i = si[slot]; }
                a[v].merge(t);
            }
        }
        const int64_t o = (int64_t)rest0 * Lc + c;
        if (p.split == 1) {
#pragma unroll
            for (int v = 0; v < V; ++v) emit<OP>(p, o + v, a[v]);
        } else {
            float* wv = p.ws + (int64_t)chunk_id * p.outputs + o;
            int* wi = reinterpret_cast<int*>(p.ws + (int64_t)p.split * p.outputs) + (int64_t)chunk_id * p.outputs + o;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                if constexpr (OP == 0) wv[v] = a[v].s; else { wv[v] = a[v].v; wi[v] = a[v].i; }
            }
        }
    }
}

// merges the p.split <= 64 partial results of every output: 16 lanes per output, lane l takes the pieces l, l + 16,
// l + 32, l + 48 (all its loads in flight together - a thread that walks the pieces one after the other waits a
// memory round trip for each: 0.4 us per piece), then the 16 lanes combine on DPP in a fixed order
template <int OP>
__global__ __launch_bounds__(kThreads) void reduce_finish(ReduceParams p) {
    const int64_t o = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 4;
    const int l = threadIdx.x & 15;
    const bool live = o < p.outputs;
    const int64_t oc = live ? o : 0;
    const float* wv = p.ws + oc;
    const int* wi = reinterpret_cast<const int*>(p.ws + (int64_t)p.split * p.outputs) + oc;
    float xv[4];
    int xi[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int s = l + 16 * u;
        const int64_t at = (int64_t)(s < p.split ? s : 0) * p.outputs;
        xv[u] = wv[at];
        if constexpr (OP != 0) xi[u] = wi[at];
    }
    Acc<OP> a;   // the identity: 0 for a sum, (-+inf, no index) for the arg ops
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (l + 16 * u < p.split) {
            Acc<OP> t;
            if constexpr (OP == 0) t.s = xv[u]; else { t.v = xv[u]; t.i = xi[u]; }
            a.merge(t);
        }
    }
    a.merge(dpp_acc<0xB1, OP>(a));
    a.merge(dpp_acc<0x4E, OP>(a));
    a.merge(dpp_acc<0x141, OP>(a));
    a.merge(dpp_acc<0x140, OP>(a));
    if (live && l == 0) emit<OP>(p, o, a);
}

// ---- no contiguous direction to exploit: a thread per output
template <int OP>
__global__ __launch_bounds__(kThreads) void reduce_gather(ReduceParams p) {
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o >= p.outputs) return;
    const float* src = p.in + kept_offset(p, o);
    Acc<OP> a;
    for (int r = 0; r < p.R; ++r) a.take(src[(int64_t)r * p.sR], r);
    emit<OP>(p, o, a);
}

// strides that allow 128-bit access along the contiguous kept dimension (pointers are checked at launch)
bool cols_vec_ok(const ReduceParams& p) {
    if (p.shape[p.nk - 1] % 4 || p.sR % 4) return false;
    for (int d = 0; d + 1 < p.nk; ++d)
        if (p.stride[d] % 4 && p.shape[d] > 1) return false;
    return true;
}

bool aligned4(const ReduceParams& p) {
    for (int d = 0; d < p.nk; ++d)
        if (p.stride[d] % 4 && p.shape[d] > 1) return false;
    return true;
}

template <int OP>
hipError_t launch_op(const ReduceParams& p, hipStream_t stream) {
    const bool base_ok = ((uintptr_t)p.in & 15) == 0;
    if (p.kind == 0) {
        const bool vec = base_ok && p.sR == 1 && p.R % 4 == 0 && aligned4(p);
        const bool wide = reduce_rows_per_group(p);
        const unsigned grid = wide ? (unsigned)p.outputs : (unsigned)((p.outputs + 3) / 4);
        if (wide) {
            if (vec) hipLaunchKernelGGL((reduce_rows<OP, true, 4>), dim3(grid), dim3(kThreads), 0, stream, p);
            else hipLaunchKernelGGL((reduce_rows<OP, false, 4>), dim3(grid), dim3(kThreads), 0, stream, p);
        } else {
            if (vec) hipLaunchKernelGGL((reduce_rows<OP, true, 1>), dim3(grid), dim3(kThreads), 0, stream, p);
            else hipLaunchKernelGGL((reduce_rows<OP, false, 1>), dim3(grid), dim3(kThreads), 0, stream, p);
        }
    } else if (p.kind == 1) {
        const int64_t Lc = p.shape[p.nk - 1];
        // the plan chose the strip for 128-bit access; misaligned pointers keep the strip with scalar access
        int v = p.cols_v, tc_log2 = p.cols_tc_log2;
        if (v == 4 && !(base_ok && (((uintptr_t)p.out | (uintptr_t)p.ws) & 15) == 0)) { v = 1; tc_log2 += 2; }
        const int64_t strip = (int64_t)v << tc_log2;
        const int strips = (int)((Lc + strip - 1) / strip);
        dim3 grid((unsigned)(strips * (p.outputs / Lc) * p.split));
        if (v == 4) hipLaunchKernelGGL((reduce_cols<OP, 4>), grid, dim3(kThreads), 0, stream, p, tc_log2, strips);
        else hipLaunchKernelGGL((reduce_cols<OP, 1>), grid, dim3(kThreads), 0, stream, p, tc_log2, strips);
        if (p.split > 1) {
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((reduce_finish<OP>), dim3((unsigned)((p.outputs * 16 + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, p);
        }
    } else {
        hipLaunchKernelGGL((reduce_gather<OP>), dim3((unsigned)((p.outputs + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace

// Column kernel configuration.  Candidates in order of preference: wide strips first (a wave load
// is one contiguous run, few row groups to merge), 128-bit access before 32-bit at equal width; the
// first that gives about four work-groups per CU wins.  When none does (few outputs) the reduced
// axis is split over work-groups instead, to about one work-group per CU: measured on 8192 x 4096
// over axis 0 (with the XCD-aware numbering of the kernel), 256-column strips x 16 pieces 24.2 us,
// 64-column strips x 4 pieces 24.9, 512 or 1024 smaller work-groups 24.7 - 25.3.
void reduce_plan_cols(ReduceParams& p) {
    const int64_t Lc = p.shape[p.nk - 1];
    const int64_t rest = p.outputs / Lc;
    const bool vec = cols_vec_ok(p);
    p.split = 1;
    struct Cand { int v, tc; };
    const Cand cands[] = {{4, 6}, {4, 5}, {1, 6}, {4, 4}};
    for (const Cand& c : cands) {
        if (c.v == 4 && !vec) continue;
        const int64_t strip = (int64_t)c.v << c.tc;
        p.cols_v = c.v; p.cols_tc_log2 = c.tc;
        if (rest * ((Lc + strip - 1) / strip) >= 1024) return;
    }
    // few outputs: pieces of the reduced axis on strips of up to 256 columns (a wave load is then one 1 KB run of a row)
    p.cols_v = vec ? 4 : 1;
    p.cols_tc_log2 = vec ? (Lc >= 256 ? 6 : (Lc >= 128 ? 5 : 4)) : 6;
    const int64_t strip = (int64_t)p.cols_v << p.cols_tc_log2;
    const int64_t groups = rest * ((Lc + strip - 1) / strip);
    const int tr = kThreads >> p.cols_tc_log2;
    int64_t split = (256 + groups - 1) / groups;
    const int64_t most = p.R / (2 * tr * kColsUnroll);   // at least two full unrolled passes per thread
    if (split > most) split = most;
    if (split > 64) split = 64;
    p.split = split < 1 ? 1 : (int32_t)split;
}

size_t reduce_workspace_bytes(const ReduceParams& p) {
    return p.split > 1 ? (size_t)p.split * (size_t)p.outputs * 4 * (p.op >= 2 ? 2 : 1) : 0;
}

// A work-group per output when there are too few outputs for a wave each to fill the chip, and for
// rows of 4096 elements or more: a wave then owns at least 1024 of them, i.e. one pass of four
// loads per lane, and four times as many waves stream at once (8192 x 4096: 21.3 -> 19.8 us).
bool reduce_rows_per_group(const ReduceParams& p) { return p.R >= 4096 || (p.outputs < 2048 && p.R >= 2048); }

LaunchShape reduce_shape(const ReduceParams& p) {
    LaunchShape s{};
    s.block[0] = kThreads; s.block[1] = s.block[2] = 1;
    s.grid[1] = s.grid[2] = 1;
    if (p.kind == 0) {
        const bool wide = reduce_rows_per_group(p);
        s.grid[0] = wide ? (uint32_t)p.outputs : (uint32_t)((p.outputs + 3) / 4);
        s.lds_bytes = 32;
        s.kernel = wide ? "reduce_rows<group>" : "reduce_rows<wave>";
    } else if (p.kind == 1) {
        const int64_t Lc = p.shape[p.nk - 1];
        const int64_t strip = (int64_t)p.cols_v << p.cols_tc_log2;
        s.grid[0] = (uint32_t)(((Lc + strip - 1) / strip) * (p.outputs / Lc) * p.split);
        s.lds_bytes = (uint32_t)(kThreads * p.cols_v * 4 * (p.op >= 2 ? 2 : 1));
        s.kernel = p.split > 1 ? (p.cols_v == 4 ? "reduce_cols<vec4,split>" : "reduce_cols<scalar,split>")
                               : (p.cols_v == 4 ? "reduce_cols<vec4>" : "reduce_cols<scalar>");
    } else {
        s.grid[0] = (uint32_t)((p.outputs + kThreads - 1) / kThreads);
        s.lds_bytes = 0;
        s.kernel = "reduce_gather";
    }
    return s;
}

hipError_t reduce_launch(const ReduceParams& p, hipStream_t stream) {
    switch (p.op) {
        case 0: return launch_op<0>(p, stream);
        case 2: return launch_op<2>(p, stream);
        default: return launch_op<3>(p, stream);
    }
}

}  // namespace hpct
