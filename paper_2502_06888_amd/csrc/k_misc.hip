// Layout kernels around the grouped FFN: offline expert packing, per-call token gather into
// MFMA fragment order, and the weighted combine (paper Section 2.1: the layer output of a
// token is the weighted sum of its selected experts' outputs).
//
// Fragment order (bf16).  A 16x32 operand fragment of the 16x16x32 MFMA is stored as 64
// consecutive 16-byte units, one per lane: lane l holds row (l & 15) and the eight reduction
// positions of group g = l >> 4.  For the up projections (reduction over d) position i of
// group g is element 32*ks + 8*g + i.  For the down projection (reduction over f) it is
// 32*ks + 4*g + i for i < 4 and 32*ks + 16 + 4*g + (i-4) otherwise, which is exactly how the
// up kernel's accumulator registers fall, so H never needs a shuffle between the two GEMMs.
#include "kernels.h"

namespace kmoe {
namespace {

constexpr int kThreads = 256;

// ---- offline packing of expert weights ----------------------------------------------------
// W13p: [rb = f/16][ks = d/32][mat 2][lane 64] x 16 B   (mat 0 = W1, 1 = W3)
// W2p : [nb = d/32][ks = f/32][sub 2][lane 64] x 16 B   (sub = which 16 of the 32 columns)
__global__ __launch_bounds__(kThreads) void pack_up_kernel(const uint16_t* __restrict__ w1,
                                                           const uint16_t* __restrict__ w3, int d,
                                                           int f, uint4* __restrict__ out) {
    const size_t units = (size_t)f * d * 2 / 8;
    const int nks = d / 32;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const int mat = (int)((u >> 6) & 1);
        const size_t q = u >> 7;
        const int ks = (int)(q % nks);
        const int rb = (int)(q / nks);
        const int row = rb * 16 + (lane & 15);
        const int col = ks * 32 + (lane >> 4) * 8;
        const uint16_t* src = (mat == 0 ? w1 : w3) + (size_t)row * d + col;
        out[u] = *reinterpret_cast<const uint4*>(src);
    }
}

__global__ __launch_bounds__(kThreads) void pack_down_kernel(const uint16_t* __restrict__ w2, int d,
                                                             int f, uint4* __restrict__ out) {
    const size_t units = (size_t)f * d / 8;
    const int nks = f / 32;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const int sub = (int)((u >> 6) & 1);
        const size_t q = u >> 7;
        const int ks = (int)(q % nks);
        const int nb = (int)(q / nks);
        const int row = nb * 32 + sub * 16 + (lane & 15);  // output feature (row of W2)
        const int g = lane >> 4;
        const uint16_t* src = w2 + (size_t)row * f + ks * 32 + 4 * g;
        const uint2 lo = *reinterpret_cast<const uint2*>(src);       // f = 32ks + 4g + 0..3
        const uint2 hi = *reinterpret_cast<const uint2*>(src + 16);  // f = 32ks + 16 + 4g + 0..3
        out[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
}

__global__ __launch_bounds__(kThreads) void copy_kernel(const uint4* __restrict__ src, size_t units,
                                                        uint4* __restrict__ dst) {
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads)
        dst[u] = src[u];
}

// ---- per-call gather of token rows into fragment order -------------------------------------
// Xp: [blk16][ks = d/32][lane 64] x 16 B.  Routed blocks follow the padded per-expert row
// space; the rows of shared experts (all tokens, natural order) follow them.
__global__ __launch_bounds__(kThreads) void gather_kernel(const uint16_t* __restrict__ x, Shape s,
                                                          PlanPtrs p, uint4* __restrict__ xp) {
    const int nks = s.d / 32;
    const int routed_blks = p.meta[2];
    const int shared_blks = s.S > 0 ? (s.N + kRowBlk - 1) / kRowBlk : 0;
    const size_t units = (size_t)(routed_blks + shared_blks) * nks * 64;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const size_t q = u >> 6;
        const int ks = (int)(q % nks);
        const int blk = (int)(q / nks);
        const int j = lane & 15, g = lane >> 4;
        int token = -1;
        if (blk < routed_blks) {
            const int e = p.blk_expert[blk];
            const int rank = blk * kRowBlk + j - p.poff[e];
            if (rank < p.counts[e]) token = p.perm[p.offsets[e] + rank] / s.k;
        } else {
            const int t = (blk - routed_blks) * kRowBlk + j;
            if (t < s.N) token = t;
        }
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (token >= 0)
            v = *reinterpret_cast<const uint4*>(x + (size_t)token * s.d + ks * 32 + g * 8);
        xp[u] = v;
    }
}

// ---- weighted combine ------------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void combine_kernel(Shape s, PlanPtrs p,
                                                           const float* __restrict__ o, int split_k,
                                                           int64_t split_stride,
                                                           void* __restrict__ y) {
    const int d4 = s.d / 4;
    const int shared_stride_rows = (s.N + kRowBlk - 1) / kRowBlk * kRowBlk;
    const int shared_row0 = p.meta[2] * kRowBlk;  // shared experts' rows follow the routed ones
    const size_t total = (size_t)s.N * d4;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (size_t)gridDim.x * kThreads) {
        const int t = (int)(i / d4);
        const int c = (int)(i % d4) * 4;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < s.k; ++j) {  // routed slots in order j = 0..k-1
            const int a = t * s.k + j;
            const int e = p.topk_idx[a];
            const int row = p.poff[e] + (p.inv_perm[a] - p.offsets[e]);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sp = 0; sp < split_k; ++sp) {
                const float4 q = *reinterpret_cast<const float4*>(
                    o + (size_t)sp * split_stride + (size_t)row * s.d + c);
                v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
            }
            const float w = p.topk_w[a];
            acc.x = __builtin_fmaf(w, v.x, acc.x);
            acc.y = __builtin_fmaf(w, v.y, acc.y);
            acc.z = __builtin_fmaf(w, v.z, acc.z);
            acc.w = __builtin_fmaf(w, v.w, acc.w);
        }
        for (int sh = 0; sh < s.S; ++sh) {  // then the always-on experts, weight 1
            const size_t row = (size_t)shared_row0 + (size_t)sh * shared_stride_rows + t;
            for (int sp = 0; sp < split_k; ++sp) {
                const float4 q = *reinterpret_cast<const float4*>(
                    o + (size_t)sp * split_stride + row * s.d + c);
                acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
            }
        }
        if (kBf16Out) {
            uint2 r;
            r.x = (uint32_t)f32_to_bf16_rne(acc.x) | ((uint32_t)f32_to_bf16_rne(acc.y) << 16);
            r.y = (uint32_t)f32_to_bf16_rne(acc.z) | ((uint32_t)f32_to_bf16_rne(acc.w) << 16);
            *reinterpret_cast<uint2*>((uint16_t*)y + (size_t)t * s.d + c) = r;
        } else {
            *reinterpret_cast<float4*>((float*)y + (size_t)t * s.d + c) = acc;
        }
    }
}

inline int grid_for(size_t work_items, int cap = 4096) {
    size_t g = (work_items + kThreads - 1) / kThreads;
    if (g < 1) g = 1;
    return (int)(g > (size_t)cap ? cap : g);
}

}  // namespace

void launch_pack_expert_bf16(hipStream_t st, const void* w1, const void* w3, const void* w2, int d,
                             int f, void* blob) {
    uint4* up = (uint4*)blob;
    uint4* down = up + (size_t)f * d * 2 / 8;
    hipLaunchKernelGGL(pack_up_kernel, dim3(grid_for((size_t)f * d / 4)), dim3(kThreads), 0, st,
                       (const uint16_t*)w1, (const uint16_t*)w3, d, f, up);
    hipLaunchKernelGGL(pack_down_kernel, dim3(grid_for((size_t)f * d / 8)), dim3(kThreads), 0, st,
                       (const uint16_t*)w2, d, f, down);
}

void launch_pack_expert_f32(hipStream_t st, const void* w1, const void* w3, const void* w2, int d,
                            int f, void* blob) {
    const size_t units = (size_t)f * d * 4 / 16;
    uint4* dst = (uint4*)blob;
    const void* src[3] = {w1, w3, w2};
    for (int m = 0; m < 3; ++m)
        hipLaunchKernelGGL(copy_kernel, dim3(grid_for(units)), dim3(kThreads), 0, st,
                           (const uint4*)src[m], units, dst + m * units);
}

void launch_gather_bf16(hipStream_t st, const void* x, const Shape& s, const PlanPtrs& p,
                        void* xp) {
    if (s.N <= 0) return;
    const size_t max_units = ((size_t)s.max_rows16 + (s.S > 0 ? (s.N + 15) / 16 : 0)) * (s.d / 32) * 64;
    hipLaunchKernelGGL(gather_kernel, dim3(grid_for(max_units, 2048)), dim3(kThreads), 0, st,
                       (const uint16_t*)x, s, p, (uint4*)xp);
}

void launch_combine(hipStream_t st, int out_dtype, const Shape& s, const PlanPtrs& p,
                    const float* o, int split_k, int64_t o_split_stride, void* y) {
    if (s.N <= 0) return;
    const dim3 grid(grid_for((size_t)s.N * (s.d / 4), 8192)), block(kThreads);
    if (out_dtype == 1)
        hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, st, s, p, o, split_k,
                           o_split_stride, y);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, st, s, p, o, split_k,
                           o_split_stride, y);
}

}  // namespace kmoe
