// fp32 expert FFN (SwiGLU) on the vector ALUs, for the fp32 configuration.
//
// Each expert is an FFN applied to the tokens routed to it (paper Section 2.1); rows follow
// the same padded per-expert row space as the bf16 path.  One workgroup serves one row and a
// slab of output features; a wavefront computes one dot product at a time (lanes stride the
// reduction axis, xor-butterfly sum), fp32 fused multiply-adds throughout, accurate expf.
#include "kernels.h"

namespace kmoe {
namespace {

constexpr int kWaves = 4;
constexpr int kSlab = 64;  // output features per workgroup

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Which expert and which source token does padded row `row` belong to?  token < 0: padding.
__device__ __forceinline__ void row_owner(const Shape& s, const PlanPtrs& p, int row, int& e,
                                          int& token) {
    const int routed_rows = p.meta[2] * kRowBlk;
    token = -1;
    e = -1;
    if (row < routed_rows) {
        e = p.blk_expert[row / kRowBlk];
        const int rank = row - p.poff[e];
        if (rank < p.counts[e]) token = p.perm[p.offsets[e] + rank] / s.k;
    } else {
        const int stride = (s.N + kRowBlk - 1) / kRowBlk * kRowBlk;
        const int r = row - routed_rows;
        if (stride > 0 && r < s.S * stride) {
            e = s.E + r / stride;
            const int t = r % stride;
            if (t < s.N) token = t;
        }
    }
}

// h[row, n] = silu(W1[n,:] . x) * (W3[n,:] . x)
__global__ __launch_bounds__(kWaves * 64) void ffn_up_f32_kernel(
    const float* __restrict__ x, Shape s, PlanPtrs p, const uint8_t* const* __restrict__ wtab,
    const uint8_t* __restrict__ w_single, int only_expert, float* __restrict__ h) {
    int e, token;
    row_owner(s, p, blockIdx.x, e, token);
    if (token < 0 || (only_expert >= 0 && e != only_expert)) return;
    const float* blob = reinterpret_cast<const float*>(w_single ? w_single : wtab[e]);
    const float* w1 = blob;
    const float* w3 = blob + (size_t)s.f * s.d;
    const float* xr = x + (size_t)token * s.d;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = blockIdx.y * kSlab;
    for (int n = n0 + wave; n < min(n0 + kSlab, s.f); n += kWaves) {
        float g = 0.f, u = 0.f;
        for (int i = lane; i < s.d; i += 64) {
            const float xv = xr[i];
            g = __builtin_fmaf(w1[(size_t)n * s.d + i], xv, g);
            u = __builtin_fmaf(w3[(size_t)n * s.d + i], xv, u);
        }
        g = wave_sum(g);
        u = wave_sum(u);
        if (lane == 0) h[(size_t)blockIdx.x * s.f + n] = g / (1.f + expf(-g)) * u;
    }
}

// o[row, m] = W2[m,:] . h[row,:]
__global__ __launch_bounds__(kWaves * 64) void ffn_down_f32_kernel(
    Shape s, PlanPtrs p, const uint8_t* const* __restrict__ wtab,
    const uint8_t* __restrict__ w_single, int only_expert, const float* __restrict__ h,
    float* __restrict__ o) {
    int e, token;
    row_owner(s, p, blockIdx.x, e, token);
    if (token < 0 || (only_expert >= 0 && e != only_expert)) return;
    const float* blob = reinterpret_cast<const float*>(w_single ? w_single : wtab[e]);
    const float* w2 = blob + 2 * (size_t)s.f * s.d;
    const float* hr = h + (size_t)blockIdx.x * s.f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = blockIdx.y * kSlab;
    for (int m = m0 + wave; m < min(m0 + kSlab, s.d); m += kWaves) {
        float acc = 0.f;
        for (int i = lane; i < s.f; i += 64) acc = __builtin_fmaf(w2[(size_t)m * s.f + i], hr[i], acc);
        acc = wave_sum(acc);
        if (lane == 0) o[(size_t)blockIdx.x * s.d + m] = acc;
    }
}

}  // namespace

void launch_ffn_f32(hipStream_t st, const float* x, const Shape& s, const PlanPtrs& p,
                    const uint8_t* const* wtab, const uint8_t* w_single, int32_t only_expert,
                    float* h, float* o) {
    if (s.N <= 0) return;
    const int rows = s.max_rowblks * kRowBlk + s.S * ((s.N + kRowBlk - 1) / kRowBlk * kRowBlk);
    // rows beyond the routed padded space of this call shift the shared rows down; bound by the
    // capacity and let row_owner() reject what is not there.
    hipLaunchKernelGGL(ffn_up_f32_kernel, dim3(rows, (s.f + kSlab - 1) / kSlab), dim3(kWaves * 64),
                       0, st, x, s, p, wtab, w_single, only_expert, h);
    hipLaunchKernelGGL(ffn_down_f32_kernel, dim3(rows, (s.d + kSlab - 1) / kSlab),
                       dim3(kWaves * 64), 0, st, s, p, wtab, w_single, only_expert, h, o);
}

}  // namespace kmoe
