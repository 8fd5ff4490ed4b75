// Layout kernels around the grouped FFN: offline expert packing, per-call token gather into
// MFMA fragment order, and the weighted combine (paper Section 2.1: the layer output of a
// token is the weighted sum of its selected experts' outputs).
//
// Fragment order (bf16).  A 32x16 operand fragment of the 32x32x16 MFMA is stored as 64
// consecutive 16-byte units, one per lane: lane l holds row (l & 31) and the eight reduction
// positions of half hi = l >> 5.  For the up projections (reduction over d) position i is
// element 16*ks + 8*hi + i, and the 32 rows of a weight fragment are 16 rows of W1 followed by
// the same 16 rows of W3, so that one MFMA yields gate and up values of the same features in
// the same lane.  For the down projection (reduction over f) position i is feature
// 16*ks + 8*(i/4) + 4*hi + i%4, which is exactly how those values fall in the up kernel's
// accumulator registers, so H never needs a shuffle between the two GEMMs.
#include <algorithm>

#include "kernels.h"

namespace kmoe {
namespace {

constexpr int kThreads = 256;

// ---- offline packing of expert weights ----------------------------------------------------
// W13p: [unit = f/16][ks = d/16][lane 64] x 16 B   rows 0..15 = W1, rows 16..31 = W3 of the unit
// W2p : [unit = d/32][ks = f/16][lane 64] x 16 B   rows = 32 output columns, values as fp16 (pack_down_f16_kernel)
__global__ __launch_bounds__(kThreads) void pack_up_kernel(const uint16_t* __restrict__ w1,
                                                           const uint16_t* __restrict__ w3, int d,
                                                           int f, uint4* __restrict__ out) {
    const size_t units = (size_t)f * d * 2 / 8;
    const int nks = d / 16;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const size_t q = u >> 6;
        const int ks = (int)(q % nks);
        const int unit = (int)(q / nks);
        const int r = lane & 31, hi = lane >> 5;
        const uint16_t* src = (r < 16 ? w1 + (size_t)(unit * 16 + r) * d
                                      : w3 + (size_t)(unit * 16 + r - 16) * d) + ks * 16 + hi * 8;
        out[u] = *reinterpret_cast<const uint4*>(src);
    }
}

// ---- offline packing of a 4-bit group-quantised expert -------------------------------------------
// Codes: [unit][quad = 4 steps][lane 64] x 16 B, dword i of a lane = its eight codes of step
// 4*quad + i in the lane's fragment order (the same orders as the bf16 fragments above).
// Scales: [unit][quad][fragment row 32] x (s | z << 16).
__global__ __launch_bounds__(kThreads) void pack_up_q4_kernel(const uint8_t* __restrict__ q1,
                                                              const uint8_t* __restrict__ q3, int d,
                                                              int f, uint4* __restrict__ out) {
    const int nq = d / 64;
    const size_t units = (size_t)(f / 16) * nq * 64;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const size_t qd = u >> 6;
        const int quad = (int)(qd % nq);
        const int unit = (int)(qd / nq);
        const int r = lane & 31, hi = lane >> 5;
        const uint8_t* row = r < 16 ? q1 + (size_t)(unit * 16 + r) * (d / 2)
                                    : q3 + (size_t)(unit * 16 + r - 16) * (d / 2);
        uint32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)  // codes of columns 64*quad + 16*i + 8*hi + 0..7: four bytes
            v[i] = *reinterpret_cast<const uint32_t*>(row + 32 * quad + 8 * i + 4 * hi);
        out[u] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

__global__ __launch_bounds__(kThreads) void pack_down_q4_kernel(const uint8_t* __restrict__ q2, int d,
                                                                int f, uint4* __restrict__ out) {
    const int nq = f / 64;
    const size_t units = (size_t)(d / 32) * nq * 64;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const size_t qd = u >> 6;
        const int quad = (int)(qd % nq);
        const int unit = (int)(qd / nq);
        const int col = unit * 32 + (lane & 31), hi = lane >> 5;
        const uint8_t* row = q2 + (size_t)col * (f / 2);
        uint32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // features 64q + 16i + 4hi + 0..3, then the same + 8
            const int f0 = 64 * quad + 16 * i + 4 * hi;
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(row + f0 / 2);
            const uint32_t up = *reinterpret_cast<const uint16_t*>(row + (f0 + 8) / 2);
            v[i] = lo | (up << 16);
        }
        out[u] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

// (s, z) of fragment row r of every (unit, quad); rows_per_unit fragment rows come from `a`
// (first half_rows rows, may be all) and then from `b`.
__global__ __launch_bounds__(kThreads) void pack_sz_q4_kernel(const uint16_t* __restrict__ sa,
                                                              const uint16_t* __restrict__ za,
                                                              const uint16_t* __restrict__ sb,
                                                              const uint16_t* __restrict__ zb,
                                                              int n_units, int nq, int half_rows,
                                                              float scale, uint32_t* __restrict__ out) {
    const size_t n = (size_t)n_units * nq * 32;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < n;
         u += (size_t)gridDim.x * kThreads) {
        const int r = (int)(u & 31);
        const size_t qd = u >> 5;
        const int quad = (int)(qd % nq);
        const int unit = (int)(qd / nq);
        uint32_t s, z;
        if (r < half_rows) {
            const size_t at = (size_t)(unit * half_rows + r) * nq + quad;
            s = sa[at];
            z = za[at];
        } else {
            const size_t at = (size_t)(unit * half_rows + r - half_rows) * nq + quad;
            s = sb[at];
            z = zb[at];
        }
        // scale: a power of two times the group's scale (exact in bf16 short of underflow); the
        // dequantised weight s * (code - z) scales with it, the zero point stays
        if (scale != 1.f) s = __float_as_uint(__uint_as_float(s << 16) * scale) >> 16;
        out[u] = s | (z << 16);
    }
}

// Range and row energy of a 4-bit W2 [d, f] as the kernels will see it: every weight
// bf16(fma(code, s, -z * s)) (fp32 fma, nearest-even rounding to bf16).  Same outputs as
// w2_stats_kernel.
__global__ __launch_bounds__(kThreads) void w2_stats_q4_kernel(const uint8_t* __restrict__ q2,
                                                               const uint16_t* __restrict__ s2,
                                                               const uint16_t* __restrict__ z2, int d, int f,
                                                               uint32_t* __restrict__ out) {
    __shared__ float ssum[kThreads / 64];
    __shared__ uint32_t smax[kThreads / 64];
    for (int row = blockIdx.x; row < d; row += gridDim.x) {
        float sum = 0.f;
        uint32_t amax = 0;
        for (int i = threadIdx.x; i < f; i += kThreads) {
            const uint8_t byte = q2[(size_t)row * (f / 2) + i / 2];
            const float code = (float)((i & 1) ? (byte >> 4) : (byte & 15));
            const float sc = __uint_as_float((uint32_t)s2[(size_t)row * (f / 64) + i / 64] << 16);
            const float zp = __uint_as_float((uint32_t)z2[(size_t)row * (f / 64) + i / 64] << 16);
            float w = __builtin_fmaf(code, sc, -zp * sc);
            uint32_t bits = __float_as_uint(w);
            if ((bits & 0x7fffffffu) <= 0x7f800000u) bits += 0x7fffu + ((bits >> 16) & 1u);  // to bf16, nearest even
            bits &= 0xffff0000u;
            w = __uint_as_float(bits);
            amax = max(amax, bits & 0x7fffffffu);
            sum = __builtin_fmaf(w, w, sum);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            sum += __shfl_xor(sum, m, 64);
            amax = max(amax, (uint32_t)__shfl_xor((int)amax, m, 64));
        }
        if ((threadIdx.x & 63) == 0) {
            ssum[threadIdx.x >> 6] = sum;
            smax[threadIdx.x >> 6] = amax;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            uint32_t m = 0;
            for (int w = 0; w < kThreads / 64; ++w) {
                t += ssum[w];
                m = max(m, smax[w]);
            }
            atomicMax(out, m);
            atomicMax(out + 1, __float_as_uint(t));
        }
        __syncthreads();
    }
}

// Range and row energy of W2 [d, f] (bf16), for its placement as fp16: out[0] = bits of the
// largest |w| (NaN and infinity order above every finite value), out[1] = bits of the largest
// sum of squares over a row (one output column of the down projection).  One workgroup per row,
// integer maxima, so the result does not depend on the order.  out is zeroed by the caller.
__global__ __launch_bounds__(kThreads) void w2_stats_kernel(const uint16_t* __restrict__ w2, int d, int f,
                                                            uint32_t* __restrict__ out) {
    __shared__ float ssum[kThreads / 64];
    __shared__ uint32_t smax[kThreads / 64];
    for (int row = blockIdx.x; row < d; row += gridDim.x) {
        const uint16_t* src = w2 + (size_t)row * f;
        float sum = 0.f;
        uint32_t amax = 0;
        for (int i = threadIdx.x; i < f; i += kThreads) {
            const uint32_t bits = (uint32_t)src[i] << 16;
            const float w = __uint_as_float(bits);
            amax = max(amax, bits & 0x7fffffffu);
            sum = __builtin_fmaf(w, w, sum);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            sum += __shfl_xor(sum, m, 64);
            amax = max(amax, (uint32_t)__shfl_xor((int)amax, m, 64));
        }
        if ((threadIdx.x & 63) == 0) {
            ssum[threadIdx.x >> 6] = sum;
            smax[threadIdx.x >> 6] = amax;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            uint32_t m = 0;
            for (int w = 0; w < kThreads / 64; ++w) {
                t += ssum[w];
                m = max(m, smax[w]);
            }
            atomicMax(out, m);
            atomicMax(out + 1, __float_as_uint(t));  // t >= 0 (or NaN, which orders above): bits order as values
        }
        __syncthreads();
    }
}

// W2 for the down projection, which runs on the fp16 MFMA: every bf16 weight times `scale` (a
// power of two, 1 unless the expert holds weights beyond the fp16 range: exact) converted to
// fp16 (nearest even).  Exact for scaled |w| in [2^-17, 65504] (a bf16 value has 8 significant
// bits, an fp16 subnormal at least that many down to 2^-17); smaller weights round to a multiple
// of 2^-24 (absolute error at most 2^-25 of the scaled value).
__global__ __launch_bounds__(kThreads) void pack_down_f16_kernel(const uint16_t* __restrict__ w2, int d,
                                                                 int f, float scale,
                                                                 uint4* __restrict__ out) {
    const size_t units = (size_t)f * d / 8;
    const int nks = f / 16;
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads) {
        const int lane = (int)(u & 63);
        const size_t q = u >> 6;
        const int ks = (int)(q % nks);
        const int unit = (int)(q / nks);
        const int col = unit * 32 + (lane & 31);
        const int hi = lane >> 5;
        const uint16_t* src = w2 + (size_t)col * f + ks * 16 + 4 * hi;
        uint32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // positions 2i, 2i+1: features 4hi + 2(i%2) + 8(i/2) + 0..1
            const uint16_t* pp = src + 8 * (i / 2) + 2 * (i % 2);
            uint32_t packed = 0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const float w = __uint_as_float((uint32_t)pp[t] << 16) * scale;
                const _Float16 hv = (_Float16)w;
                packed |= (uint32_t)__builtin_bit_cast(uint16_t, hv) << (16 * t);
            }
            v[i] = packed;
        }
        out[u] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

__global__ __launch_bounds__(kThreads) void zero_u64_kernel(unsigned long long* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
        p[i] = 0ull;
}

__global__ __launch_bounds__(kThreads) void copy_kernel(const uint4* __restrict__ src, size_t units,
                                                        uint4* __restrict__ dst) {
    for (size_t u = (size_t)blockIdx.x * kThreads + threadIdx.x; u < units;
         u += (size_t)gridDim.x * kThreads)
        dst[u] = src[u];
}

// ---- per-call gather of token rows into fragment order -------------------------------------
// Xp: [row block][ks = d/16][lane 64] x 16 B.  Routed blocks follow the padded per-expert row
// space; the rows of shared experts (all tokens, natural order) follow them.
// A wavefront takes one row block and `quads` groups of four reduction steps (one group on small
// layers, so that there are wavefronts for every compute unit; up to kGatherQuads on large ones,
// where the look-ups are then shared by more traffic).  Per group it
// moves four fragments (4 KiB) with four loads and four stores per lane, laid out so that both
// sides work in whole 128-byte lines: lane (r = lane / 8, c = lane % 8) reads, for rows r, r + 8,
// r + 16, r + 24 of the block, the 16 bytes c of the row's 128-byte piece (step c / 2 of the
// group, half c % 2), and eight consecutive lanes store eight consecutive 16-byte units of one
// fragment.  The token of a row is looked up once per wavefront item, not once per unit.
constexpr int kGatherQuads = 8;
__global__ __launch_bounds__(kThreads) void gather_kernel(const uint16_t* __restrict__ x, Shape s,
                                                          PlanPtrs p, uint4* __restrict__ xp,
                                                          unsigned long long* __restrict__ herr, int quads) {
    const int nks = s.d / 16;  // a multiple of 4: the bf16 path needs d_model % 64 == 0
    const int routed_blks = p.meta[2];
    const int shared_blks = s.S > 0 ? (s.N + kRowBlk - 1) / kRowBlk : 0;
    // the up kernel adds the remainder energy of every H row of this call to herr: start at zero
    const size_t h_rows = ((size_t)routed_blks + (size_t)s.S * ((s.N + kRowBlk - 1) / kRowBlk)) * kRowBlk;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < h_rows; i += (size_t)gridDim.x * kThreads)
        herr[i] = 0ull;
    const int nquads = nks / 4;
    const int groups = (nquads + quads - 1) / quads;
    const int lane = threadIdx.x & 63, r = lane >> 3, c = lane & 7;
    const int waves = kThreads / 64;
    const long items = (long)(routed_blks + shared_blks) * groups;
    for (long item = (long)blockIdx.x * waves + (threadIdx.x >> 6); item < items; item += (long)gridDim.x * waves) {
        const int blk = (int)(item / groups), g = (int)(item % groups);
        // tokens of rows r, r + 8, r + 16, r + 24: the block's expert and its offsets once, then the
        // four look-ups side by side (clamped indices, no branch between them)
        const uint16_t* src[4];
        if (blk < routed_blks) {
            const int e = p.blk_expert[blk];
            const int first = blk * kRowBlk - p.poff[e], cnt = p.counts[e], off = p.offsets[e];
            int a[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = p.perm[off + min(first + i * 8 + r, cnt - 1)];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                src[i] = first + i * 8 + r < cnt ? x + (size_t)(a[i] / s.k) * s.d + c * 8 : nullptr;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = (blk - routed_blks) * kRowBlk + i * 8 + r;
                src[i] = t < s.N ? x + (size_t)t * s.d + c * 8 : nullptr;
            }
        }
        uint4* dst = xp + ((size_t)blk * nks) * 64 + (size_t)(c >> 1) * 64 + (c & 1) * 32 + r;
        const int q1 = min((g + 1) * quads, nquads);
        for (int q = g * quads; q < q1; ++q) {
            uint4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                v[i] = src[i] ? *reinterpret_cast<const uint4*>(src[i] + (size_t)q * 64) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[(size_t)q * 256 + i * 8] = v[i];
        }
    }
}

// ---- weighted combine ------------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));  // first-class 16-byte value for streaming loads

// A wavefront item is one token x kCombineCols float4 columns per lane: the token's rows and routing
// weights are looked up once per item (uniform over the wavefront), and all partial rows of the
// item are requested before the first addition.  O is read exactly once: streaming loads.
constexpr int kCombineCols = 2;
template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void combine_kernel(Shape s, PlanPtrs p,
                                                           const float* __restrict__ o, int split_k,
                                                           int64_t split_stride,
                                                           void* __restrict__ y) {
    const int d4 = s.d / 4;
    const int shared_stride_rows = (s.N + kRowBlk - 1) / kRowBlk * kRowBlk;
    const int shared_row0 = p.meta[2] * kRowBlk;  // shared experts' rows follow the routed ones
    const int lane = threadIdx.x & 63, waves = kThreads / 64;
    const int chunks = (d4 + 64 * kCombineCols - 1) / (64 * kCombineCols);
    const long items = (long)s.N * chunks;
    for (long item = (long)blockIdx.x * waves + (threadIdx.x >> 6); item < items; item += (long)gridDim.x * waves) {
        const int t = (int)(item / chunks), ch = (int)(item % chunks);
        float4 acc[kCombineCols];
        int col[kCombineCols];
#pragma unroll
        for (int u = 0; u < kCombineCols; ++u) {
            acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            col[u] = (ch * kCombineCols + u) * 64 + lane;  // float4 column of this lane
        }
        for (int j = 0; j < s.k; ++j) {  // routed slots in order j = 0..k-1
            const int a = t * s.k + j;
            const int e = p.topk_idx[a];
            const int row = p.poff[e] + (p.inv_perm[a] - p.offsets[e]);
            const float w = p.topk_w[a];
            float4 v[kCombineCols];
#pragma unroll
            for (int u = 0; u < kCombineCols; ++u) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sp = 0; sp < split_k; ++sp) {
                const float4* src = reinterpret_cast<const float4*>(o + (size_t)sp * split_stride + (size_t)row * s.d);
#pragma unroll
                for (int u = 0; u < kCombineCols; ++u) {
                    if (col[u] < d4) {
                        const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + col[u]));
                        v[u].x += q.x; v[u].y += q.y; v[u].z += q.z; v[u].w += q.w;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kCombineCols; ++u) {
                acc[u].x = __builtin_fmaf(w, v[u].x, acc[u].x);
                acc[u].y = __builtin_fmaf(w, v[u].y, acc[u].y);
                acc[u].z = __builtin_fmaf(w, v[u].z, acc[u].z);
                acc[u].w = __builtin_fmaf(w, v[u].w, acc[u].w);
            }
        }
        for (int sh = 0; sh < s.S; ++sh) {  // then the always-on experts, weight 1
            const size_t row = (size_t)shared_row0 + (size_t)sh * shared_stride_rows + t;
            for (int sp = 0; sp < split_k; ++sp) {
                const float4* src = reinterpret_cast<const float4*>(o + (size_t)sp * split_stride + row * s.d);
#pragma unroll
                for (int u = 0; u < kCombineCols; ++u) {
                    if (col[u] < d4) {
                        const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + col[u]));
                        acc[u].x += q.x; acc[u].y += q.y; acc[u].z += q.z; acc[u].w += q.w;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kCombineCols; ++u) {
            if (col[u] >= d4) continue;
            if (kBf16Out) {
                uint2 r;
                r.x = (uint32_t)f32_to_bf16_rne(acc[u].x) | ((uint32_t)f32_to_bf16_rne(acc[u].y) << 16);
                r.y = (uint32_t)f32_to_bf16_rne(acc[u].z) | ((uint32_t)f32_to_bf16_rne(acc[u].w) << 16);
                *reinterpret_cast<uint2*>((uint16_t*)y + (size_t)t * s.d + (size_t)col[u] * 4) = r;
            } else {
                *reinterpret_cast<float4*>((float*)y + (size_t)t * s.d + (size_t)col[u] * 4) = acc[u];
            }
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
                             int f, void* blob, float w2_scale) {
    uint4* up = (uint4*)blob;
    uint4* down = up + (size_t)f * d * 2 / 8;
    hipLaunchKernelGGL(pack_up_kernel, dim3(grid_for((size_t)f * d / 4)), dim3(kThreads), 0, st,
                       (const uint16_t*)w1, (const uint16_t*)w3, d, f, up);
    hipLaunchKernelGGL(pack_down_f16_kernel, dim3(grid_for((size_t)f * d / 8)), dim3(kThreads), 0, st,
                       (const uint16_t*)w2, d, f, w2_scale, down);
}

void launch_w2_stats(hipStream_t st, const void* w2, int d, int f, uint32_t* out2) {
    hipLaunchKernelGGL(w2_stats_kernel, dim3(d < 2048 ? d : 2048), dim3(kThreads), 0, st, (const uint16_t*)w2,
                       d, f, out2);
}

void launch_zero_u64(hipStream_t st, unsigned long long* p, size_t n) {
    if (n == 0) return;
    hipLaunchKernelGGL(zero_u64_kernel, dim3(grid_for(n, 1024)), dim3(kThreads), 0, st, p, n);
}

void launch_pack_expert_q4(hipStream_t st, const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                           const uint8_t* q3, const uint16_t* s3, const uint16_t* z3, const uint8_t* q2,
                           const uint16_t* s2, const uint16_t* z2, int d, int f, void* blob, float w2_scale) {
    const size_t df = (size_t)d * f;
    uint8_t* b = (uint8_t*)blob;
    hipLaunchKernelGGL(pack_up_q4_kernel, dim3(grid_for(df / 16)), dim3(kThreads), 0, st, q1, q3, d, f,
                       (uint4*)b);
    hipLaunchKernelGGL(pack_sz_q4_kernel, dim3(grid_for(df / 32)), dim3(kThreads), 0, st, s1, z1, s3, z3,
                       f / 16, d / 64, 16, 1.f, (uint32_t*)(b + df));
    hipLaunchKernelGGL(pack_down_q4_kernel, dim3(grid_for(df / 32)), dim3(kThreads), 0, st, q2, d, f,
                       (uint4*)(b + df + df / 8));
    hipLaunchKernelGGL(pack_sz_q4_kernel, dim3(grid_for(df / 64)), dim3(kThreads), 0, st, s2, z2, s2, z2,
                       d / 32, f / 64, 32, w2_scale, (uint32_t*)(b + df + df / 8 + df / 2));
}

void launch_w2_stats_q4(hipStream_t st, const uint8_t* q2, const uint16_t* s2, const uint16_t* z2, int d, int f,
                        uint32_t* out2) {
    hipLaunchKernelGGL(w2_stats_q4_kernel, dim3(d < 2048 ? d : 2048), dim3(kThreads), 0, st, q2, s2, z2, d, f, out2);
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
                        void* xp, unsigned long long* herr) {
    if (s.N <= 0) return;
    const size_t max_units =
        ((size_t)s.max_rowblks + (s.S > 0 ? (s.N + kRowBlk - 1) / kRowBlk : 0)) * (s.d / 16) * 64;
    // a wavefront item is 4 * quads fragments of 64 units; four wavefronts per workgroup; at least
    // some thousands of items, so that every compute unit has several wavefronts in flight
    const size_t blocks_now = std::min<size_t>((size_t)s.max_rowblks, ((size_t)s.N * s.k + kRowBlk - 1) / kRowBlk + s.E) +
                              (s.S > 0 ? (s.N + kRowBlk - 1) / kRowBlk : 0);
    const size_t total_quads = blocks_now * (s.d / 64);
    int quads = (int)(total_quads / 4096);
    quads = quads < 1 ? 1 : (quads > kGatherQuads ? kGatherQuads : quads);
    hipLaunchKernelGGL(gather_kernel, dim3(grid_for(max_units / (4 * quads) + kThreads, 2048)), dim3(kThreads), 0, st,
                       (const uint16_t*)x, s, p, (uint4*)xp, herr, quads);
}

void launch_combine(hipStream_t st, int out_dtype, const Shape& s, const PlanPtrs& p,
                    const float* o, int split_k, int64_t o_split_stride, void* y) {
    if (s.N <= 0) return;
    // one wavefront per (token, 64 * kCombineCols float4 columns)
    const int chunks = (s.d / 4 + 64 * kCombineCols - 1) / (64 * kCombineCols);
    const dim3 grid(grid_for((size_t)s.N * chunks * 64, 8192)), block(kThreads);
    if (out_dtype == 1)
        hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, st, s, p, o, split_k,
                           o_split_stride, y);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, st, s, p, o, split_k,
                           o_split_stride, y);
}

}  // namespace kmoe
