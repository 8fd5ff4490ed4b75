// Router: gate logits in a fixed fp32 summation order, wavefront top-k, routing weights.
//
// The gating network scores every expert for every token and the k best are activated
// (paper Section 2.1).  One 64-lane wavefront serves one token.  The logit of (token, expert)
// is accumulated in an order that a scalar program can reproduce exactly: the row is cut into
// 16-byte vectors, vector c belongs to lane c mod 64, a lane folds its elements in increasing
// index with fused multiply-adds, and the 64 partial sums meet in an xor butterfly
// (32,16,...,1).  IEEE addition is commutative, so every lane ends with the same value.
#include "kernels.h"

namespace kmoe {
namespace {

constexpr int kRouterWaves = 2;
constexpr int kCB = 4;  // vectors per lane loaded together
constexpr int kEG = 8;  // experts accumulated together

template <typename T>
struct Chunk;

template <>
struct Chunk<float> {
    static constexpr int V = 4;
    typedef float4 Raw;
    static __device__ __forceinline__ Raw raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ void widen(const Raw q, float (&v)[4]) {
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    static __device__ __forceinline__ void load(const float* p, float (&v)[4]) { widen(raw(p), v); }
};

struct bf16raw {
    uint16_t bits;
};

template <>
struct Chunk<bf16raw> {
    static constexpr int V = 8;
    typedef uint4 Raw;
    static __device__ __forceinline__ Raw raw(const bf16raw* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ __forceinline__ void load(const bf16raw* p, float (&v)[8]) { widen(raw(p), v); }
    static __device__ __forceinline__ void widen(const Raw q, float (&v)[8]) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);            // low half = lower index
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

struct Cand {
    float v;
    int e;  // -1: none
};

__device__ __forceinline__ bool better(const Cand& a, const Cand& b) {
    if (a.e < 0) return false;
    if (b.e < 0) return true;
    return a.v > b.v || (a.v == b.v && a.e < b.e);
}

// Top-k by (logit desc, index asc) and the routing weights of one token; every lane holds in
// mine[s] the logit of expert lane + 64 s.  One wavefront.
__device__ __forceinline__ void select_and_write(const float (&mine)[4], int lane, int t, int E, int k,
                                                 int renorm, int32_t* __restrict__ idx_out,
                                                 float* __restrict__ w_out) {
    bool taken[4] = {false, false, false, false};
    float selv[kMaxTopK];
    int sele[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        selv[j] = 0.f;
        sele[j] = 0;
        if (j < k) {
            Cand best{0.f, -1};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int e = lane + 64 * s;
                Cand c{mine[s], (e < E && !taken[s]) ? e : -1};
                if (better(c, best)) best = c;
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                Cand o{__shfl_xor(best.v, m, 64), __shfl_xor(best.e, m, 64)};
                if (better(o, best)) best = o;
            }
            best.v = __shfl(best.v, 0, 64);
            best.e = __shfl(best.e, 0, 64);
            selv[j] = best.v;
            sele[j] = best.e;
#pragma unroll
            for (int s = 0; s < 4; ++s)
                if (best.e == lane + 64 * s) taken[s] = true;
        }
    }

    // routing weights: softmax over all experts, renormalised over the winners (or not)
    const float mx = selv[0];
    float den = 0.f;
    if (renorm) {
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j)
            if (j < k) den += expf(selv[j] - mx);
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (lane + 64 * s < E) den += expf(mine[s] - mx);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) den += __shfl_xor(den, m, 64);
    }
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < k) {
                idx_out[(size_t)t * k + j] = sele[j];
                w_out[(size_t)t * k + j] = expf(selv[j] - mx) / den;
            }
        }
    }
}

// Sum over the 64 lanes of eight values at once, in the order of the xor butterfly (32, 16, ..., 1)
// stated at the top.  At step m a lane only needs lane[l] + lane[l ^ m] for the values it will
// still hold afterwards, so the lanes split the values between them: after the steps 32, 16 and
// 8 lane l holds value (l >> 3) & 7 alone, and the steps 4, 2, 1 finish it.  Each sum a lane
// forms is the one the full butterfly forms in that lane (IEEE addition is commutative), so the
// totals are bit for bit the butterfly's: 10 cross-lane moves instead of 48.  Returns the eight
// totals, uniform over the wavefront.
__device__ __forceinline__ void butterfly8(const float (&a)[kEG], int lane, float (&tot)[kEG]) {
    static_assert(kEG == 8, "three halving steps");
    float b[4], c[2], dsum;
    const bool h5 = (lane & 32) != 0, h4 = (lane & 16) != 0, h3 = (lane & 8) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float keep = h5 ? a[4 + i] : a[i], send = h5 ? a[i] : a[4 + i];
        b[i] = keep + __shfl_xor(send, 32, 64);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float keep = h4 ? b[2 + i] : b[i], send = h4 ? b[i] : b[2 + i];
        c[i] = keep + __shfl_xor(send, 16, 64);
    }
    {
        const float keep = h3 ? c[1] : c[0], send = h3 ? c[0] : c[1];
        dsum = keep + __shfl_xor(send, 8, 64);
    }
#pragma unroll
    for (int m = 4; m >= 1; m >>= 1) dsum = dsum + __shfl_xor(dsum, m, 64);
#pragma unroll
    for (int j = 0; j < kEG; ++j)
        tot[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dsum), 8 * j));
}

// Top-k and renormalised routing weights of one token with at most kEG experts, from logits that
// are uniform over the wavefront: every lane selects for itself (no cross-lane traffic), lane 0
// writes.  Same order (logit descending, index ascending) and the same weight arithmetic as
// select_and_write with renorm set.
__device__ __forceinline__ void select_uniform_and_write(const float (&lg)[kEG], int E, int lane, int t,
                                                         int k, int32_t* __restrict__ idx_out,
                                                         float* __restrict__ w_out) {
    unsigned taken = 0u;
    float selv[kMaxTopK];
    int sele[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        selv[j] = 0.f;
        sele[j] = 0;
        if (j < k) {
            int best = -1;
            float bv = 0.f;
#pragma unroll
            for (int e = 0; e < kEG; ++e) {
                const bool free_e = e < E && ((taken >> e) & 1u) == 0u;
                if (free_e && (best < 0 || lg[e] > bv)) {
                    best = e;
                    bv = lg[e];
                }
            }
            taken |= 1u << best;
            selv[j] = bv;
            sele[j] = best;
        }
    }
    const float mx = selv[0];
    float den = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j)
        if (j < k) den += expf(selv[j] - mx);
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < k) {
                idx_out[(size_t)t * k + j] = sele[j];
                w_out[(size_t)t * k + j] = expf(selv[j] - mx) / den;
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kRouterWaves * 64) void router_kernel(
    const T* __restrict__ X, const T* __restrict__ Wg, int N, int d, int E, int k, int renorm,
    float* __restrict__ logits_out, int32_t* __restrict__ idx_out, float* __restrict__ w_out) {
    constexpr int V = Chunk<T>::V;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * kRouterWaves + (threadIdx.x >> 6);
    if (t >= N) return;  // whole wavefront leaves; no block-wide synchronisation below
    const int nchunk = d / V;
    const T* xrow = X + (size_t)t * d;

    float mine[4];  // logits of experts lane, lane+64, lane+128, lane+192
#pragma unroll
    for (int s = 0; s < 4; ++s) mine[s] = 0.f;

    const int cpl = (nchunk + 63) / 64;  // vectors per lane
    for (int e0 = 0; e0 < E; e0 += kEG) {
        float acc[kEG];
#pragma unroll
        for (int j = 0; j < kEG; ++j) acc[j] = 0.f;
        // kCB vectors per lane at a time: all their loads are independent and issued together,
        // the fused multiply-adds then run in increasing element index per (expert, lane)
        for (int c0 = 0; c0 < cpl; c0 += kCB) {
            float xv[kCB][V];
#pragma unroll
            for (int q = 0; q < kCB; ++q) {
                const int c = (c0 + q) * 64 + lane;
                if (c < nchunk) {
                    Chunk<T>::load(xrow + (size_t)c * V, xv[q]);
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i) xv[q][i] = 0.f;
                }
            }
#pragma unroll
            for (int j = 0; j < kEG; ++j) {
                if (e0 + j < E) {
                    float wv[kCB][V];
#pragma unroll
                    for (int q = 0; q < kCB; ++q) {
                        const int c = min((c0 + q) * 64 + lane, nchunk - 1);  // clamped: x is 0 there
                        Chunk<T>::load(Wg + (size_t)(e0 + j) * d + (size_t)c * V, wv[q]);
                    }
#pragma unroll
                    for (int q = 0; q < kCB; ++q) {
                        if ((c0 + q) * 64 + lane < nchunk) {
#pragma unroll
                            for (int i = 0; i < V; ++i)
                                acc[j] = __builtin_fmaf(xv[q][i], wv[q][i], acc[j]);
                        }
                    }
                }
            }
        }
        float tot[kEG];
        butterfly8(acc, lane, tot);
#pragma unroll
        for (int j = 0; j < kEG; ++j) {
            const int e = e0 + j;
            if (e < E) {
                if (logits_out != nullptr && lane == 0) logits_out[(size_t)t * E + e] = tot[j];
                if ((e & 63) == lane) {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        if ((e >> 6) == s) mine[s] = tot[j];
                }
            }
        }
        if (E <= kEG && renorm) {  // one group holds every expert: select in registers
            select_uniform_and_write(tot, E, lane, t, k, idx_out, w_out);
            return;
        }
    }

    select_and_write(mine, lane, t, E, k, renorm, idx_out, w_out);
}


// The same arithmetic for large batch groups: one wavefront serves kMT tokens at a time, so that
// every vector of the gate matrix it loads (and widens) feeds kMT tokens, and the loop body has no
// branch: it serves shapes in which every lane holds a whole number of kMCB-vector groups and the
// experts come in whole groups of kEG (anything else takes router_kernel), so all loads of a
// group are in flight together.  Per (token, expert, lane) the order of the fused multiply-adds
// is the one stated at the top.  Tokens past the end re-read the last row and write nothing.
constexpr int kMT = 4;   // tokens per wavefront
constexpr int kMCB = 2;  // vectors per lane loaded together
template <typename T>
__global__ __launch_bounds__(kRouterWaves * 64) void router_multi_kernel(
    const T* __restrict__ X, const T* __restrict__ Wg, int N, int d, int E, int k, int renorm,
    float* __restrict__ logits_out, int32_t* __restrict__ idx_out, float* __restrict__ w_out) {
    constexpr int V = Chunk<T>::V;
    const int lane = threadIdx.x & 63;
    const int t0 = (blockIdx.x * kRouterWaves + (threadIdx.x >> 6)) * kMT;
    if (t0 >= N) return;  // whole wavefront leaves; no block-wide synchronisation below
    const int cpl = d / (V * 64);  // vectors per lane, a multiple of kMCB
    const T* xrow[kMT];
#pragma unroll
    for (int q = 0; q < kMT; ++q) xrow[q] = X + (size_t)min(t0 + q, N - 1) * d + (size_t)lane * V;

    float mine[kMT][4];  // per token: logits of experts lane, lane+64, lane+128, lane+192
#pragma unroll
    for (int q = 0; q < kMT; ++q)
#pragma unroll
        for (int s = 0; s < 4; ++s) mine[q][s] = 0.f;

    for (int e0 = 0; e0 < E; e0 += kEG) {
        float acc[kMT][kEG];
#pragma unroll
        for (int q = 0; q < kMT; ++q)
#pragma unroll
            for (int j = 0; j < kEG; ++j) acc[q][j] = 0.f;
        const T* wrow = Wg + (size_t)e0 * d + (size_t)lane * V;
        for (int c0 = 0; c0 < cpl; c0 += kMCB) {
            typename Chunk<T>::Raw xr[kMT][kMCB], wr[kEG][kMCB];
#pragma unroll
            for (int q = 0; q < kMT; ++q)
#pragma unroll
                for (int b = 0; b < kMCB; ++b) xr[q][b] = Chunk<T>::raw(xrow[q] + (size_t)(c0 + b) * 64 * V);
#pragma unroll
            for (int j = 0; j < kEG; ++j)
#pragma unroll
                for (int b = 0; b < kMCB; ++b)
                    wr[j][b] = Chunk<T>::raw(wrow + (size_t)j * d + (size_t)(c0 + b) * 64 * V);
            float xv[kMT][kMCB][V];
#pragma unroll
            for (int q = 0; q < kMT; ++q)
#pragma unroll
                for (int b = 0; b < kMCB; ++b) Chunk<T>::widen(xr[q][b], xv[q][b]);
#pragma unroll
            for (int j = 0; j < kEG; ++j) {
#pragma unroll
                for (int b = 0; b < kMCB; ++b) {
                    float wv[V];
                    Chunk<T>::widen(wr[j][b], wv);
#pragma unroll
                    for (int q = 0; q < kMT; ++q)
#pragma unroll
                        for (int i = 0; i < V; ++i) acc[q][j] = __builtin_fmaf(xv[q][b][i], wv[i], acc[q][j]);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < kMT; ++q) {
            float tot[kEG];
            butterfly8(acc[q], lane, tot);
#pragma unroll
            for (int j = 0; j < kEG; ++j) {
                const int e = e0 + j;
                if (logits_out != nullptr && lane == 0 && t0 + q < N) logits_out[(size_t)(t0 + q) * E + e] = tot[j];
                if ((e & 63) == lane) {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        if ((e >> 6) == s) mine[q][s] = tot[j];
                }
            }
            if (E <= kEG && renorm && t0 + q < N)  // one group holds every expert: select in registers
                select_uniform_and_write(tot, E, lane, t0 + q, k, idx_out, w_out);
        }
    }
    if (E <= kEG && renorm) return;
#pragma unroll
    for (int q = 0; q < kMT; ++q)
        if (t0 + q < N) select_and_write(mine[q], lane, t0 + q, E, k, renorm, idx_out, w_out);
}


// The same arithmetic with one workgroup per token: wavefront w scores experts w*kSG, w*kSG+1,
// then (w+kSW)*kSG, ...; the token's row stays in registers (at most kSC vectors per lane) and
// the loads of a group's gate rows are all in flight together.  Logits meet in LDS and the first
// wavefront selects.  Used for small batch groups, where one wavefront per token leaves most
// of the chip idle.  The summation order per (token, expert) is the one stated at the top.
constexpr int kSW = 4;   // wavefronts per token
constexpr int kSG = 2;   // experts scored together by a wavefront
constexpr int kSC = 16;  // vectors of the row per lane, at most (template parameter SC: 2, 8 or 16)
template <typename T, int SC>
__global__ __launch_bounds__(kSW * 64) void router_split_kernel(
    const T* __restrict__ X, const T* __restrict__ Wg, int N, int d, int E, int k, int renorm,
    float* __restrict__ logits_out, int32_t* __restrict__ idx_out, float* __restrict__ w_out) {
    constexpr int V = Chunk<T>::V;
    __shared__ float slog[kMaxExperts];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    const int nchunk = d / V;
    const int cpl = (nchunk + 63) / 64;
    const T* xrow = X + (size_t)t * d;
    typename Chunk<T>::Raw xr[SC];  // the token's row, as stored; lanes past the end re-read the last vector
#pragma unroll
    for (int q = 0; q < SC; ++q)
        if (q < cpl) xr[q] = Chunk<T>::raw(xrow + (size_t)min(q * 64 + lane, nchunk - 1) * V);
    for (int e0 = wave * kSG; e0 < E; e0 += kSW * kSG) {
        // all gate vectors of the group are requested before the first multiply-add
        typename Chunk<T>::Raw wr[kSG][SC];
#pragma unroll
        for (int j = 0; j < kSG; ++j) {
            const int e = min(e0 + j, E - 1);  // clamped: the result of a surplus expert is dropped
#pragma unroll
            for (int q = 0; q < SC; ++q)
                if (q < cpl) wr[j][q] = Chunk<T>::raw(Wg + (size_t)e * d + (size_t)min(q * 64 + lane, nchunk - 1) * V);
        }
        float acc[kSG];
#pragma unroll
        for (int j = 0; j < kSG; ++j) {
            acc[j] = 0.f;
#pragma unroll
            for (int q = 0; q < SC; ++q) {
                if (q < cpl && q * 64 + lane < nchunk) {
                    float wv[V], xv[V];
                    Chunk<T>::widen(wr[j][q], wv);
                    Chunk<T>::widen(xr[q], xv);
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[j] = __builtin_fmaf(xv[i], wv[i], acc[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < kSG; ++j) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc[j] = acc[j] + __shfl_xor(acc[j], m, 64);
            const int e = e0 + j;
            if (e < E && lane == 0) {
                slog[e] = acc[j];
                if (logits_out != nullptr) logits_out[(size_t)t * E + e] = acc[j];
            }
        }
    }
    __syncthreads();
    if (wave != 0) return;
    if (E <= kEG && renorm) {  // few experts: every lane reads them all and selects in registers
        float lg[kEG];
#pragma unroll
        for (int e = 0; e < kEG; ++e) lg[e] = e < E ? slog[e] : 0.f;
        select_uniform_and_write(lg, E, lane, t, k, idx_out, w_out);
        return;
    }
    float mine[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) mine[s4] = lane + 64 * s4 < E ? slog[lane + 64 * s4] : 0.f;
    select_and_write(mine, lane, t, E, k, renorm, idx_out, w_out);
}

}  // namespace

void launch_router(hipStream_t st, int dtype, const void* x, const void* wg, const Shape& s,
                   float* logits_out, int32_t* idx_out, float* w_out) {
    if (s.N <= 0) return;
    const int V = dtype == 0 ? 4 : 8;
    const int cpl = (s.d / V + 63) / 64;
    if (s.N <= 2048 && cpl <= kSC) {  // small batch group: one workgroup per token
        dim3 grid(s.N), block(kSW * 64);
#define KMOE_SPLIT(T, SC)                                                                              \
    hipLaunchKernelGGL((router_split_kernel<T, SC>), grid, block, 0, st, (const T*)x, (const T*)wg, s.N, \
                       s.d, s.E, s.k, s.renorm, logits_out, idx_out, w_out)
        if (dtype == 0) {
            if (cpl <= 2) KMOE_SPLIT(float, 2); else if (cpl <= 8) KMOE_SPLIT(float, 8); else KMOE_SPLIT(float, 16);
        } else {
            if (cpl <= 2) KMOE_SPLIT(bf16raw, 2); else if (cpl <= 8) KMOE_SPLIT(bf16raw, 8); else KMOE_SPLIT(bf16raw, 16);
        }
#undef KMOE_SPLIT
        return;
    }
    // large bf16 batch groups of a shape the branch-free kernel serves: kMT tokens share every gate vector
    if (dtype != 0 && s.N >= 8192 && s.d % (8 * 64 * kMCB) == 0 && s.E % kEG == 0) {
        const int per_block = kRouterWaves * kMT;
        dim3 grid((s.N + per_block - 1) / per_block), block(kRouterWaves * 64);
        hipLaunchKernelGGL(router_multi_kernel<bf16raw>, grid, block, 0, st, (const bf16raw*)x,
                           (const bf16raw*)wg, s.N, s.d, s.E, s.k, s.renorm, logits_out, idx_out,
                           w_out);
        return;
    }
    dim3 grid((s.N + kRouterWaves - 1) / kRouterWaves), block(kRouterWaves * 64);
    if (dtype == 0) {
        hipLaunchKernelGGL(router_kernel<float>, grid, block, 0, st, (const float*)x,
                           (const float*)wg, s.N, s.d, s.E, s.k, s.renorm, logits_out, idx_out,
                           w_out);
    } else {
        hipLaunchKernelGGL(router_kernel<bf16raw>, grid, block, 0, st, (const bf16raw*)x,
                           (const bf16raw*)wg, s.N, s.d, s.E, s.k, s.renorm, logits_out, idx_out,
                           w_out);
    }
}

}  // namespace kmoe
