// Kernels of the attention (non-expert) layer for one decoding step of one batch.
//
// Algorithm 1 of the paper runs the non-expert layer batch by batch; the arithmetic is the
// attention layer of the paper's model family (Section 2.1) with its normalisation folded in
// (Section 4): RMS norm, q/k/v projections, rotary embedding, cache append, grouped-query
// softmax attention of the one new token over the cached positions, output projection and
// residual.  The projections are dense contractions and run on bf16 MFMA (32x32x16, fp32
// accumulate) with weights pre-packed in fragment order so that a wavefront streams one
// contiguous run of 1 KiB fragments; with few rows they are bound by the weight bytes, so the
// reduction is split across wavefronts until the chip is full and the partial sums are added in
// a fixed order by the kernel that consumes them.  The attention core is bound by the cache
// bytes: one workgroup per (sequence, key-value head) reads every K and V row once, 16 bytes
// per lane, all query heads of the group sharing each row.  Cache rows are read with
// non-temporal loads and the weights with ordinary ones: the layer's weights (tens of MB) are
// read again for every batch of the group and fit the last-level cache, the caches of a batch are
// read once and would only evict them.
#include <type_traits>

#include "attn_kernels.h"

namespace kattn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf_bits(float a) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)a);  // round to nearest even
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return bf_bits(lo) | (bf_bits(hi) << 16); }
__device__ __forceinline__ void widen8(const u32x4 v, float (&f)[8]) {
    f[0] = bf_lo(v.x); f[1] = bf_hi(v.x); f[2] = bf_lo(v.y); f[3] = bf_hi(v.y);
    f[4] = bf_lo(v.z); f[5] = bf_hi(v.z); f[6] = bf_lo(v.w); f[7] = bf_hi(v.w);
}
__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// 16-byte piece index of element (row, k) of a [rows, K] matrix in fragment order.
__device__ __forceinline__ size_t frag_piece(int row, int chunk, int S) {
    return ((size_t)(row >> 5) * S + (chunk >> 1)) * 64 + (row & 31) + 32 * (chunk & 1);
}

// Batch that owns activation row `row` (the table has at most kMaxGroup entries).
__device__ __forceinline__ int find_batch(const GroupTab& tab, int row) {
    int b = 0;
    while (b + 1 < tab.n && row >= tab.row0[b + 1]) ++b;
    return b;
}

__global__ __launch_bounds__(256) void pack_weight_kernel(const u32x4* __restrict__ w, int rows, int K,
                                                          u32x4* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)rows * K / 8) return;
    const int lane = (int)(i & 63), S = K / 16;
    const size_t unit = i >> 6;
    const int s = (int)(unit % S), rb = (int)(unit / S);
    const int row = rb * 32 + (lane & 31), k0 = s * 16 + (lane >> 5) * 8;
    out[i] = w[((size_t)row * K + k0) / 8];
}

// One workgroup per row; a thread keeps its 16-byte pieces of the row in registers between the
// sum of squares and the scaling (rows of up to 256 * 8 * kNormPieces elements).
constexpr int kNormPieces = 4;
__global__ __launch_bounds__(256) void rmsnorm_kernel(GroupTab tab, const u32x4* __restrict__ g, int d,
                                                      float eps, u32x4* __restrict__ a) {
    __shared__ float part[4];
    const int row = blockIdx.x, nch = d / 8, S = d / 16;
    const int bt = find_batch(tab, row);
    const u32x4* xr = (const u32x4*)tab.h_in[bt] + (size_t)(row - tab.row0[bt]) * nch;
    u32x4 xv[kNormPieces], gv[kNormPieces];
#pragma unroll
    for (int i = 0; i < kNormPieces; ++i) {
        const int c = threadIdx.x + i * 256;
        if (c < nch) {
            xv[i] = xr[c];
            gv[i] = g[c];
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kNormPieces; ++i) {
        if (threadIdx.x + i * 256 < nch) {
            float f[8];
            widen8(xv[i], f);
#pragma unroll
            for (int j = 0; j < 8; ++j) ss = __builtin_fmaf(f[j], f[j], ss);
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = (part[0] + part[1]) + (part[2] + part[3]);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < kNormPieces; ++i) {
        const int c = threadIdx.x + i * 256;
        if (c < nch) {
            float f[8], gg[8];
            widen8(xv[i], f);
            widen8(gv[i], gg);
            u32x4 o;
            o.x = pack2(f[0] * r * gg[0], f[1] * r * gg[1]);
            o.y = pack2(f[2] * r * gg[2], f[3] * r * gg[3]);
            o.z = pack2(f[4] * r * gg[4], f[5] * r * gg[5]);
            o.w = pack2(f[6] * r * gg[6], f[7] * r * gg[7]);
            a[frag_piece(row, c, S)] = o;
        }
    }
}

// One wavefront per (U column blocks of 32 outputs, split of the reduction, row tile of NB
// blocks): every activation fragment it loads feeds U MFMAs, every weight fragment NB.
template <int NB, int U>
__global__ __launch_bounds__(256, 2) void proj_kernel(const u32x4* __restrict__ A,
                                                   const u32x4* __restrict__ W, float* __restrict__ out,
                                                   int S, int CB, int splits, int n_rt, int n_out,
                                                   int64_t split_stride) {
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int CG = CB / U;  // column groups (host-checked: U divides CB)
    if (w >= CG * splits * n_rt) return;
    const int cg = w % CG, sp = (w / CG) % splits, rt = w / (CG * splits);
    const int SS = S / splits;  // a multiple of 8 (host-checked)
    const u32x4* wp = W + ((size_t)cg * U * S + (size_t)sp * SS) * 64 + lane;
    const u32x4* ap = A + ((size_t)rt * NB * S + (size_t)sp * SS) * 64 + lane;
    constexpr int C = U == 1 ? 4 : 2;
    f32x16 acc[U][NB];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[u][b][r] = 0.f;
    u32x4 w0[C][U], w1[C][U], a0[C][NB], a1[C][NB];
    auto load = [&](u32x4(&wb)[C][U], u32x4(&ab)[C][NB], int s) {
#pragma unroll
        for (int j = 0; j < C; ++j) {
#pragma unroll
            for (int u = 0; u < U; ++u) wb[j][u] = wp[((size_t)u * S + s + j) * 64];
#pragma unroll
            for (int b = 0; b < NB; ++b) ab[j][b] = ap[((size_t)b * S + s + j) * 64];
        }
    };
    auto mac = [&](const u32x4(&wb)[C][U], const u32x4(&ab)[C][NB]) {
#pragma unroll
        for (int j = 0; j < C; ++j)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int u = 0; u < U; ++u)
                    acc[u][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ab[j][b]), as_bf16x8(wb[j][u]),
                                                                        acc[u][b], 0, 0, 0);
    };
    load(w0, a0, 0);
    for (int s = 0; s < SS; s += 2 * C) {
        load(w1, a1, s + C);
        mac(w0, a0);
        if (s + 2 * C < SS) load(w0, a0, s + 2 * C);
        mac(w1, a1);
    }
    float* o = out + (size_t)sp * split_stride;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int col = (cg * U + u) * 32 + (lane & 31);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const size_t row = (size_t)(rt * NB + b) * kRowBlk + 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
                o[row * n_out + col] = acc[u][b][r];
            }
    }
}

// One thread per rotated pair of q or k, or per element of v, of one sequence.
__global__ __launch_bounds__(256) void qkv_finish_kernel(const float* __restrict__ part, int splits,
                                                         int64_t split_stride, Dims dm, GroupTab tab,
                                                         const double* __restrict__ inv_freq,
                                                         float* __restrict__ q) {
    const int row_g = blockIdx.y, hd = dm.hd, half = hd / 2;
    const int bt = find_batch(tab, row_g);
    const int s = row_g - tab.row0[bt], n_seq = tab.row0[bt + 1] - tab.row0[bt], pos = tab.pos[bt];
    uint16_t* kc = (uint16_t*)tab.kc[bt];
    uint16_t* vc = (uint16_t*)tab.vc[bt];
    uint16_t* new_rows = (uint16_t*)tab.new_rows[bt];
    const int dq = dm.Hq * hd, dkv = dm.Hkv * hd, n_out = dq + 2 * dkv;
    const int n_pairs = (dm.Hq + dm.Hkv) * half;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_pairs + dkv) return;
    const float* row = part + (size_t)row_g * n_out;
    auto total = [&](int col) {
        float a = 0.f;
        for (int sp = 0; sp < splits; ++sp) a += row[(size_t)sp * split_stride + col];
        return a;
    };
    if (i < n_pairs) {
        const int h = i / half, j = i % half;  // heads 0..Hq-1 are q, then k
        const float a = total(h * hd + j), b = total(h * hd + j + half);
        // angle reduced to [-pi, pi] in double, sine and cosine of the remainder in single
        const double ang = (double)pos * inv_freq[j];
        const double turns = rint(ang * 0.15915494309189535);
        const float red = (float)(ang - turns * 6.283185307179586);
        float sf, c;
        sincosf(red, &sf, &c);
        const float r0 = a * c - b * sf, r1 = b * c + a * sf;
        if (h < dm.Hq) {
            // 1/sqrt(hd) and log2(e) folded in: the attention kernel works with base-2 exponentials
            const float qscale = 1.4426950408889634f / sqrtf((float)hd);
            q[((size_t)row_g * dm.Hq + h) * hd + j] = r0 * qscale;
            q[((size_t)row_g * dm.Hq + h) * hd + j + half] = r1 * qscale;
        } else {
            const int hk = h - dm.Hq;
            const uint16_t b0 = (uint16_t)bf_bits(r0), b1 = (uint16_t)bf_bits(r1);
            uint16_t* dst = kc + (((size_t)s * dm.Hkv + hk) * dm.max_len + pos) * hd;
            dst[j] = b0;
            dst[j + half] = b1;
            if (new_rows != nullptr) {
                uint16_t* nr = new_rows + ((size_t)s * dm.Hkv + hk) * hd;
                nr[j] = b0;
                nr[j + half] = b1;
            }
        }
    } else {
        const int e = i - n_pairs, hk = e / hd, j = e % hd;
        const uint16_t b = (uint16_t)bf_bits(total(dq + dkv + e));
        vc[(((size_t)s * dm.Hkv + hk) * dm.max_len + pos) * hd + j] = b;
        if (new_rows != nullptr) new_rows[((size_t)(n_seq + s) * dm.Hkv + hk) * hd + j] = b;
    }
}

// Sum over the LPR (4, 8 or 16) consecutive lanes that share a row, by data-parallel-primitive
// adds: lane pairs, quad halves, then the mirrored half row and the mirrored row (after the
// first two steps every quad holds one value, so a mirror acts as the xor exchange).
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, false));
    };
    v += dpp(v, std::integral_constant<int, 0xB1>{});                  // quad_perm [1,0,3,2]
    v += dpp(v, std::integral_constant<int, 0x4E>{});                  // quad_perm [2,3,0,1]
    if (LPR > 4) v += dpp(v, std::integral_constant<int, 0x141>{});    // row_half_mirror
    if (LPR > 8) v += dpp(v, std::integral_constant<int, 0x140>{});    // row_mirror
    return v;
}

struct Soft {  // running softmax (base 2) of one (query head, 8-element slice)
    float m, l, acc[8];
};
__device__ __forceinline__ void merge(Soft& a, float m2, float l2, const float (&acc2)[8]) {
    const float mn = fmaxf(a.m, m2);
    const float sa = __builtin_amdgcn_exp2f(a.m - mn), sb = __builtin_amdgcn_exp2f(m2 - mn);
    a.l = a.l * sa + l2 * sb;
#pragma unroll
    for (int j = 0; j < 8; ++j) a.acc[j] = a.acc[j] * sa + acc2[j] * sb;
    a.m = mn;
}

constexpr float kEmpty = -1.0e30f;  // finite stand-in for "no position seen yet"

// One workgroup (4 wavefronts, four workgroups per compute unit) per (sequence, key-value head); G query heads share the rows.
// A row of HD elements is read by HD/8 lanes (16 bytes each); a wavefront covers 512/HD rows per
// load, issues the K and V loads of kChunk such row groups together, and keeps one running
// softmax per row slot (rescaled once per chunk), merged at the end.
constexpr int kAttnWaves = 4, kChunk = 2;
template <int HD, int G>
__global__ __launch_bounds__(kAttnWaves * 64, 4) void attn_decode_kernel(const float* __restrict__ q,
                                                                     Dims dm, GroupTab tab,
                                                                     u32x4* __restrict__ o_frag) {
    constexpr int LPR = HD / 8, RPW = 64 / LPR;
    __shared__ float sm[kAttnWaves][G * LPR][10];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row_g = blockIdx.x / dm.Hkv, hk = blockIdx.x % dm.Hkv;
    const int bt = find_batch(tab, row_g);
    const int s = row_g - tab.row0[bt], pos = tab.pos[bt];
    const int sub = lane % LPR, slot = lane / LPR;
    float qr[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int j = 0; j < 8; ++j) qr[g][j] = q[((size_t)row_g * dm.Hq + hk * G + g) * HD + sub * 8 + j];
    const size_t base = ((size_t)s * dm.Hkv + hk) * dm.max_len * LPR + sub;
    const u32x4* K = (const u32x4*)tab.kc[bt] + base;
    const u32x4* V = (const u32x4*)tab.vc[bt] + base;
    Soft st[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        st[g].m = kEmpty;
        st[g].l = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) st[g].acc[j] = 0.f;
    }
    for (int p0 = wave * RPW * kChunk; p0 <= pos; p0 += kAttnWaves * RPW * kChunk) {
        u32x4 kraw[kChunk], vraw[kChunk];
        bool valid[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) {
            const int p = p0 + c * RPW + slot;
            valid[c] = p <= pos;
            const int pc = valid[c] ? p : pos;
            kraw[c] = __builtin_nontemporal_load(K + (size_t)pc * LPR);
            vraw[c] = __builtin_nontemporal_load(V + (size_t)pc * LPR);
        }
        float sc[G][kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) {
            float kf[8];
            widen8(kraw[c], kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) dot = __builtin_fmaf(qr[g][j], kf[j], dot);
                dot = row_sum<LPR>(dot);
                sc[g][c] = valid[c] ? dot : kEmpty;
            }
        }
        float pr[G][kChunk];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mn = st[g].m;
#pragma unroll
            for (int c = 0; c < kChunk; ++c) mn = fmaxf(mn, sc[g][c]);
            const float sa = __builtin_amdgcn_exp2f(st[g].m - mn);
            float add = 0.f;
#pragma unroll
            for (int c = 0; c < kChunk; ++c) {
                pr[g][c] = valid[c] ? __builtin_amdgcn_exp2f(sc[g][c] - mn) : 0.f;
                add += pr[g][c];
            }
            st[g].l = st[g].l * sa + add;
            st[g].m = mn;
#pragma unroll
            for (int j = 0; j < 8; ++j) st[g].acc[j] *= sa;
        }
#pragma unroll
        for (int c = 0; c < kChunk; ++c) {
            float vf[8];
            widen8(vraw[c], vf);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int j = 0; j < 8; ++j) st[g].acc[j] = __builtin_fmaf(pr[g][c], vf[j], st[g].acc[j]);
        }
    }
    // row slots of the wavefront
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m2 = __shfl_xor(st[g].m, off, 64), l2 = __shfl_xor(st[g].l, off, 64);
            float a2[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a2[j] = __shfl_xor(st[g].acc[j], off, 64);
            merge(st[g], m2, l2, a2);
        }
    }
    if (slot == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float* e = sm[wave][g * LPR + sub];
            e[0] = st[g].m;
            e[1] = st[g].l;
#pragma unroll
            for (int j = 0; j < 8; ++j) e[2 + j] = st[g].acc[j];
        }
    }
    __syncthreads();
    if (threadIdx.x < G * LPR) {
        const int g = threadIdx.x / LPR, sb = threadIdx.x % LPR;
        Soft t;
        t.m = kEmpty;
        t.l = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) t.acc[j] = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float* e = sm[w][threadIdx.x];
            float a2[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a2[j] = e[2 + j];
            merge(t, e[0], e[1], a2);
        }
        const float inv = 1.0f / t.l;  // position pos is always valid, so l > 0
        u32x4 o;
        o.x = pack2(t.acc[0] * inv, t.acc[1] * inv);
        o.y = pack2(t.acc[2] * inv, t.acc[3] * inv);
        o.z = pack2(t.acc[4] * inv, t.acc[5] * inv);
        o.w = pack2(t.acc[6] * inv, t.acc[7] * inv);
        const int chunk = ((hk * G + g) * HD) / 8 + sb;
        o_frag[frag_piece(row_g, chunk, dm.Hq * HD / 16)] = o;
    }
}

__global__ __launch_bounds__(256) void out_finish_kernel(const float* __restrict__ part, int splits,
                                                         int64_t split_stride, GroupTab tab, int d) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // 8 consecutive elements
    const int nch = d / 8;
    if (i >= (size_t)tab.row0[tab.n] * nch) return;
    const int row = (int)(i / nch), bt = find_batch(tab, row);
    const size_t at = (size_t)(row - tab.row0[bt]) * nch + i % nch;
    float f[8];
    widen8(((const u32x4*)tab.h_in[bt])[at], f);
    for (int sp = 0; sp < splits; ++sp) {
        const float4* p = reinterpret_cast<const float4*>(part + (size_t)sp * split_stride + i * 8);
        const float4 a = p[0], b = p[1];
        f[0] += a.x; f[1] += a.y; f[2] += a.z; f[3] += a.w;
        f[4] += b.x; f[5] += b.y; f[6] += b.z; f[7] += b.w;
    }
    u32x4 o;
    o.x = pack2(f[0], f[1]);
    o.y = pack2(f[2], f[3]);
    o.z = pack2(f[4], f[5]);
    o.w = pack2(f[6], f[7]);
    ((u32x4*)tab.h_out[bt])[at] = o;
}

}  // namespace

void launch_pack_weight(hipStream_t st, const void* w, int rows, int K, void* out) {
    const size_t pieces = (size_t)rows * K / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st,
                       (const u32x4*)w, rows, K, (u32x4*)out);
}

void launch_rmsnorm(hipStream_t st, const GroupTab& tab, const void* g, int d, float eps, void* a_frag) {
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(tab.row0[tab.n]), dim3(256), 0, st, tab, (const u32x4*)g, d, eps,
                       (u32x4*)a_frag);
}

int pick_row_tile(int row_blocks) { return row_blocks >= 3 ? 4 : row_blocks == 2 ? 2 : 1; }

// Column blocks per wavefront: two once a row tile is full (128 rows), where the activation
// fragments re-read from L2 are what the kernel moves most of.
static int pick_col_units(int row_blocks, int n_out) { return row_blocks >= 4 && (n_out / 32) % 2 == 0 ? 2 : 1; }

int pick_splits(int row_blocks, int K, int n_out) {
    const int U = pick_col_units(row_blocks, n_out);
    const int S = K / 16, CG = n_out / 32 / U;
    const int nb = pick_row_tile(row_blocks), n_rt = (row_blocks + nb - 1) / nb;
    int splits = 1;
    while (splits < kMaxSplit && CG * n_rt * splits < (U == 2 ? 768 : 1024) && S % (splits * 2 * 8) == 0) splits *= 2;
    return splits;
}

void launch_proj(hipStream_t st, const void* a_frag, const void* w_frag, int row_blocks, int K,
                 int n_out, int splits, float* out, int64_t split_stride) {
    const int S = K / 16, CB = n_out / 32;
    const int nb = pick_row_tile(row_blocks), n_rt = (row_blocks + nb - 1) / nb;
    const int U = pick_col_units(row_blocks, n_out);
    const int waves = CB / U * splits * n_rt;
    const dim3 grid((waves + 3) / 4), block(256);
    const u32x4* A = (const u32x4*)a_frag;
    const u32x4* W = (const u32x4*)w_frag;
    if (nb == 4 && U == 2)
        hipLaunchKernelGGL((proj_kernel<4, 2>), grid, block, 0, st, A, W, out, S, CB, splits, n_rt, n_out, split_stride);
    else if (nb == 4)
        hipLaunchKernelGGL((proj_kernel<4, 1>), grid, block, 0, st, A, W, out, S, CB, splits, n_rt, n_out, split_stride);
    else if (nb == 2)
        hipLaunchKernelGGL((proj_kernel<2, 1>), grid, block, 0, st, A, W, out, S, CB, splits, n_rt, n_out, split_stride);
    else
        hipLaunchKernelGGL((proj_kernel<1, 1>), grid, block, 0, st, A, W, out, S, CB, splits, n_rt, n_out, split_stride);
}

void launch_qkv_finish(hipStream_t st, const float* part, int splits, int64_t split_stride,
                       const Dims& dm, const GroupTab& tab, const double* inv_freq, float* q) {
    const int items = (dm.Hq + dm.Hkv) * (dm.hd / 2) + dm.Hkv * dm.hd;
    hipLaunchKernelGGL(qkv_finish_kernel, dim3((items + 255) / 256, tab.row0[tab.n]), dim3(256), 0, st, part,
                       splits, split_stride, dm, tab, inv_freq, q);
}

template <int HD>
static int launch_attention_hd(hipStream_t st, const float* q, const Dims& dm, const GroupTab& tab,
                               void* o_frag) {
    const dim3 grid(tab.row0[tab.n] * dm.Hkv), block(kAttnWaves * 64);
    u32x4* O = (u32x4*)o_frag;
    switch (dm.Hq / dm.Hkv) {
#define KATTN_CASE(G) \
    case G: hipLaunchKernelGGL((attn_decode_kernel<HD, G>), grid, block, 0, st, q, dm, tab, O); return 0;
        KATTN_CASE(1) KATTN_CASE(2) KATTN_CASE(3) KATTN_CASE(4) KATTN_CASE(5) KATTN_CASE(6) KATTN_CASE(7) KATTN_CASE(8)
#undef KATTN_CASE
    }
    return -1;
}

int launch_attention(hipStream_t st, const float* q, const Dims& dm, const GroupTab& tab, void* o_frag) {
    switch (dm.hd) {
        case 32: return launch_attention_hd<32>(st, q, dm, tab, o_frag);
        case 64: return launch_attention_hd<64>(st, q, dm, tab, o_frag);
        case 128: return launch_attention_hd<128>(st, q, dm, tab, o_frag);
    }
    return -1;
}

void launch_out_finish(hipStream_t st, const float* part, int splits, int64_t split_stride,
                       const GroupTab& tab, int d) {
    const size_t n = (size_t)tab.row0[tab.n] * d / 8;
    hipLaunchKernelGGL(out_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, splits,
                       split_stride, tab, d);
}

}  // namespace kattn
