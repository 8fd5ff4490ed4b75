// Grouped SwiGLU expert FFN on bf16 MFMA (v_mfma_f32_16x16x32_bf16), fp32 accumulate.
//
// Every expert is an FFN evaluated once over all of its tokens from all batches of the batch
// group, experts in execution order (paper Section 2.1 and Section 5).  Two launches:
//   up  : H = silu(X W1^T) .* (X W3^T)   reduction over d, H stored as bf16 in fragment order
//   down: O = H W2^T                      reduction over f, fp32, optional split-K partials
//
// Work split.  A tile is one expert x up to 16 row blocks of 16 tokens.  A workgroup takes a
// tile and WAVES output units; a wavefront owns one unit -- 16 features of W1 and the same 16
// of W3 (up), or 32 output columns of W2 (down) -- for all rows of the tile, so every weight
// byte is fetched from HBM once per tile.  Weights are pre-packed so that a wavefront's stream
// is one contiguous run of 1 KiB fragments (two per 32-deep reduction step), read straight
// into registers through a PD-stage software prefetch ring.  The activations of the tile are
// staged through LDS, double buffered, in the same fragment order, so LDS reads are one
// conflict-free 16-byte read per lane.  The workgroup -> tile map deals consecutive tiles of
// one expert to the same XCD so that the expert's activations stay in that XCD's L2.
#include "kernels.h"

namespace kmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte unit as a first-class value
typedef const __attribute__((address_space(1))) u32x4* gptr;  // global (HBM) address space

constexpr int kXcd = 8;
constexpr int kBlkStageUnits = 128;  // 16-byte units of one row block per LDS stage (SK * PL = 2)
constexpr int kLdsUnits = 2 * kTileBlks * kBlkStageUnits;
constexpr int kLdsBytes = kLdsUnits * 16;  // 64 KiB, double buffered

__device__ __forceinline__ gptr as_global(const void* p) { return (gptr)(uintptr_t)p; }

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t bf16_bits_rne(float v) {
    uint32_t a = __float_as_uint(v);
    a += 0x7fffu + ((a >> 16) & 1u);
    return a >> 16;
}

// A stage of the reduction loop covers SK steps of 32 for PL planes of the activations
// (SK * PL == 2): SK = 2, PL = 1 normally; SK = 1, PL = 2 when H is carried as a bf16 pair
// (high part + rounding remainder) through the down projection.
struct TileCtx {
    gptr wbase;     // this wavefront's weight stream (+lane), 128 units per reduction step
    gptr actbase;   // packed activations at the tile's first row block (plane 0)
    size_t plane;   // units between activation planes
    u32x4* lds;
    int nks;        // reduction steps of 32
    int s0, s1;     // stage range of this workgroup
    int nblk;       // live row blocks of the tile
    bool active;    // wavefront owns a real unit
};

template <int SK>
__device__ __forceinline__ void load_w(const TileCtx& c, u32x4 (&dst)[SK][2], int stage) {
#pragma unroll
    for (int ks = 0; ks < SK; ++ks) {
        gptr q = c.wbase + (size_t)(stage * SK + ks) * 128;
        dst[ks][0] = q[0];
        dst[ks][1] = q[64];
    }
}

// Unit u of a stage is (row block b, plane pl, step ks, lane): u = ((b*PL + pl)*SK + ks)*64 + lane.
template <int PASSES, int T, int SK, int PL>
__device__ __forceinline__ void load_x(const TileCtx& c, u32x4 (&xr)[PASSES], int stage) {
    const int live_units = c.nblk * kBlkStageUnits;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        int u = (int)threadIdx.x + p * T;
        u = u < live_units ? u : 0;  // out-of-tile lanes re-read unit 0 (in bounds, not stored)
        const int b = u / kBlkStageUnits, r = u % kBlkStageUnits;
        const int pl = PL == 1 ? 0 : r / (SK * 64);
        const int w = r % (SK * 64);  // ks*64 + lane
        xr[p] = c.actbase[(size_t)pl * c.plane + ((size_t)b * c.nks + (size_t)stage * SK) * 64 + w];
    }
}

template <int PASSES, int T>
__device__ __forceinline__ void store_x(const TileCtx& c, const u32x4 (&xr)[PASSES], int buf) {
    const int live_units = c.nblk * kBlkStageUnits;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int u = (int)threadIdx.x + p * T;
        if (u < live_units) c.lds[buf * (kLdsUnits / 2) + u] = xr[p];
    }
}

template <int MODE, int NB, int WAVES, int PD, int SK, int PL>
__device__ __forceinline__ void ffn_tile(const TileCtx& c, f32x4 (&acc0)[NB], f32x4 (&acc1)[NB]) {
    static_assert(SK * PL == 2 && PD % 2 == 0, "stage geometry");
    constexpr int T = WAVES * 64;
    constexpr int UNITS = NB * kBlkStageUnits;
    constexpr int PASSES = (UNITS + T - 1) / T;
    const int lane = threadIdx.x & 63;

    u32x4 wr[PD][SK][2];
    u32x4 xr[PASSES];

#pragma unroll
    for (int b = 0; b < NB; ++b) {
        acc0[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // prologue: fill the weight ring, stage the first activations
    if (c.active) {
#pragma unroll
        for (int u = 0; u < PD; ++u)
            if (c.s0 + u < c.s1) load_w<SK>(c, wr[u], c.s0 + u);
    }
    load_x<PASSES, T, SK, PL>(c, xr, c.s0);
    store_x<PASSES, T>(c, xr, 0);
    __syncthreads();

    for (int s = c.s0; s < c.s1; s += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int cur = s + u;
            if (cur < c.s1) {  // uniform over the workgroup
                const int buf = u & 1;  // PD is even and s - s0 is a multiple of PD
                const bool more = cur + 1 < c.s1;
                if (more) load_x<PASSES, T, SK, PL>(c, xr, cur + 1);
                if (c.active) {
                    const u32x4* L = c.lds + buf * (kLdsUnits / 2) + lane;
#pragma unroll
                    for (int ks = 0; ks < SK; ++ks) {
                        const bf16x8 wa = as_bf16x8(wr[u][ks][0]);
                        const bf16x8 wb = as_bf16x8(wr[u][ks][1]);
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
#pragma unroll
                            for (int pl = 0; pl < PL; ++pl) {
                                const bf16x8 xa = as_bf16x8(L[((b * PL + pl) * SK + ks) * 64]);
                                if (MODE == 0) {  // rows = features, cols = tokens
                                    acc0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, xa, acc0[b], 0, 0, 0);
                                    acc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, xa, acc1[b], 0, 0, 0);
                                } else {  // rows = tokens, cols = output columns
                                    acc0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wa, acc0[b], 0, 0, 0);
                                    acc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wb, acc1[b], 0, 0, 0);
                                }
                            }
                        }
                    }
                    if (cur + PD < c.s1) load_w<SK>(c, wr[u], cur + PD);
                }
                if (more) store_x<PASSES, T>(c, xr, buf ^ 1);
                __syncthreads();
            }
        }
    }
}

struct Wg {
    int tile, grp, sp;
    bool live;
};

// XCD-aware map from the hardware workgroup id (dealt round-robin to the 8 XCDs) to a logical
// id such that each XCD walks a contiguous range of (tile, split, group) items.
__device__ __forceinline__ Wg locate(const FfnArgs& a, int n_groups, int split) {
    Wg w;
    const int ntile = *a.tile_count;
    const int per_tile = n_groups * split;
    const int live = ntile * per_tile;
    const int per_xcd = (live + kXcd - 1) / kXcd;
    const int id = blockIdx.x;
    const int seq = id / kXcd;
    const int L = (id % kXcd) * per_xcd + seq;
    w.live = seq < per_xcd && L < live;
    w.tile = (a.tile_first ? *a.tile_first : 0) + L / per_tile;
    const int r = L % per_tile;
    w.sp = r / n_groups;
    w.grp = r % n_groups;
    return w;
}

// Up projections + SwiGLU.  The accumulator of lane (token j = lane & 15, group g = lane >> 4)
// holds features 16*unit + 4g + r, r = 0..3: exactly half of the lane's 16-byte unit in the
// fragment order of the down projection, so H is written with one 8-byte store per row block.
template <int NB, int WAVES, int PD>
__device__ __forceinline__ void up_tile(const FfnArgs& a, const TileCtx& c, int unit, int hblk0) {
    f32x4 g[NB], u[NB];
    ffn_tile<0, NB, WAVES, PD, 2, 1>(c, g, u);
    if (!c.active) return;
    const int lane = threadIdx.x & 63;
    uint2* hp = reinterpret_cast<uint2*>(a.out);
    const size_t ksteps_h = (size_t)a.f / 32;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < c.nblk) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float gv = g[b][r];
                const float h = gv / (1.f + __expf(-gv)) * u[b][r];
                hi[r] = bf16_bits_rne(h);
                lo[r] = bf16_bits_rne(h - __uint_as_float(hi[r] << 16));
            }
            const size_t unit16 = ((size_t)(hblk0 + b) * ksteps_h + (size_t)(unit >> 1)) * 64 + lane;
            hp[unit16 * 2 + (unit & 1)] = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
            if (a.h_planes == 2)
                hp[(unit16 + (size_t)a.h_plane_units) * 2 + (unit & 1)] =
                    make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
        }
    }
}

template <int NB, int WAVES, int PD, int PL>
__device__ __forceinline__ void down_tile(const FfnArgs& a, const TileCtx& c, int unit, int hblk0,
                                          int sp) {
    f32x4 p0[NB], p1[NB];
    ffn_tile<1, NB, WAVES, PD, 2 / PL, PL>(c, p0, p1);
    if (!c.active) return;
    const int lane = threadIdx.x & 63;
    float* o = reinterpret_cast<float*>(a.out) + (size_t)sp * a.o_split_stride;
    const int col = unit * 32 + (lane & 15);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < c.nblk) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const size_t row = (size_t)(hblk0 + b) * kRowBlk + 4 * (lane >> 4) + r;
                o[row * a.d + col] = p0[b][r];
                o[row * a.d + col + 16] = p1[b][r];
            }
        }
    }
}

#define NB_SWITCH(CALL)                       \
    if (nblk <= 1) { CALL(1); }               \
    else if (nblk <= 2) { CALL(2); }          \
    else if (nblk <= 4) { CALL(4); }          \
    else if (nblk <= 6) { CALL(6); }          \
    else if (nblk <= 8) { CALL(8); }          \
    else if (nblk <= 10) { CALL(10); }        \
    else if (nblk <= 12) { CALL(12); }        \
    else { CALL(16); }

template <int WAVES, int PD>
__global__ __launch_bounds__(WAVES * 64) void ffn_up_kernel(FfnArgs a, int n_groups) {
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, 1);
    if (!w.live) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = a.w_single ? a.w_single : a.wtab[e];
    const int unit = w.grp * WAVES + wave;
    TileCtx c;
    c.nks = a.d / 32;
    c.active = unit < a.f / 16;
    c.wbase = as_global(blob) + (size_t)unit * c.nks * 128 + lane;
    c.actbase = as_global(a.act) + (size_t)a.tile_xblk[w.tile] * c.nks * 64;
    c.plane = 0;
    c.lds = lds;
    c.s0 = 0;
    c.s1 = c.nks / 2;
    c.nblk = nblk;
#define CALL(NB) up_tile<NB, WAVES, PD>(a, c, unit, hblk0)
    NB_SWITCH(CALL)
#undef CALL
}

template <int WAVES, int PD, int PL>
__global__ __launch_bounds__(WAVES * 64) void ffn_down_kernel(FfnArgs a, int n_groups) {
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, a.split_k);
    if (!w.live) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = a.w_single ? a.w_single : a.wtab[e];
    const int unit = w.grp * WAVES + wave;
    TileCtx c;
    c.nks = a.f / 32;
    c.active = unit < a.d / 32;
    c.wbase = as_global(blob + (size_t)a.d * a.f * 4) + (size_t)unit * c.nks * 128 + lane;
    c.actbase = as_global(a.act) + (size_t)hblk0 * c.nks * 64;
    c.plane = (size_t)a.h_plane_units;
    c.lds = lds;
    const int nstage = c.nks / (2 / PL);
    c.s0 = (int)((long long)w.sp * nstage / a.split_k);
    c.s1 = (int)((long long)(w.sp + 1) * nstage / a.split_k);
    c.nblk = nblk;
#define CALL(NB) down_tile<NB, WAVES, PD, PL>(a, c, unit, hblk0, w.sp)
    NB_SWITCH(CALL)
#undef CALL
}

template <int WAVES, int PD>
void launch_up(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.f / 16 + WAVES - 1) / WAVES;
    const int grid = (a.max_tiles * n_groups + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_up_kernel<WAVES, PD>), dim3(grid), dim3(WAVES * 64), kLdsBytes, st, a,
                       n_groups);
}

template <int WAVES, int PD, int PL>
void launch_down(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.d / 32 + WAVES - 1) / WAVES;
    const int grid = (a.max_tiles * n_groups * a.split_k + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_down_kernel<WAVES, PD, PL>), dim3(grid), dim3(WAVES * 64), kLdsBytes,
                       st, a, n_groups);
}

template <typename K>
hipError_t allow_lds(K kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

}  // namespace

int ffn_configure() {
    hipError_t e = allow_lds(&ffn_up_kernel<8, 2>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<8, 2, 1>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<8, 4, 2>);
    return (int)e;
}

void launch_ffn_up_bf16(hipStream_t st, const FfnArgs& a) { launch_up<8, 2>(st, a); }

void launch_ffn_down_bf16(hipStream_t st, const FfnArgs& a) {
    if (a.h_planes == 2)
        launch_down<8, 4, 2>(st, a);
    else
        launch_down<8, 2, 1>(st, a);
}

}  // namespace kmoe
