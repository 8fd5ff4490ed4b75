// Grouped SwiGLU expert FFN on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// Every expert is an FFN evaluated once over all of its tokens from all batches of the batch
// group, experts in execution order (paper Section 2.1 and Section 5).  Two launches:
//   up  : H = silu(X W1^T) .* (X W3^T)   reduction over d, H stored as bf16 in fragment order
//   down: O = H W2^T                      reduction over f, fp32, optional split-K partials
//
// Work split.  A tile is one expert x up to 8 row blocks of 32 tokens.  A workgroup takes a tile
// and WAVES output units; a wavefront owns one unit for all rows of the tile, so every weight
// byte is fetched from HBM once per tile.  An up unit is 16 features: its weight fragment
// stacks the 16 rows of W1 on the 16 rows of W3, so one 32x32x16 MFMA yields the gate and the up
// value of the same feature in the same lane and SwiGLU needs no data movement.  A down unit is
// 32 output columns of W2.  Weights are pre-packed so that a wavefront's stream is one
// contiguous run of 1 KiB fragments (one per 16-deep reduction step), read straight into
// registers through a software prefetch ring.  The activations of the tile are staged through
// LDS, double buffered, in the same fragment order, so LDS reads are one conflict-free 16-byte
// read per lane.  The workgroup -> tile map deals consecutive tiles of one expert to the same
// XCD so that the expert's activations stay in that XCD's L2.
#include "kernels.h"

namespace kmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte unit as a first-class value
typedef const __attribute__((address_space(1))) u32x4* gptr;  // global (HBM) address space

constexpr int kXcd = 8;
constexpr int kFragsPerBlk = 8;  // fragments of one row block in one LDS stage
constexpr int kBlkStageUnits = kFragsPerBlk * 64;  // 16-byte units of one row block per stage
constexpr int kBufUnits = kTileBlks * kBlkStageUnits;
constexpr int kLdsBytes = 2 * kBufUnits * 16;  // 128 KiB, double buffered

__device__ __forceinline__ gptr as_global(const void* p) { return (gptr)(uintptr_t)p; }

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t bf16_bits_rne(float v) {
    uint32_t a = __float_as_uint(v);
    a += 0x7fffu + ((a >> 16) & 1u);
    return a >> 16;
}

// One LDS stage holds, per row block, SX reduction steps of 16 for PL planes of the activations
// (SX * PL == 8): SX = 8, PL = 1 normally; SX = 4, PL = 2 when H is carried as a bf16 pair
// (value + rounding remainder) through the down projection.  The weight ring in registers is
// SX steps deep, one slot per step of the stage.  The activation loads of the next stage are
// issued before any weight load of this stage, so by the time they are waited for (end of the
// stage) every older load in the in-order memory counter has long been consumed: waiting for
// the activations never forces a weight prefetch to complete early.
struct TileCtx {
    gptr wbase;     // this wavefront's weight stream (+lane), 64 units per reduction step
    gptr actbase;   // packed activations at the tile's first row block (plane 0)
    size_t plane;   // units between activation planes
    u32x4* lds;
    int nks;        // reduction steps of 16 in the whole reduction
    int k0, k1;     // reduction steps of this workgroup: [k0, k1), k0 a multiple of SX
    int nblk;       // live row blocks of the tile
    bool active;    // wavefront owns a real unit
};

// Unit u of a stage is (row block b, plane pl, step j, lane): u = ((b*PL + pl)*SX + j)*64 + lane.
// Lanes past the live part of the tile re-read unit 0, steps past the end of the reduction
// re-read the last step: both in bounds, and what is then stored lands in LDS slots that no
// live MFMA reads.
template <int PASSES, int T, int SX, int PL>
__device__ __forceinline__ void load_x(const TileCtx& c, u32x4 (&xr)[PASSES], int kbase) {
    const int live_units = c.nblk * kBlkStageUnits;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        int u = (int)threadIdx.x + p * T;
        u = u < live_units ? u : 0;
        const int b = u / kBlkStageUnits, r = u % kBlkStageUnits;
        const int pl = r / (SX * 64);
        const int j = (r / 64) % SX;
        const int ks = min(kbase + j, c.nks - 1);
        xr[p] = c.actbase[(size_t)pl * c.plane + ((size_t)b * c.nks + ks) * 64 + (r & 63)];
    }
}

// When PASSES * T fits one LDS buffer the stores need no guard.
template <int PASSES, int T>
__device__ __forceinline__ void store_x(const TileCtx& c, const u32x4 (&xr)[PASSES], int buf) {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int u = (int)threadIdx.x + p * T;
        if (PASSES * T <= kBufUnits || u < kBufUnits) c.lds[buf * kBufUnits + u] = xr[p];
    }
}

// MFMAs of one reduction step: NB*PL fragments read from LDS through a rolling window of D
// registers, so that D reads are in flight ahead of the matrix core; the interleaving is
// pinned with scheduling groups (D reads, then one read per MFMA).
template <int MODE, int NB, int SX, int PL, int D>
__device__ __forceinline__ void step_mfma(const u32x4* L, int j, const u32x4 w, f32x16 (&acc)[NB]) {
    constexpr int NF = NB * PL;
    constexpr int DD = D < NF ? D : NF;
    u32x4 win[DD];
    const bf16x8 wf = as_bf16x8(w);
#pragma unroll
    for (int i = 0; i < DD; ++i) win[i] = L[(i * SX + j) * 64];  // fragment i = (b, pl) = i/PL, i%PL
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int b = i / PL;
        const bf16x8 xa = as_bf16x8(win[i % DD]);
        if (MODE == 0)  // rows = 16 gate + 16 up features, cols = tokens
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xa, acc[b], 0, 0, 0);
        else  // rows = tokens, cols = output columns
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, wf, acc[b], 0, 0, 0);
        if (i + DD < NF) win[i % DD] = L[((i + DD) * SX + j) * 64];
    }
    __builtin_amdgcn_sched_group_barrier(0x100, DD, 0);
#pragma unroll
    for (int i = 0; i < NF - DD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, DD, 0);
}

template <int MODE, int NB, int WAVES, int SX, int PL>
__device__ __forceinline__ void ffn_tile(const TileCtx& c, f32x16 (&acc)[NB]) {
    static_assert(SX * PL == kFragsPerBlk, "stage geometry");
    constexpr int T = WAVES * 64;
    constexpr int UNITS = NB * kBlkStageUnits;
    constexpr int PASSES = (UNITS + T - 1) / T;
    constexpr int D = 3;
    // weight ring: RS stages of SX steps.  Small tiles leave registers for a ring of 16 steps
    // (16 KiB per wavefront in flight), full tiles get 8.
    constexpr int RS = (NB <= 5 ? 16 : 8) / SX;
    const int lane = threadIdx.x & 63;

    u32x4 wr[RS][SX];
    u32x4 xr[PASSES];

#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

    // prologue: stage the first activations, fill the weight ring
    load_x<PASSES, T, SX, PL>(c, xr, c.k0);
#pragma unroll
    for (int rs = 0; rs < RS; ++rs)
#pragma unroll
        for (int j = 0; j < SX; ++j)
            if (c.k0 + rs * SX + j < c.k1) wr[rs][j] = c.wbase[(size_t)(c.k0 + rs * SX + j) * 64];
    store_x<PASSES, T>(c, xr, 0);
    __syncthreads();

    int k = c.k0, buf = 0;
    // steady state: every stage of the group is complete, has a successor to stage and a slot to
    // reload, so the body is branch-free
    for (; k + 2 * RS * SX <= c.k1; k += RS * SX) {
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            const int kk = k + rs * SX;
            load_x<PASSES, T, SX, PL>(c, xr, kk + SX);
            __builtin_amdgcn_sched_barrier(0);
            const u32x4* L = c.lds + buf * kBufUnits + lane;
#pragma unroll
            for (int j = 0; j < SX; ++j) {
                step_mfma<MODE, NB, SX, PL, D>(L, j, wr[rs][j], acc);
                wr[rs][j] = c.wbase[(size_t)(kk + RS * SX + j) * 64];
                __builtin_amdgcn_sched_barrier(0);
            }
            store_x<PASSES, T>(c, xr, buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    // drain: the last stages, guarded step by step
    for (; k < c.k1; k += RS * SX) {
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            const int kk = k + rs * SX;
            if (kk < c.k1) {  // uniform over the workgroup
                const bool more = kk + SX < c.k1;
                if (more) load_x<PASSES, T, SX, PL>(c, xr, kk + SX);
                const u32x4* L = c.lds + buf * kBufUnits + lane;
#pragma unroll
                for (int j = 0; j < SX; ++j) {
                    if (kk + j < c.k1) {
                        step_mfma<MODE, NB, SX, PL, D>(L, j, wr[rs][j], acc);
                        if (kk + RS * SX + j < c.k1)
                            wr[rs][j] = c.wbase[(size_t)(kk + RS * SX + j) * 64];
                    }
                }
                if (more) store_x<PASSES, T>(c, xr, buf ^ 1);
                __syncthreads();
                buf ^= 1;
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

// Up projections + SwiGLU.  The accumulator of lane (token j = lane & 31, half hi = lane >> 5)
// holds, in register r < 8, the gate value of feature 16*unit + 8*(r/4) + 4*hi + r%4 and in
// register r + 8 the up value of the same feature: exactly the lane's 16-byte unit in the
// fragment order of the down projection, so H is written with one 16-byte store per row block.
template <int NB, int WAVES>
__device__ __forceinline__ void up_tile(const FfnArgs& a, const TileCtx& c, int unit, int hblk0) {
    f32x16 acc[NB];
    ffn_tile<0, NB, WAVES, 8, 1>(c, acc);
    if (!c.active) return;
    const int lane = threadIdx.x & 63;
    u32x4* hp = reinterpret_cast<u32x4*>(a.out);
    const size_t ksteps_h = (size_t)a.f / 16;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < c.nblk) {
            uint32_t hi[8], lo[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float gv = acc[b][r];
                const float h = gv / (1.f + __expf(-gv)) * acc[b][r + 8];
                hi[r] = bf16_bits_rne(h);
                lo[r] = bf16_bits_rne(h - __uint_as_float(hi[r] << 16));
            }
            const size_t at = ((size_t)(hblk0 + b) * ksteps_h + (size_t)unit) * 64 + lane;
            hp[at] = u32x4{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16),
                           hi[6] | (hi[7] << 16)};
            if (a.h_planes == 2)
                hp[at + (size_t)a.h_plane_units] =
                    u32x4{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16),
                          lo[6] | (lo[7] << 16)};
        }
    }
}

// Down projection: lane (column n = lane & 31, half hi) holds in register r the token row
// 8*(r/4) + 4*hi + r%4 of the row block.
template <int NB, int WAVES, int PL>
__device__ __forceinline__ void down_tile(const FfnArgs& a, const TileCtx& c, int unit, int hblk0,
                                          int sp) {
    f32x16 acc[NB];
    ffn_tile<1, NB, WAVES, 8 / PL, PL>(c, acc);
    if (!c.active) return;
    const int lane = threadIdx.x & 63;
    float* o = reinterpret_cast<float*>(a.out) + (size_t)sp * a.o_split_stride;
    const int col = unit * 32 + (lane & 31);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < c.nblk) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const size_t row = (size_t)(hblk0 + b) * kRowBlk + 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
                o[row * a.d + col] = acc[b][r];
            }
        }
    }
}

#define NB_SWITCH(CALL)                       \
    if (nblk <= 2) { CALL(2); }               \
    else if (nblk <= 4) { CALL(4); }          \
    else if (nblk <= 5) { CALL(5); }          \
    else if (nblk <= 6) { CALL(6); }          \
    else { CALL(8); }

template <int WAVES>
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
    c.nks = a.d / 16;
    c.active = unit < a.f / 16;
    const int wunit = c.active ? unit : a.f / 16 - 1;  // idle wavefronts shadow the last unit
    c.wbase = as_global(blob) + (size_t)wunit * c.nks * 64 + lane;
    c.actbase = as_global(a.act) + (size_t)a.tile_xblk[w.tile] * c.nks * 64;
    c.plane = 0;
    c.lds = lds;
    c.k0 = 0;
    c.k1 = c.nks;
    c.nblk = nblk;
#define CALL(NB) up_tile<NB, WAVES>(a, c, unit, hblk0)
    NB_SWITCH(CALL)
#undef CALL
}

template <int WAVES, int PL>
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
    c.nks = a.f / 16;
    c.active = unit < a.d / 32;
    const int wunit = c.active ? unit : a.d / 32 - 1;  // idle wavefronts shadow the last unit
    c.wbase = as_global(blob + (size_t)a.d * a.f * 4) + (size_t)wunit * c.nks * 64 + lane;
    c.actbase = as_global(a.act) + (size_t)hblk0 * c.nks * 64;
    c.plane = (size_t)a.h_plane_units;
    c.lds = lds;
    constexpr int SX = 8 / PL;
    const int nstage = (c.nks + SX - 1) / SX;
    c.k0 = (int)((long long)w.sp * nstage / a.split_k) * SX;
    c.k1 = min((int)((long long)(w.sp + 1) * nstage / a.split_k) * SX, c.nks);
    c.nblk = nblk;
#define CALL(NB) down_tile<NB, WAVES, PL>(a, c, unit, hblk0, w.sp)
    NB_SWITCH(CALL)
#undef CALL
}

template <int WAVES>
void launch_up(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.f / 16 + WAVES - 1) / WAVES;
    const int grid = (a.max_tiles * n_groups + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_up_kernel<WAVES>), dim3(grid), dim3(WAVES * 64), kLdsBytes, st, a,
                       n_groups);
}

template <int WAVES, int PL>
void launch_down(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.d / 32 + WAVES - 1) / WAVES;
    const int grid = (a.max_tiles * n_groups * a.split_k + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_down_kernel<WAVES, PL>), dim3(grid), dim3(WAVES * 64), kLdsBytes, st,
                       a, n_groups);
}

template <typename K>
hipError_t allow_lds(K kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

// 8 or 7 wavefronts per workgroup, whichever leaves the smaller idle tail in the last round
// of workgroups over the 256 compute units (one workgroup per unit at a time).
int pick_waves(int units, int64_t tiles_times_split, int variant) {
    if (variant == 1) return 8;
    if (variant == 2) return 7;
    double best = 0.0;
    int pick = 8;
    for (int w : {8, 7}) {
        const int64_t wgs = tiles_times_split * ((units + w - 1) / w);
        const int64_t rounds = (wgs + 255) / 256;
        const double busy = (double)units * tiles_times_split / ((double)rounds * 256 * w);
        if (busy > best + 1e-9) {
            best = busy;
            pick = w;
        }
    }
    return pick;
}

}  // namespace

int ffn_configure() {
    hipError_t e = allow_lds(&ffn_up_kernel<8>);
    if (e == hipSuccess) e = allow_lds(&ffn_up_kernel<7>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<8, 1>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<8, 2>);
    return (int)e;
}

void launch_ffn_up_bf16(hipStream_t st, const FfnArgs& a) {
    if (pick_waves(a.f / 16, a.est_tiles, a.variant) == 7)
        launch_up<7>(st, a);
    else
        launch_up<8>(st, a);
}

void launch_ffn_down_bf16(hipStream_t st, const FfnArgs& a) {
    if (a.h_planes == 2)
        launch_down<8, 2>(st, a);
    else
        launch_down<8, 1>(st, a);
}

}  // namespace kmoe
