// Grouped SwiGLU expert FFN on the 32x32x16 MFMA (bf16 for the up projections, fp16 for the down
// projection), fp32 accumulate.
//
// Every expert is an FFN evaluated once over all of its tokens from all batches of the batch
// group, experts in execution order (paper Section 2.1 and Section 5).  Two launches:
//   up  : H = silu(X W1^T) .* (X W3^T)   reduction over d on the bf16 MFMA; H stored in fragment order as
//                                        fp16 plus a plane with its rounding remainder (bf16 experts)
//   down: O = H W2^T                      reduction over f on the fp16 MFMA (W2 placed as fp16), the
//                                        remainder plane only where needed; fp32 split-K partials
//
// Work split.  A tile is one expert x up to 8 row blocks of 32 tokens.  A workgroup takes a tile
// and WAVES * U output units; a wavefront owns U units for all rows of the tile, so every weight
// byte is fetched from HBM once per tile and every activation fragment read from LDS feeds U
// MFMAs (with one unit per wavefront the LDS read port, one KiB per MFMA, is what bounds the
// matrix cores).  An up unit is 16 features: its weight fragment
// stacks the 16 rows of W1 on the 16 rows of W3, so one 32x32x16 MFMA yields the gate and the up
// value of the same feature in the same lane and SwiGLU needs no data movement.  A down unit is
// 32 output columns of W2.  Weights are pre-packed so that a wavefront's stream is one
// contiguous run of 1 KiB fragments (one per 16-deep reduction step), read straight into
// registers through a software prefetch ring.  The activations of the tile are staged through
// LDS, double buffered, in the same fragment order, so LDS reads are one conflict-free 16-byte
// read per lane.  All of that traffic (weight reloads, activation loads of a later stage, LDS
// stores of the next one) is issued between the MFMAs in a pinned order, never in bursts.  The
// workgroup -> tile map keeps what the workgroups of an XCD share in that XCD's L2: a tile's
// activations on small tiles, and on full tiles (an expert spans many tiles that all stream its
// weights) panels of a few tiles x a few weight streams.
#include "kernels.h"

namespace kmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte unit as a first-class value
typedef const __attribute__((address_space(1))) u32x4* gptr;  // global (HBM) address space

constexpr int kXcd = 8;
constexpr int kFragsPerBlk = 8;  // fragments of one row block in one LDS stage
constexpr int kBlkStageUnits = kFragsPerBlk * 64;  // 16-byte units of one row block per stage
constexpr int kBufUnits = kTileBlks * kBlkStageUnits;
constexpr int kLdsBytes = 2 * kBufUnits * 16;  // 128 KiB, double buffered

__device__ __forceinline__ gptr as_global(const void* p) { return (gptr)(uintptr_t)p; }

// Weights are read exactly once per tile: a streaming (non-temporal) load keeps them from
// taking cache lines that the re-read activations need, and measurably raises the HBM rate.
__device__ __forceinline__ u32x4 load_stream(gptr p) { return __builtin_nontemporal_load(p); }
// Reloads of the weight ring.  The down projection on full tiles (two-unit shape) is the one place
// where ordinary loads measure faster (1-2 %): the four tiles of a panel read the same W2 stream
// right behind each other and find more of it in L2 when the lines are not marked as streaming.
template <int MODE, int U>
__device__ __forceinline__ u32x4 load_ring(gptr p) {
    if (MODE == 1 && U == 2) return *p;
    return __builtin_nontemporal_load(p);
}

// The activations of a tile are loaded through a buffer descriptor: the address of a load is then
// a scalar byte offset (kept and advanced by the scalar unit) plus the lane's constant 16-byte
// slot, and costs no vector instruction.  (Through plain pointers every activation load of the
// reduction loop cost a 64-bit vector add; with one wavefront per SIMD those adds sit between
// the MFMAs.  The weight stream stays on plain non-temporal loads: through a descriptor it
// streamed measurably slower from HBM.)  A descriptor covers the live row blocks of one plane.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(gptr base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)(uintptr_t)base, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load(rsrc_t r, uint32_t byte_offset) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (threadIdx.x & 63u) * 16u, byte_offset, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// One LDS stage holds, per row block, SX reduction steps of 16 for PL planes of the activations
// (SX * PL == 8): SX = 8, PL = 1 normally; SX = 4, PL = 2 when the down projection also
// multiplies the rounding remainder of H (second plane).
struct TileCtx {
    gptr wbase;      // weight stream of this wavefront's first unit (+lane), 64 units per step
    size_t ustride;  // 16-byte units between the streams of consecutive output units
    gptr actbase;    // packed activations at the tile's first row block (plane 0)
    size_t plane;    // units between activation planes
    rsrc_t ars[2];   // descriptors of the tile's activations, plane 0 and plane 1 (bind_activations)
    u32x4* lds;
    int nks;         // reduction steps of 16 in the whole reduction
    int k0, k1;      // reduction steps of this workgroup: [k0, k1), k0 a multiple of SX
    int nblk;        // live row blocks of the tile
};

// Descriptors of the tile's activations: the live row blocks of each plane (at most 8 blocks of
// nks KiB: far below the 4 GiB a descriptor's offsets reach).  The scalar offset of a load is not
// range-checked by the hardware; it is in bounds by the same argument as the pointer it replaces.
__device__ __forceinline__ void bind_activations(TileCtx& c) {
    const uint32_t bytes = (uint32_t)c.nblk * (uint32_t)c.nks * 1024u;
    c.ars[0] = make_rsrc(c.actbase, bytes);
    c.ars[1] = make_rsrc(c.actbase + c.plane, bytes);
}

// Unit u of a stage is (row block b, plane pl, step j, lane): u = ((b*PL + pl)*SX + j)*64 + lane.
// Lanes past the live part of the tile re-read unit 0, steps past the end of the reduction
// re-read the last step: both in bounds, and what is then stored lands in LDS slots that no
// live MFMA reads.
// Where the units of a stage come from.  The workgroup is whole wavefronts of 64 and a row
// block's stage part is a multiple of 64 units, so the 64 units a wavefront loads in one pass are
// one fragment: (row block, plane, step) is the same for all its lanes and everything but the
// lane offset is scalar, computed once per tile.  (Computed per lane and per stage, the 16 passes
// of the four-wavefront shape cost a hundred vector instructions per stage and forty registers,
// whose spills are reloaded before the loop and then waited for in every stage.)
template <int PASSES, int T, int SX, int PL>
struct XMap {
    static_assert(T % 64 == 0 && kBlkStageUnits % 64 == 0, "a pass of a wavefront is one fragment");
    uint32_t off[PASSES];  // bytes from the plane's start to the row block of pass p at step 0, uniform
    int pl[PASSES];        // plane of pass p, uniform
    int step[PASSES];      // step of the stage, uniform
    __device__ __forceinline__ void init(const TileCtx& c) {
        const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
        const int live = c.nblk * (kBlkStageUnits / 64);
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            int fr = wave + p * (T / 64);  // fragment of the stage; past the live part: fragment 0
            fr = fr < live ? fr : 0;
            const int b = fr / (kBlkStageUnits / 64), r = fr % (kBlkStageUnits / 64);
            off[p] = (uint32_t)b * (uint32_t)c.nks * 1024u;
            pl[p] = r / SX;
            step[p] = r % SX;
        }
    }
    // CLAMP: steps past the end of the reduction re-read the last step; the steady state never
    // gets there and skips the test.
    template <bool CLAMP>
    __device__ __forceinline__ u32x4 load(const TileCtx& c, int p, int kbase) const {
        const int ks = CLAMP ? min(kbase + step[p], c.nks - 1) : kbase + step[p];
        return buf_load(PL == 1 || pl[p] == 0 ? c.ars[0] : c.ars[1], off[p] + (uint32_t)ks * 1024u);
    }
};

// When PASSES * T fits one LDS buffer the stores need no guard.
template <int PASSES, int T>
__device__ __forceinline__ void store_x(const TileCtx& c, const u32x4 (&xr)[PASSES], int buf) {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int u = (int)threadIdx.x + p * T;
        if (PASSES * T <= kBufUnits || u < kBufUnits) c.lds[buf * kBufUnits + u] = xr[p];
    }
}
// HT = 0: bf16 operands; HT = 1: fp16 operands (down projection with H carried as fp16).
template <int MODE, int HT = 0>
__device__ __forceinline__ f32x16 mfma(const bf16x8 wf, const bf16x8 xa, const f32x16 acc) {
    if (HT == 1)  // rows = tokens, cols = output columns; same bits, read as fp16
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, xa),
                                                      __builtin_bit_cast(f16x8, wf), acc, 0, 0, 0);
    if (MODE == 0)  // rows = 16 gate + 16 up features, cols = tokens
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xa, acc, 0, 0, 0);
    // rows = tokens, cols = output columns
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, wf, acc, 0, 0, 0);
}

// MFMAs of one reduction step for the U units of a wavefront: NB*PL activation fragments read
// from LDS through a rolling window of D registers, each fragment feeding U MFMAs.  Used by the
// guarded drain.
template <int MODE, int NB, int U, int SX, int PL, int D, int HT = 0>
__device__ __forceinline__ void step_mfma(const u32x4* L, int j, const u32x4 (&w)[U],
                                          f32x16 (&acc)[U][NB]) {
    constexpr int NF = NB * PL;
    constexpr int DD = D < NF ? D : NF;
    u32x4 win[DD];
#pragma unroll
    for (int i = 0; i < DD; ++i) win[i] = L[(i * SX + j) * 64];  // fragment i = (b, pl) = i/PL, i%PL
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int b = i / PL;
        const bf16x8 xa = as_bf16x8(win[i % DD]);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u][b] = mfma<MODE, HT>(as_bf16x8(w[u]), xa, acc[u][b]);
        if (i + DD < NF) win[i % DD] = L[((i + DD) * SX + j) * 64];
    }
    __builtin_amdgcn_sched_group_barrier(0x100, DD, 0);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, U, 0);
        if (i + DD < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
}

// MFMAs of a whole stage (SX steps) with the weight reloads of the next ring turn.  The LDS
// window rolls across the step boundaries, so only the first D reads of a stage are exposed;
// each ring slot is reloaded right after the last MFMA that reads it.  Order pinned: D reads,
// then per fragment U MFMAs and one read (while any are left) and, after the last fragment of a
// step, the U reloads of that step's slot.
template <int MODE, int NB, int U, int SX, int PL, int D, int HT, int PASSES, int T, int DX>
__device__ __forceinline__ void stage_mfma(const u32x4* L, u32x4 (&w)[SX][U], gptr wnext,
                                           size_t ustride, f32x16 (&acc)[U][NB],
                                           u32x4* next_buf, const u32x4 (&xs)[PASSES],
                                           const TileCtx& c, const XMap<PASSES, T, SX, PL>& xm,
                                           int kload, u32x4 (&xl)[PASSES]) {
    constexpr int NS = NB * PL;   // fragments per step
    constexpr int NF = NS * SX;   // fragments per stage
    constexpr int DD = D < NF ? D : NF;
    // The traffic of the activations rides between the MFMAs: with one wavefront per SIMD every
    // instruction issued ahead of the first MFMA of a stage, and every burst that holds a port,
    // is time the matrix cores idle.  xl (the stage at reduction step kload) is loaded from
    // memory one pass per fragment, xs (the next stage) goes to the other LDS buffer the same
    // way.  With a look-ahead of one stage xl and xs are the same registers: loads in the first
    // quarter of the stage, stores in its second half; otherwise both spread over the stage.
    constexpr int L1 = DX == 1 ? (NF / 4 > PASSES ? NF / 4 : PASSES) : NF;
    constexpr int S0 = DX == 1 ? NF / 2 : 0;
    u32x4 win[DD];
    // fragment t of the stage: step t / NS, (row block, plane) t % NS
#define KMOE_FRAG_AT(t) L[(((t) % NS) * SX + (t) / NS) * 64]
#define KMOE_LOAD_AT(p) (((p) * L1) / PASSES)
#define KMOE_STORE_AT(p) (S0 + ((p) * (NF - S0)) / PASSES)
    static_assert(PASSES <= NF / 2, "one pass per fragment at most");
#pragma unroll
    for (int t = 0; t < DD; ++t) win[t] = KMOE_FRAG_AT(t);
#pragma unroll
    for (int t = 0; t < NF; ++t) {
        const int j = t / NS, b = (t % NS) / PL;
        const bf16x8 xa = as_bf16x8(win[t % DD]);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u][b] = mfma<MODE, HT>(as_bf16x8(w[j][u]), xa, acc[u][b]);
        if (t + DD < NF) win[t % DD] = KMOE_FRAG_AT(t + DD);
        {   // the pass stored at this fragment, if any (both maps are strictly increasing in p)
            const int p = t < S0 ? PASSES : ((t - S0) * PASSES + (NF - S0) - 1) / (NF - S0);
            if (p < PASSES && KMOE_STORE_AT(p) == t) {
                const int u = (int)threadIdx.x + p * T;
                if (PASSES * T <= kBufUnits || u < kBufUnits) next_buf[u] = xs[p];
            }
        }
        {   // the pass loaded at this fragment, if any
            const int p = (t * PASSES + L1 - 1) / L1;
            if (p < PASSES && KMOE_LOAD_AT(p) == t) xl[p] = xm.template load<false>(c, p, kload);
        }
        if (t % NS == NS - 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) w[j][u] = load_ring<MODE, U>(wnext + (size_t)u * ustride + (size_t)j * 64);
        }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, DD, 0);
#pragma unroll
    for (int t = 0; t < NF; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, U, 0);
        if (t + DD < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        const int ps = t < S0 ? PASSES : ((t - S0) * PASSES + (NF - S0) - 1) / (NF - S0);
        if (ps < PASSES && KMOE_STORE_AT(ps) == t) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        const int pl = (t * PASSES + L1 - 1) / L1;
        if (pl < PASSES && KMOE_LOAD_AT(pl) == t) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        if (t % NS == NS - 1) __builtin_amdgcn_sched_group_barrier(0x020, U, 0);
    }
#undef KMOE_FRAG_AT
#undef KMOE_LOAD_AT
#undef KMOE_STORE_AT
}

// Register budget of one shape: the weight ring is RING steps deep (U KiB per step in flight
// per wavefront), the activation look-ahead DX stages.
template <int NB, int WAVES, int U>
struct Shape2 {
    static constexpr int RING = (U == 1) ? (NB <= 5 ? 16 : 8) : 8;
    // two stages ahead wherever the registers allow: small tiles, and the two-unit shape (one
    // wavefront per SIMD, accumulators in AGPRs), whose full tiles miss L2 most often
    static constexpr int DX = (NB <= 5 || U == 2) ? 2 : 1;
};

// Registers of the software pipeline of one tile pass: the weight ring (RS stages of SX steps,
// U units) and the activations in flight to LDS (DX stages ahead).
template <int NB, int WAVES, int U, int SX>
struct Pipe {
    static constexpr int T = WAVES * 64;
    static constexpr int PASSES = (NB * kBlkStageUnits + T - 1) / T;
    static constexpr int RS = Shape2<NB, WAVES, U>::RING / SX;
    // Activation look-ahead in stages.  The memory counter retires loads in issue order, so the
    // wait for a stage's activations (before they are stored to LDS) also waits for every
    // weight load issued before them.  With a look-ahead of one stage that cuts the useful
    // depth of the weight ring to one stage whatever its size; with DX stages between the issue
    // of the activation loads and their wait, all older weight loads have been consumed by
    // then and the ring keeps its full depth.
    static constexpr int DX = Shape2<NB, WAVES, U>::DX;
    static constexpr int G = RS > DX ? RS : DX;  // stages per unrolled group (RS, DX in {1,2,4})
    static_assert(RS >= 1 && G % RS == 0 && G % DX == 0, "group must cycle ring and look-ahead");
    u32x4 wr[RS][SX][U];
    u32x4 xr[DX][PASSES];
    XMap<PASSES, T, SX, 8 / SX> xm;
    __device__ __forceinline__ void init(const TileCtx& c) { xm.init(c); }
    template <int PL>
    __device__ __forceinline__ void load(const TileCtx& c, int slot, int kbase) {
        static_assert(PL == 8 / SX, "planes per stage");
#pragma unroll
        for (int p = 0; p < PASSES; ++p) xr[slot][p] = xm.template load<true>(c, p, kbase);
    }
};

// Issue the loads that open a pass: activations of the first DX stages and the whole weight
// ring, interleaved in the order the steady state issues them, so that the wait counts at the
// loop head are the same on entry and on the back edge.  Nothing is waited for here: a
// workgroup calls this for its next pass before the epilogue of the current one, so the
// memory latency of the ring fill hides behind the epilogue.
template <int NB, int WAVES, int U, int SX, int PL>
__device__ __forceinline__ void open_pass(const TileCtx& c, Pipe<NB, WAVES, U, SX>& pp) {
    using P = Pipe<NB, WAVES, U, SX>;
#pragma unroll
    for (int i = 0; i < P::G; ++i) {
        if (i < P::DX) pp.template load<PL>(c, i, c.k0 + i * SX);
        if (i < P::RS) {
#pragma unroll
            for (int j = 0; j < SX; ++j)  // past the end: re-read the last step (in bounds, unused)
#pragma unroll
                for (int u = 0; u < U; ++u)
                    pp.wr[i][j][u] = load_stream(c.wbase + (size_t)u * c.ustride +
                                                 (size_t)min(c.k0 + i * SX + j, c.k1 - 1) * 64);
        }
    }
}

// One pass over the reduction range of the tile for the U units of every wavefront; the pass
// must have been opened.  On return all LDS reads of the pass are behind a barrier.
template <int MODE, int NB, int WAVES, int U, int SX, int PL, int HT = 0>
__device__ __forceinline__ void run_pass(const TileCtx& c, Pipe<NB, WAVES, U, SX>& pp,
                                         f32x16 (&acc)[U][NB]) {
    static_assert(SX * PL == kFragsPerBlk, "stage geometry");
    using P = Pipe<NB, WAVES, U, SX>;
    constexpr int T = P::T, PASSES = P::PASSES, RS = P::RS, DX = P::DX, G = P::G;
    constexpr int D = 3;
    const int lane = threadIdx.x & 63;

#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[u][b][i] = 0.f;

    store_x<PASSES, T>(c, pp.xr[0], 0);
    __syncthreads();

    int k = c.k0, buf = 0;
    // steady state: every stage of the group is complete, has a successor to stage and a slot to
    // reload, so the body is branch-free (activation loads past the end re-read the last step)
    // (the ring reloads reach RS stages ahead, the unclamped activation loads DX: the further one
    // must stay inside the range)
    for (; k + (G + (RS > DX ? RS : DX)) * SX <= c.k1; k += G * SX) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int kk = k + g * SX;
            __builtin_amdgcn_sched_barrier(0);
            const u32x4* L = c.lds + buf * kBufUnits + lane;
            stage_mfma<MODE, NB, U, SX, PL, D, HT, PASSES, T, DX>(
                L, pp.wr[g % RS], c.wbase + (size_t)(kk + RS * SX) * 64, c.ustride, acc,
                c.lds + (buf ^ 1) * kBufUnits, pp.xr[(g + 1) % DX], c, pp.xm, kk + DX * SX, pp.xr[g % DX]);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            buf ^= 1;
        }
    }
    // drain: the last stages, guarded step by step
    for (; k < c.k1; k += G * SX) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int kk = k + g * SX;
            if (kk < c.k1) {  // uniform over the workgroup
                const bool more = kk + SX < c.k1;
                if (kk + DX * SX < c.k1)
                    pp.template load<PL>(c, g % DX, kk + DX * SX);
                const u32x4* L = c.lds + buf * kBufUnits + lane;
#pragma unroll
                for (int j = 0; j < SX; ++j) {
                    if (kk + j < c.k1) {
                        step_mfma<MODE, NB, U, SX, PL, D, HT>(L, j, pp.wr[g % RS][j], acc);
                        if (kk + RS * SX + j < c.k1) {
#pragma unroll
                            for (int u = 0; u < U; ++u)
                                pp.wr[g % RS][j][u] =
                                    load_ring<MODE, U>(c.wbase + (size_t)u * c.ustride +
                                                       (size_t)(kk + RS * SX + j) * 64);
                        }
                    }
                }
                if (more) store_x<PASSES, T>(c, pp.xr[(g + 1) % DX], buf ^ 1);
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

// Packed weights of expert e for this launch: one blob for all tiles (a streamed expert run on
// its own), a window slot named in the launch's group list, or the layer's table of resident blobs.
__device__ __forceinline__ const uint8_t* blob_of(const FfnArgs& a, int e) {
    if (a.w_single) return a.w_single;
    const uint8_t* blob = nullptr;
#pragma unroll
    for (int i = 0; i < kMaxLaunchGroup; ++i)
        if (i < a.n_group && a.group_expert[i] == e) blob = a.w_group[i];
    return blob ? blob : a.wtab[e];
}

// XCD-aware map from the hardware workgroup id (dealt round-robin to the 8 XCDs) to a logical
// id such that each XCD walks a contiguous range of (tile, split, group) items.  Two orders of
// that range.  Small tiles (an expert is one tile; the weights are read once whatever the
// order): all items of a tile, then the next tile, so the tile's activations stay in the XCD's
// L2.  Full tiles (an expert spans many tiles and each of them streams the expert's weights
// again): panels of kPanelTiles tiles x kPanelCols items, so that the workgroups an XCD runs at
// the same time share both the activations of a few tiles and a few weight streams, and most
// weight reads are L2 hits behind the first workgroup of a column.  (Dealing the panels round
// robin instead, so that all XCDs work on the same expert at the same time and share its weights
// through the memory-side cache, was measured 10-20 % slower: every XCD then asks the same
// memory channels for the same lines at once.)
constexpr int kPanelTiles = 4, kPanelCols = 8;
__device__ __forceinline__ Wg locate(const FfnArgs& a, int n_groups, int split) {
    Wg w;
    const int ntile = a.tile_count ? *a.tile_count : a.tile_count_v;
    const int per_tile = n_groups * split;
    const int live = ntile * per_tile;
    const int per_xcd = (live + kXcd - 1) / kXcd;
    const int id = blockIdx.x;
    const int seq = id / kXcd;
    const int L = (id % kXcd) * per_xcd + seq;
    w.live = seq < per_xcd && L < live;
    int tile, r;
    if (a.full_tiles) {
        const int pt = a.panel ? 1 << (a.panel - 1) : kPanelTiles, pc = a.panel ? max(1, 32 >> (a.panel - 1)) : kPanelCols;
        const int panel_items = pt * per_tile;
        const int tp = L / panel_items, l = L - tp * panel_items;
        const int rows = max(1, min(pt, ntile - tp * pt));  // the last panel may be short (ids past the end: 1)
        const int cb = l / (rows * pc), m = l - cb * rows * pc;
        tile = tp * pt + m % rows;
        r = cb * pc + m / rows;  // < per_tile: the last column block holds rows * (its width) items
    } else {
        tile = L / per_tile;
        r = L % per_tile;
    }
    w.tile = (a.tile_first ? *a.tile_first : a.tile_first_v) + tile;
    w.sp = r / n_groups;
    w.grp = r % n_groups;
    return w;
}

// Up projections + SwiGLU.  The accumulator of lane (token j = lane & 31, half hi = lane >> 5)
// holds, in register r < 8, the gate value of feature 16*unit + 8*(r/4) + 4*hi + r%4 and in
// register r + 8 the up value of the same feature: exactly the lane's 16-byte unit in the
// fragment order of the down projection, so H is written with one 16-byte store per row block.
//
// Format of H: fp16 (nearest even, clamped to the largest finite value; clamped values are
// counted), plus a second plane with the rounding remainder h - fp16(h), also fp16.  The down
// projection multiplies the remainder plane only for tiles that need it: the up kernel adds, per
// token row, the energy of the remainders (sum of squares over the features of this workgroup) to
// herr[row], in integer units of 2^-20 of the expert's threshold, so that the total does not
// depend on the order of the atomic additions.
constexpr float kErrUnit = 1048576.f;  // herr counts in units of threshold / 2^20
template <int NB, int WAVES, int U>
__device__ __forceinline__ void store_up(const FfnArgs& a, const f32x16 (&acc)[U][NB], int nblk,
                                         int wunit, int unit0, int hblk0, int expert, u32x4* lds) {
    const int lane = threadIdx.x & 63;
    u32x4* hp = reinterpret_cast<u32x4*>(a.out);
    const size_t ksteps_h = (size_t)a.f / 16;
    float esum[NB];
    int sat = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b) esum[b] = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (wunit + u < unit0) continue;  // streamed only to stay in bounds: another wavefront's
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
                // H = silu(gate) * up; silu through the hardware reciprocal (1 ulp), far inside
                // the rounding of H
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float h[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float gv = acc[u][b][2 * q + t];
                        h[t] = gv * __builtin_amdgcn_rcpf(1.f + __expf(-gv)) * acc[u][b][2 * q + t + 8];
                    }
                    float r[2];
                    f16x2 v, l;
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        sat += __builtin_fabsf(h[t]) > 65504.f ? 1 : 0;
                        v[t] = (_Float16)__builtin_fminf(__builtin_fmaxf(h[t], -65504.f), 65504.f);
                        r[t] = h[t] - (float)v[t];  // exact in fp32
                        l[t] = (_Float16)__builtin_fminf(__builtin_fmaxf(r[t], -65504.f), 65504.f);
                        esum[b] = __builtin_fmaf(r[t], r[t], esum[b]);
                    }
                    hi[q] = __builtin_bit_cast(uint32_t, v);
                    lo[q] = __builtin_bit_cast(uint32_t, l);
                }
                const size_t at = ((size_t)(hblk0 + b) * ksteps_h + (size_t)(wunit + u)) * 64 + lane;
                // streaming stores: measurably cheaper next to the weight stream than cached ones
                __builtin_nontemporal_store(u32x4{hi[0], hi[1], hi[2], hi[3]}, hp + at);
                __builtin_nontemporal_store(u32x4{lo[0], lo[1], lo[2], lo[3]},
                                            hp + at + (size_t)a.h_plane_units);
            }
        }
    }
    if (sat) atomicAdd(a.sat_count, sat);
    if (a.h_mode != 0) return;  // remainder always multiplied: no energies needed (uniform over the launch)
    // remainder energy per token row of the tile: lanes l and l + 32 hold the same token, the
    // wavefronts meet in LDS (free: every LDS read of the pass is behind a barrier), one integer
    // atomic per row and workgroup
    float* red = reinterpret_cast<float*>(lds);
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        esum[b] += __shfl_xor(esum[b], 32, 64);
        if (lane < 32) red[(wave * NB + b) * 32 + lane] = esum[b];
    }
    __syncthreads();
    const float inv_tau = a.wmeta[expert].y * kErrUnit;
    for (int i = threadIdx.x; i < nblk * 32; i += WAVES * 64) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w * NB * 32 + i];
        const unsigned long long q = (unsigned long long)__builtin_fminf(sum * inv_tau, 1.7e13f);
        if (q) atomicAdd(a.herr + (size_t)hblk0 * 32 + i, q);
    }
}

// Down projection: lane (column n = lane & 31, half hi) holds in register r the token row
// 8*(r/4) + 4*hi + r%4 of the row block.  `scale` undoes the power-of-two scaling of W2 (1 unless
// the expert holds weights beyond the fp16 range).
template <int NB, int U>
__device__ __forceinline__ void store_down(const FfnArgs& a, const f32x16 (&acc)[U][NB], int nblk,
                                           int wunit, int unit0, int hblk0, int sp, float scale) {
    const int lane = threadIdx.x & 63;
    float* o = reinterpret_cast<float*>(a.out) + (size_t)sp * a.o_split_stride;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (wunit + u < unit0) continue;
        const int col = (wunit + u) * 32 + (lane & 31);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nblk) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const size_t row =
                        (size_t)(hblk0 + b) * kRowBlk + 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
                    __builtin_nontemporal_store(acc[u][b][r] * scale, o + row * a.d + col);
                }
            }
        }
    }
}

// One workgroup, one tile, WAVES * U consecutive output units: wavefront w owns the units
// unit0 = (grp * WAVES + w) * U .. unit0 + U - 1, as far as they exist.  It always streams U real
// units, wunit = min(unit0, n_units - U) onwards, so that every load stays in bounds, and stores
// only those it owns (wunit + u >= unit0).  (Several such runs per workgroup, with the next
// run's loads issued before the epilogue, were measured to gain nothing, and the loop around
// the reduction loop made the compiler wait in every stage for reloads it had placed on the
// outer back edge.)
template <int MODE, int NB, int WAVES, int U, int PL, int HT = 0>
__device__ __forceinline__ void run_tile(const FfnArgs& a, TileCtx c, gptr wsection, int n_units,
                                         int grp, int hblk0, int sp, int expert, float scale) {
    constexpr int SX = 8 / PL;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), lane = threadIdx.x & 63;
    Pipe<NB, WAVES, U, SX> pp;
    f32x16 acc[U][NB];
    const int unit0 = (grp * WAVES + wave) * U;
    const int wunit = min(unit0, n_units - U);
    c.wbase = wsection + (size_t)wunit * c.ustride + lane;
    pp.init(c);
    open_pass<NB, WAVES, U, SX, PL>(c, pp);
    run_pass<MODE, NB, WAVES, U, SX, PL, HT>(c, pp, acc);
    if (MODE == 0)
        store_up<NB, WAVES, U>(a, acc, c.nblk, wunit, unit0, hblk0, expert, c.lds);
    else
        store_down<NB, U>(a, acc, c.nblk, wunit, unit0, hblk0, sp, scale);
}

#define NB_SWITCH(CALL)                       \
    if (nblk <= 2) { CALL(2); }               \
    else if (nblk <= 4) { CALL(4); }          \
    else if (nblk <= 5) { CALL(5); }          \
    else if (nblk <= 6) { CALL(6); }          \
    else { CALL(8); }
static_assert(kTileBlks == 8, "row-block classes above cover tiles of up to 8 blocks");

template <int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void ffn_up_kernel(FfnArgs a, int n_groups) {
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, 1);
    if (!w.live) return;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = blob_of(a, e);
    TileCtx c;
    c.nks = a.d / 16;
    c.ustride = (size_t)c.nks * 64;
    c.actbase = as_global(a.act) + (size_t)a.tile_xblk[w.tile] * c.nks * 64;
    c.plane = 0;
    c.lds = lds;
    c.k0 = 0;
    c.k1 = c.nks;
    c.nblk = nblk;
    bind_activations(c);
#define CALL(NB) run_tile<0, NB, WAVES, U, 1>(a, c, as_global(blob), a.f / 16, w.grp, hblk0, 0, e, 1.f)
    NB_SWITCH(CALL)
#undef CALL
}

// True when the down projection of this tile must multiply the remainder plane of H too: the
// launch asks for it (h_mode 1), or some token row of the tile recorded a remainder energy above
// the expert's threshold (h_mode 0).  Uniform over the workgroup; one thread per row.
__device__ __forceinline__ int wants_remainder(const FfnArgs& a, int nblk, int hblk0) {
    int two = a.h_mode == 1;
    if (a.h_mode == 0) {
        const int over = (int)threadIdx.x < nblk * kRowBlk &&
                         a.herr[(size_t)hblk0 * kRowBlk + threadIdx.x] > (unsigned long long)kErrUnit;
        two = __syncthreads_or(over);
        if (two && threadIdx.x == 0) atomicAdd(a.sat_count + 1, 1);  // workgroups that took the remainder plane
    }
    return two;
}

// Down projection of bf16 experts: H and W2 as fp16 on the fp16 MFMA.  The remainder plane of H
// is multiplied as well (two planes per stage, twice the MFMAs) when the launch asks for it
// (h_mode 1) or when, for some token row of the tile, the energy of the remainders recorded by
// the up kernel exceeds the expert's threshold (h_mode 0); the test is uniform over the workgroup.
template <int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void ffn_down_kernel(FfnArgs a, int n_groups) {
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, a.split_k);
    if (!w.live) return;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = blob_of(a, e);
    const float scale = a.wmeta[e].x;
    static_assert(WAVES * 64 >= kTileBlks * kRowBlk, "one thread per token row of the tile");
    const int two = wants_remainder(a, nblk, hblk0);
    TileCtx c;
    c.nks = a.f / 16;
    c.ustride = (size_t)c.nks * 64;
    c.actbase = as_global(a.act) + (size_t)hblk0 * c.nks * 64;
    c.plane = (size_t)a.h_plane_units;
    c.lds = lds;
    c.nblk = nblk;
    bind_activations(c);
    const gptr wsec = as_global(blob + (size_t)a.d * a.f * 4);
    if (two) {
        constexpr int SX = 4;
        const int nstage = (c.nks + SX - 1) / SX;
        c.k0 = (int)((long long)w.sp * nstage / a.split_k) * SX;
        c.k1 = min((int)((long long)(w.sp + 1) * nstage / a.split_k) * SX, c.nks);
#define CALL(NB) run_tile<1, NB, WAVES, U, 2, 1>(a, c, wsec, a.d / 32, w.grp, hblk0, w.sp, e, scale)
        NB_SWITCH(CALL)
#undef CALL
    } else {
        constexpr int SX = 8;
        const int nstage = (c.nks + SX - 1) / SX;
        c.k0 = (int)((long long)w.sp * nstage / a.split_k) * SX;
        c.k1 = min((int)((long long)(w.sp + 1) * nstage / a.split_k) * SX, c.nks);
#define CALL(NB) run_tile<1, NB, WAVES, U, 1, 1>(a, c, wsec, a.d / 32, w.grp, hblk0, w.sp, e, scale)
        NB_SWITCH(CALL)
#undef CALL
    }
}

// ---- 4-bit group-quantised expert weights ------------------------------------------------------
//
// Experts may be kept and moved as 4-bit codes with one scale and one zero point per group of 64
// weights along the reduction axis, W = s * (W_q - z) (paper Section 7, "Quantization", Eq. 8);
// they are converted back to bf16 right before the multiplication (and handed to the fp16 MFMA of
// the down projection as fp16, exactly).  A group of 64 is exactly
// four reduction steps of one fragment row, so the packed stream of an output unit is, per
// step quad, 1 KiB of codes (lane l: four dwords = steps 4q..4q+3, eight codes each, in the
// lane's fragment order) and 128 bytes of (s, z) bf16 pairs (one per fragment row).  The ring
// holds quads; a step's weight fragment is dequantised in registers (fp32 fma, hardware bf16
// rounding) before its MFMAs.  One output unit per wavefront.
typedef const __attribute__((address_space(1))) uint32_t* gptr32;

struct QCtx {
    gptr nib;     // codes of this wavefront's unit (+lane), 64 units per quad
    gptr32 sz;    // (s | z << 16) of this wavefront's unit (+ lane & 31), 32 dwords per quad
};

// HT = 0: the dequantised weights as bf16 (one hardware rounding of the fp32 fma).  HT = 1: the
// same bf16 values handed over as fp16, for the down projection on the fp16 MFMA (exact: the
// placement scales an expert's (s) by a power of two when its weights would leave the fp16 range).
template <int HT>
__device__ __forceinline__ bf16x8 dequant8(uint32_t codes, uint32_t sz) {
    const float s = __uint_as_float(sz << 16);
    const float z = __uint_as_float(sz & 0xffff0000u);
    const float zs = -z * s;
    float v[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) v[p] = __builtin_fmaf((float)((codes >> (4 * p)) & 15u), s, zs);
    bf16x8 r;
#pragma unroll
    for (int p = 0; p < 8; ++p) r[p] = (__bf16)v[p];
    if (HT == 1) {
        f16x8 h;
#pragma unroll
        for (int p = 0; p < 8; ++p) h[p] = (_Float16)(float)r[p];
        return __builtin_bit_cast(bf16x8, h);
    }
    return r;
}

template <int NB, int WAVES, int SX>
struct PipeQ {
    static constexpr int T = WAVES * 64;
    static constexpr int PASSES = (NB * kBlkStageUnits + T - 1) / T;
    static constexpr int RQ = 4;                  // ring depth in quads (16 reduction steps)
    static constexpr int QS = SX / 4;             // quads per stage
    static constexpr int RS = RQ / QS;            // ring depth in stages
    static constexpr int DX = (NB <= 5) ? 2 : 1;  // activation look-ahead in stages
    static constexpr int G = RS > DX ? RS : DX;
    static_assert(SX % 4 == 0 && RQ % QS == 0 && G % RS == 0 && G % DX == 0, "ring geometry");
    u32x4 wq[RQ];
    uint32_t sz[RQ];
    u32x4 xr[DX][PASSES];
    XMap<PASSES, T, SX, 8 / SX> xm;
    __device__ __forceinline__ void load(const TileCtx& c, int slot, int kbase) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) xr[slot][p] = xm.template load<true>(c, p, kbase);
    }
};

template <int NB, int WAVES, int SX, int PL>
__device__ __forceinline__ void open_pass_q4(const TileCtx& c, const QCtx& q, PipeQ<NB, WAVES, SX>& pp) {
    using P = PipeQ<NB, WAVES, SX>;
#pragma unroll
    for (int i = 0; i < P::G; ++i) {
        if (i < P::DX) pp.load(c, i, c.k0 + i * SX);
        if (i < P::RS) {
#pragma unroll
            for (int h = 0; h < P::QS; ++h) {  // past the end: re-read the last quad (in bounds, unused)
                const int quad = min(c.k0 / 4 + i * P::QS + h, c.k1 / 4 - 1);
                pp.wq[i * P::QS + h] = load_stream(q.nib + (size_t)quad * 64);
                pp.sz[i * P::QS + h] = q.sz[(size_t)quad * 32];
            }
        }
    }
}

template <int MODE, int NB, int WAVES, int SX, int PL, int HT>
__device__ __forceinline__ void run_pass_q4(const TileCtx& c, const QCtx& q, PipeQ<NB, WAVES, SX>& pp,
                                            f32x16 (&acc)[1][NB]) {
    static_assert(SX * PL == kFragsPerBlk, "stage geometry");
    using P = PipeQ<NB, WAVES, SX>;
    constexpr int T = P::T, PASSES = P::PASSES, RS = P::RS, DX = P::DX, G = P::G, QS = P::QS;
    constexpr int NS = NB * PL, NF = NS * SX, D = 3, DD = D < NF ? D : NF;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[0][b][i] = 0.f;
    store_x<PASSES, T>(c, pp.xr[0], 0);
    __syncthreads();

    int k = c.k0, buf = 0;
#define KMOE_FRAG_AT(t) L[(((t) % NS) * SX + (t) / NS) * 64]
    for (; k + (G + RS) * SX <= c.k1; k += G * SX) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int kk = k + g * SX;
            pp.load(c, g % DX, kk + DX * SX);
            __builtin_amdgcn_sched_barrier(0);
            const u32x4* L = c.lds + buf * kBufUnits + lane;
            u32x4 win[DD];
#pragma unroll
            for (int t = 0; t < DD; ++t) win[t] = KMOE_FRAG_AT(t);
            bf16x8 wf;
#pragma unroll
            for (int t = 0; t < NF; ++t) {
                const int j = t / NS, b = (t % NS) / PL;
                const int slot = (g % RS) * QS + j / 4;
                if (t % NS == 0) wf = dequant8<HT>(pp.wq[slot][j % 4], pp.sz[slot]);
                acc[0][b] = mfma<MODE, HT>(wf, as_bf16x8(win[t % DD]), acc[0][b]);
                if (t + DD < NF) win[t % DD] = KMOE_FRAG_AT(t + DD);
                if (t % NS == NS - 1 && j % 4 == 3) {  // the quad is consumed: next ring turn
                    const size_t quad = (size_t)((kk + RS * SX) / 4 + j / 4);
                    pp.wq[slot] = load_stream(q.nib + quad * 64);
                    pp.sz[slot] = q.sz[quad * 32];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            store_x<PASSES, T>(c, pp.xr[(g + 1) % DX], buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    // drain: the last stages, guarded step by step
    for (; k < c.k1; k += G * SX) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int kk = k + g * SX;
            if (kk < c.k1) {  // uniform over the workgroup
                const bool more = kk + SX < c.k1;
                if (kk + DX * SX < c.k1)
                    pp.load(c, g % DX, kk + DX * SX);
                const u32x4* L = c.lds + buf * kBufUnits + lane;
#pragma unroll
                for (int j = 0; j < SX; ++j) {
                    if (kk + j < c.k1) {
                        const int slot = (g % RS) * QS + j / 4;
                        const bf16x8 wf = dequant8<HT>(pp.wq[slot][j % 4], pp.sz[slot]);
#pragma unroll
                        for (int i = 0; i < NS; ++i)
                            acc[0][i / PL] = mfma<MODE, HT>(wf, as_bf16x8(L[(i * SX + j) * 64]), acc[0][i / PL]);
                        if (j % 4 == 3 && kk + RS * SX + j < c.k1) {
                            const size_t quad = (size_t)((kk + RS * SX) / 4 + j / 4);
                            pp.wq[slot] = load_stream(q.nib + quad * 64);
                            pp.sz[slot] = q.sz[quad * 32];
                        }
                    }
                }
                if (more) store_x<PASSES, T>(c, pp.xr[(g + 1) % DX], buf ^ 1);
                __syncthreads();
                buf ^= 1;
            }
        }
    }
#undef KMOE_FRAG_AT
}

template <int MODE, int NB, int WAVES, int PL>
__device__ __forceinline__ void run_tile_q4(const FfnArgs& a, TileCtx c, const uint8_t* nib_section,
                                            const uint8_t* sz_section, int n_units, int grp,
                                            int hblk0, int sp, int expert, float scale) {
    constexpr int SX = 8 / PL;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int unit0 = grp * WAVES + wave;
    const int wunit = min(unit0, n_units - 1);
    const size_t quads = (size_t)c.nks / 4;
    QCtx q;
    q.nib = as_global(nib_section) + (size_t)wunit * quads * 64 + lane;
    q.sz = (gptr32)(uintptr_t)sz_section + (size_t)wunit * quads * 32 + (lane & 31);
    PipeQ<NB, WAVES, SX> pp;
    pp.xm.init(c);
    f32x16 acc[1][NB];
    open_pass_q4<NB, WAVES, SX, PL>(c, q, pp);
    run_pass_q4<MODE, NB, WAVES, SX, PL, MODE>(c, q, pp, acc);  // up: bf16 MFMA; down: fp16 MFMA
    if (MODE == 0)
        store_up<NB, WAVES, 1>(a, acc, c.nblk, wunit, unit0, hblk0, expert, c.lds);
    else
        store_down<NB, 1>(a, acc, c.nblk, wunit, unit0, hblk0, sp, scale);
}

// Blob of a 4-bit expert: [up codes d*f | up (s,z) d*f/8 | down codes d*f/2 | down (s,z) d*f/16] bytes.
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void ffn_up_q4_kernel(FfnArgs a, int n_groups) {
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, 1);
    if (!w.live) return;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = blob_of(a, e);
    TileCtx c;
    c.nks = a.d / 16;
    c.ustride = 0;
    c.wbase = nullptr;
    c.actbase = as_global(a.act) + (size_t)a.tile_xblk[w.tile] * c.nks * 64;
    c.plane = 0;
    c.lds = lds;
    c.k0 = 0;
    c.k1 = c.nks;
    c.nblk = nblk;
    bind_activations(c);
    const size_t df = (size_t)a.d * a.f;
#define CALL(NB) run_tile_q4<0, NB, WAVES, 1>(a, c, blob, blob + df, a.f / 16, w.grp, hblk0, 0, e, 1.f)
    NB_SWITCH(CALL)
#undef CALL
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void ffn_down_q4_kernel(FfnArgs a, int n_groups) {
    static_assert(WAVES * 64 >= kTileBlks * kRowBlk, "one thread per token row of the tile");
    extern __shared__ u32x4 lds[];
    const Wg w = locate(a, n_groups, a.split_k);
    if (!w.live) return;
    const int e = a.tile_expert[w.tile];
    const int nblk = a.tile_nblk[w.tile];
    const int hblk0 = a.tile_hblk[w.tile];
    const uint8_t* blob = blob_of(a, e);
    const float scale = a.wmeta[e].x;
    const int two = wants_remainder(a, nblk, hblk0);
    TileCtx c;
    c.nks = a.f / 16;
    c.ustride = 0;
    c.wbase = nullptr;
    c.actbase = as_global(a.act) + (size_t)hblk0 * c.nks * 64;
    c.plane = (size_t)a.h_plane_units;
    c.lds = lds;
    c.nblk = nblk;
    bind_activations(c);
    const size_t df = (size_t)a.d * a.f;
    const uint8_t* down = blob + df + df / 8;
    if (two) {
        constexpr int SX = 4;
        const int nstage = (c.nks + SX - 1) / SX;
        c.k0 = (int)((long long)w.sp * nstage / a.split_k) * SX;
        c.k1 = min((int)((long long)(w.sp + 1) * nstage / a.split_k) * SX, c.nks);
#define CALL(NB) run_tile_q4<1, NB, WAVES, 2>(a, c, down, down + df / 2, a.d / 32, w.grp, hblk0, w.sp, e, scale)
        NB_SWITCH(CALL)
#undef CALL
    } else {
        constexpr int SX = 8;
        const int nstage = (c.nks + SX - 1) / SX;
        c.k0 = (int)((long long)w.sp * nstage / a.split_k) * SX;
        c.k1 = min((int)((long long)(w.sp + 1) * nstage / a.split_k) * SX, c.nks);
#define CALL(NB) run_tile_q4<1, NB, WAVES, 1>(a, c, down, down + df / 2, a.d / 32, w.grp, hblk0, w.sp, e, scale)
        NB_SWITCH(CALL)
#undef CALL
    }
}

template <int WAVES, int U>
void launch_up(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.f / 16 + WAVES * U - 1) / (WAVES * U);
    const int grid = (a.max_tiles * n_groups + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_up_kernel<WAVES, U>), dim3(grid), dim3(WAVES * 64), kLdsBytes, st, a,
                       n_groups);
}

template <int WAVES, int U>
void launch_down(hipStream_t st, const FfnArgs& a) {
    const int n_groups = (a.d / 32 + WAVES * U - 1) / (WAVES * U);
    const int grid = (a.max_tiles * n_groups * a.split_k + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((ffn_down_kernel<WAVES, U>), dim3(grid), dim3(WAVES * 64), kLdsBytes, st, a,
                       n_groups);
}

template <typename K>
hipError_t allow_lds(K kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

}  // namespace

int ffn_configure() {
    hipError_t e = allow_lds(&ffn_up_kernel<8, 1>);
    if (e == hipSuccess) e = allow_lds(&ffn_up_q4_kernel<8>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_q4_kernel<8>);
    if (e == hipSuccess) e = allow_lds(&ffn_up_kernel<7, 1>);
    if (e == hipSuccess) e = allow_lds(&ffn_up_kernel<4, 2>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<8, 1>);
    if (e == hipSuccess) e = allow_lds(&ffn_down_kernel<4, 2>);
    return (int)e;
}

// Launch shapes.  variant 1 / 2: eight / seven wavefronts per workgroup, one output unit each;
// variant 3: four wavefronts with two units each (every activation fragment read from LDS feeds
// two MFMAs).  Default: tiles expected to be full (many rows per expert, MFMA-bound) take the
// two-unit shape, small tiles (weight streaming dominates) eight single-unit wavefronts.
void launch_ffn_up_bf16(hipStream_t st, const FfnArgs& a) {
    if (a.weight_bits == 4) {
        const int n_groups = (a.f / 16 + 7) / 8;
        const int grid = (a.max_tiles * n_groups + kXcd - 1) / kXcd * kXcd;
        hipLaunchKernelGGL((ffn_up_q4_kernel<8>), dim3(grid), dim3(512), kLdsBytes, st, a, n_groups);
        return;
    }
    const int units = a.f / 16;
    int v = a.variant;
    if (v == 0) {
        v = a.full_tiles ? 3 : 1;
        if (!a.full_tiles) {
            // small tiles: the chip works through the workgroups in rounds of one per compute unit
            // (LDS); seven wavefronts per workgroup instead of eight when that fills the last
            // round better (rounds x units per workgroup is what the launch costs)
            const long tiles = a.est_tiles > 0 ? a.est_tiles : 1;
            auto cost = [&](int w) { return ((tiles * ((units + w - 1) / w) + 255) / 256) * w; };
            if (cost(7) < cost(8)) v = 2;
        }
    }
    if (v == 3 && units >= 2)
        launch_up<4, 2>(st, a);
    else if (v == 2)
        launch_up<7, 1>(st, a);
    else
        launch_up<8, 1>(st, a);
}

void launch_ffn_down_bf16(hipStream_t st, const FfnArgs& a) {
    if (a.weight_bits == 4) {  // 4-bit experts: weights dequantised in registers, same H format
        const int n_groups = (a.d / 32 + 7) / 8;
        const int grid = (a.max_tiles * n_groups * a.split_k + kXcd - 1) / kXcd * kXcd;
        hipLaunchKernelGGL((ffn_down_q4_kernel<8>), dim3(grid), dim3(512), kLdsBytes, st, a, n_groups);
        return;
    }
    // Two units per wavefront halve the LDS reads per MFMA: faster on full tiles (prefill layer)
    // and whenever the remainder plane is multiplied too (twice the MFMAs per weight byte); with
    // one plane on small tiles (decode layer) eight single-unit wavefronts are 2-3 % faster.
    const int units = a.d / 32;
    const bool two = (a.variant == 3 || (a.variant == 0 && (a.full_tiles || a.h_mode == 1))) && units >= 2;
    if (two) launch_down<4, 2>(st, a); else launch_down<8, 1>(st, a);
}

}  // namespace kmoe
