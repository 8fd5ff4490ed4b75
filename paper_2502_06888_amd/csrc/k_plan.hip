// Dispatch plan: per-expert counts, prefix sums, stable grouping of assignments by expert,
// execution order of the experts, and the tile tables the grouped FFN walks.
//
// The expert layer is evaluated expert by expert over the tokens of all batches of the batch
// group, experts that serve the most batches / tokens first (paper Section 5).  Everything
// here is integer work with a unique answer: histograms use LDS atomics (order-free), stable
// ranks come from wavefront ballots and per-segment prefix sums.
#include "kernels.h"

namespace kmoe {
namespace {

constexpr int kThreads = 256;
constexpr int kRounds = kPlanChunk / kThreads;  // 4
constexpr int kSegs = kRounds * (kThreads / 64);  // 16 (round, wave) segments per chunk

// The batch offsets arrive as a kernel argument; a per-lane index into them would be a chain of
// dependent global loads, so they are first copied to LDS (sbo, kMaxBatches + 1 ints).
__device__ __forceinline__ void stage_offsets(const BatchOffsets& bo, int32_t* sbo) {
    for (int b = threadIdx.x; b <= kMaxBatches; b += kThreads) sbo[b] = bo.v[b];
}

__device__ __forceinline__ int batch_of(const int32_t* sbo, int n, int t) {
    int lo = 0, hi = n;  // find b with v[b] <= t < v[b+1]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (sbo[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// P1: per chunk of assignments, tokens per expert and the set of batches touching each expert.
__global__ __launch_bounds__(kThreads) void plan_count_kernel(const int32_t* __restrict__ idx,
                                                              int A, int E, int k, BatchOffsets bo,
                                                              int32_t* __restrict__ blk_counts,
                                                              unsigned long long* __restrict__ blk_mask) {
    __shared__ int32_t cnt[kMaxExperts];
    __shared__ unsigned long long msk[kMaxExperts];
    __shared__ int32_t sbo[kMaxBatches + 1];
    stage_offsets(bo, sbo);
    for (int e = threadIdx.x; e < E; e += kThreads) {
        cnt[e] = 0;
        msk[e] = 0ull;
    }
    __syncthreads();
    const int base = blockIdx.x * kPlanChunk;
    for (int r = 0; r < kRounds; ++r) {
        const int a = base + r * kThreads + threadIdx.x;
        if (a < A) {
            const int e = idx[a];
            atomicAdd(&cnt[e], 1);
            atomicOr(&msk[e], 1ull << batch_of(sbo, bo.n, a / k));
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kThreads) {
        blk_counts[(size_t)blockIdx.x * E + e] = cnt[e];
        blk_mask[(size_t)blockIdx.x * E + e] = msk[e];
    }
}

// Totals -> scans, execution order, tile tables, host mail.  cnt[] and nbt[] hold the tokens
// and the batches of every expert on entry; off[], pof[], ord[] and nact are LDS scratch.
__device__ __forceinline__ void scan_body(const Shape& s, const PlanPtrs& p, int max_tiles,
                                          int32_t* cnt, int32_t* nbt, int32_t* off, int32_t* pof,
                                          int32_t* ord, int32_t* nact_p) {
    const int E = s.E, tid = threadIdx.x;
    if (tid == 0) {
        *nact_p = 0;
        int o = 0, po = 0;
        for (int e = 0; e < E; ++e) {
            off[e] = o;
            pof[e] = po;
            o += cnt[e];
            po += (cnt[e] + kRowBlk - 1) / kRowBlk * kRowBlk;
        }
        off[E] = o;
        pof[E] = po;
    }
    for (int e = tid; e < E; e += kThreads) ord[e] = -1;
    __syncthreads();
    // execution order: rank of e among the activated experts by (nbatch desc, count desc, e asc)
    for (int e = tid; e < E; e += kThreads) {
        if (cnt[e] > 0) {
            int rank = 0;
            for (int q = 0; q < E; ++q) {
                if (q == e || cnt[q] == 0) continue;
                const bool q_first = nbt[q] > nbt[e] ||
                                     (nbt[q] == nbt[e] && (cnt[q] > cnt[e] || (cnt[q] == cnt[e] && q < e)));
                rank += q_first ? 1 : 0;
            }
            ord[rank] = e;
            atomicAdd(nact_p, 1);
        }
    }
    __syncthreads();
    const int nact = *nact_p;
    for (int e = tid; e < E; e += kThreads) {
        p.counts[e] = cnt[e];
        p.offsets[e] = off[e];
        p.poff[e] = pof[e];
        p.nbatch[e] = nbt[e];
        p.exec_order[e] = ord[e];
        p.mail[e] = cnt[e];
        p.mail[E + e] = ord[e];
        p.exp_tile0[e] = 0;
        p.exp_ntiles[e] = 0;
        const int b0 = pof[e] / kRowBlk, nb = (cnt[e] + kRowBlk - 1) / kRowBlk;
        for (int b = 0; b < nb; ++b) p.blk_expert[b0 + b] = e;
    }
    __syncthreads();  // exp_tile0 / exp_ntiles are zeroed before thread 0 fills them
    if (tid == 0) {
        p.offsets[E] = off[E];
        p.poff[E] = pof[E];
        p.mail[2 * E] = nact;
        // tiles: shared experts first (they serve every batch), then routed in execution order
        int nt = 0;
        const int routed_blks = pof[E] / kRowBlk;
        const int nblk_tok = (s.N + kRowBlk - 1) / kRowBlk;
        for (int sh = 0; sh < s.S; ++sh) {
            const int first = nt;  // kept in a register: reading exp_tile0 back would wait on the store
            p.exp_tile0[E + sh] = first;
            for (int b = 0; b < nblk_tok && nt < max_tiles; b += kTileBlks) {
                p.tile_expert[nt] = E + sh;
                p.tile_xblk[nt] = routed_blks + b;
                p.tile_hblk[nt] = routed_blks + sh * nblk_tok + b;
                p.tile_nblk[nt] = min(kTileBlks, nblk_tok - b);
                ++nt;
            }
            p.exp_ntiles[E + sh] = nt - first;
        }
        for (int i = 0; i < nact; ++i) {
            const int e = ord[i];
            const int b0 = pof[e] / kRowBlk, nb = (cnt[e] + kRowBlk - 1) / kRowBlk;
            const int first = nt;
            p.exp_tile0[e] = first;
            for (int b = 0; b < nb && nt < max_tiles; b += kTileBlks) {
                p.tile_expert[nt] = e;
                p.tile_xblk[nt] = b0 + b;
                p.tile_hblk[nt] = b0 + b;
                p.tile_nblk[nt] = min(kTileBlks, nb - b);
                ++nt;
            }
            p.exp_ntiles[e] = nt - first;
        }
        p.meta[0] = nact;
        p.meta[1] = nt;
        p.meta[2] = routed_blks;
        p.meta[3] = s.N;
    }
}

// P2: one block.  Sums the per-chunk histograms, then scan_body.  The chunk histograms pass through
// LDS in panels of kScanPanel entries (whole chunks): all threads load a panel (coalesced), one
// thread per expert runs down its column in LDS, all threads store the exclusive bases.  (One
// thread per expert walking global memory chunk by chunk took 34 us on a 32-chunk layer: a chain
// of dependent loads.)
constexpr int kScanPanel = 4096;
__global__ __launch_bounds__(kThreads) void plan_scan_kernel(Shape s, int nchunks, PlanPtrs p,
                                                             int max_tiles) {
    __shared__ int32_t cnt[kMaxExperts];
    __shared__ int32_t nbt[kMaxExperts];
    __shared__ int32_t off[kMaxExperts + 1];
    __shared__ int32_t pof[kMaxExperts + 1];
    __shared__ int32_t ord[kMaxExperts];
    __shared__ int32_t nact;
    __shared__ int32_t panel[kScanPanel];
    __shared__ unsigned long long pmask[kMaxExperts];
    static_assert(kScanPanel >= kMaxExperts, "a panel holds at least one chunk");
    const int E = s.E;
    for (int e = threadIdx.x; e < E; e += kThreads) {
        cnt[e] = 0;
        pmask[e] = 0ull;
    }
    __syncthreads();
    const int per_panel = kScanPanel / E;  // whole chunks per panel
    for (int c0 = 0; c0 < nchunks; c0 += per_panel) {
        const int nc = min(per_panel, nchunks - c0);
        const size_t g0 = (size_t)c0 * E;
        for (int i = threadIdx.x; i < nc * E; i += kThreads) panel[i] = p.blk_counts[g0 + i];
        // batch masks: or-reduced per expert (order-free)
        for (int i = threadIdx.x; i < nc * E; i += kThreads) {
            const unsigned long long m = p.blk_mask[g0 + i];
            if (m) atomicOr(&pmask[i % E], m);
        }
        __syncthreads();
        for (int e = threadIdx.x; e < E; e += kThreads) {
            int run = cnt[e];
            for (int c = 0; c < nc; ++c) {
                const int v = panel[c * E + e];
                panel[c * E + e] = run;
                run += v;
            }
            cnt[e] = run;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < nc * E; i += kThreads) p.blk_base[g0 + i] = panel[i];
        __syncthreads();
    }
    for (int e = threadIdx.x; e < E; e += kThreads) nbt[e] = __popcll(pmask[e]);
    __syncthreads();
    scan_body(s, p, max_tiles, cnt, nbt, off, pof, ord, &nact);
}

// Stable position of every assignment of one chunk inside its expert's group.  off[] are the
// exclusive expert offsets, base[] (may be null = zeros) the tokens of earlier chunks.
__device__ __forceinline__ void rank_body(const int32_t* __restrict__ idx, int A, int E,
                                          const PlanPtrs& p, int chunk, int32_t (*seg)[kMaxExperts],
                                          const int32_t* off, const int32_t* base_of_chunk,
                                          const int32_t* preloaded = nullptr) {
    for (int i = threadIdx.x; i < kSegs * kMaxExperts; i += kThreads) (&seg[0][0])[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = chunk * kPlanChunk;
    int my_e[kRounds], my_rank[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int a = base + r * kThreads + threadIdx.x;
        const int e = preloaded ? preloaded[r] : (a < A ? idx[a] : -1);
        my_e[r] = e;
        my_rank[r] = 0;
        bool done = e < 0;
        // group the wavefront's lanes by expert; every pass retires the leader's group
        while (true) {
            const unsigned long long pending = __ballot(!done);
            if (pending == 0ull) break;
            const int leader = __ffsll((long long)pending) - 1;
            const int ev = __shfl(e, leader, 64);
            const unsigned long long same = __ballot(e == ev);
            if (e == ev) {
                my_rank[r] = __popcll(same & ((1ull << lane) - 1ull));
                if (lane == leader) seg[r * (kThreads / 64) + wave][ev] = __popcll(same);
                done = true;
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kThreads) {  // exclusive scan over the 16 segments
        int run = 0;
#pragma unroll
        for (int sg = 0; sg < kSegs; ++sg) {
            const int c = seg[sg][e];
            seg[sg][e] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int a = base + r * kThreads + threadIdx.x;
        const int e = my_e[r];
        if (e >= 0) {
            const int pos = off[e] + (base_of_chunk ? base_of_chunk[e] : 0) +
                            seg[r * (kThreads / 64) + wave][e] + my_rank[r];
            p.inv_perm[a] = pos;
            p.perm[pos] = a;
        }
    }
}

// P3: one block per chunk.
__global__ __launch_bounds__(kThreads) void plan_rank_kernel(const int32_t* __restrict__ idx, int A,
                                                             int E, PlanPtrs p) {
    __shared__ int32_t seg[kSegs][kMaxExperts];  // tokens of expert e in (round, wave) segment
    rank_body(idx, A, E, p, blockIdx.x, seg, p.offsets, p.blk_base + (size_t)blockIdx.x * E);
}

// All three phases in one block, for batch groups of at most one chunk of assignments.
__global__ __launch_bounds__(kThreads) void plan_fused_kernel(const int32_t* __restrict__ idx,
                                                              Shape s, BatchOffsets bo, PlanPtrs p,
                                                              int max_tiles) {
    __shared__ int32_t cnt[kMaxExperts];
    __shared__ unsigned long long msk[kMaxExperts];
    __shared__ int32_t nbt[kMaxExperts];
    __shared__ int32_t off[kMaxExperts + 1];
    __shared__ int32_t pof[kMaxExperts + 1];
    __shared__ int32_t ord[kMaxExperts];
    __shared__ int32_t nact;
    __shared__ int32_t seg[kSegs][kMaxExperts];
    __shared__ int32_t sbo[kMaxBatches + 1];
    const int A = s.N * s.k;
    int32_t mine[kRounds];  // this thread's assignments, loaded once for both phases
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int a = r * kThreads + threadIdx.x;
        mine[r] = a < A ? idx[a] : -1;
    }
    stage_offsets(bo, sbo);
    for (int e = threadIdx.x; e < s.E; e += kThreads) {
        cnt[e] = 0;
        msk[e] = 0ull;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int a = r * kThreads + threadIdx.x;
        if (mine[r] >= 0) {
            atomicAdd(&cnt[mine[r]], 1);
            atomicOr(&msk[mine[r]], 1ull << batch_of(sbo, bo.n, a / s.k));
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < s.E; e += kThreads) nbt[e] = __popcll(msk[e]);
    __syncthreads();
    scan_body(s, p, max_tiles, cnt, nbt, off, pof, ord, &nact);
    __syncthreads();
    rank_body(idx, A, s.E, p, 0, seg, off, nullptr, mine);
}

// Correlation table update (paper Section 6.2, path length 1): one thread per token adds its
// k x k (previous expert, current expert) pairs to the layer's table.  Integer atomics: the
// result does not depend on the order.
__global__ __launch_bounds__(kThreads) void corr_update_kernel(const int32_t* __restrict__ idx_prev,
                                                               const int32_t* __restrict__ idx_cur,
                                                               int N, int k, int E,
                                                               int32_t* __restrict__ table) {
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= N) return;
    for (int a = 0; a < k; ++a) {
        const int p = idx_prev[(size_t)t * k + a];
        for (int b = 0; b < k; ++b) atomicAdd(&table[(size_t)p * E + idx_cur[(size_t)t * k + b]], 1);
    }
}

}  // namespace

void launch_corr_update(hipStream_t st, const int32_t* idx_prev, const int32_t* idx_cur, int N, int k,
                        int E, int32_t* table) {
    if (N <= 0) return;
    hipLaunchKernelGGL(corr_update_kernel, dim3((N + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                       idx_prev, idx_cur, N, k, E, table);
}

void launch_plan(hipStream_t st, const Shape& s, const BatchOffsets& bo, const PlanPtrs& p,
                 int max_tiles) {
    const int A = s.N * s.k;
    const int nchunks = (A + kPlanChunk - 1) / kPlanChunk;
    if (nchunks <= 1) {
        hipLaunchKernelGGL(plan_fused_kernel, dim3(1), dim3(kThreads), 0, st, p.topk_idx, s, bo, p,
                           max_tiles);
        return;
    }
    if (nchunks > 0) {
        hipLaunchKernelGGL(plan_count_kernel, dim3(nchunks), dim3(kThreads), 0, st, p.topk_idx, A,
                           s.E, s.k, bo, p.blk_counts, p.blk_mask);
    }
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(kThreads), 0, st, s, nchunks, p, max_tiles);
    if (nchunks > 0) {
        hipLaunchKernelGGL(plan_rank_kernel, dim3(nchunks), dim3(kThreads), 0, st, p.topk_idx, A,
                           s.E, p);
    }
}

}  // namespace kmoe
