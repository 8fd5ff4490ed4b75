/*
 * moe.h -- C ABI of the MI355X MoE-layer hot path (expert-aware multi-batch pipeline).
 *
 * One call sequence evaluates one Mixture-of-Experts layer for a whole batch group
 * (the tokens of B batches concatenated), expert by expert rather than batch by batch,
 * while the expert weights may live in pinned host memory and be streamed into a window
 * of device slots (paper Section 5 and Algorithm 1, expert-layer branch; Section 6.1 for
 * pinned host residency; Section 8, "Overlapping Computation and I/O", for the streams).
 *
 * Conventions
 *  - Every entry point returns a moe_status; nothing throws or aborts.  The library keeps no
 *    process-global state except the last error text of calls that have no context (kept per
 *    thread) and the static device scratch of moe_route_static.  A failed call leaves the
 *    context usable; the reason is available from moe_last_error().
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses,
 *    "pinned" host pointers must come from hipHostMalloc (e.g. a pin_memory tensor).
 *  - The caller owns all tensors, the workspace, the window and both streams
 *    (hipStream_t passed as void*).  The library owns only the context, a few events
 *    and a small pinned host mailbox.
 *  - moe_route, moe_stream_experts and moe_layer_forward enqueue work and return;
 *    results are valid once the compute stream has been synchronised.
 *  - Row-major everywhere.  X, Y: [n_tokens, d_model].  W1, W3: [d_ff, d_model].
 *    W2: [d_model, d_ff].  Wg: [n_experts, d_model].  Element type = config dtype.
 *  - Assignment a = t*top_k + j sends token t to expert topk_idx[a] (slot j).
 */
#ifndef KLOTSKI_MOE_H
#define KLOTSKI_MOE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque, library-owned */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1, /* null pointer, bad enum, index out of range */
    MOE_ERR_SHAPE = 2,       /* sizes the kernels do not support, or beyond the configured maxima */
    MOE_ERR_STATE = 3,       /* call order violated (e.g. forward before route, weights not set) */
    MOE_ERR_OOM = 4,         /* workspace or window too small */
    MOE_ERR_NOT_PINNED = 5,  /* a host pointer that must be pinned is not */
    MOE_ERR_HIP = 6          /* a HIP runtime call failed */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;
typedef enum { MOE_RESIDENT = 0, MOE_HOST_PINNED = 1 } moe_residency;

/* flags of moe_stream_experts */
#define MOE_PREFETCH 1  /* issued before the gate ran: the caller's guess of the hot experts */
#define MOE_ON_DEMAND 2 /* issued after the gate: experts the gate selected that are not in flight */

#define MOE_MAX_EXPERTS 256 /* routed experts per layer */
#define MOE_MAX_TOPK 8
#define MOE_MAX_BATCHES 64
#define MOE_MAX_SHARED 8

typedef struct {
    int32_t d_model;       /* d; bf16: multiple of 64, f32: multiple of 4 */
    int32_t d_ff;          /* f; bf16: multiple of 64, f32: multiple of 4 */
    int32_t n_experts;     /* E routed experts, 1..MOE_MAX_EXPERTS */
    int32_t top_k;         /* k, 1..min(E, MOE_MAX_TOPK) */
    int32_t n_shared;      /* S always-on experts (ids E..E+S-1), 0..MOE_MAX_SHARED */
    int32_t n_layers;      /* MoE layers handled by one context */
    int32_t window_layers; /* 0: all routed experts resident; >0: window of window_layers*E slots */
    int32_t max_tokens;    /* largest batch group (tokens) a call may bring */
    int32_t max_batches;   /* largest number of batches in a group, <= MOE_MAX_BATCHES */
    int32_t dtype;         /* moe_dtype of X, Y and all weights */
    int32_t renormalize;   /* 1: routing weights renormalised over the k winners; 0: full softmax */
    int32_t weight_bits;   /* 0 or 16: expert weights as dtype; 4 (bf16 only): 4-bit codes in groups
                              of 64 with a bf16 scale and zero point each, set with moe_set_expert_q4 */
} moe_config;

/* Sizes and first-order time estimates for one configuration (moe_plan). */
typedef struct {
    int64_t workspace_bytes; /* device scratch moe_create needs */
    int64_t expert_bytes;    /* packed size of one expert = size of one window slot */
    int64_t window_bytes;    /* n_slots * expert_bytes (0 when window_layers == 0) */
    int32_t n_slots;         /* window_layers * n_experts */
    int32_t reserved;
    double t_io_expert_s;    /* expert_bytes / link_Bps: one expert over the host link */
    double t_c_expert_s;     /* max(expert_bytes/hbm_Bps, flops/mfma_flops) at n_tokens*k/E rows */
    double t_c_gate_s;       /* gate: bytes of X over hbm_Bps */
} moe_plan_t;

/* Counters of the pipeline, cumulative since moe_create or moe_reset_stats. */
typedef struct {
    int64_t tokens;          /* tokens routed */
    int64_t bytes_h2d;       /* expert bytes copied host -> device */
    int64_t n_copies;        /* expert copies issued */
    int64_t n_prefetch_hits; /* experts needed by a layer that were already in flight or resident */
    int64_t n_prefetch_unused; /* prefetched experts that the gate then did not select */
    int64_t n_forward;       /* moe_layer_forward calls */
    int64_t n_active_sum;    /* sum over forwards of activated routed experts */
    int64_t h_saturated;     /* values of the intermediate H clamped to the fp16 range (0 in any sane layer) */
    int64_t h_remainder_wgs; /* down-projection workgroups that multiplied the remainder plane of H because the
                                recorded remainder energy of their tile asked for it (h_planes 1, see moe_set_tuning) */
    /* The three times below cover the work enqueued while profiling was on (moe_set_profiling)
     * since the last moe_reset_stats, measured with HIP events around every expert copy and
     * every group of kernels; 0 when nothing was recorded.  The pipeline's bubble (paper
     * Section 3 and Section 7, T = T_c + T_b) is 1 - compute_busy_ns / wall_ns; the idle
     * fraction of the host link is 1 - copy_busy_ns / wall_ns. */
    int64_t copy_busy_ns;    /* time with at least one expert copy in progress (union over the copy streams) */
    int64_t compute_busy_ns; /* time the compute stream spent in this library's kernels */
    int64_t wall_ns;         /* first recorded start to last recorded end */
} moe_stats;

/*
 * moe_plan -- host only, pure.  Sizes the workspace and the window for `cfg`, and prices one
 * expert's transfer and compute at the given rates (bytes/s, bytes/s, flop/s) for a batch
 * group of n_tokens tokens: the per-shape quantities the paper's planner measures
 * (Section 7, stage "measurement"; t_IO_E and t_c_E of the inequality group).
 * Errors: MOE_ERR_INVALID_ARG (null), MOE_ERR_SHAPE (unsupported sizes).
 */
moe_status moe_plan(const moe_config* cfg, int32_t n_tokens, double hbm_Bps, double link_Bps,
                    double mfma_flops, moe_plan_t* out);

/*
 * moe_plan_batches -- host only, pure.  Smallest integer n (batches per batch group) that
 * satisfies the four overlap inequalities of the paper's planner (Section 7, inequality
 * group; the legend's t_c_topk-E is the formulas' t_c_hot-E; the sum runs over the queue Q
 * of activated non-hot experts).  All times in seconds; t_c_E has len_q entries.
 * Returns n >= 1 in *n_out; MOE_ERR_INVALID_ARG when t_c_A + t_c_G <= 0 while I/O is not.
 */
moe_status moe_plan_batches(double t_c_A, double t_c_G, double t_c_hotE, const double* t_c_E,
                            int32_t len_q, double t_io_A, double t_io_G, double t_io_E, int32_t K,
                            int32_t* n_out);

/*
 * moe_create -- build a context.  workspace_dev: device scratch of at least
 * moe_plan().workspace_bytes, 256-byte aligned.  window_dev: device memory of at least
 * window_bytes when cfg->window_layers > 0, else ignored (may be null).  Streams are
 * hipStream_t; the copy stream must differ from the compute stream when a window is used.
 * The buffers and streams must outlive the context.  The HIP runtime maps streams onto a few
 * hardware queues; a copy stream that shares its queue with the compute stream has its copies
 * wait behind the expert kernels (seen as a link idle of 15-20 % on small experts).  Creating the
 * compute stream and the copy stream first, one after the other, and keeping them for the life of
 * the process has kept them on queues of their own.
 */
moe_status moe_create(const moe_config* cfg, void* compute_stream, void* copy_stream,
                      void* workspace_dev, int64_t workspace_bytes, void* window_dev,
                      int64_t window_bytes, moe_ctx** out);

/* moe_destroy -- synchronises both streams, releases events and the mailbox. */
moe_status moe_destroy(moe_ctx* ctx);

/* moe_set_gate -- register the gate matrix Wg [E, d] (device) of a layer: the gating network
 * whose softmax scores select the top-k experts of every token (paper Section 2.1).  Not copied. */
moe_status moe_set_gate(moe_ctx* ctx, int32_t layer, const void* wg_dev);

/*
 * moe_set_expert -- offline placement of one expert (paper Section 4: placement happens in
 * an offline phase before inference).  Reads W1, W3, W2 (device, row-major) and writes the
 * expert's packed blob (moe_plan().expert_bytes bytes, a layout private to the library) to
 * packed_dst: device memory when where == MOE_RESIDENT, pinned host memory when
 * where == MOE_HOST_PINNED (requires a window; shared experts must be resident).
 * Synchronous.  packed_dst must stay valid while the context lives; the sources need not.
 * expert in [0, E) routed, [E, E+S) shared.
 */
moe_status moe_set_expert(moe_ctx* ctx, int32_t layer, int32_t expert, const void* w1_dev,
                          const void* w3_dev, const void* w2_dev, int32_t where, void* packed_dst);

/*
 * moe_set_expert_q4 -- placement of one 4-bit group-quantised expert (contexts created with
 * weight_bits == 4).  Quantisation and dequantisation follow the paper's Eq. 8 (Section 7,
 * "Quantization"): W = s * (W_q - z) with one scale s and one real zero point z per group of 64
 * consecutive weights of a row.  For each of W1, W3 ([f, d]) and W2 ([d, f]), all device
 * pointers: q = codes, uint8 [rows, cols / 2], the even column in the low nibble; s, z = bf16
 * [rows, cols / 64].  How s and z were fitted is the caller's business.  The kernels turn a
 * weight back into bf16 (fp32 fma, one rounding) right before it is multiplied.  (If an expert's
 * dequantised W2 would leave the fp16 range of the down projection, the packed copy of its scales
 * is multiplied by a power of two, undone on the outputs: exact.)  Everything
 * else as moe_set_expert; the packed blob has moe_plan().expert_bytes = 27/16 * d * f bytes.
 */
moe_status moe_set_expert_q4(moe_ctx* ctx, int32_t layer, int32_t expert, const void* q1_dev,
                             const void* s1_dev, const void* z1_dev, const void* q3_dev,
                             const void* s3_dev, const void* z3_dev, const void* q2_dev,
                             const void* s2_dev, const void* z2_dev, int32_t where, void* packed_dst);

/*
 * moe_route -- gate + dispatch plan of one layer for a batch group (Section 2.1: softmax gate,
 * top-k; Section 5: expert layer divided by experts, hot experts first).
 *   x_dev [n_tokens, d]; batch_offsets_host[n_batches+1], non-decreasing, starts at 0,
 *   n_tokens = batch_offsets_host[n_batches] <= max_tokens (0 is allowed: no work).
 * Optional device outputs (null = not wanted), all valid after the compute stream syncs:
 *   logits_dev [n_tokens, E] f32      fp32 gate logits (fixed summation order)
 *   topk_idx_dev [n_tokens, k] i32    winners by (logit desc, index asc)
 *   topk_w_dev [n_tokens, k] f32      routing weights
 *   counts_dev [E], offsets_dev [E+1] tokens per expert and their exclusive scan
 *   perm_dev, inv_perm_dev [n_tokens*k] stable grouping of assignments by expert
 *   exec_order_dev [E]                activated experts by (batches touching desc, tokens desc,
 *                                     index asc); -1 beyond the activated ones
 * counts and exec_order are also mailed to the host (see moe_route_wait).
 */
moe_status moe_route(moe_ctx* ctx, int32_t layer, const void* x_dev,
                     const int32_t* batch_offsets_host, int32_t n_batches, float* logits_dev,
                     int32_t* topk_idx_dev, float* topk_w_dev, int32_t* counts_dev,
                     int32_t* offsets_dev, int32_t* perm_dev, int32_t* inv_perm_dev,
                     int32_t* exec_order_dev);

/*
 * moe_route_wait -- block until the last moe_route's counts reached the host, then copy them
 * out: counts_host[E], exec_order_host[E] (-1 padded), *n_active (any may be null).
 * This is the point where the paper's pipeline learns which experts the gate selected and
 * starts their on-demand transfers (Section 5).
 */
moe_status moe_route_wait(moe_ctx* ctx, int32_t* counts_host, int32_t* exec_order_host,
                          int32_t* n_active);

/*
 * moe_route_static -- for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The gate + dispatch plan of moe_route without
 * a context and without a workspace: the scratch the dispatch kernels need beyond their inputs
 * and outputs (per-chunk histograms, padded offsets, batches per expert, tile tables, and any
 * of the outputs below that the caller does not ask for) lives in a fixed array of 1.5 MiB in
 * the library's device image, one copy per GPU, held until the process ends.  The call
 * allocates nothing (no hipMalloc, hipFree, hipHostMalloc, event or stream creation); it
 * enqueues the router and the dispatch kernels on `stream` (hipStream_t) and returns.
 *   dtype: moe_dtype of x_dev [n_tokens, d_model] and wg_dev [n_experts, d_model], both device.
 *   batch_offsets_host[n_batches + 1]: as for moe_route; must end at n_tokens.
 *   Outputs: as for moe_route, device pointers, each optional; same values bit for bit.
 * Limits: n_tokens <= MOE_STATIC_MAX_TOKENS and n_tokens * top_k <= MOE_STATIC_MAX_ASSIGNMENTS
 * (beyond: MOE_ERR_SHAPE, nothing is launched); d_model a multiple of 64 (bf16) or 4 (f32).
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (the
 * kernels rewrite all they read, nothing needs clearing): calls that overlap on one GPU -- from
 * two streams or two threads -- race; calls on one stream are ordered and safe.
 * The error text of a failed call is available from moe_last_error(NULL) on the calling thread.
 */
#define MOE_STATIC_MAX_TOKENS 65536
#define MOE_STATIC_MAX_ASSIGNMENTS 65536
moe_status moe_route_static(void* stream, int32_t dtype, const void* x_dev, const void* wg_dev,
                            int32_t n_tokens, int32_t d_model, int32_t n_experts, int32_t top_k,
                            int32_t renormalize, const int32_t* batch_offsets_host, int32_t n_batches,
                            float* logits_dev, int32_t* topk_idx_dev, float* topk_w_dev,
                            int32_t* counts_dev, int32_t* offsets_dev, int32_t* perm_dev,
                            int32_t* inv_perm_dev, int32_t* exec_order_dev);

/*
 * moe_stream_experts -- enqueue host->device copies of routed experts of `layer` on the copy
 * stream, in the order given (Section 5: prefetch the hot experts before the gate, transfer
 * the rest on demand after it, never transfer experts nobody selected).  Each expert goes to
 * a free window slot; a slot is reused only after the kernels that read it have finished.
 * Experts already resident or in flight for this layer are skipped.  With MOE_ON_DEMAND the
 * ids must be among the experts the last moe_route activated.  Returns MOE_ERR_OOM if no
 * slot can be freed (window smaller than one layer's activated experts plus prefetches).
 */
moe_status moe_stream_experts(moe_ctx* ctx, int32_t layer, const int32_t* expert_ids_host,
                              int32_t n_ids, int32_t flags);

/*
 * moe_layer_forward -- Y = MoE layer(X) for the batch group of the last moe_route on this
 * layer: grouped SwiGLU experts over each expert's tokens, in exec_order, then
 * Y[t] = sum_j w[t,j]*FFN_{idx[t,j]}(X[t]) + sum_s FFN_{E+s}(X[t]) (Section 2.1).
 * With a window, activated experts not yet in flight are transferred on demand first, each
 * expert's kernels wait for its copy, and its slot is released right after its last kernel
 * (Section 5, last sentence of "minimizing intra-layer bubbles").
 * x_dev must be the tensor given to moe_route.  y_dev [n_tokens, d] in the config dtype.
 */
moe_status moe_layer_forward(moe_ctx* ctx, int32_t layer, const void* x_dev, void* y_dev);

/* moe_get_stats blocks until the compute stream (and, for the three times, the recorded copies)
 * are done.  moe_reset_stats zeroes the counters and drops the recorded spans. */
moe_status moe_get_stats(moe_ctx* ctx, moe_stats* out);
moe_status moe_reset_stats(moe_ctx* ctx);

/*
 * moe_set_tuning -- knobs, 0 keeps the current value.  split_k: split of the down projection's
 * reduction (auto by default).
 * h_planes (bf16 path): the intermediate H = silu(X W1^T) .* (X W3^T) is handed from the up
 * projections to the down projection as fp16 (W2 is placed as fp16 as well, times a power of two
 * when it holds weights beyond the fp16 range, undone on the outputs), together with a second
 * fp16 plane holding the rounding remainder H - fp16(H).  1 (default): the down projection
 * multiplies the remainder plane only for the tiles that need it -- the up kernel records the
 * energy of the remainders per token row, and a tile whose rows all stay below the expert's
 * threshold (6 standard deviations of the remainders' contribution to an output within 0.8 of
 * the 1e-2 absolute tolerance, from the row energies of W2 taken at placement) is computed from
 * the value plane alone, at half the matrix-core work.  2: the remainder plane is always
 * multiplied (outputs then never depend on which tokens share a tile).  4-bit experts use the same
 * format: their W2 is turned back into bf16 in registers and handed to the fp16 MFMA as fp16.
 * variant: launch shape of the bf16 expert kernels, ones digit: 1 = 8 wavefronts x 1 output unit,
 * 2 = 7 x 1, 3 = 4 x 2 (0 = chosen by tile size); tens digit p (1..6): on full tiles the workgroups
 * an XCD runs together cover 2^(p-1) tiles x 32/2^(p-1) unit groups (0 = 4 x 8); -1 selects the
 * defaults again.
 */
moe_status moe_set_tuning(moe_ctx* ctx, int32_t split_k, int32_t h_planes, int32_t variant);

/*
 * Measurement stage of the constraint-sensitive planner (paper Section 7: before inference the
 * computation and transfer times of the layer's parts are measured on the machine at hand and
 * then applied to the inequality group, see moe_plan_batches).  Runs on the given batch group:
 * the gate + dispatch plan, `reps` times; one expert's transfer from pinned host memory into a
 * window slot, `reps` times (0 when the layer has no host-resident expert); then gather, the two
 * expert kernels of every activated routed expert on its own tokens, one expert at a time in
 * execution order, and the combine.  Blocks until done; leaves no expert in the window and the
 * context as after a moe_route of this group.  y_dev receives the layer output of the group
 * only if every expert of the layer is resident (otherwise the timed kernels run on a stand-in
 * blob and y_dev is scratch).  All times in seconds, device time between HIP events.
 */
typedef struct {
    double t_c_gate_group_s;                /* router + plan for the whole group */
    double t_io_expert_s;                   /* one expert blob over the host link */
    double t_c_gather_s, t_c_combine_s;     /* once per group */
    double t_c_expert_s[MOE_MAX_EXPERTS];   /* up + down of expert e over the group's tokens; 0 = not activated */
    int32_t n_active;
    int32_t exec_order[MOE_MAX_EXPERTS];    /* activated experts, execution order */
    int32_t counts[MOE_MAX_EXPERTS];        /* tokens per expert */
} moe_measured;
moe_status moe_measure(moe_ctx* ctx, int32_t layer, const void* x_dev,
                       const int32_t* batch_offsets_host, int32_t n_batches, void* y_dev,
                       int32_t reps, moe_measured* out);

/*
 * Correlation-aware expert prefetcher, path length 1 (paper Section 6.2).  Per layer the library
 * keeps a table T[layer][p][e]: how often a token that activated expert p in layer - 1 activated
 * expert e in this layer (every pair of a previous and a current top-k slot counts once).
 *
 * moe_corr_enable(mode): 0 = off, 1 = learn and predict, 2 = predict from the table as it is.
 * While learning, every moe_route(layer) that follows a moe_route(layer - 1)
 * of the same number of tokens adds the transitions of the batch group to T[layer] (one small
 * kernel with integer atomics on the compute stream) and refreshes the host mirror of T[layer].
 * The table lives in the caller's workspace and is zeroed by moe_create and moe_corr_reset
 * (both stream-ordered on the compute stream).
 *
 * moe_corr_predict(layer, K): the K experts of `layer` that the batch group routed last (which
 * must have been routed through layer - 1) tends to: score[e] = sum over previous experts p of
 * counts[p] * T[layer][p][e] / rowsum(T[layer][p]) in fp64, p ascending; best K by (score desc,
 * index asc), zero scores never returned.  Host only; blocks until the last moe_route has
 * delivered its counts.  experts_out_host has room for K ids; *n_out <= K.
 * Errors: MOE_ERR_STATE (not enabled, or the last routed layer is not layer - 1).
 *
 * moe_corr_table: copies the host mirror of T[layer] (E*E int32, row = previous expert).
 * moe_corr_rank: the ranking alone, pure host function (no context): table [E][E] int32, the
 * previous layer's tokens per expert; score_out (E doubles) may be null.
 */
moe_status moe_corr_enable(moe_ctx* ctx, int32_t mode);
moe_status moe_corr_reset(moe_ctx* ctx);
moe_status moe_corr_predict(moe_ctx* ctx, int32_t layer, int32_t K, int32_t* experts_out_host,
                            int32_t* n_out);
moe_status moe_corr_table(moe_ctx* ctx, int32_t layer, int32_t* table_out_host);
moe_status moe_corr_rank(const int32_t* table_host, const int32_t* counts_prev_host, int32_t E,
                         int32_t K, int32_t* experts_out_host, int32_t* n_out, double* score_out);

/*
 * moe_set_profiling(1) turns on two things: HIP events around every expert copy and every group
 * of kernels, from which moe_get_stats derives copy_busy_ns, compute_busy_ns and wall_ns (the
 * events cost a few microseconds each: time throughput with profiling off); and the
 * per-kernel timing of the last moe_route + moe_layer_forward pair (all-resident layers only),
 * taken with HIP events on the compute stream between the launches.  For the fp32 path up_ms is
 * 0 and down_ms covers both expert kernels.  moe_get_profile blocks until that forward is done.
 */
typedef struct {
    float router_ms, plan_ms, gather_ms, up_ms, down_ms, combine_ms;
} moe_profile;
moe_status moe_set_profiling(moe_ctx* ctx, int32_t enable);
moe_status moe_get_profile(moe_ctx* ctx, moe_profile* out);

/* Last error text of the context (or of the last failed moe_create/moe_plan when ctx is null). */
const char* moe_last_error(const moe_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* KLOTSKI_MOE_H */
