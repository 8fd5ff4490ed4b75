/*
 * moe_attn.h -- C ABI of the non-expert (attention) layer of the multi-batch pipeline.
 *
 * The expert layer works on all batches of a batch group at once; the non-expert layer is
 * run batch by batch, each batch bringing its own hidden state h and key-value cache c, which
 * may live in pinned host memory (paper Algorithm 1, else-branch: load the next batch's h and
 * c, compute this batch, store this batch's h and c; Section 8, "Overlapping Computation and
 * I/O": one stream prefetches the cache, another stores the new cache).  One call here runs
 * that inner loop for one layer and one decoding step over the whole batch group.
 *
 * The layer itself is the attention layer of the paper's model family with its normalisation
 * folded in (Section 2.1 and Section 4):
 *     xn = rmsnorm(x) * g;  q, k, v = Wq xn, Wk xn, Wv xn;  q, k rotated by position
 *     (rotary embedding, pairs (i, i + head_dim/2), angle pos * theta^(-2i/head_dim));
 *     cache[pos] = (k, v);  o_h = softmax(q_h K_g^T / sqrt(head_dim)) V_g over positions
 *     0..pos with g = h / (n_q_heads / n_kv_heads);  y = x + Wo concat(o_h).
 *
 * Conventions: as in moe.h (status codes, "dev" / "host" / "pinned", caller-owned memory and
 * streams, asynchronous calls).  All tensors are bf16, row-major.
 *   hidden state  : [n_seq, d_model]
 *   Wq            : [n_q_heads*head_dim, d_model];  Wk, Wv: [n_kv_heads*head_dim, d_model]
 *   Wo            : [d_model, n_q_heads*head_dim];  g: [d_model]
 *   K / V cache   : [n_seq, n_kv_heads, max_len, head_dim]; positions 0..pos-1 valid on entry,
 *                   position pos written by the call
 */
#ifndef KLOTSKI_MOE_ATTN_H
#define KLOTSKI_MOE_ATTN_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_attn_ctx moe_attn_ctx; /* opaque, library-owned */

typedef struct {
    int32_t d_model;    /* multiple of 128, at most 8192 */
    int32_t n_q_heads;  /* a multiple of n_kv_heads, at most 8 times it */
    int32_t n_kv_heads;
    int32_t head_dim;   /* 32, 64 or 128; n_q_heads*head_dim a multiple of 128 */
    int32_t max_seqs;   /* sequences per batch, at most */
    int32_t max_len;    /* capacity of every cache, in positions */
    int32_t n_layers;   /* attention layers whose weights one context holds (>= 1) */
    int32_t max_group_seqs; /* 0, or the sequences of a whole batch group at most: a group whose
                           batches all live on the device and whose sequences fit is run with
                           one launch per kernel, the projection weights read once for all */
    float rope_theta;
    float rms_eps;
} moe_attn_config;

/* One batch of the group. */
typedef struct {
    int32_t n_seq;      /* 1..max_seqs */
    int32_t pos;        /* cached positions of every sequence of the batch, 0..max_len-1 */
    int32_t kv_on_host; /* 1: k_cache / v_cache are pinned host memory and are streamed through a
                           device staging pair; 0: device memory, used in place */
    int32_t h_on_host;  /* the same for h_in / h_out */
    void* k_cache;      /* read 0..pos-1, written at pos */
    void* v_cache;
    const void* h_in;
    void* h_out;        /* may equal h_in */
} moe_attn_batch;

/* Timing of the last moe_attn_forward_group with profiling on (it then waits for the streams). */
typedef struct {
    double wall_s;         /* first copy or kernel start -> last store end */
    double load_busy_s;    /* sum over batches of the load stream's copy time */
    double store_busy_s;   /* the same for the store stream */
    double compute_busy_s; /* sum over batches of kernel time */
    double kernel_s[6];    /* the same per kernel: norm, q|k|v projection, rotation + cache append,
                              attention, output projection, residual */
    int64_t bytes_loaded;  /* host -> device */
    int64_t bytes_stored;  /* device -> host */
} moe_attn_profile;

/*
 * moe_attn_workspace_bytes -- host only, pure.  Device scratch a context needs (the packed
 * weights of n_layers layers, the two cache staging buffers shared by all layers, activations
 * and partial sums).  MOE_ERR_SHAPE on unsupported
 * sizes, MOE_ERR_INVALID_ARG on null.
 */
moe_status moe_attn_workspace_bytes(const moe_attn_config* cfg, int64_t* bytes_out);

/*
 * moe_attn_create -- workspace_dev: 256-byte aligned device memory of at least
 * moe_attn_workspace_bytes().  The three streams (hipStream_t as void*) must differ and have the
 * default priority; compute runs the kernels, load the host -> device copies of h and c, store
 * the device -> host copies.  The caller keeps ownership of all of them.
 */
moe_status moe_attn_create(const moe_attn_config* cfg, void* workspace_dev, int64_t workspace_bytes,
                           void* compute_stream, void* load_stream, void* store_stream,
                           moe_attn_ctx** out);
void moe_attn_destroy(moe_attn_ctx* ctx);

/*
 * moe_attn_set_weights -- packs the weights of `layer` into the workspace (device resident; the
 * weight stream of Algorithm 1, load(layers[j+1]), is the caller's: call this for the next
 * attention layer while the expert layer computes).  Pointers are device addresses unless
 * on_host != 0 (then plain or pinned host memory; the call copies synchronously).  Enqueued on
 * the compute stream.
 */
moe_status moe_attn_set_weights(moe_attn_ctx* ctx, int32_t layer, const void* g, const void* wq,
                                const void* wk, const void* wv, const void* wo, int32_t on_host);

/*
 * moe_attn_forward_group -- Algorithm 1, non-expert branch, for one decoding step of `layer`
 * (the caches of a batch are that layer's): for batch
 * b = 0..n_batches-1, wait for b's h and c on the load stream, start loading batch b+1 into
 * the other staging buffer, compute b, then store b's new cache row and hidden state on the
 * store stream.  (A group that is entirely on the device and fits max_group_seqs needs no such
 * order and is computed in one pass, see moe_attn_config.)  Returns after enqueueing; results are valid once the compute stream is
 * synchronised (it is made to wait for the last store).  The batches array is read during the
 * call only.  Errors: MOE_ERR_INVALID_ARG (null, layer, pos or n_seq out of range), MOE_ERR_STATE
 * (the layer has no weights), MOE_ERR_NOT_PINNED (a host pointer that is not pinned), MOE_ERR_HIP.
 */
moe_status moe_attn_forward_group(moe_attn_ctx* ctx, int32_t layer, int32_t n_batches,
                                  const moe_attn_batch* batches);

/*
 * moe_attn_prefetch -- Algorithm 1, expert-layer branch, "load(c[i][j+1][0])": while the expert
 * layer computes, start bringing the caches of the first batch of the next attention layer into
 * staging buffer 0 (load stream; it first waits for the compute work enqueued so far).  The next
 * moe_attn_forward_group whose first batch has the same caches, n_seq and pos uses them and
 * copies only that batch's hidden state; any other first batch is loaded as usual.  No-op for
 * device-resident caches.  Errors as for a batch of moe_attn_forward_group.
 */
moe_status moe_attn_prefetch(moe_attn_ctx* ctx, const moe_attn_batch* first);

/* Profiling: when on (1..64), every forward_group call times its streams with events and
 * synchronises.  With on = n > 1 each kernel but the last (the residual, which may work in place)
 * is launched n times back to back between its two events, same inputs and same outputs, so that
 * kernel_s is free of the event pair's own cost; wall_s and compute_busy_s then include the
 * repeats. */
moe_status moe_attn_set_profiling(moe_attn_ctx* ctx, int32_t on);
moe_status moe_attn_get_profile(moe_attn_ctx* ctx, moe_attn_profile* out);

/* Last error message of the context (or of the calling thread when ctx is null). */
const char* moe_attn_last_error(const moe_attn_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif
