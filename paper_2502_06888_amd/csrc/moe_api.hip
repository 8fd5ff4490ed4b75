// C-ABI of the MoE-layer hot path: context, offline placement, routing, expert streaming and
// the layer forward.  Host logic only; the kernels live in the k_*.hip files.
//
// Pipeline (paper Section 5 / Algorithm 1, expert-layer branch): prefetch the experts the
// caller expects to be hot before the gate runs; run the gate for all batches of the group at
// once; start on-demand transfers for the activated experts that are not in flight; run the
// experts in execution order, each one as soon as its weights have landed; release an
// expert's slot right after its last kernel.  Copies run on a dedicated stream and are tied
// to the compute stream by per-slot events (Section 8, "Overlapping Computation and I/O").
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/moe.h"
#include "kernels.h"

using namespace kmoe;

namespace {
constexpr int kTileRows = kRowBlk * kTileBlks;
// experts smaller than this (bytes) are copied over two alternating streams (four were measured slower)
constexpr int64_t kSecondCopyStreamBelow = 64ll << 20;
// consecutive small experts share a pair of launches while their blobs stay below this
constexpr int64_t kGroupBytes = 24ll << 20;


thread_local std::string g_last_error;

struct Layout {
    int64_t A = 0, max_rowblks = 0, tok_rows16 = 0, x_rows16 = 0, h_rows16 = 0;
    int32_t nchunks = 0, max_tiles = 0, split_cap = 1;
    int64_t expert_bytes = 0;
    // byte offsets into the workspace
    int64_t topk_idx, topk_w, counts, offsets, poff, nbatch, exec_order, meta, perm, inv_perm,
        blk_counts, blk_base, blk_mask, tile_expert, tile_xblk, tile_hblk, tile_nblk, exp_tile0,
        exp_ntiles, blk_expert, mail, wtab, wmeta, herr, xp, h, o;
    int64_t o_split_stride = 0;  // elements
    int64_t h_plane_units = 0;   // 16-byte units between the value plane and the remainder plane of H
    int64_t corr_table = 0;      // int32 [n_layers][E][E]
    int64_t prev_idx = 0;        // top-k ids of the previously routed layer
    int64_t total = 0;
};

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

moe_status check_config(const moe_config* c, std::string& err) {
    auto bad = [&](const char* m, moe_status s) {
        err = m;
        return s;
    };
    if (!c) return bad("config is null", MOE_ERR_INVALID_ARG);
    if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) return bad("dtype must be MOE_F32 or MOE_BF16", MOE_ERR_INVALID_ARG);
    if (c->d_model <= 0 || c->d_ff <= 0) return bad("d_model and d_ff must be positive", MOE_ERR_SHAPE);
    const int mult = c->dtype == MOE_BF16 ? 64 : 4;
    if (c->d_model % mult || c->d_ff % mult)
        return bad(c->dtype == MOE_BF16 ? "bf16 needs d_model and d_ff to be multiples of 64"
                                        : "f32 needs d_model and d_ff to be multiples of 4",
                   MOE_ERR_SHAPE);
    if (c->n_experts < 1 || c->n_experts > MOE_MAX_EXPERTS) return bad("n_experts out of range", MOE_ERR_SHAPE);
    if (c->top_k < 1 || c->top_k > MOE_MAX_TOPK || c->top_k > c->n_experts) return bad("top_k out of range", MOE_ERR_SHAPE);
    if (c->n_shared < 0 || c->n_shared > MOE_MAX_SHARED) return bad("n_shared out of range", MOE_ERR_SHAPE);
    if (c->n_layers < 1) return bad("n_layers must be >= 1", MOE_ERR_SHAPE);
    if (c->window_layers < 0 || c->window_layers > c->n_layers) return bad("window_layers out of range", MOE_ERR_SHAPE);
    if (c->max_tokens < 1 || (int64_t)c->max_tokens * c->top_k > (1 << 28)) return bad("max_tokens out of range", MOE_ERR_SHAPE);
    if (c->max_batches < 1 || c->max_batches > MOE_MAX_BATCHES) return bad("max_batches out of range", MOE_ERR_SHAPE);
    if (c->weight_bits != 0 && c->weight_bits != 16 && c->weight_bits != 4) return bad("weight_bits must be 0, 16 or 4", MOE_ERR_INVALID_ARG);
    if (c->weight_bits == 4 && c->dtype != MOE_BF16) return bad("4-bit expert weights need the bf16 path", MOE_ERR_INVALID_ARG);
    return MOE_OK;
}

void compute_layout(const moe_config& c, Layout& L) {
    const int64_t E = c.n_experts, S = c.n_shared, k = c.top_k, d = c.d_model, f = c.d_ff;
    const int64_t elt = c.dtype == MOE_BF16 ? 2 : 4;
    L.A = (int64_t)c.max_tokens * k;
    L.max_rowblks = (L.A + kRowBlk - 1) / kRowBlk + E;
    L.tok_rows16 = ((int64_t)c.max_tokens + kRowBlk - 1) / kRowBlk;
    L.x_rows16 = L.max_rowblks + (S > 0 ? L.tok_rows16 : 0);
    L.h_rows16 = L.max_rowblks + S * L.tok_rows16;
    L.nchunks = (int32_t)((L.A + kPlanChunk - 1) / kPlanChunk);
    L.max_tiles = max_tiles_for((int)L.max_rowblks, (int)E, (int)S, c.max_tokens);
    L.split_cap = (c.dtype == MOE_BF16 && L.A <= 8192) ? 8 : 1;
    L.expert_bytes = c.weight_bits == 4 ? d * f * 27 / 16 : 3 * d * f * elt;  // q4: codes + (s, z) pairs
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        int64_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.topk_idx = take(L.A * 4);
    L.topk_w = take(L.A * 4);
    L.counts = take(E * 4);
    L.offsets = take((E + 1) * 4);
    L.poff = take((E + 1) * 4);
    L.nbatch = take(E * 4);
    L.exec_order = take(E * 4);
    L.meta = take(16 * 4);
    L.perm = take(L.A * 4);
    L.inv_perm = take(L.A * 4);
    L.blk_counts = take((int64_t)L.nchunks * E * 4);
    L.blk_base = take((int64_t)L.nchunks * E * 4);
    L.blk_mask = take((int64_t)L.nchunks * E * 8);
    L.tile_expert = take((int64_t)L.max_tiles * 4);
    L.tile_xblk = take((int64_t)L.max_tiles * 4);
    L.tile_hblk = take((int64_t)L.max_tiles * 4);
    L.tile_nblk = take((int64_t)L.max_tiles * 4);
    L.exp_tile0 = take((E + S) * 4);
    L.exp_ntiles = take((E + S) * 4);
    L.blk_expert = take(L.max_rowblks * 4);
    L.mail = take((2 * E + 1) * 4);
    L.wtab = take((int64_t)c.n_layers * (E + S) * 8);
    L.wmeta = take((int64_t)c.n_layers * (E + S) * 8);
    const int64_t h_rows = L.h_rows16 * kRowBlk;
    L.herr = take(h_rows * 8);
    if (c.dtype == MOE_BF16) {
        L.xp = take(L.x_rows16 * kRowBlk * d * 2);
        L.h_plane_units = h_rows * f * 2 / 16;
        L.h = take(2 * h_rows * f * 2);  // H: value plane + remainder plane, 2 bytes per element each
    } else {
        L.xp = off;
        L.h = take(h_rows * f * 4);
    }
    L.o_split_stride = h_rows * d;
    L.o = take((int64_t)L.split_cap * L.o_split_stride * 4);
    L.corr_table = take((int64_t)c.n_layers * E * E * 4);
    L.prev_idx = take(L.A * 4);
    L.total = off;
}

enum SlotState { SLOT_FREE = 0, SLOT_LOADED = 1 };

struct Slot {
    uint8_t* ptr = nullptr;
    int layer = -1, expert = -1;
    SlotState state = SLOT_FREE;
    bool prefetched = false;
    hipEvent_t ready = nullptr;  // copy landed (recorded on the copy stream)
    hipEvent_t done = nullptr;   // last reader finished (recorded on the compute stream)
    bool done_pending = false;
    bool ready_recorded = false;  // a copy into this slot has been issued at some time
    uint64_t released_at = 0;     // order in which slots were released (0 = never used)
};

struct LayerState {
    const void* wg = nullptr;
    std::vector<const uint8_t*> resident;  // E+S device blobs (null if not resident)
    std::vector<const uint8_t*> host;      // E pinned host blobs (null if resident)
    std::vector<int> slot_of;              // E: window slot holding the expert, or -1
};

struct HostTile {
    int first = 0, count = 0;
};

}  // namespace

struct moe_ctx {
    moe_config cfg{};
    Layout L;
    hipStream_t compute = nullptr, copy = nullptr;
    std::vector<hipStream_t> copy_extra;  // library-owned additional copy streams (small experts only)
    uint64_t copies_issued = 0;
    uint64_t release_clock = 0;
    uint8_t* ws = nullptr;
    uint8_t* window = nullptr;
    PlanPtrs plan{};
    const uint8_t** wtab_dev = nullptr;  // [n_layers][E+S]
    std::vector<LayerState> layers;
    std::vector<Slot> slots;
    int32_t* mailbox = nullptr;  // pinned host, 2E+1
    hipEvent_t route_ev = nullptr;
    // state of the last moe_route
    int routed_layer = -1;
    int routed_tokens = 0;
    const void* routed_x = nullptr;
    bool route_pending = false;  // mailbox not read yet
    bool host_plan_valid = false;
    std::vector<int32_t> h_counts, h_order;
    int h_nactive = 0;
    std::vector<HostTile> h_tiles;  // per expert id (E+S)
    int split_k_user = 0;
    int variant = 0;   // kernel shape selector of the bf16 FFN (0 = default)
    int h_mode = 0;    // bf16 experts: 0 = the remainder plane of H is multiplied where its recorded energy
                       // asks for it (default), 1 = always
    float2* wmeta_dev = nullptr;         // [n_layers][E+S]: (down-projection output scale, 1 / remainder threshold)
    // timed spans of the pipeline, recorded while profiling is on (moe_get_stats harvests them)
    struct Span {
        hipEvent_t a, b;
        int kind;  // 0: host->device copy, 1: kernels on the compute stream
        bool closed;
    };
    std::vector<Span> spans;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    // correlation-aware prefetcher
    bool corr_on = false;      // predictions allowed
    bool corr_learn = false;   // moe_route adds transitions to the table
    int32_t* corr_host = nullptr;  // pinned host mirror, [n_layers][E][E]
    int prev_idx_layer = -1, prev_idx_tokens = -1;
    moe_stats stats{};
    bool profiling = false;
    hipEvent_t pev[8] = {};  // router start, router end, plan end, fwd start, gather, up, down, combine
    bool prof_route = false, prof_fwd = false;
    mutable std::string err;
};

namespace {

// Remainder plane of H: when is one fp16 plane enough?  The down projection of an expert turns the
// rounding remainders r_i = h_i - fp16(h_i) of a token row into an output error sum_i r_i * W2[n,i].
// Rounding remainders are as good as independent of the weights, so that error has variance
// sum_i r_i^2 W2[n,i]^2 ~ (sum_i r_i^2) * (sum_i W2[n,i]^2) / f.  A token's output adds at most one
// such term with total weight 1 for the routed experts (the routing weights sum to at most 1) and
// one per shared expert.  The remainder plane is skipped for a tile while, for each of its rows,
// kSigmas standard deviations of that sum stay below kErrBudget (0.8 of the 1e-2 absolute
// tolerance the layer is held to; the rest covers the final rounding and fp32 reassociation):
//     energy(row) = sum_i r_i^2  <=  tau = kErrBudget^2 * f / (kSigmas^2 * (1 + S) * R),
// R = the largest sum of squares over a row of W2, taken at placement.
constexpr double kErrBudget = 8e-3, kSigmas = 6.0;

// Timing event from the context's pool (created on first use, reused after moe_reset_stats).
hipEvent_t pool_event(moe_ctx* c) {
    if (c->ev_used == c->ev_pool.size()) {
        hipEvent_t ev = nullptr;
        if (hipEventCreate(&ev) != hipSuccess) return nullptr;
        c->ev_pool.push_back(ev);
    }
    return c->ev_pool[c->ev_used++];
}

// Opens a timed span on `st` while profiling is on; returns its index or -1.
int span_open(moe_ctx* c, hipStream_t st, int kind) {
    if (!c->profiling || c->spans.size() >= (1u << 16)) return -1;
    hipEvent_t a = pool_event(c), b = pool_event(c);
    if (!a || !b) return -1;
    if (hipEventRecord(a, st) != hipSuccess) return -1;
    c->spans.push_back({a, b, kind, false});
    return (int)c->spans.size() - 1;
}
void span_close(moe_ctx* c, hipStream_t st, int idx) {
    if (idx >= 0 && hipEventRecord(c->spans[idx].b, st) == hipSuccess) c->spans[idx].closed = true;
}

moe_status fail(const moe_ctx* ctx, moe_status s, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    g_last_error = buf;
    return s;
}

#define HIP_TRY(ctx, expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(ctx, MOE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

bool is_pinned_host(const void* p) {
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // clear the sticky error of an unregistered pointer
        return false;
    }
    return at.type == hipMemoryTypeHost;
}

Shape make_shape(const moe_ctx* c, int n_tokens) {
    Shape s;
    s.N = n_tokens;
    s.d = c->cfg.d_model;
    s.f = c->cfg.d_ff;
    s.E = c->cfg.n_experts;
    s.k = c->cfg.top_k;
    s.S = c->cfg.n_shared;
    s.renorm = c->cfg.renormalize;
    s.max_rowblks = (int32_t)c->L.max_rowblks;
    return s;
}

bool all_resident_layer(const moe_ctx* c, int layer) {
    for (const uint8_t* p : c->layers[layer].resident)
        if (!p) return false;
    return true;
}

int auto_split_k(const moe_ctx* c, int n_tokens) {
    if (c->cfg.dtype != MOE_BF16) return 1;
    int cap = c->L.split_cap;
    const int nstage = c->cfg.d_ff / 64;
    cap = std::min(cap, nstage);
    if (c->split_k_user > 0) return std::min(c->split_k_user, cap);
    const int64_t A = (int64_t)n_tokens * c->cfg.top_k;
    const int64_t tiles = std::max<int64_t>(std::min<int64_t>(c->cfg.n_experts, A), (A + kTileRows - 1) / kTileRows) +
                          (int64_t)c->cfg.n_shared * ((n_tokens + kTileRows - 1) / kTileRows);
    const int64_t groups = (c->cfg.d_model / 32 + 7) / 8;
    const int64_t wgs = std::max<int64_t>(1, tiles * groups);
    int64_t want = (256 + wgs - 1) / wgs;  // one workgroup per compute unit; partial sums cost the combine
    return (int)std::max<int64_t>(1, std::min<int64_t>(want, cap));
}

// Host mirror of the device tile enumeration (plan_scan_kernel): shared experts first, then the
// routed experts in execution order, 16 row blocks per tile.
void build_host_tiles(moe_ctx* c) {
    const int E = c->cfg.n_experts, S = c->cfg.n_shared;
    c->h_tiles.assign(E + S, HostTile{});
    int nt = 0;
    const int nblk_tok = (c->routed_tokens + kRowBlk - 1) / kRowBlk;
    for (int sh = 0; sh < S; ++sh) {
        c->h_tiles[E + sh].first = nt;
        nt += (nblk_tok + kTileBlks - 1) / kTileBlks;
        c->h_tiles[E + sh].count = nt - c->h_tiles[E + sh].first;
    }
    for (int i = 0; i < c->h_nactive; ++i) {
        const int e = c->h_order[i];
        const int nb = (c->h_counts[e] + kRowBlk - 1) / kRowBlk;
        c->h_tiles[e].first = nt;
        nt += (nb + kTileBlks - 1) / kTileBlks;
        c->h_tiles[e].count = nt - c->h_tiles[e].first;
    }
}

moe_status wait_route(moe_ctx* ctx) {
    if (ctx->routed_layer < 0) return fail(ctx, MOE_ERR_STATE, "moe_route has not been called");
    if (ctx->route_pending) {
        HIP_TRY(ctx, hipEventSynchronize(ctx->route_ev));
        const int E = ctx->cfg.n_experts;
        ctx->h_counts.assign(ctx->mailbox, ctx->mailbox + E);
        ctx->h_order.assign(ctx->mailbox + E, ctx->mailbox + 2 * E);
        ctx->h_nactive = ctx->mailbox[2 * E];
        ctx->route_pending = false;
        ctx->host_plan_valid = true;
        ctx->stats.n_active_sum += ctx->h_nactive;
        build_host_tiles(ctx);
    }
    return MOE_OK;
}

void release_slot(moe_ctx* ctx, Slot& s, bool record_done) {
    if (s.layer >= 0 && s.expert >= 0) ctx->layers[s.layer].slot_of[s.expert] = -1;
    if (record_done) {
        (void)hipEventRecord(s.done, ctx->compute);
        s.done_pending = true;
    }
    s.layer = -1;
    s.expert = -1;
    s.state = SLOT_FREE;
    s.prefetched = false;
    s.released_at = ++ctx->release_clock;
}

moe_status stream_one(moe_ctx* ctx, int layer, int e, bool prefetch) {
    LayerState& ls = ctx->layers[layer];
    if (ls.resident[e]) return MOE_OK;  // nothing to move
    if (!ls.host[e]) return fail(ctx, MOE_ERR_STATE, "layer %d expert %d has no weights", layer, e);
    if (ls.slot_of[e] >= 0) return MOE_OK;  // already in flight or loaded
    // The free slot released longest ago: its readers are the furthest behind the head of the
    // compute stream, so the copy stream's wait for them is the least likely to stall.
    int pick = -1;
    for (size_t i = 0; i < ctx->slots.size(); ++i)
        if (ctx->slots[i].state == SLOT_FREE &&
            (pick < 0 || ctx->slots[i].released_at < ctx->slots[pick].released_at))
            pick = (int)i;
    if (pick < 0) return fail(ctx, MOE_ERR_OOM, "no free window slot for layer %d expert %d", layer, e);
    Slot& s = ctx->slots[pick];
    // Small experts alternate between two copy streams: the fixed start-up gap of one copy then
    // hides behind the other stream's transfer and the link stays busy.  Every slot still has
    // its own ready event, so nothing depends on the order in which the copies land.
    hipStream_t cs = ctx->copy;
    if (!ctx->copy_extra.empty()) {
        const size_t which = (size_t)(ctx->copies_issued++ % (ctx->copy_extra.size() + 1));
        if (which > 0) cs = ctx->copy_extra[which - 1];
    }
    if (s.done_pending) {  // the slot's previous readers must finish before it is overwritten
        HIP_TRY(ctx, hipStreamWaitEvent(cs, s.done, 0));
        s.done_pending = false;
    }
    // ... and so must its previous copy, which may have gone over the other copy stream (a
    // dropped prefetch guess frees a slot without any reader)
    if (!ctx->copy_extra.empty() && s.ready_recorded) HIP_TRY(ctx, hipStreamWaitEvent(cs, s.ready, 0));
    const int span = span_open(ctx, cs, 0);
    HIP_TRY(ctx, hipMemcpyAsync(s.ptr, ls.host[e], (size_t)ctx->L.expert_bytes, hipMemcpyHostToDevice, cs));
    span_close(ctx, cs, span);
    HIP_TRY(ctx, hipEventRecord(s.ready, cs));
    s.ready_recorded = true;
    s.layer = layer;
    s.expert = e;
    s.state = SLOT_LOADED;
    s.prefetched = prefetch;
    ls.slot_of[e] = pick;
    ctx->stats.bytes_h2d += ctx->L.expert_bytes;
    ctx->stats.n_copies += 1;
    return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_last_error(const moe_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

moe_status moe_plan(const moe_config* cfg, int32_t n_tokens, double hbm_Bps, double link_Bps,
                    double mfma_flops, moe_plan_t* out) {
    std::string err;
    moe_status st = check_config(cfg, err);
    if (st != MOE_OK) return fail(nullptr, st, "%s", err.c_str());
    if (!out) return fail(nullptr, MOE_ERR_INVALID_ARG, "out is null");
    if (n_tokens < 0 || n_tokens > cfg->max_tokens)
        return fail(nullptr, MOE_ERR_SHAPE, "n_tokens %d outside [0, max_tokens]", n_tokens);
    Layout L;
    compute_layout(*cfg, L);
    memset(out, 0, sizeof *out);
    out->workspace_bytes = L.total;
    out->expert_bytes = L.expert_bytes;
    out->n_slots = cfg->window_layers * cfg->n_experts;
    out->window_bytes = (int64_t)out->n_slots * L.expert_bytes;
    const double elt = cfg->dtype == MOE_BF16 ? 2.0 : 4.0;
    const double rows = (double)n_tokens * cfg->top_k / cfg->n_experts;
    const double flops = 6.0 * cfg->d_model * (double)cfg->d_ff * rows;
    out->t_io_expert_s = link_Bps > 0 ? (double)L.expert_bytes / link_Bps : 0.0;
    const double t_mem = hbm_Bps > 0 ? (double)L.expert_bytes / hbm_Bps : 0.0;
    const double t_alu = mfma_flops > 0 ? flops / mfma_flops : 0.0;
    out->t_c_expert_s = std::max(t_mem, t_alu);
    out->t_c_gate_s = hbm_Bps > 0 ? (double)n_tokens * cfg->d_model * elt / hbm_Bps : 0.0;
    return MOE_OK;
}

moe_status moe_plan_batches(double t_c_A, double t_c_G, double t_c_hotE, const double* t_c_E,
                            int32_t len_q, double t_io_A, double t_io_G, double t_io_E, int32_t K,
                            int32_t* n_out) {
    if (!n_out || len_q < 0 || K < 0 || (len_q > 0 && !t_c_E))
        return fail(nullptr, MOE_ERR_INVALID_ARG, "bad argument to moe_plan_batches");
    const double vals[] = {t_c_A, t_c_G, t_c_hotE, t_io_A, t_io_G, t_io_E};
    for (double v : vals)
        if (!(v >= 0.0)) return fail(nullptr, MOE_ERR_INVALID_ARG, "times must be >= 0");
    double sum_q = 0.0;
    for (int i = 0; i < len_q; ++i) {
        if (!(t_c_E[i] >= 0.0)) return fail(nullptr, MOE_ERR_INVALID_ARG, "times must be >= 0");
        sum_q += t_c_E[i];
    }
    // n * rate + hot + queue >= rhs, one row per arrow of the pipeline figure (I..IV)
    struct Row {
        double rate, hot, queue, rhs;
    };
    std::vector<Row> rows;
    rows.push_back({t_c_A, 0.0, 0.0, t_io_G});
    rows.push_back({t_c_A + t_c_G, 0.0, 0.0, t_io_G + K * t_io_E});
    if (len_q > 0) {  // with no cold expert queued the last two conditions do not apply
        rows.push_back({t_c_A + t_c_G, t_c_hotE, 0.0, t_io_G + (K + 1) * t_io_E});
        rows.push_back({t_c_A + t_c_G, t_c_hotE, sum_q, t_io_G + (K + len_q) * t_io_E + t_io_A});
    }
    long long n = 1;
    for (const Row& r : rows) {  // first guess: the ceiling of each row's quotient
        const double need = r.rhs - r.hot - r.queue;
        if (need <= 0.0) continue;
        if (!(r.rate > 0.0))
            return fail(nullptr, MOE_ERR_INVALID_ARG, "no compute time to overlap the I/O with");
        const double x = need / r.rate;
        if (x >= 2.0e9) {
            n = INT32_MAX;
            continue;
        }
        long long c = (long long)x;
        if ((double)c < x) ++c;
        n = std::max(n, c);
    }
    // The quotients can be off by an ulp: settle on the smallest n that satisfies every
    // inequality evaluated as printed.
    auto holds = [&](long long m) {
        for (const Row& r : rows)
            if (!((double)m * r.rate + r.hot + r.queue >= r.rhs)) return false;
        return true;
    };
    while (n > 1 && holds(n - 1)) --n;
    while (n < INT32_MAX && !holds(n)) ++n;
    if (n > INT32_MAX) n = INT32_MAX;
    *n_out = (int32_t)n;
    return MOE_OK;
}

moe_status moe_create(const moe_config* cfg, void* compute_stream, void* copy_stream,
                      void* workspace_dev, int64_t workspace_bytes, void* window_dev,
                      int64_t window_bytes, moe_ctx** out) {
    std::string err;
    moe_status st = check_config(cfg, err);
    if (st != MOE_OK) return fail(nullptr, st, "%s", err.c_str());
    if (!out) return fail(nullptr, MOE_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!workspace_dev) return fail(nullptr, MOE_ERR_INVALID_ARG, "workspace is null");
    if (((uintptr_t)workspace_dev & 255u) != 0) return fail(nullptr, MOE_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    Layout L;
    compute_layout(*cfg, L);
    if (workspace_bytes < L.total)
        return fail(nullptr, MOE_ERR_OOM, "workspace of %lld bytes, need %lld", (long long)workspace_bytes, (long long)L.total);
    const int n_slots = cfg->window_layers * cfg->n_experts;
    if (n_slots > 0) {
        if (!window_dev) return fail(nullptr, MOE_ERR_INVALID_ARG, "window is null");
        if (((uintptr_t)window_dev & 255u) != 0) return fail(nullptr, MOE_ERR_INVALID_ARG, "window must be 256-byte aligned");
        if (window_bytes < (int64_t)n_slots * L.expert_bytes)
            return fail(nullptr, MOE_ERR_OOM, "window of %lld bytes, need %lld", (long long)window_bytes, (long long)n_slots * L.expert_bytes);
        if (compute_stream == copy_stream)
            return fail(nullptr, MOE_ERR_INVALID_ARG, "streaming needs a copy stream distinct from the compute stream");
    }
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return fail(nullptr, MOE_ERR_OOM, "out of host memory");
    c->cfg = *cfg;
    c->L = L;
    c->compute = (hipStream_t)compute_stream;
    c->copy = (hipStream_t)copy_stream;
    c->ws = (uint8_t*)workspace_dev;
    c->window = (uint8_t*)window_dev;
    uint8_t* w = c->ws;
    PlanPtrs& p = c->plan;
    p.topk_idx = (int32_t*)(w + L.topk_idx);
    p.topk_w = (float*)(w + L.topk_w);
    p.counts = (int32_t*)(w + L.counts);
    p.offsets = (int32_t*)(w + L.offsets);
    p.poff = (int32_t*)(w + L.poff);
    p.nbatch = (int32_t*)(w + L.nbatch);
    p.exec_order = (int32_t*)(w + L.exec_order);
    p.meta = (int32_t*)(w + L.meta);
    p.perm = (int32_t*)(w + L.perm);
    p.inv_perm = (int32_t*)(w + L.inv_perm);
    p.blk_counts = (int32_t*)(w + L.blk_counts);
    p.blk_base = (int32_t*)(w + L.blk_base);
    p.blk_mask = (unsigned long long*)(w + L.blk_mask);
    p.tile_expert = (int32_t*)(w + L.tile_expert);
    p.tile_xblk = (int32_t*)(w + L.tile_xblk);
    p.tile_hblk = (int32_t*)(w + L.tile_hblk);
    p.tile_nblk = (int32_t*)(w + L.tile_nblk);
    p.exp_tile0 = (int32_t*)(w + L.exp_tile0);
    p.exp_ntiles = (int32_t*)(w + L.exp_ntiles);
    p.blk_expert = (int32_t*)(w + L.blk_expert);
    c->wtab_dev = (const uint8_t**)(w + L.wtab);
    c->wmeta_dev = (float2*)(w + L.wmeta);
    const int E = cfg->n_experts, S = cfg->n_shared;
    c->layers.resize(cfg->n_layers);
    for (auto& ls : c->layers) {
        ls.resident.assign(E + S, nullptr);
        ls.host.assign(E, nullptr);
        ls.slot_of.assign(E, -1);
    }
    auto cleanup = [&](moe_status s, const char* what, hipError_t e) {
        moe_status r = fail(nullptr, s, "%s failed: %s", what, hipGetErrorString(e));
        moe_destroy(c);
        return r;
    };
    hipError_t e;
    e = hipMemsetAsync(w + L.wtab, 0, (size_t)cfg->n_layers * (E + S) * 8, c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipMemsetAsync", e);
    e = hipMemsetAsync(w + L.meta, 0, 64, c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipMemsetAsync", e);
    e = hipMemsetAsync(w + L.wmeta, 0, (size_t)cfg->n_layers * (E + S) * 8, c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipMemsetAsync", e);
    e = hipMemsetAsync(w + L.herr, 0, (size_t)L.h_rows16 * kRowBlk * 8, c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipMemsetAsync", e);
    e = hipMemsetAsync(w + L.corr_table, 0, (size_t)cfg->n_layers * E * E * 4, c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipMemsetAsync", e);
    e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipStreamSynchronize", e);
    e = hipHostMalloc((void**)&c->mailbox, (size_t)(2 * E + 1) * 4, hipHostMallocDefault);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipHostMalloc", e);
    // The plan kernel writes counts and execution order straight into this pinned block (device
    // stores to mapped host memory, visible to the host once the route event has completed): no
    // copy node sits between the plan and the expert kernels.
    void* mail_dev = nullptr;
    e = hipHostGetDevicePointer(&mail_dev, c->mailbox, 0);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipHostGetDevicePointer", e);
    p.mail = (int32_t*)mail_dev;
    e = hipHostMalloc((void**)&c->corr_host, (size_t)cfg->n_layers * E * E * 4, hipHostMallocDefault);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipHostMalloc", e);
    memset(c->corr_host, 0, (size_t)cfg->n_layers * E * E * 4);
    e = hipEventCreateWithFlags(&c->route_ev, hipEventDisableTiming);
    if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipEventCreate", e);
    for (auto& ev : c->pev) {
        e = hipEventCreate(&ev);
        if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipEventCreate", e);
    }
    if (n_slots > 0 && L.expert_bytes < kSecondCopyStreamBelow) {
        const int extra = 1;
        for (int i = 0; i < extra; ++i) {
            hipStream_t cs = nullptr;
            e = hipStreamCreateWithFlags(&cs, hipStreamNonBlocking);  // default priority
            if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipStreamCreateWithFlags", e);
            c->copy_extra.push_back(cs);
        }
    }
    c->slots.resize(n_slots);
    for (int i = 0; i < n_slots; ++i) {
        Slot& s = c->slots[i];
        s.ptr = c->window + (size_t)i * L.expert_bytes;
        e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipEventCreate", e);
        e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup(MOE_ERR_HIP, "hipEventCreate", e);
    }
    if (cfg->dtype == MOE_BF16) {
        int r = ffn_configure();
        if (r != 0) return cleanup(MOE_ERR_HIP, "hipFuncSetAttribute", (hipError_t)r);
    }
    *out = c;
    return MOE_OK;
}

moe_status moe_destroy(moe_ctx* ctx) {
    if (!ctx) return MOE_OK;
    (void)hipStreamSynchronize(ctx->compute);  // a null handle is the default stream
    if (ctx->copy != ctx->compute) (void)hipStreamSynchronize(ctx->copy);
    for (hipStream_t cs : ctx->copy_extra) {
        (void)hipStreamSynchronize(cs);
        (void)hipStreamDestroy(cs);
    }
    for (Slot& s : ctx->slots) {
        if (s.ready) (void)hipEventDestroy(s.ready);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    if (ctx->route_ev) (void)hipEventDestroy(ctx->route_ev);
    for (auto& ev : ctx->pev)
        if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : ctx->ev_pool) (void)hipEventDestroy(ev);
    if (ctx->mailbox) (void)hipHostFree(ctx->mailbox);
    if (ctx->corr_host) (void)hipHostFree(ctx->corr_host);
    delete ctx;
    return MOE_OK;
}

moe_status moe_set_gate(moe_ctx* ctx, int32_t layer, const void* wg_dev) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!wg_dev) return fail(ctx, MOE_ERR_INVALID_ARG, "gate matrix is null");
    ctx->layers[layer].wg = wg_dev;
    return MOE_OK;
}

}  // extern "C"

namespace {

// Range and row energy of an expert's W2, taken on the device by `stats` (two words: bits of the
// largest |w|, bits of the largest row sum of squares), turned into the power of two that brings
// W2 into the fp16 range (*w2_scale, applied at packing; its inverse goes to meta->x and is
// applied to the outputs) and into 1 / threshold of the remainder energy (meta->y, see kErrBudget).
template <typename StatsFn>
moe_status w2_placement_figures(moe_ctx* ctx, int layer, int expert, StatsFn stats, float* w2_scale, float2* meta) {
    const int f = ctx->cfg.d_ff, S = ctx->cfg.n_shared;
    uint32_t* stats_dev = (uint32_t*)(ctx->ws + ctx->L.meta) + 8;  // two spare words of the meta block
    uint32_t st[2] = {0, 0};
    HIP_TRY(ctx, hipMemsetAsync(stats_dev, 0, 8, ctx->compute));
    stats(stats_dev);
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipMemcpyAsync(st, stats_dev, 8, hipMemcpyDeviceToHost, ctx->compute));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    if (st[0] >= 0x7f800000u || st[1] >= 0x7f800000u)
        return fail(ctx, MOE_ERR_SHAPE, "W2 of layer %d expert %d holds non-finite weights (or its row energy overflows)", layer, expert);
    float amax, rowsq;
    memcpy(&amax, &st[0], 4);
    memcpy(&rowsq, &st[1], 4);
    int shift = 0;
    while (std::ldexp((double)amax, -shift) > 65504.0) ++shift;
    *w2_scale = (float)std::ldexp(1.0, -shift);
    const double inv_tau = kSigmas * kSigmas * (1.0 + S) * (double)rowsq / ((double)f * kErrBudget * kErrBudget);
    *meta = make_float2((float)std::ldexp(1.0, shift), (float)std::min(inv_tau, 3.0e38));
    return MOE_OK;
}

// Common part of expert placement: validation, staging through window slot 0 for pinned
// destinations, the pack launches (given as a callable), bookkeeping of where the blob lives.
template <typename PackFn>
moe_status place_expert(moe_ctx* ctx, int32_t layer, int32_t expert, int32_t where, void* packed_dst,
                        PackFn pack) {
    const int E = ctx->cfg.n_experts, S = ctx->cfg.n_shared;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (expert < 0 || expert >= E + S) return fail(ctx, MOE_ERR_INVALID_ARG, "expert %d out of range", expert);
    if (!packed_dst) return fail(ctx, MOE_ERR_INVALID_ARG, "null weight pointer");
    if (where != MOE_RESIDENT && where != MOE_HOST_PINNED) return fail(ctx, MOE_ERR_INVALID_ARG, "bad residency");
    if (((uintptr_t)packed_dst & 15u) != 0) return fail(ctx, MOE_ERR_INVALID_ARG, "packed_dst must be 16-byte aligned");
    LayerState& ls = ctx->layers[layer];
    void* pack_to = packed_dst;
    if (where == MOE_HOST_PINNED) {
        if (expert >= E) return fail(ctx, MOE_ERR_INVALID_ARG, "shared experts must be resident");
        if (ctx->slots.empty()) return fail(ctx, MOE_ERR_STATE, "host-resident experts need a window (window_layers > 0)");
        if (!is_pinned_host(packed_dst)) return fail(ctx, MOE_ERR_NOT_PINNED, "packed_dst is not pinned host memory");
        for (const Slot& s : ctx->slots)
            if (s.state != SLOT_FREE) return fail(ctx, MOE_ERR_STATE, "placement while experts are in the window");
        HIP_TRY(ctx, hipStreamSynchronize(ctx->copy));
        for (hipStream_t cs : ctx->copy_extra) HIP_TRY(ctx, hipStreamSynchronize(cs));
        pack_to = ctx->slots[0].ptr;  // staging: slot 0 is idle during the offline phase
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    pack(pack_to);
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    if (where == MOE_HOST_PINNED) {
        HIP_TRY(ctx, hipMemcpy(packed_dst, pack_to, (size_t)ctx->L.expert_bytes, hipMemcpyDeviceToHost));
        ctx->slots[0].done_pending = false;
        ls.host[expert] = (const uint8_t*)packed_dst;
        ls.resident[expert] = nullptr;
        const uint8_t* nul = nullptr;
        HIP_TRY(ctx, hipMemcpy((void*)(ctx->wtab_dev + (size_t)layer * (E + S) + expert), &nul, 8, hipMemcpyHostToDevice));
    } else {
        ls.resident[expert] = (const uint8_t*)packed_dst;
        if (expert < E) ls.host[expert] = nullptr;
        const uint8_t* ptr = (const uint8_t*)packed_dst;
        HIP_TRY(ctx, hipMemcpy((void*)(ctx->wtab_dev + (size_t)layer * (E + S) + expert), &ptr, 8, hipMemcpyHostToDevice));
    }
    return MOE_OK;
}

}  // namespace

extern "C" {

moe_status moe_set_expert(moe_ctx* ctx, int32_t layer, int32_t expert, const void* w1_dev,
                          const void* w3_dev, const void* w2_dev, int32_t where, void* packed_dst) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (!w1_dev || !w3_dev || !w2_dev) return fail(ctx, MOE_ERR_INVALID_ARG, "null weight pointer");
    if (ctx->cfg.weight_bits == 4) return fail(ctx, MOE_ERR_STATE, "this context holds 4-bit experts: use moe_set_expert_q4");
    const int d = ctx->cfg.d_model, f = ctx->cfg.d_ff;
    const int E = ctx->cfg.n_experts, S = ctx->cfg.n_shared;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (expert < 0 || expert >= E + S) return fail(ctx, MOE_ERR_INVALID_ARG, "expert %d out of range", expert);
    float2 meta = make_float2(1.f, 0.f);
    float w2_scale = 1.f;
    if (ctx->cfg.dtype == MOE_BF16) {
        moe_status ws = w2_placement_figures(ctx, layer, expert, [&](uint32_t* stats_dev) {
            launch_w2_stats(ctx->compute, w2_dev, d, f, stats_dev);
        }, &w2_scale, &meta);
        if (ws != MOE_OK) return ws;
    }
    moe_status st = place_expert(ctx, layer, expert, where, packed_dst, [&](void* to) {
        if (ctx->cfg.dtype == MOE_BF16)
            launch_pack_expert_bf16(ctx->compute, w1_dev, w3_dev, w2_dev, d, f, to, w2_scale);
        else
            launch_pack_expert_f32(ctx->compute, w1_dev, w3_dev, w2_dev, d, f, to);
    });
    if (st != MOE_OK) return st;
    HIP_TRY(ctx, hipMemcpy((void*)(ctx->wmeta_dev + (size_t)layer * (E + S) + expert), &meta, 8, hipMemcpyHostToDevice));
    return MOE_OK;
}

moe_status moe_set_expert_q4(moe_ctx* ctx, int32_t layer, int32_t expert, const void* q1_dev,
                             const void* s1_dev, const void* z1_dev, const void* q3_dev,
                             const void* s3_dev, const void* z3_dev, const void* q2_dev,
                             const void* s2_dev, const void* z2_dev, int32_t where, void* packed_dst) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (ctx->cfg.weight_bits != 4) return fail(ctx, MOE_ERR_STATE, "the context was not created with weight_bits = 4");
    const void* all[9] = {q1_dev, s1_dev, z1_dev, q3_dev, s3_dev, z3_dev, q2_dev, s2_dev, z2_dev};
    for (const void* p : all)
        if (!p) return fail(ctx, MOE_ERR_INVALID_ARG, "null weight pointer");
    for (const void* p : all)
        if (((uintptr_t)p & 3u) != 0) return fail(ctx, MOE_ERR_INVALID_ARG, "quantised tensors must be 4-byte aligned");
    const int d = ctx->cfg.d_model, f = ctx->cfg.d_ff;
    const int E = ctx->cfg.n_experts, S = ctx->cfg.n_shared;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (expert < 0 || expert >= E + S) return fail(ctx, MOE_ERR_INVALID_ARG, "expert %d out of range", expert);
    float2 meta = make_float2(1.f, 0.f);
    float w2_scale = 1.f;
    moe_status ws = w2_placement_figures(ctx, layer, expert, [&](uint32_t* stats_dev) {
        launch_w2_stats_q4(ctx->compute, (const uint8_t*)q2_dev, (const uint16_t*)s2_dev, (const uint16_t*)z2_dev, d, f, stats_dev);
    }, &w2_scale, &meta);
    if (ws != MOE_OK) return ws;
    moe_status st = place_expert(ctx, layer, expert, where, packed_dst, [&](void* to) {
        launch_pack_expert_q4(ctx->compute, (const uint8_t*)q1_dev, (const uint16_t*)s1_dev,
                              (const uint16_t*)z1_dev, (const uint8_t*)q3_dev, (const uint16_t*)s3_dev,
                              (const uint16_t*)z3_dev, (const uint8_t*)q2_dev, (const uint16_t*)s2_dev,
                              (const uint16_t*)z2_dev, d, f, to, w2_scale);
    });
    if (st != MOE_OK) return st;
    HIP_TRY(ctx, hipMemcpy((void*)(ctx->wmeta_dev + (size_t)layer * (E + S) + expert), &meta, 8, hipMemcpyHostToDevice));
    return MOE_OK;
}

moe_status moe_route(moe_ctx* ctx, int32_t layer, const void* x_dev,
                     const int32_t* batch_offsets_host, int32_t n_batches, float* logits_dev,
                     int32_t* topk_idx_dev, float* topk_w_dev, int32_t* counts_dev,
                     int32_t* offsets_dev, int32_t* perm_dev, int32_t* inv_perm_dev,
                     int32_t* exec_order_dev) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!batch_offsets_host) return fail(ctx, MOE_ERR_INVALID_ARG, "batch_offsets is null");
    if (n_batches < 1 || n_batches > ctx->cfg.max_batches) return fail(ctx, MOE_ERR_SHAPE, "n_batches %d outside [1, %d]", n_batches, ctx->cfg.max_batches);
    if (batch_offsets_host[0] != 0) return fail(ctx, MOE_ERR_INVALID_ARG, "batch_offsets must start at 0");
    BatchOffsets bo;
    bo.n = n_batches;
    for (int b = 0; b <= n_batches; ++b) {
        if (b > 0 && batch_offsets_host[b] < batch_offsets_host[b - 1])
            return fail(ctx, MOE_ERR_INVALID_ARG, "batch_offsets must be non-decreasing");
        bo.v[b] = batch_offsets_host[b];
    }
    for (int b = n_batches + 1; b <= kMaxBatches; ++b) bo.v[b] = batch_offsets_host[n_batches];
    const int N = batch_offsets_host[n_batches];
    if (N > ctx->cfg.max_tokens) return fail(ctx, MOE_ERR_SHAPE, "%d tokens exceed max_tokens %d", N, ctx->cfg.max_tokens);
    if (N > 0 && !x_dev) return fail(ctx, MOE_ERR_INVALID_ARG, "x is null");
    LayerState& ls = ctx->layers[layer];
    if (!ls.wg) return fail(ctx, MOE_ERR_STATE, "gate of layer %d not set", layer);
    const int E = ctx->cfg.n_experts, k = ctx->cfg.top_k;
    const Shape s = make_shape(ctx, N);
    hipStream_t st = ctx->compute;
    const bool prof = ctx->profiling;
    const int span = span_open(ctx, st, 1);
    if (prof) (void)hipEventRecord(ctx->pev[0], st);
    launch_router(st, ctx->cfg.dtype, x_dev, ls.wg, s, logits_dev, ctx->plan.topk_idx, ctx->plan.topk_w);
    if (prof) (void)hipEventRecord(ctx->pev[1], st);
    launch_plan(st, s, bo, ctx->plan, ctx->L.max_tiles);
    if (prof) (void)hipEventRecord(ctx->pev[2], st);
    span_close(ctx, st, span);
    ctx->prof_route = prof;
    HIP_TRY(ctx, hipGetLastError());
    const size_t A = (size_t)N * k;
    auto out = [&](void* dst, const void* src, size_t bytes) -> hipError_t {
        if (!dst || bytes == 0) return hipSuccess;
        return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st);
    };
    HIP_TRY(ctx, out(topk_idx_dev, ctx->plan.topk_idx, A * 4));
    HIP_TRY(ctx, out(topk_w_dev, ctx->plan.topk_w, A * 4));
    HIP_TRY(ctx, out(counts_dev, ctx->plan.counts, (size_t)E * 4));
    HIP_TRY(ctx, out(offsets_dev, ctx->plan.offsets, (size_t)(E + 1) * 4));
    HIP_TRY(ctx, out(perm_dev, ctx->plan.perm, A * 4));
    HIP_TRY(ctx, out(inv_perm_dev, ctx->plan.inv_perm, A * 4));
    HIP_TRY(ctx, out(exec_order_dev, ctx->plan.exec_order, (size_t)E * 4));
    if (ctx->corr_learn) {
        int32_t* prev = (int32_t*)(ctx->ws + ctx->L.prev_idx);
        if (layer > 0 && ctx->prev_idx_layer == layer - 1 && ctx->prev_idx_tokens == N && N > 0) {
            int32_t* tab = (int32_t*)(ctx->ws + ctx->L.corr_table) + (size_t)layer * E * E;
            launch_corr_update(st, prev, ctx->plan.topk_idx, N, k, E, tab);
            HIP_TRY(ctx, hipGetLastError());
            HIP_TRY(ctx, hipMemcpyAsync(ctx->corr_host + (size_t)layer * E * E, tab, (size_t)E * E * 4,
                                        hipMemcpyDeviceToHost, st));
        }
        if (A > 0) HIP_TRY(ctx, hipMemcpyAsync(prev, ctx->plan.topk_idx, A * 4, hipMemcpyDeviceToDevice, st));
        ctx->prev_idx_layer = layer;
        ctx->prev_idx_tokens = N;
    }
    HIP_TRY(ctx, hipEventRecord(ctx->route_ev, st));
    ctx->routed_layer = layer;
    ctx->routed_tokens = N;
    ctx->routed_x = x_dev;
    ctx->route_pending = true;
    ctx->host_plan_valid = false;
    ctx->stats.tokens += N;
    return MOE_OK;
}

moe_status moe_route_wait(moe_ctx* ctx, int32_t* counts_host, int32_t* exec_order_host,
                          int32_t* n_active) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    moe_status st = wait_route(ctx);
    if (st != MOE_OK) return st;
    const int E = ctx->cfg.n_experts;
    if (counts_host) memcpy(counts_host, ctx->h_counts.data(), (size_t)E * 4);
    if (exec_order_host) memcpy(exec_order_host, ctx->h_order.data(), (size_t)E * 4);
    if (n_active) *n_active = ctx->h_nactive;
    return MOE_OK;
}

moe_status moe_stream_experts(moe_ctx* ctx, int32_t layer, const int32_t* expert_ids_host,
                              int32_t n_ids, int32_t flags) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (n_ids < 0 || (n_ids > 0 && !expert_ids_host)) return fail(ctx, MOE_ERR_INVALID_ARG, "bad expert id list");
    if (flags != MOE_PREFETCH && flags != MOE_ON_DEMAND) return fail(ctx, MOE_ERR_INVALID_ARG, "flags must be MOE_PREFETCH or MOE_ON_DEMAND");
    if (ctx->slots.empty()) return fail(ctx, MOE_ERR_STATE, "context has no window (window_layers == 0)");
    const int E = ctx->cfg.n_experts;
    for (int i = 0; i < n_ids; ++i)
        if (expert_ids_host[i] < 0 || expert_ids_host[i] >= E)
            return fail(ctx, MOE_ERR_INVALID_ARG, "expert id %d out of range", expert_ids_host[i]);
    if (flags == MOE_ON_DEMAND) {
        if (ctx->routed_layer != layer) return fail(ctx, MOE_ERR_STATE, "on-demand transfer for layer %d, but the last moe_route was for layer %d", layer, ctx->routed_layer);
        moe_status st = wait_route(ctx);
        if (st != MOE_OK) return st;
        for (int i = 0; i < n_ids; ++i)
            if (ctx->h_counts[expert_ids_host[i]] == 0)
                return fail(ctx, MOE_ERR_INVALID_ARG, "expert %d was not activated: it is never transferred", expert_ids_host[i]);
    }
    for (int i = 0; i < n_ids; ++i) {
        moe_status st = stream_one(ctx, layer, expert_ids_host[i], flags == MOE_PREFETCH);
        if (st != MOE_OK) return st;
    }
    return MOE_OK;
}

moe_status moe_layer_forward(moe_ctx* ctx, int32_t layer, const void* x_dev, void* y_dev) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (ctx->routed_layer != layer) return fail(ctx, MOE_ERR_STATE, "moe_route(layer %d) must precede moe_layer_forward", layer);
    if (x_dev != ctx->routed_x) return fail(ctx, MOE_ERR_STATE, "x differs from the tensor given to moe_route");
    const int N = ctx->routed_tokens;
    ctx->stats.n_forward += 1;
    if (N == 0) return MOE_OK;
    if (!y_dev) return fail(ctx, MOE_ERR_INVALID_ARG, "y is null");
    const int E = ctx->cfg.n_experts, S = ctx->cfg.n_shared;
    LayerState& ls = ctx->layers[layer];
    bool all_resident = true;
    for (int e = 0; e < E + S; ++e) {
        if (!ls.resident[e]) {
            all_resident = false;
            if (e >= E || !ls.host[e]) return fail(ctx, MOE_ERR_STATE, "weights of layer %d expert %d not set", layer, e);
        }
    }
    const Shape s = make_shape(ctx, N);
    const PlanPtrs& p = ctx->plan;
    hipStream_t st = ctx->compute;
    const uint8_t* const* wtab = ctx->wtab_dev + (size_t)layer * (E + S);
    uint8_t* w = ctx->ws;
    const bool bf16 = ctx->cfg.dtype == MOE_BF16;
    const int split = auto_split_k(ctx, N);
    float* o = (float*)(w + ctx->L.o);

    FfnArgs a{};
    a.wtab = wtab;
    a.tile_expert = p.tile_expert;
    a.tile_xblk = p.tile_xblk;
    a.tile_hblk = p.tile_hblk;
    a.tile_nblk = p.tile_nblk;
    a.d = s.d;
    a.f = s.f;
    a.o_split_stride = ctx->L.o_split_stride;
    a.variant = ctx->variant % 10;
    a.panel = ctx->variant / 10;
    a.full_tiles = ((int64_t)N * s.k / std::max(1, E) > 160) ? 1 : 0;
    a.h_mode = ctx->h_mode;
    a.h_plane_units = ctx->L.h_plane_units;
    a.herr = (unsigned long long*)(w + ctx->L.herr);
    a.wmeta = ctx->wmeta_dev + (size_t)layer * (E + S);
    a.sat_count = (int32_t*)(w + ctx->L.meta) + 10;
    a.weight_bits = ctx->cfg.weight_bits;

    const bool prof = ctx->profiling && all_resident_layer(ctx, layer);
    ctx->prof_fwd = false;
    if (prof) (void)hipEventRecord(ctx->pev[3], st);
    int span = span_open(ctx, st, 1);
    if (bf16) launch_gather_bf16(st, x_dev, s, p, w + ctx->L.xp, a.herr);
    if (prof) (void)hipEventRecord(ctx->pev[4], st);

    if (all_resident) {
        if (bf16) {
            a.w_single = nullptr;
            a.tile_first = nullptr;
            a.tile_count = p.meta + 1;
            const int64_t A = (int64_t)N * s.k;
            a.max_tiles = (int)std::min<int64_t>(ctx->L.max_tiles,
                                                 (A / kRowBlk + E) / kTileBlks + std::min<int64_t>(E, A) +
                                                     (int64_t)S * ((N + kTileRows - 1) / kTileRows) + 1);
            a.est_tiles = (int)(std::max<int64_t>(std::min<int64_t>(E, A), (A + kTileRows - 1) / kTileRows) +
                                (int64_t)S * ((N + kTileRows - 1) / kTileRows));
            a.act = w + ctx->L.xp;
            a.out = w + ctx->L.h;
            a.split_k = 1;
            launch_ffn_up_bf16(st, a);
            if (prof) (void)hipEventRecord(ctx->pev[5], st);
            a.act = w + ctx->L.h;
            a.out = o;
            a.split_k = split;
            launch_ffn_down_bf16(st, a);
        } else {
            if (prof) (void)hipEventRecord(ctx->pev[5], st);
            launch_ffn_f32(st, (const float*)x_dev, s, p, wtab, nullptr, -1, (float*)(w + ctx->L.h), o);
        }
        if (prof) (void)hipEventRecord(ctx->pev[6], st);
    } else {
        span_close(ctx, st, span);  // the gather; every expert and the combine get spans of their own
        span = -1;
        moe_status rs = wait_route(ctx);
        if (rs != MOE_OK) return rs;
        // experts of this layer in the window that the gate did not select are dropped
        for (Slot& sl : ctx->slots) {
            if (sl.state == SLOT_LOADED && sl.layer == layer && ctx->h_counts[sl.expert] == 0) {
                ctx->stats.n_prefetch_unused += 1;
                release_slot(ctx, sl, false);
            }
        }
        // on-demand transfers for activated experts that are neither resident nor in flight
        for (int i = 0; i < ctx->h_nactive; ++i) {
            const int e = ctx->h_order[i];
            if (ls.resident[e]) continue;
            if (ls.slot_of[e] >= 0) {
                if (ctx->slots[ls.slot_of[e]].prefetched) ctx->stats.n_prefetch_hits += 1;
                continue;
            }
            moe_status ss = stream_one(ctx, layer, e, false);
            if (ss != MOE_OK) return ss;
        }
        // device-side tile ranges are addressed through exp_tile0 / exp_ntiles
        auto run_expert = [&](int e, const uint8_t* blob) {
            const int sp = span_open(ctx, st, 1);
            if (bf16) {
                a.w_single = blob;
                a.tile_first = p.exp_tile0 + e;
                a.tile_count = p.exp_ntiles + e;
                a.max_tiles = ctx->h_tiles[e].count;
                a.est_tiles = a.max_tiles;
                if (a.max_tiles > 0) {
                    a.act = w + ctx->L.xp;
                    a.out = w + ctx->L.h;
                    a.split_k = 1;
                    launch_ffn_up_bf16(st, a);
                    a.act = w + ctx->L.h;
                    a.out = o;
                    a.split_k = split;
                    launch_ffn_down_bf16(st, a);
                }
            } else {
                launch_ffn_f32(st, (const float*)x_dev, s, p, wtab, blob, e, (float*)(w + ctx->L.h), o);
            }
            span_close(ctx, st, sp);
        };
        for (int sh = 0; sh < S; ++sh) run_expert(E + sh, ls.resident[E + sh]);
        // experts whose weights were on the device before the gate ran (resident or prefetched)
        // go first, then the rest in execution order, which is also their copy order
        std::vector<int> seq;  // positions in the execution order, in launch order
        for (int pass = 0; pass < 2; ++pass)
            for (int i = 0; i < ctx->h_nactive; ++i) {
                const int e = ctx->h_order[i];
                const bool early = ls.resident[e] != nullptr ||
                                   (ls.slot_of[e] >= 0 && ctx->slots[ls.slot_of[e]].prefetched);
                if ((pass == 0) == early) seq.push_back(i);
            }
        // Small experts are computed in groups.  A pair of launches per expert costs about as much
        // as moving a 5 MB expert over the link, so the compute stream, not the link, would set
        // the pace.  Experts that follow each other both in the launch sequence and in execution
        // order own one contiguous range of tiles: they share one pair of launches, issued once
        // the last of them has landed, while the group's blobs stay below kGroupBytes.
        size_t at = 0;
        while (at < seq.size()) {
            size_t end = at + 1;
            if (bf16) {
                int64_t bytes = ctx->L.expert_bytes;
                while (end < seq.size() && end - at < (size_t)kMaxLaunchGroup && seq[end] == seq[end - 1] + 1 &&
                       bytes + ctx->L.expert_bytes <= kGroupBytes) {
                    ++end;
                    bytes += ctx->L.expert_bytes;
                }
            }
            const int sp = end - at > 1 ? span_open(ctx, st, 1) : -1;
            int tiles = 0;
            for (size_t j = at; j < end; ++j) {
                const int e = ctx->h_order[seq[j]];
                const uint8_t* blob = ls.resident[e];
                if (!blob) {
                    if (ls.slot_of[e] < 0)
                        return fail(ctx, MOE_ERR_STATE, "layer %d expert %d is not in the window", layer, e);
                    Slot& sl = ctx->slots[ls.slot_of[e]];
                    HIP_TRY(ctx, hipStreamWaitEvent(st, sl.ready, 0));
                    blob = sl.ptr;
                }
                if (end - at == 1) {
                    run_expert(e, blob);
                } else {
                    a.w_group[j - at] = blob;
                    a.group_expert[j - at] = e;
                    tiles += ctx->h_tiles[e].count;
                }
            }
            if (end - at > 1) {
                a.w_single = nullptr;
                a.n_group = (int32_t)(end - at);
                a.tile_first = nullptr;
                a.tile_count = nullptr;
                a.tile_first_v = ctx->h_tiles[ctx->h_order[seq[at]]].first;
                a.tile_count_v = tiles;
                a.max_tiles = tiles;
                a.est_tiles = tiles;
                if (tiles > 0) {
                    a.act = w + ctx->L.xp;
                    a.out = w + ctx->L.h;
                    a.split_k = 1;
                    launch_ffn_up_bf16(st, a);
                    a.act = w + ctx->L.h;
                    a.out = o;
                    a.split_k = split;
                    launch_ffn_down_bf16(st, a);
                }
                a.n_group = 0;
                span_close(ctx, st, sp);
            }
            for (size_t j = at; j < end; ++j) {  // slots are freed as soon as their last kernel is queued
                const int e = ctx->h_order[seq[j]];
                if (!ls.resident[e]) release_slot(ctx, ctx->slots[ls.slot_of[e]], true);
            }
            at = end;
        }
    }
    if (span < 0) span = span_open(ctx, st, 1);
    launch_combine(st, bf16 ? 1 : 0, s, p, o, bf16 ? split : 1, ctx->L.o_split_stride, y_dev);
    span_close(ctx, st, span);
    if (prof) {
        (void)hipEventRecord(ctx->pev[7], st);
        ctx->prof_fwd = true;
    }
    HIP_TRY(ctx, hipGetLastError());
    return MOE_OK;
}

moe_status moe_get_stats(moe_ctx* ctx, moe_stats* out) {
    if (!ctx || !out) return fail(ctx, MOE_ERR_INVALID_ARG, "null argument");
    // device counters since the last reset (stream-ordered read): H values clamped to the fp16 range,
    // down-projection workgroups that multiplied the remainder plane
    int32_t cnt[2] = {0, 0};
    HIP_TRY(ctx, hipMemcpyAsync(cnt, (int32_t*)(ctx->ws + ctx->L.meta) + 10, 8, hipMemcpyDeviceToHost, ctx->compute));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    ctx->stats.h_saturated = cnt[0];
    ctx->stats.h_remainder_wgs = cnt[1];
    // timed spans recorded while profiling was on: busy time of the link (union of the copy
    // intervals: two copy streams may overlap), of the compute stream, and the wall time from the
    // first start to the last end
    ctx->stats.copy_busy_ns = ctx->stats.compute_busy_ns = ctx->stats.wall_ns = 0;
    std::vector<std::pair<double, double>> copies;
    double lo = 0.0, hi = 0.0, compute_ms = 0.0;
    bool any = false;
    hipEvent_t ref = nullptr;
    for (const moe_ctx::Span& sp : ctx->spans) {
        if (!sp.closed) continue;
        HIP_TRY(ctx, hipEventSynchronize(sp.b));
        if (!ref) ref = sp.a;
        float t0 = 0.f, dt = 0.f;
        if (hipEventElapsedTime(&t0, ref, sp.a) != hipSuccess || hipEventElapsedTime(&dt, sp.a, sp.b) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        const double a0 = t0, a1 = (double)t0 + dt;
        lo = any ? std::min(lo, a0) : a0;
        hi = any ? std::max(hi, a1) : a1;
        any = true;
        if (sp.kind == 0) copies.emplace_back(a0, a1); else compute_ms += dt;
    }
    std::sort(copies.begin(), copies.end());
    double busy = 0.0, cur0 = 0.0, cur1 = 0.0;
    bool open = false;
    for (const auto& iv : copies) {
        if (open && iv.first <= cur1) {
            cur1 = std::max(cur1, iv.second);
        } else {
            if (open) busy += cur1 - cur0;
            cur0 = iv.first;
            cur1 = iv.second;
            open = true;
        }
    }
    if (open) busy += cur1 - cur0;
    ctx->stats.copy_busy_ns = (int64_t)(busy * 1e6);
    ctx->stats.compute_busy_ns = (int64_t)(compute_ms * 1e6);
    ctx->stats.wall_ns = any ? (int64_t)((hi - lo) * 1e6) : 0;
    *out = ctx->stats;
    return MOE_OK;
}

moe_status moe_reset_stats(moe_ctx* ctx) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    // spans still in flight keep their events until the streams have passed them
    if (!ctx->spans.empty()) {
        HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
        if (ctx->copy && ctx->copy != ctx->compute) HIP_TRY(ctx, hipStreamSynchronize(ctx->copy));
        for (hipStream_t cs : ctx->copy_extra) HIP_TRY(ctx, hipStreamSynchronize(cs));
    }
    ctx->spans.clear();
    ctx->ev_used = 0;
    launch_zero_u64(ctx->compute, (unsigned long long*)((int32_t*)(ctx->ws + ctx->L.meta) + 10), 1);  // meta[10..11]
    HIP_TRY(ctx, hipGetLastError());
    ctx->stats = moe_stats{};
    return MOE_OK;
}

moe_status moe_set_profiling(moe_ctx* ctx, int32_t enable) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    ctx->profiling = enable != 0;
    ctx->prof_route = ctx->prof_fwd = false;
    return MOE_OK;
}

moe_status moe_get_profile(moe_ctx* ctx, moe_profile* out) {
    if (!ctx || !out) return fail(ctx, MOE_ERR_INVALID_ARG, "null argument");
    memset(out, 0, sizeof *out);
    if (!ctx->prof_route || !ctx->prof_fwd)
        return fail(ctx, MOE_ERR_STATE, "no profiled moe_route + resident moe_layer_forward pair yet");
    HIP_TRY(ctx, hipEventSynchronize(ctx->pev[7]));
    float* dst[7] = {&out->router_ms, &out->plan_ms, nullptr, &out->gather_ms, &out->up_ms,
                     &out->down_ms, &out->combine_ms};
    for (int i = 0; i < 7; ++i) {
        if (!dst[i]) continue;
        HIP_TRY(ctx, hipEventElapsedTime(dst[i], ctx->pev[i], ctx->pev[i + 1]));
    }
    return MOE_OK;
}

moe_status moe_measure(moe_ctx* ctx, int32_t layer, const void* x_dev,
                       const int32_t* batch_offsets_host, int32_t n_batches, void* y_dev,
                       int32_t reps, moe_measured* out) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (!out || !y_dev) return fail(ctx, MOE_ERR_INVALID_ARG, "null argument");
    if (reps < 1 || reps > 1000) return fail(ctx, MOE_ERR_INVALID_ARG, "reps outside [1, 1000]");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (ctx->cfg.dtype != MOE_BF16) return fail(ctx, MOE_ERR_STATE, "measurement covers the bf16 path");
    memset(out, 0, sizeof *out);
    const int E = ctx->cfg.n_experts, S = ctx->cfg.n_shared;
    LayerState& ls = ctx->layers[layer];
    for (int e = 0; e < E + S; ++e)
        if (!ls.resident[e] && (e >= E || !ls.host[e]))
            return fail(ctx, MOE_ERR_STATE, "weights of layer %d expert %d not set", layer, e);
    hipStream_t st = ctx->compute;
    std::vector<hipEvent_t> evs;
    bool hip_failed = false;  // any HIP call of the measurement failed: the figures are void
    auto check = [&](hipError_t e) {
        if (e != hipSuccess) hip_failed = true;
    };
    // A timing event recorded on `on`; on failure the index of the first event is returned (so
    // that later look-ups stay in bounds) and the measurement is reported as failed at the end.
    auto mark = [&](hipStream_t on) -> int {
        hipEvent_t ev = nullptr;
        if (hipEventCreate(&ev) != hipSuccess) {
            hip_failed = true;
            return 0;
        }
        evs.push_back(ev);
        check(hipEventRecord(ev, on));
        return (int)evs.size() - 1;
    };
    auto done = [&](moe_status r) {
        for (hipEvent_t ev : evs) (void)hipEventDestroy(ev);
        return r;
    };
    auto secs = [&](int a, int b) {
        float ms = 0.f;
        if (evs.empty() || a < 0 || b < 0 || (size_t)a >= evs.size() || (size_t)b >= evs.size()) {
            hip_failed = true;
            return 0.0;
        }
        check(hipEventElapsedTime(&ms, evs[a], evs[b]));
        return (double)ms * 1e-3;
    };
    const bool learn = ctx->corr_learn;  // repeated routing of one group must not feed the table
    ctx->corr_learn = false;
    // gate + plan
    const int g0 = mark(st);
    moe_status r = MOE_OK;
    for (int i = 0; i < reps && r == MOE_OK; ++i)
        r = moe_route(ctx, layer, x_dev, batch_offsets_host, n_batches, nullptr, nullptr, nullptr, nullptr,
                      nullptr, nullptr, nullptr, nullptr);
    const int g1 = mark(st);
    ctx->corr_learn = learn;
    if (r != MOE_OK) return done(r);
    r = wait_route(ctx);
    if (r != MOE_OK) return done(r);
    const int N = ctx->routed_tokens;
    out->n_active = ctx->h_nactive;
    for (int e = 0; e < E; ++e) out->counts[e] = ctx->h_counts[e];
    for (int i = 0; i < ctx->h_nactive; ++i) out->exec_order[i] = ctx->h_order[i];
    // one expert over the link, into a free slot that then serves as a stand-in blob
    const uint8_t* standin = nullptr;
    int io0 = -1, io1 = -1, slot = -1;
    int host_e = -1;
    for (int i = 0; i < ctx->h_nactive && host_e < 0; ++i)
        if (!ls.resident[ctx->h_order[i]]) host_e = ctx->h_order[i];
    if (host_e >= 0) {
        for (size_t i = 0; i < ctx->slots.size() && slot < 0; ++i)
            if (ctx->slots[i].state == SLOT_FREE) slot = (int)i;
        if (slot < 0) return done(fail(ctx, MOE_ERR_OOM, "no free window slot to measure a transfer"));
        Slot& sl = ctx->slots[slot];
        if (sl.done_pending) {
            check(hipStreamWaitEvent(ctx->copy, sl.done, 0));
            sl.done_pending = false;
        }
        if (sl.ready_recorded) check(hipStreamWaitEvent(ctx->copy, sl.ready, 0));
        io0 = mark(ctx->copy);
        for (int i = 0; i < reps; ++i)
            check(hipMemcpyAsync(sl.ptr, ls.host[host_e], (size_t)ctx->L.expert_bytes, hipMemcpyHostToDevice, ctx->copy));
        io1 = mark(ctx->copy);
        check(hipEventRecord(sl.ready, ctx->copy));
        sl.ready_recorded = true;
        check(hipStreamWaitEvent(st, sl.ready, 0));
        standin = sl.ptr;
    }
    if (N > 0) {
        const Shape s = make_shape(ctx, N);
        const PlanPtrs& p = ctx->plan;
        uint8_t* w = ctx->ws;
        const int split = auto_split_k(ctx, N);
        float* o = (float*)(w + ctx->L.o);
        FfnArgs a{};
        a.wtab = ctx->wtab_dev + (size_t)layer * (E + S);
        a.tile_expert = p.tile_expert;
        a.tile_xblk = p.tile_xblk;
        a.tile_hblk = p.tile_hblk;
        a.tile_nblk = p.tile_nblk;
        a.d = s.d;
        a.f = s.f;
        a.o_split_stride = ctx->L.o_split_stride;
        a.variant = ctx->variant % 10;
        a.panel = ctx->variant / 10;
        a.full_tiles = ((int64_t)N * s.k / std::max(1, E) > 160) ? 1 : 0;
        a.h_mode = ctx->h_mode;
        a.h_plane_units = ctx->L.h_plane_units;
        a.herr = (unsigned long long*)(w + ctx->L.herr);
        a.wmeta = ctx->wmeta_dev + (size_t)layer * (E + S);
        a.sat_count = (int32_t*)(w + ctx->L.meta) + 10;
        a.weight_bits = ctx->cfg.weight_bits;
        const size_t herr_rows = (size_t)ctx->L.h_rows16 * kRowBlk;
        auto run_expert = [&](int e, const uint8_t* blob) {
            launch_zero_u64(st, a.herr, herr_rows);  // repeated runs must not add up their remainder energies
            a.w_single = blob;
            a.tile_first = p.exp_tile0 + e;
            a.tile_count = p.exp_ntiles + e;
            a.max_tiles = ctx->h_tiles[e].count;
            a.est_tiles = a.max_tiles;
            if (a.max_tiles == 0) return;
            a.act = w + ctx->L.xp;
            a.out = w + ctx->L.h;
            a.split_k = 1;
            launch_ffn_up_bf16(st, a);
            a.act = w + ctx->L.h;
            a.out = o;
            a.split_k = split;
            launch_ffn_down_bf16(st, a);
        };
        const int q0 = mark(st);
        for (int i = 0; i < reps; ++i) launch_gather_bf16(st, x_dev, s, p, w + ctx->L.xp, a.herr);
        const int q1 = mark(st);
        for (int sh = 0; sh < S; ++sh) run_expert(E + sh, ls.resident[E + sh]);
        std::vector<int> e0(ctx->h_nactive), e1(ctx->h_nactive);
        for (int i = 0; i < ctx->h_nactive; ++i) {
            const int e = ctx->h_order[i];
            const uint8_t* blob = ls.resident[e] ? ls.resident[e] : standin;
            e0[i] = mark(st);
            for (int j = 0; j < reps; ++j) run_expert(e, blob);
            e1[i] = mark(st);
        }
        const int c0 = mark(st);
        for (int i = 0; i < reps; ++i) launch_combine(st, 1, s, p, o, split, ctx->L.o_split_stride, y_dev);
        const int c1 = mark(st);
        if (hipStreamSynchronize(st) != hipSuccess || hipStreamSynchronize(ctx->copy) != hipSuccess)
            return done(fail(ctx, MOE_ERR_HIP, "synchronisation failed during measurement"));
        out->t_c_gather_s = secs(q0, q1) / reps;
        out->t_c_combine_s = secs(c0, c1) / reps;
        for (int i = 0; i < ctx->h_nactive; ++i) out->t_c_expert_s[ctx->h_order[i]] = secs(e0[i], e1[i]) / reps;
    } else {
        (void)hipStreamSynchronize(st);
        (void)hipStreamSynchronize(ctx->copy);
    }
    out->t_c_gate_group_s = secs(g0, g1) / reps;
    if (io0 >= 0) out->t_io_expert_s = secs(io0, io1) / reps;
    if (hipGetLastError() != hipSuccess || hip_failed)
        return done(fail(ctx, MOE_ERR_HIP, "a HIP call of the measurement failed: the reported times are void"));
    return done(MOE_OK);
}

moe_status moe_corr_rank(const int32_t* table_host, const int32_t* counts_prev_host, int32_t E,
                         int32_t K, int32_t* experts_out_host, int32_t* n_out, double* score_out) {
    if (!table_host || !counts_prev_host || !n_out || (K > 0 && !experts_out_host))
        return fail(nullptr, MOE_ERR_INVALID_ARG, "null argument");
    if (E < 1 || E > MOE_MAX_EXPERTS || K < 0) return fail(nullptr, MOE_ERR_INVALID_ARG, "E or K out of range");
    std::vector<double> score((size_t)E, 0.0);
    for (int p = 0; p < E; ++p) {  // previous experts in increasing index: fixed fp64 summation order
        const int32_t n = counts_prev_host[p];
        if (n <= 0) continue;
        const int32_t* row = table_host + (size_t)p * E;
        int64_t total = 0;
        for (int e = 0; e < E; ++e) total += row[e];
        if (total <= 0) continue;  // never observed: says nothing
        const double dn = (double)n, dt = (double)total;
        for (int e = 0; e < E; ++e) {
            const double freq = (double)row[e] / dt;
            const double term = dn * freq;
            score[e] = score[e] + term;
        }
    }
    std::vector<char> taken((size_t)E, 0);
    int n = 0;
    for (; n < K && n < E; ++n) {
        int best = -1;
        for (int e = 0; e < E; ++e)
            if (!taken[e] && score[e] > 0.0 && (best < 0 || score[e] > score[best])) best = e;
        if (best < 0) break;
        taken[best] = 1;
        experts_out_host[n] = best;
    }
    *n_out = n;
    if (score_out) memcpy(score_out, score.data(), (size_t)E * sizeof(double));
    return MOE_OK;
}

moe_status moe_corr_enable(moe_ctx* ctx, int32_t on) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (on < 0 || on > 2) return fail(ctx, MOE_ERR_INVALID_ARG, "mode must be 0, 1 or 2");
    ctx->corr_on = on != 0;
    ctx->corr_learn = on == 1;
    ctx->prev_idx_layer = -1;
    ctx->prev_idx_tokens = -1;
    return MOE_OK;
}

moe_status moe_corr_reset(moe_ctx* ctx) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    const size_t bytes = (size_t)ctx->cfg.n_layers * ctx->cfg.n_experts * ctx->cfg.n_experts * 4;
    HIP_TRY(ctx, hipMemsetAsync(ctx->ws + ctx->L.corr_table, 0, bytes, ctx->compute));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));  // no mirror refresh may still be in flight
    memset(ctx->corr_host, 0, bytes);
    ctx->prev_idx_layer = -1;
    ctx->prev_idx_tokens = -1;
    return MOE_OK;
}

moe_status moe_corr_table(moe_ctx* ctx, int32_t layer, int32_t* table_out_host) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!table_out_host) return fail(ctx, MOE_ERR_INVALID_ARG, "output is null");
    if (ctx->route_pending) {
        moe_status st = wait_route(ctx);  // mirror refreshes are ordered before the route event
        if (st != MOE_OK) return st;
    }
    const size_t EE = (size_t)ctx->cfg.n_experts * ctx->cfg.n_experts;
    memcpy(table_out_host, ctx->corr_host + (size_t)layer * EE, EE * 4);
    return MOE_OK;
}

moe_status moe_corr_predict(moe_ctx* ctx, int32_t layer, int32_t K, int32_t* experts_out_host,
                            int32_t* n_out) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 1 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d has no previous expert layer", layer);
    if (!ctx->corr_on) return fail(ctx, MOE_ERR_STATE, "correlation table is not enabled");
    if (ctx->routed_layer != layer - 1) return fail(ctx, MOE_ERR_STATE, "prediction for layer %d needs the routing of layer %d, the last moe_route was for layer %d", layer, layer - 1, ctx->routed_layer);
    moe_status st = wait_route(ctx);
    if (st != MOE_OK) return st;
    const size_t EE = (size_t)ctx->cfg.n_experts * ctx->cfg.n_experts;
    return moe_corr_rank(ctx->corr_host + (size_t)layer * EE, ctx->h_counts.data(), ctx->cfg.n_experts, K,
                         experts_out_host, n_out, nullptr);
}

// ---- routing for callers that cannot allocate ---------------------------------------------------
// The dispatch plan needs device scratch beyond its inputs and outputs (per-chunk histograms and
// bases, padded offsets, batches per expert, tile tables, the selected experts when the caller
// does not ask for them).  moe_route takes it from the context's workspace; this entry point
// takes it from a fixed array in the library's device image, so that nothing is allocated.
}  // extern "C"

namespace {
constexpr int64_t kStaticScratchBytes = 1536 * 1024;
constexpr int kStaticMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
// Device address of `scratch` on each GPU (every GPU holds its own copy of the array at its own
// address).  Host code never passes the array's name to a kernel or a copy: only these pointers.
unsigned char* g_scratch_ptr[kStaticMaxDevices] = {};
std::mutex g_scratch_mutex;

moe_status static_scratch(unsigned char** out) {
    int dev = -1;
    HIP_TRY(nullptr, hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return fail(nullptr, MOE_ERR_HIP, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(nullptr, MOE_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace

extern "C" {

moe_status moe_route_static(void* stream, int32_t dtype, const void* x_dev, const void* wg_dev,
                            int32_t n_tokens, int32_t d_model, int32_t n_experts, int32_t top_k,
                            int32_t renormalize, const int32_t* batch_offsets_host, int32_t n_batches,
                            float* logits_dev, int32_t* topk_idx_dev, float* topk_w_dev,
                            int32_t* counts_dev, int32_t* offsets_dev, int32_t* perm_dev,
                            int32_t* inv_perm_dev, int32_t* exec_order_dev) {
    if (dtype != MOE_F32 && dtype != MOE_BF16) return fail(nullptr, MOE_ERR_INVALID_ARG, "dtype must be MOE_F32 or MOE_BF16");
    const int mult = dtype == MOE_BF16 ? 64 : 4;
    if (d_model <= 0 || d_model % mult) return fail(nullptr, MOE_ERR_SHAPE, "d_model must be a positive multiple of %d", mult);
    if (n_experts < 1 || n_experts > MOE_MAX_EXPERTS) return fail(nullptr, MOE_ERR_SHAPE, "n_experts out of range");
    if (top_k < 1 || top_k > MOE_MAX_TOPK || top_k > n_experts) return fail(nullptr, MOE_ERR_SHAPE, "top_k out of range");
    if (!batch_offsets_host) return fail(nullptr, MOE_ERR_INVALID_ARG, "batch_offsets is null");
    if (n_batches < 1 || n_batches > MOE_MAX_BATCHES) return fail(nullptr, MOE_ERR_SHAPE, "n_batches %d outside [1, %d]", n_batches, MOE_MAX_BATCHES);
    if (batch_offsets_host[0] != 0) return fail(nullptr, MOE_ERR_INVALID_ARG, "batch_offsets must start at 0");
    BatchOffsets bo;
    bo.n = n_batches;
    for (int b = 0; b <= n_batches; ++b) {
        if (b > 0 && batch_offsets_host[b] < batch_offsets_host[b - 1])
            return fail(nullptr, MOE_ERR_INVALID_ARG, "batch_offsets must be non-decreasing");
        bo.v[b] = batch_offsets_host[b];
    }
    for (int b = n_batches + 1; b <= kMaxBatches; ++b) bo.v[b] = batch_offsets_host[n_batches];
    if (batch_offsets_host[n_batches] != n_tokens)
        return fail(nullptr, MOE_ERR_INVALID_ARG, "batch_offsets end at %d, n_tokens is %d", batch_offsets_host[n_batches], n_tokens);
    if (n_tokens < 0 || n_tokens > MOE_STATIC_MAX_TOKENS || (int64_t)n_tokens * top_k > MOE_STATIC_MAX_ASSIGNMENTS)
        return fail(nullptr, MOE_ERR_SHAPE, "%d tokens x top-%d exceed what moe_route_static serves (%d tokens, %d assignments)",
                    n_tokens, top_k, MOE_STATIC_MAX_TOKENS, MOE_STATIC_MAX_ASSIGNMENTS);
    if (n_tokens > 0 && (!x_dev || !wg_dev)) return fail(nullptr, MOE_ERR_INVALID_ARG, "x or the gate matrix is null");

    // carve the scratch array; whatever the caller asks for is written in place instead
    const int64_t E = n_experts, A = (int64_t)n_tokens * top_k;
    const int64_t max_rowblks = (A + kRowBlk - 1) / kRowBlk + E;
    const int64_t nchunks = (A + kPlanChunk - 1) / kPlanChunk;
    const int max_tiles = max_tiles_for((int)max_rowblks, (int)E, 0, n_tokens);
    unsigned char* base = nullptr;
    moe_status rs = static_scratch(&base);
    if (rs != MOE_OK) return rs;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        unsigned char* at = base + off;
        off = align_up(off + bytes, 256);
        return at;
    };
    PlanPtrs p{};
    p.meta = (int32_t*)take(16 * 4);
    p.topk_idx = topk_idx_dev ? topk_idx_dev : (int32_t*)take(A * 4);
    p.topk_w = topk_w_dev ? topk_w_dev : (float*)take(A * 4);
    p.counts = counts_dev ? counts_dev : (int32_t*)take(E * 4);
    p.offsets = offsets_dev ? offsets_dev : (int32_t*)take((E + 1) * 4);
    p.poff = (int32_t*)take((E + 1) * 4);
    p.nbatch = (int32_t*)take(E * 4);
    p.exec_order = exec_order_dev ? exec_order_dev : (int32_t*)take(E * 4);
    p.perm = perm_dev ? perm_dev : (int32_t*)take(A * 4);
    p.inv_perm = inv_perm_dev ? inv_perm_dev : (int32_t*)take(A * 4);
    p.blk_counts = (int32_t*)take(nchunks * E * 4);
    p.blk_base = (int32_t*)take(nchunks * E * 4);
    p.blk_mask = (unsigned long long*)take(nchunks * E * 8);
    p.tile_expert = (int32_t*)take((int64_t)max_tiles * 4);
    p.tile_xblk = (int32_t*)take((int64_t)max_tiles * 4);
    p.tile_hblk = (int32_t*)take((int64_t)max_tiles * 4);
    p.tile_nblk = (int32_t*)take((int64_t)max_tiles * 4);
    p.exp_tile0 = (int32_t*)take(E * 4);
    p.exp_ntiles = (int32_t*)take(E * 4);
    p.blk_expert = (int32_t*)take(max_rowblks * 4);
    p.mail = (int32_t*)take((2 * E + 1) * 4);
    if (off > kStaticScratchBytes)  // cannot happen within the limits above; kept as the bound's proof
        return fail(nullptr, MOE_ERR_SHAPE, "routing scratch of %lld bytes exceeds the static %lld", (long long)off, (long long)kStaticScratchBytes);
    Shape s{};
    s.N = n_tokens;
    s.d = d_model;
    s.f = 0;
    s.E = n_experts;
    s.k = top_k;
    s.S = 0;
    s.renorm = renormalize ? 1 : 0;
    s.max_rowblks = (int32_t)max_rowblks;
    hipStream_t st = (hipStream_t)stream;
    launch_router(st, dtype, x_dev, wg_dev, s, logits_dev, p.topk_idx, p.topk_w);
    launch_plan(st, s, bo, p, max_tiles);
    HIP_TRY(nullptr, hipGetLastError());
    return MOE_OK;
}

moe_status moe_set_tuning(moe_ctx* ctx, int32_t split_k, int32_t h_planes, int32_t variant) {
    if (variant < -1 || variant > 69) return fail(ctx, MOE_ERR_INVALID_ARG, "variant out of range");
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (split_k < 0 || split_k > 64) return fail(ctx, MOE_ERR_INVALID_ARG, "split_k out of range");
    if (h_planes < 0 || h_planes > 2) return fail(ctx, MOE_ERR_INVALID_ARG, "h_planes must be 0 (keep), 1 (automatic) or 2 (always both planes)");
    ctx->split_k_user = split_k;
    if (h_planes > 0) ctx->h_mode = h_planes == 2 ? 1 : 0;
    if (variant != 0) ctx->variant = variant < 0 ? 0 : variant;
    return MOE_OK;
}

}  // extern "C"
