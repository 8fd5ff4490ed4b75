// C ABI of the attention (non-expert) layer: the per-batch loop of Algorithm 1's else-branch
// with the hidden state and the key-value cache of each batch moved by a load stream and a
// store stream around the compute stream.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/moe_attn.h"
#include "attn_kernels.h"

using namespace kattn;

struct moe_attn_ctx {
    moe_attn_config cfg;
    Dims dm;
    hipStream_t compute, load, store;
    uint8_t* ws;
    // offsets into the workspace
    size_t o_wqkv, o_wo, o_g, layer_stride, o_freq, o_ax, o_ao, o_part, o_q, o_kv[2][2], o_new[2], o_hin[2], o_hout[2], total;
    int rows_alloc;   // rows the activation buffers hold (multiple of 128)
    int part_rows;    // rows x splits the partial-sum buffer holds
    size_t widest;    // columns of the widest projection
    std::vector<char> has_weights;  // per layer
    hipEvent_t entry, finish, loaded[2], done[2], stored[2];
    int profiling;  // 0 off, n >= 1: kernels launched n times between their events
    std::vector<hipEvent_t> ev;  // kEv per batch when profiling
    moe_attn_profile prof;
    bool prof_valid;
    bool pre_valid;        // staging buffer 0 holds the caches of `pre` (moe_attn_prefetch)
    moe_attn_batch pre;
    mutable std::string err;
};

namespace {

thread_local std::string g_attn_error;

// profiling events of one batch: load begin / end, store begin / end, then the 7 boundaries of
// the 6 kernels on the compute stream
constexpr int kEv = 11, kEvLoad = 0, kEvStore = 2, kEvKernel = 4;

moe_status fail(const moe_attn_ctx* ctx, moe_status s, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    g_attn_error = buf;
    return s;
}

#define HIP_TRY(ctx, expr)                                                                \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess)                                                             \
            return fail(ctx, MOE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

int pointer_kind(const void* p) {  // 0 unknown / pageable, 1 pinned host, 2 device
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, p) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    if (at.type == hipMemoryTypeHost) return 1;
    if (at.type == hipMemoryTypeDevice) return 2;
    return 0;
}

size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

moe_status check_config(const moe_attn_config* c, std::string* why) {
    auto bad = [&](const char* m) {
        *why = m;
        return MOE_ERR_SHAPE;
    };
    if (c->d_model <= 0 || c->d_model % 128 != 0 || c->d_model > 8192) return bad("d_model must be a multiple of 128 in 128..8192");
    if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 32, 64 or 128");
    if (c->n_kv_heads <= 0 || c->n_q_heads <= 0 || c->n_q_heads % c->n_kv_heads != 0) return bad("n_q_heads must be a multiple of n_kv_heads");
    const int g = c->n_q_heads / c->n_kv_heads;
    if (g > 8) return bad("n_q_heads / n_kv_heads must be at most 8");
    if ((c->n_q_heads * c->head_dim) % 128 != 0) return bad("n_q_heads*head_dim must be a multiple of 128");
    if ((c->n_kv_heads * c->head_dim) % 32 != 0) return bad("n_kv_heads*head_dim must be a multiple of 32");
    if (c->max_seqs <= 0 || c->max_seqs > 4096) return bad("max_seqs must be in 1..4096");
    if (c->max_len <= 0 || c->max_len > (1 << 20)) return bad("max_len must be in 1..2^20");
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return bad("rope_theta must be > 0 and rms_eps >= 0");
    if (c->n_layers < 1 || c->n_layers > 1024) return bad("n_layers must be in 1..1024");
    if (c->max_group_seqs < 0 || c->max_group_seqs > 65536) return bad("max_group_seqs must be in 0..65536");
    return MOE_OK;
}

void layout(moe_attn_ctx* c) {
    const moe_attn_config& g = c->cfg;
    const size_t d = g.d_model, dq = (size_t)g.n_q_heads * g.head_dim, dkv = (size_t)g.n_kv_heads * g.head_dim;
    const size_t n_qkv = dq + 2 * dkv;
    const int most = g.max_group_seqs > g.max_seqs ? g.max_group_seqs : g.max_seqs;
    c->rows_alloc = ((most + 127) / 128) * 128;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o += up256(bytes);
        return at;
    };
    c->o_wqkv = take(n_qkv * d * 2);  // layer 0; layer l at + l * layer_stride
    c->o_wo = take(d * dq * 2);
    c->o_g = take(d * 2);
    c->layer_stride = o;
    o *= (size_t)g.n_layers;
    c->o_freq = take((size_t)g.head_dim / 2 * sizeof(double));
    c->o_ax = take((size_t)c->rows_alloc * d * 2);
    c->o_ao = take((size_t)c->rows_alloc * dq * 2);
    c->widest = n_qkv > d ? n_qkv : d;
    c->part_rows = c->rows_alloc > kMaxSplit * 128 ? c->rows_alloc : kMaxSplit * 128;
    c->o_part = take((size_t)c->part_rows * c->widest * 4);
    c->o_q = take((size_t)c->rows_alloc * dq * 4);
    const size_t cache = (size_t)g.max_seqs * dkv * g.max_len * 2;
    for (int b = 0; b < 2; ++b) {
        c->o_kv[b][0] = take(cache);
        c->o_kv[b][1] = take(cache);
        c->o_new[b] = take(2 * (size_t)g.max_seqs * dkv * 2);
        c->o_hin[b] = take((size_t)g.max_seqs * d * 2);
        c->o_hout[b] = take((size_t)g.max_seqs * d * 2);
    }
    c->total = o;
}

moe_status check_batch(const moe_attn_ctx* ctx, const moe_attn_batch& B, int b) {
    const moe_attn_config& c = ctx->cfg;
    if (B.n_seq < 1 || B.n_seq > c.max_seqs) return fail(ctx, MOE_ERR_INVALID_ARG, "batch %d: n_seq %d outside 1..max_seqs", b, B.n_seq);
    if (B.pos < 0 || B.pos >= c.max_len) return fail(ctx, MOE_ERR_INVALID_ARG, "batch %d: pos %d outside 0..max_len-1", b, B.pos);
    if (!B.k_cache || !B.v_cache || !B.h_in || !B.h_out) return fail(ctx, MOE_ERR_INVALID_ARG, "batch %d: null pointer", b);
    const int want_kv = B.kv_on_host ? 1 : 2, want_h = B.h_on_host ? 1 : 2;
    if (pointer_kind(B.k_cache) != want_kv || pointer_kind(B.v_cache) != want_kv)
        return fail(ctx, B.kv_on_host ? MOE_ERR_NOT_PINNED : MOE_ERR_INVALID_ARG, "batch %d: cache pointers are not %s memory", b, B.kv_on_host ? "pinned host" : "device");
    if (pointer_kind(B.h_in) != want_h || pointer_kind(B.h_out) != want_h)
        return fail(ctx, B.h_on_host ? MOE_ERR_NOT_PINNED : MOE_ERR_INVALID_ARG, "batch %d: hidden-state pointers are not %s memory", b, B.h_on_host ? "pinned host" : "device");
    return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_attn_last_error(const moe_attn_ctx* ctx) { return ctx ? ctx->err.c_str() : g_attn_error.c_str(); }

moe_status moe_attn_workspace_bytes(const moe_attn_config* cfg, int64_t* bytes_out) {
    if (!cfg || !bytes_out) return fail(nullptr, MOE_ERR_INVALID_ARG, "null argument");
    std::string why;
    moe_status s = check_config(cfg, &why);
    if (s != MOE_OK) return fail(nullptr, s, "%s", why.c_str());
    moe_attn_ctx tmp{};
    tmp.cfg = *cfg;
    layout(&tmp);
    *bytes_out = (int64_t)tmp.total;
    return MOE_OK;
}

moe_status moe_attn_create(const moe_attn_config* cfg, void* workspace_dev, int64_t workspace_bytes,
                           void* compute_stream, void* load_stream, void* store_stream,
                           moe_attn_ctx** out) {
    if (!cfg || !out) return fail(nullptr, MOE_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    std::string why;
    moe_status s = check_config(cfg, &why);
    if (s != MOE_OK) return fail(nullptr, s, "%s", why.c_str());
    if (!workspace_dev || ((uintptr_t)workspace_dev & 255u) != 0) return fail(nullptr, MOE_ERR_INVALID_ARG, "workspace must be non-null and 256-byte aligned");
    if (!compute_stream || !load_stream || !store_stream || compute_stream == load_stream ||
        compute_stream == store_stream || load_stream == store_stream)
        return fail(nullptr, MOE_ERR_INVALID_ARG, "three distinct non-null streams are required");
    moe_attn_ctx* c = new moe_attn_ctx{};
    c->cfg = *cfg;
    c->dm = Dims{cfg->d_model, cfg->n_q_heads, cfg->n_kv_heads, cfg->head_dim, cfg->max_len};
    layout(c);
    if ((int64_t)c->total > workspace_bytes) {
        const long long need = (long long)c->total;
        delete c;
        return fail(nullptr, MOE_ERR_OOM, "workspace of %lld bytes, need %lld", (long long)workspace_bytes, need);
    }
    if (pointer_kind(workspace_dev) != 2) {
        delete c;
        return fail(nullptr, MOE_ERR_INVALID_ARG, "workspace is not device memory");
    }
    c->ws = (uint8_t*)workspace_dev;
    c->has_weights.assign(cfg->n_layers, 0);
    c->compute = (hipStream_t)compute_stream;
    c->load = (hipStream_t)load_stream;
    c->store = (hipStream_t)store_stream;
    hipEvent_t* plain[] = {&c->entry, &c->finish, &c->loaded[0], &c->loaded[1], &c->done[0], &c->done[1], &c->stored[0], &c->stored[1]};
    for (hipEvent_t* e : plain) {
        if (hipEventCreate(e) != hipSuccess) {  // timing enabled: entry / finish bracket the wall time
            moe_attn_destroy(c);  // releases the events created so far
            return fail(nullptr, MOE_ERR_HIP, "hipEventCreate failed");
        }
    }
    // rotary frequencies theta^(-2i/hd) in double; activation buffers start as zeros so that the
    // padding rows of a row block are finite
    std::vector<double> f(cfg->head_dim / 2);
    for (int i = 0; i < cfg->head_dim / 2; ++i) f[i] = std::pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
    hipError_t e = hipMemcpy(c->ws + c->o_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + c->o_ax, 0, c->o_part - c->o_ax, c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) {
        moe_attn_destroy(c);
        return fail(nullptr, MOE_ERR_HIP, "workspace initialisation failed: %s", hipGetErrorString(e));
    }
    *out = c;
    return MOE_OK;
}

void moe_attn_destroy(moe_attn_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->compute);
    (void)hipStreamSynchronize(c->load);
    (void)hipStreamSynchronize(c->store);
    hipEvent_t plain[] = {c->entry, c->finish, c->loaded[0], c->loaded[1], c->done[0], c->done[1], c->stored[0], c->stored[1]};
    for (hipEvent_t e : plain)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    delete c;
}

moe_status moe_attn_set_weights(moe_attn_ctx* ctx, int32_t layer, const void* g, const void* wq,
                                const void* wk, const void* wv, const void* wo, int32_t on_host) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d outside 0..%d", layer, ctx->cfg.n_layers - 1);
    const size_t lo = (size_t)layer * ctx->layer_stride;
    if (!g || !wq || !wk || !wv || !wo) return fail(ctx, MOE_ERR_INVALID_ARG, "null weight pointer");
    const moe_attn_config& c = ctx->cfg;
    const size_t d = c.d_model, dq = (size_t)c.n_q_heads * c.head_dim, dkv = (size_t)c.n_kv_heads * c.head_dim;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    // row-major staging: the partial-sum buffer is idle here and large enough for any one matrix
    uint8_t* stage = ctx->ws + ctx->o_part;
    const size_t stage_bytes = (size_t)ctx->part_rows * ctx->widest * 4;
    struct Item {
        const void* src;
        size_t rows, K;
        size_t dst_off;
    } items[4] = {{wq, dq, d, lo + ctx->o_wqkv},
                  {wk, dkv, d, lo + ctx->o_wqkv + dq * d * 2},
                  {wv, dkv, d, lo + ctx->o_wqkv + (dq + dkv) * d * 2},
                  {wo, d, dq, lo + ctx->o_wo}};
    for (const Item& it : items) {
        const size_t bytes = it.rows * it.K * 2;
        const void* src = it.src;
        if (on_host) {
            if (bytes > stage_bytes) return fail(ctx, MOE_ERR_OOM, "weight matrix larger than the staging area");
            HIP_TRY(ctx, hipMemcpy(stage, it.src, bytes, hipMemcpyHostToDevice));
            src = stage;
        } else if (pointer_kind(it.src) != 2) {
            return fail(ctx, MOE_ERR_INVALID_ARG, "weight pointer is not device memory");
        }
        launch_pack_weight(ctx->compute, src, (int)it.rows, (int)it.K, ctx->ws + it.dst_off);
        HIP_TRY(ctx, hipGetLastError());
        HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
    }
    HIP_TRY(ctx, hipMemcpy(ctx->ws + lo + ctx->o_g, g, d * 2, on_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice));
    ctx->has_weights[layer] = 1;
    return MOE_OK;
}

moe_status moe_attn_set_profiling(moe_attn_ctx* ctx, int32_t on) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (on < 0 || on > 64) return fail(ctx, MOE_ERR_INVALID_ARG, "profiling level %d outside 0..64", on);
    ctx->profiling = on;
    ctx->prof_valid = false;
    return MOE_OK;
}

moe_status moe_attn_get_profile(moe_attn_ctx* ctx, moe_attn_profile* out) {
    if (!ctx || !out) return fail(ctx, MOE_ERR_INVALID_ARG, "null argument");
    if (!ctx->prof_valid) return fail(ctx, MOE_ERR_STATE, "no profiled moe_attn_forward_group yet");
    *out = ctx->prof;
    return MOE_OK;
}

moe_status moe_attn_prefetch(moe_attn_ctx* ctx, const moe_attn_batch* first) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (!first) return fail(ctx, MOE_ERR_INVALID_ARG, "first is null");
    moe_status bs = check_batch(ctx, *first, 0);
    if (bs != MOE_OK) return bs;
    ctx->pre_valid = false;
    if (!first->kv_on_host || first->pos == 0) return MOE_OK;  // nothing to move
    const moe_attn_config& c = ctx->cfg;
    const size_t hd = c.head_dim, pitch = (size_t)c.max_len * hd * 2;
    const size_t width = (size_t)first->pos * hd * 2, height = (size_t)first->n_seq * c.n_kv_heads;
    // staging buffer 0 is free once everything enqueued on the compute stream so far has run
    HIP_TRY(ctx, hipEventRecord(ctx->entry, ctx->compute));
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->load, ctx->entry, 0));
    HIP_TRY(ctx, hipMemcpy2DAsync(ctx->ws + ctx->o_kv[0][0], pitch, first->k_cache, pitch, width, height, hipMemcpyHostToDevice, ctx->load));
    HIP_TRY(ctx, hipMemcpy2DAsync(ctx->ws + ctx->o_kv[0][1], pitch, first->v_cache, pitch, width, height, hipMemcpyHostToDevice, ctx->load));
    ctx->pre = *first;
    ctx->pre_valid = true;
    return MOE_OK;
}

moe_status moe_attn_forward_group(moe_attn_ctx* ctx, int32_t layer, int32_t n_batches,
                                  const moe_attn_batch* batches) {
    if (!ctx) return fail(nullptr, MOE_ERR_INVALID_ARG, "ctx is null");
    if (!batches || n_batches < 0) return fail(ctx, MOE_ERR_INVALID_ARG, "bad batches argument");
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, MOE_ERR_INVALID_ARG, "layer %d outside 0..%d", layer, ctx->cfg.n_layers - 1);
    if (!ctx->has_weights[layer]) return fail(ctx, MOE_ERR_STATE, "moe_attn_set_weights has not been called for layer %d", layer);
    const size_t lo = (size_t)layer * ctx->layer_stride;
    const moe_attn_config& c = ctx->cfg;
    const size_t d = c.d_model, hd = c.head_dim, dkv = (size_t)c.n_kv_heads * hd, dq = (size_t)c.n_q_heads * hd;
    for (int b = 0; b < n_batches; ++b) {
        moe_status bs = check_batch(ctx, batches[b], b);
        if (bs != MOE_OK) return bs;
    }
    if (n_batches == 0) return MOE_OK;
    const bool prof = ctx->profiling > 0;
    const int reps = prof ? ctx->profiling : 1;
    if (prof) {
        ctx->prof_valid = false;
        while (ctx->ev.size() < (size_t)n_batches * kEv) {
            hipEvent_t e;
            HIP_TRY(ctx, hipEventCreate(&e));
            ctx->ev.push_back(e);
        }
    }
    hipStream_t st = ctx->compute, ld = ctx->load, sv = ctx->store;
    uint8_t* w = ctx->ws;
    const size_t pitch = (size_t)c.max_len * hd * 2;  // bytes between (sequence, head) rows of a cache
    int64_t bytes_loaded = 0, bytes_stored = 0;

    // the staging buffers may still be read by work enqueued earlier on the compute stream
    // a batch that lives on the device needs neither stream: no event is recorded or waited for
    // on its behalf (a group that is all on the device is a plain run of kernels)
    auto on_device = [&](int b) { return !batches[b].kv_on_host && !batches[b].h_on_host; };
    bool any_host = false;
    for (int b = 0; b < n_batches; ++b) any_host = any_host || !on_device(b);
    if (any_host || prof) {
        HIP_TRY(ctx, hipEventRecord(ctx->entry, st));
        HIP_TRY(ctx, hipStreamWaitEvent(ld, ctx->entry, 0));
        HIP_TRY(ctx, hipStreamWaitEvent(sv, ctx->entry, 0));
    }
    bool used_done[2] = {false, false}, used_stored[2] = {false, false}, used_loaded[2] = {false, false};

    auto issue_load = [&](int b, bool caches_there) -> moe_status {
        const moe_attn_batch& B = batches[b];
        const int buf = b & 1;
        used_loaded[buf] = false;
        if (on_device(b) && !prof) return MOE_OK;
        if (used_done[buf]) HIP_TRY(ctx, hipStreamWaitEvent(ld, ctx->done[buf], 0));
        if (prof) HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvLoad], ld));
        if (B.kv_on_host && B.pos > 0 && !caches_there) {
            const size_t width = (size_t)B.pos * hd * 2, height = (size_t)B.n_seq * c.n_kv_heads;
            HIP_TRY(ctx, hipMemcpy2DAsync(w + ctx->o_kv[buf][0], pitch, B.k_cache, pitch, width, height, hipMemcpyHostToDevice, ld));
            HIP_TRY(ctx, hipMemcpy2DAsync(w + ctx->o_kv[buf][1], pitch, B.v_cache, pitch, width, height, hipMemcpyHostToDevice, ld));
            bytes_loaded += 2 * (int64_t)(width * height);
        }
        if (B.h_on_host) {
            HIP_TRY(ctx, hipMemcpyAsync(w + ctx->o_hin[buf], B.h_in, (size_t)B.n_seq * d * 2, hipMemcpyHostToDevice, ld));
            bytes_loaded += (int64_t)B.n_seq * d * 2;
        }
        if (prof) HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvLoad + 1], ld));
        HIP_TRY(ctx, hipEventRecord(ctx->loaded[buf], ld));
        used_loaded[buf] = true;
        return MOE_OK;
    };

    // the six kernels of the layer for the rows of `tab`; profiling events go to slot `slot`
    auto launch_layer = [&](const GroupTab& tab, int slot) -> moe_status {
        auto mark = [&](int i) -> hipError_t { return prof ? hipEventRecord(ctx->ev[slot * kEv + kEvKernel + i], st) : hipSuccess; };
        float* part = (float*)(w + ctx->o_part);
        float* q = (float*)(w + ctx->o_q);
        const int rows = tab.row0[tab.n];
        const int nrb = (rows + kRowBlk - 1) / kRowBlk;
        const int rows_pad = ((rows + 127) / 128) * 128;  // the row tile of a projection is at most 128 rows
        const int n_qkv = (int)(dq + 2 * dkv);
        auto splits_for = [&](int K, int n_out) {
            int sp = pick_splits(nrb, K, n_out);
            while (sp > 1 && sp * rows_pad > ctx->part_rows) sp /= 2;
            return sp;
        };
        const int64_t stride = (int64_t)rows_pad * (int64_t)ctx->widest;
        HIP_TRY(ctx, mark(0));
        for (int r = 0; r < reps; ++r) launch_rmsnorm(st, tab, w + lo + ctx->o_g, (int)d, c.rms_eps, w + ctx->o_ax);
        HIP_TRY(ctx, mark(1));
        const int sp1 = splits_for((int)d, n_qkv);
        for (int r = 0; r < reps; ++r) launch_proj(st, w + ctx->o_ax, w + lo + ctx->o_wqkv, nrb, (int)d, n_qkv, sp1, part, stride);
        HIP_TRY(ctx, mark(2));
        for (int r = 0; r < reps; ++r) launch_qkv_finish(st, part, sp1, stride, ctx->dm, tab, (const double*)(w + ctx->o_freq), q);
        HIP_TRY(ctx, mark(3));
        for (int r = 0; r < reps; ++r)
            if (launch_attention(st, q, ctx->dm, tab, w + ctx->o_ao) != 0)
                return fail(ctx, MOE_ERR_SHAPE, "no attention kernel for this head shape");
        HIP_TRY(ctx, mark(4));
        const int sp2 = splits_for((int)dq, (int)d);
        for (int r = 0; r < reps; ++r) launch_proj(st, w + ctx->o_ao, w + lo + ctx->o_wo, nrb, (int)dq, (int)d, sp2, part, stride);
        HIP_TRY(ctx, mark(5));
        launch_out_finish(st, part, sp2, stride, tab, (int)d);
        HIP_TRY(ctx, hipGetLastError());
        HIP_TRY(ctx, mark(6));
        return MOE_OK;
    };

    // A group that lives on the device needs no per-batch order: the weights are shared across
    // its batches as the expert layer shares an expert's (one pass over the projection weights
    // for all rows of the group, one launch of each kernel), provided the rows fit the buffers.
    int total_rows = 0;
    for (int b = 0; b < n_batches; ++b) total_rows += batches[b].n_seq;
    const int group_cap = c.max_group_seqs > c.max_seqs ? c.max_group_seqs : c.max_seqs;  // as configured, not as padded
    const bool grouped = !any_host && n_batches <= kMaxGroup && total_rows <= group_cap;
    const int n_units = grouped ? 1 : n_batches;
    if (grouped) {
        GroupTab tab{};
        tab.n = n_batches;
        for (int b = 0; b < n_batches; ++b) {
            tab.row0[b + 1] = tab.row0[b] + batches[b].n_seq;
            tab.pos[b] = batches[b].pos;
            tab.h_in[b] = batches[b].h_in;
            tab.h_out[b] = batches[b].h_out;
            tab.kc[b] = batches[b].k_cache;
            tab.vc[b] = batches[b].v_cache;
            tab.new_rows[b] = nullptr;
        }
        ctx->pre_valid = false;
        if (prof) {
            HIP_TRY(ctx, hipEventRecord(ctx->ev[kEvLoad], ld));
            HIP_TRY(ctx, hipEventRecord(ctx->ev[kEvLoad + 1], ld));
            HIP_TRY(ctx, hipEventRecord(ctx->ev[kEvStore], sv));
            HIP_TRY(ctx, hipEventRecord(ctx->ev[kEvStore + 1], sv));
        }
        moe_status grc = launch_layer(tab, 0);
        if (grc != MOE_OK) return grc;
    }

    // the caches of the first batch may have been brought in ahead of the call
    const moe_attn_batch& F = batches[0];
    const bool pre = ctx->pre_valid && F.kv_on_host && ctx->pre.k_cache == F.k_cache && ctx->pre.v_cache == F.v_cache &&
                     ctx->pre.n_seq == F.n_seq && ctx->pre.pos == F.pos;
    ctx->pre_valid = false;
    moe_status rc = grouped ? MOE_OK : issue_load(0, pre);
    if (rc != MOE_OK) return rc;
    for (int b = 0; b < (grouped ? 0 : n_batches); ++b) {
        const moe_attn_batch& B = batches[b];
        const int buf = b & 1;
        if (b + 1 < n_batches) {
            rc = issue_load(b + 1, false);
            if (rc != MOE_OK) return rc;
        }
        if (used_loaded[buf]) HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->loaded[buf], 0));
        if (used_stored[buf] && !on_device(b)) HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->stored[buf], 0));
        GroupTab tab{};
        tab.n = 1;
        tab.row0[0] = 0;
        tab.row0[1] = B.n_seq;
        tab.pos[0] = B.pos;
        tab.h_in[0] = B.h_on_host ? (const void*)(w + ctx->o_hin[buf]) : B.h_in;
        tab.h_out[0] = B.h_on_host ? (void*)(w + ctx->o_hout[buf]) : B.h_out;
        tab.kc[0] = B.kv_on_host ? (void*)(w + ctx->o_kv[buf][0]) : B.k_cache;
        tab.vc[0] = B.kv_on_host ? (void*)(w + ctx->o_kv[buf][1]) : B.v_cache;
        tab.new_rows[0] = B.kv_on_host ? (void*)(w + ctx->o_new[buf]) : nullptr;
        rc = launch_layer(tab, b);
        if (rc != MOE_OK) return rc;
        if (any_host) {  // a later batch may load into this staging buffer
            HIP_TRY(ctx, hipEventRecord(ctx->done[buf], st));
            used_done[buf] = true;
        }

        if (B.kv_on_host || B.h_on_host) {
            HIP_TRY(ctx, hipStreamWaitEvent(sv, ctx->done[buf], 0));
            if (prof) HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvStore], sv));
            if (B.kv_on_host) {
                const size_t height = (size_t)B.n_seq * c.n_kv_heads, row = hd * 2;
                const uint8_t* nr = w + ctx->o_new[buf];
                HIP_TRY(ctx, hipMemcpy2DAsync((uint8_t*)B.k_cache + (size_t)B.pos * row, pitch, nr, row, row, height, hipMemcpyDeviceToHost, sv));
                HIP_TRY(ctx, hipMemcpy2DAsync((uint8_t*)B.v_cache + (size_t)B.pos * row, pitch, nr + height * row, row, row, height, hipMemcpyDeviceToHost, sv));
                bytes_stored += 2 * (int64_t)(height * row);
            }
            if (B.h_on_host) {
                HIP_TRY(ctx, hipMemcpyAsync(B.h_out, w + ctx->o_hout[buf], (size_t)B.n_seq * d * 2, hipMemcpyDeviceToHost, sv));
                bytes_stored += (int64_t)B.n_seq * d * 2;
            }
            if (prof) HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvStore + 1], sv));
            HIP_TRY(ctx, hipEventRecord(ctx->stored[buf], sv));
            used_stored[buf] = true;
        } else if (prof) {
            HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvStore], sv));
            HIP_TRY(ctx, hipEventRecord(ctx->ev[b * kEv + kEvStore + 1], sv));
        }
    }
    for (int buf = 0; buf < 2; ++buf)
        if (used_stored[buf]) HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->stored[buf], 0));
    if (prof) HIP_TRY(ctx, hipEventRecord(ctx->finish, st));
    if (prof) {
        HIP_TRY(ctx, hipStreamSynchronize(st));
        HIP_TRY(ctx, hipStreamSynchronize(ld));
        HIP_TRY(ctx, hipStreamSynchronize(sv));
        moe_attn_profile p{};
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->entry, ctx->finish));
        p.wall_s = ms * 1e-3;
        for (int b = 0; b < n_units; ++b) {
            hipEvent_t* e = &ctx->ev[(size_t)b * kEv];
            HIP_TRY(ctx, hipEventElapsedTime(&ms, e[kEvLoad], e[kEvLoad + 1]));
            p.load_busy_s += ms * 1e-3;
            HIP_TRY(ctx, hipEventElapsedTime(&ms, e[kEvStore], e[kEvStore + 1]));
            p.store_busy_s += ms * 1e-3;
            HIP_TRY(ctx, hipEventElapsedTime(&ms, e[kEvKernel], e[kEvKernel + 6]));
            p.compute_busy_s += ms * 1e-3;
            for (int i = 0; i < 6; ++i) {
                HIP_TRY(ctx, hipEventElapsedTime(&ms, e[kEvKernel + i], e[kEvKernel + i + 1]));
                p.kernel_s[i] += ms * 1e-3 / (i < 5 ? reps : 1);
            }
        }
        p.bytes_loaded = bytes_loaded;
        p.bytes_stored = bytes_stored;
        ctx->prof = p;
        ctx->prof_valid = true;
    }
    return MOE_OK;
}

}  // extern "C"
