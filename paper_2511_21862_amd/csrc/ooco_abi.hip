// Host side of libooco: context, argument validation, the work-list planner and the C ABI.
#include "../../include/ooco.h"
#include "ooco_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

using namespace ooco;

namespace {

thread_local char g_create_error[512] = "";

constexpr size_t kDefaultWorkspace = 128ull << 20;
constexpr size_t kPlanBytes = 16ull << 20;   // pinned + device staging for the work lists
constexpr int kProfSlots = 1024;             // profiled calls between two ooco_profile_read

}  // namespace

namespace {
// Geometry and knobs the planner needs (no device state).
struct PlanGeometry {
    int Hq, Hkv, hd, BS, max_blocks_per_seq, num_cus;
    size_t ws_bytes;
    int64_t split_blocks, target_items, force_splits;
};

struct HostPlan {
    std::vector<DecodeItem> d;
    std::vector<PrefillTile> p;
    std::vector<MergeItem> m;
    int64_t parts = 0;
    int total_q = 0;
};

// Validates the length arrays and builds the three work lists.  Pure host code.
ooco_status build_plan(const PlanGeometry &geo, int num_seqs, const int32_t *h_seq_lens,
                       const int32_t *h_query_start_loc, const int32_t *h_ctx_lens, HostPlan &out, char *err)
{
    auto bad = [&](ooco_status code, const char *fmt, ...) __attribute__((format(printf, 3, 4))) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, 512, fmt, ap);
        va_end(ap);
        return code;
    };
    out.d.clear();
    out.p.clear();
    out.m.clear();
    out.parts = 0;
    out.total_q = 0;
    if (num_seqs < 0) return bad(OOCO_EINVAL, "ooco_plan: num_seqs=%d", num_seqs);
    if (num_seqs > 0 && (!h_seq_lens || !h_query_start_loc || !h_ctx_lens))
        return bad(OOCO_EINVAL, "ooco_plan: NULL length array");
    const int BS = geo.BS;

    // ---- validation and classification
    if (num_seqs > 0 && h_query_start_loc[0] != 0)
        return bad(OOCO_ESHAPE, "ooco_plan: query_start_loc[0]=%d, expected 0", h_query_start_loc[0]);
    int64_t dec_blocks = 0;
    for (int i = 0; i < num_seqs; ++i) {
        const int64_t ql = (int64_t)h_query_start_loc[i + 1] - h_query_start_loc[i];
        if (ql < 0) return bad(OOCO_ESHAPE, "ooco_plan: query_start_loc decreases at sequence %d", i);
        if (h_ctx_lens[i] < 0 || h_seq_lens[i] < 0)
            return bad(OOCO_ESHAPE, "ooco_plan: negative length at sequence %d", i);
        if ((int64_t)h_ctx_lens[i] + ql != h_seq_lens[i])
            return bad(OOCO_ESHAPE, "ooco_plan: sequence %d has ctx_len %d + q_len %lld != seq_len %d", i,
                       h_ctx_lens[i], (long long)ql, h_seq_lens[i]);
        const int64_t nb = ((int64_t)h_seq_lens[i] + BS - 1) / BS;
        if (nb > geo.max_blocks_per_seq)
            return bad(OOCO_ESHAPE, "ooco_plan: sequence %d needs %lld blocks > max_blocks_per_seq %d", i,
                       (long long)nb, geo.max_blocks_per_seq);
        if (ql == 1) dec_blocks += nb;
    }
    out.total_q = num_seqs > 0 ? h_query_start_loc[num_seqs] : 0;

    // ---- split quantum for decode (KV blocks per work item)
    const size_t part_bytes = (size_t)geo.Hq * (geo.hd + 2) * sizeof(float);
    int64_t quantum = geo.split_blocks;
    if (quantum <= 0) {
        // Aim at `target` wave-sized items per kv head: enough to keep every CU busy with several
        // waves and to even out the tail, not so many that partial results cost bandwidth.
        const int64_t target =
            geo.target_items > 0 ? geo.target_items : std::max<int64_t>(1, (int64_t)geo.num_cus * 16 / geo.Hkv);
        quantum = (dec_blocks + target - 1) / target;
        quantum = std::min<int64_t>(std::max<int64_t>(quantum, 8), 512);
    }
    auto parts_of = [&](int64_t nb) {
        const int64_t n = geo.force_splits > 0 ? std::min<int64_t>(geo.force_splits, nb) : (nb + quantum - 1) / quantum;
        return std::max<int64_t>(n, 1);
    };
    for (;;) {
        int64_t n_parts = 0;
        for (int i = 0; i < num_seqs; ++i) {
            if (h_query_start_loc[i + 1] - h_query_start_loc[i] != 1) continue;
            const int64_t n = parts_of(((int64_t)h_seq_lens[i] + BS - 1) / BS);
            if (n > 1) n_parts += n;
        }
        if ((size_t)n_parts * part_bytes <= geo.ws_bytes) break;
        if (geo.force_splits > 0 || geo.split_blocks > 0 || quantum > (1 << 24))
            return bad(OOCO_ENOMEM, "ooco_plan: workspace of %zu bytes cannot hold %lld partial results", geo.ws_bytes,
                       (long long)n_parts);
        quantum *= 2;
    }

    int64_t part = 0;
    for (int i = 0; i < num_seqs; ++i) {
        const int q0 = h_query_start_loc[i];
        const int ql = h_query_start_loc[i + 1] - q0;
        if (ql == 1) {
            const int64_t nb = ((int64_t)h_seq_lens[i] + BS - 1) / BS;
            const int64_t n = parts_of(nb);
            if (n > 1) out.m.push_back(MergeItem{q0, (int32_t)part, (int32_t)n, 0});
            for (int64_t s = 0; s < n; ++s) {
                DecodeItem d;
                d.seq = i;
                d.q_row = q0;
                d.blk_begin = (int32_t)(nb * s / n);
                d.blk_end = (int32_t)(nb * (s + 1) / n);
                d.seq_len = h_seq_lens[i];
                d.part = n > 1 ? (int32_t)part++ : -1;
                d.pad0 = d.pad1 = 0;
                out.d.push_back(d);
            }
        } else if (ql > 1) {
            for (int t0 = 0; t0 < ql; t0 += kPrefillRows) {
                PrefillTile t;
                t.seq = i;
                t.q_row0 = q0 + t0;
                t.rows = std::min(kPrefillRows, ql - t0);
                t.pos0 = h_ctx_lens[i] + t0;
                t.seq_len = h_seq_lens[i];
                t.pad0 = t.pad1 = t.pad2 = 0;
                out.p.push_back(t);
            }
        }
    }
    // longest work first: the hardware dispatches workgroups in index order
    std::stable_sort(out.d.begin(), out.d.end(), [](const DecodeItem &a, const DecodeItem &b) {
        return (a.blk_end - a.blk_begin) > (b.blk_end - b.blk_begin);
    });
    std::stable_sort(out.p.begin(), out.p.end(),
                     [](const PrefillTile &a, const PrefillTile &b) { return (a.pos0 + a.rows) > (b.pos0 + b.rows); });
    out.parts = part;
    return OOCO_OK;
}

}  // namespace

struct ooco_ctx {
    int Hq = 0, Hkv = 0, g = 0, hd = 0, BS = 0;
    int64_t num_blocks = 0;
    int max_blocks_per_seq = 0;
    float scale = 0.f;
    int device = 0;
    int num_cus = 256;

    void *ws = nullptr;
    size_t ws_bytes = 0;
    bool own_ws = false;

    char *plan_h = nullptr;   // pinned host staging
    char *plan_d = nullptr;   // device copy
    hipEvent_t upload_done = nullptr;
    bool upload_pending = false;

    // current plan
    bool plan_valid = false;
    bool plan_dirty = false;
    bool plan_one_shot = false;   // planned inside ooco_attn_mixed from device lengths
    int plan_num_seqs = -1;
    int plan_total_q = -1;
    int64_t n_ditems = 0, n_ptiles = 0, n_mitems = 0, n_parts = 0;
    size_t off_d = 0, off_p = 0, off_m = 0, plan_used = 0;
    size_t ws_used = 0;

    // options
    int64_t opt_split_blocks = 0;
    int64_t opt_target_items = 0;
    int64_t opt_force_splits = 0;
    int64_t opt_profile = 0;

    // per-kernel timing (option "profile"): 4 events per call in a ring
    std::vector<hipEvent_t> prof_ev;
    int64_t prof_calls = 0;

    HostPlan plan;
    std::vector<int32_t> h_len_scratch;   // for the plan-less path
    mutable char err[512] = "";
};

namespace {

ooco_status fail(const ooco_ctx *ctx, ooco_status code, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_create_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

extern "C" {

ooco_status ooco_ctx_create(ooco_ctx **out, int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                            int64_t num_blocks, int max_blocks_per_seq, float softmax_scale, void *workspace,
                            size_t workspace_bytes)
{
    if (!out) return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: out is NULL");
    *out = nullptr;
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: num_q_heads=%d must be a positive multiple of num_kv_heads=%d",
                    num_q_heads, num_kv_heads);
    if (num_q_heads / num_kv_heads > 16)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: GQA group size %d > 16 is not supported",
                    num_q_heads / num_kv_heads);
    if (head_dim != 64 && head_dim != 128)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: head_dim=%d (supported: 64, 128)", head_dim);
    if (block_size != kBlockSize)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: block_size=%d (supported: %d)", block_size, kBlockSize);
    if (num_blocks <= 0 || max_blocks_per_seq <= 0)
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: num_blocks and max_blocks_per_seq must be positive");
    if (workspace && workspace_bytes == 0)
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: caller workspace given with workspace_bytes == 0");
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: workspace must be 256-byte aligned");

    ooco_ctx *c = new (std::nothrow) ooco_ctx();
    if (!c) return fail(nullptr, OOCO_ENOMEM, "ooco_ctx_create: out of host memory");
    c->Hq = num_q_heads;
    c->Hkv = num_kv_heads;
    c->g = num_q_heads / num_kv_heads;
    c->hd = head_dim;
    c->BS = block_size;
    c->num_blocks = num_blocks;
    c->max_blocks_per_seq = max_blocks_per_seq;
    c->scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)head_dim);

    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
            c->num_cus = cus;
    }
    if (e == hipSuccess) {
        if (workspace) {
            c->ws = workspace;
            c->ws_bytes = workspace_bytes;
        } else {
            c->ws_bytes = workspace_bytes ? workspace_bytes : kDefaultWorkspace;
            e = hipMalloc(&c->ws, c->ws_bytes);
            c->own_ws = (e == hipSuccess);
        }
    }
    if (e == hipSuccess) e = hipHostMalloc((void **)&c->plan_h, kPlanBytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc((void **)&c->plan_d, kPlanBytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->upload_done, hipEventDisableTiming);
    if (e != hipSuccess) {
        fail(nullptr, e == hipErrorOutOfMemory ? OOCO_ENOMEM : OOCO_EHIP, "ooco_ctx_create: %s", hipGetErrorString(e));
        ooco_status st = e == hipErrorOutOfMemory ? OOCO_ENOMEM : OOCO_EHIP;
        (void)hipGetLastError();
        if (c->upload_done) (void)hipEventDestroy(c->upload_done);
        if (c->plan_d) (void)hipFree(c->plan_d);
        if (c->plan_h) (void)hipHostFree(c->plan_h);
        if (c->own_ws && c->ws) (void)hipFree(c->ws);
        delete c;
        return st;
    }
    *out = c;
    return OOCO_OK;
}

ooco_status ooco_ctx_destroy(ooco_ctx *ctx)
{
    if (!ctx) return OOCO_OK;
    if (ctx->upload_pending) (void)hipEventSynchronize(ctx->upload_done);
    (void)hipDeviceSynchronize();
    if (ctx->upload_done) (void)hipEventDestroy(ctx->upload_done);
    for (hipEvent_t x : ctx->prof_ev)
        if (x) (void)hipEventDestroy(x);
    if (ctx->plan_d) (void)hipFree(ctx->plan_d);
    if (ctx->plan_h) (void)hipHostFree(ctx->plan_h);
    if (ctx->own_ws && ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
    return OOCO_OK;
}

ooco_status ooco_profile_read(ooco_ctx *ctx, double *ms_sum, int64_t *calls)
{
    if (!ctx) return OOCO_EINVAL;
    double sum[3] = {0.0, 0.0, 0.0};
    for (int64_t c = 0; c < ctx->prof_calls; ++c) {
        hipEvent_t *ev = ctx->prof_ev.data() + 4 * c;
        hipError_t e = hipEventSynchronize(ev[3]);
        for (int k = 0; k < 3 && e == hipSuccess; ++k) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, ev[k], ev[k + 1]);
            sum[k] += ms;
        }
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_profile_read: %s", hipGetErrorString(e));
    }
    if (ms_sum) ms_sum[0] = sum[0], ms_sum[1] = sum[1], ms_sum[2] = sum[2];
    if (calls) *calls = ctx->prof_calls;
    ctx->prof_calls = 0;
    return OOCO_OK;
}

const char *ooco_last_error(const ooco_ctx *ctx) { return ctx ? ctx->err : g_create_error; }

ooco_status ooco_set_option(ooco_ctx *ctx, const char *name, int64_t value)
{
    if (!ctx) return OOCO_EINVAL;
    if (!name) return fail(ctx, OOCO_EINVAL, "ooco_set_option: name is NULL");
    if (value < 0) return fail(ctx, OOCO_EINVAL, "ooco_set_option: %s must be >= 0", name);
    if (!strcmp(name, "decode_split_blocks"))
        ctx->opt_split_blocks = value;
    else if (!strcmp(name, "decode_target_items"))
        ctx->opt_target_items = value;
    else if (!strcmp(name, "force_splits"))
        ctx->opt_force_splits = value;
    else if (!strcmp(name, "profile")) {
        ctx->opt_profile = value;
        ctx->prof_calls = 0;
        return OOCO_OK;   // does not invalidate the plan
    }
    else
        return fail(ctx, OOCO_EINVAL, "ooco_set_option: unknown option '%s'", name);
    ctx->plan_valid = false;
    return OOCO_OK;
}

ooco_status ooco_plan(ooco_ctx *ctx, int num_seqs, const int32_t *h_seq_lens, const int32_t *h_query_start_loc,
                      const int32_t *h_ctx_lens)
{
    if (!ctx) return OOCO_EINVAL;
    ctx->plan_valid = false;
    PlanGeometry geo;
    geo.Hq = ctx->Hq;
    geo.Hkv = ctx->Hkv;
    geo.hd = ctx->hd;
    geo.BS = ctx->BS;
    geo.max_blocks_per_seq = ctx->max_blocks_per_seq;
    geo.num_cus = ctx->num_cus;
    geo.ws_bytes = ctx->ws_bytes;
    geo.split_blocks = ctx->opt_split_blocks;
    geo.target_items = ctx->opt_target_items;
    geo.force_splits = ctx->opt_force_splits;
    ooco_status st = build_plan(geo, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens, ctx->plan, ctx->err);
    if (st != OOCO_OK) return st;
    const HostPlan &pl = ctx->plan;

    // layout of the lists in the staging buffer
    const size_t off_d = 0;
    const size_t off_p = align_up(off_d + pl.d.size() * sizeof(DecodeItem), 256);
    const size_t off_m = align_up(off_p + pl.p.size() * sizeof(PrefillTile), 256);
    const size_t used = align_up(off_m + pl.m.size() * sizeof(MergeItem), 256);
    if (used > kPlanBytes)
        return fail(ctx, OOCO_ENOMEM, "ooco_plan: work lists need %zu bytes > %zu", used, (size_t)kPlanBytes);

    // the previous upload may still be reading the pinned buffer
    if (ctx->upload_pending) {
        hipError_t e = hipEventSynchronize(ctx->upload_done);
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_plan: %s", hipGetErrorString(e));
        ctx->upload_pending = false;
    }
    if (!pl.d.empty()) memcpy(ctx->plan_h + off_d, pl.d.data(), pl.d.size() * sizeof(DecodeItem));
    if (!pl.p.empty()) memcpy(ctx->plan_h + off_p, pl.p.data(), pl.p.size() * sizeof(PrefillTile));
    if (!pl.m.empty()) memcpy(ctx->plan_h + off_m, pl.m.data(), pl.m.size() * sizeof(MergeItem));

    ctx->n_ditems = (int64_t)pl.d.size();
    ctx->n_ptiles = (int64_t)pl.p.size();
    ctx->n_mitems = (int64_t)pl.m.size();
    ctx->n_parts = pl.parts;
    ctx->off_d = off_d;
    ctx->off_p = off_p;
    ctx->off_m = off_m;
    ctx->plan_used = used;
    ctx->ws_used = (size_t)pl.parts * ((size_t)ctx->Hq * (ctx->hd + 2) * sizeof(float));
    ctx->plan_num_seqs = num_seqs;
    ctx->plan_total_q = pl.total_q;
    ctx->plan_valid = true;
    ctx->plan_dirty = true;
    ctx->plan_one_shot = false;
    return OOCO_OK;
}

ooco_status ooco_plan_dry_run(int num_q_heads, int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                              int num_cus, size_t workspace_bytes, int64_t split_blocks, int64_t target_items,
                              int64_t force_splits, int num_seqs, const int32_t *h_seq_lens,
                              const int32_t *h_query_start_loc, const int32_t *h_ctx_lens, int32_t *decode_items_out,
                              int64_t decode_cap, int32_t *prefill_tiles_out, int64_t prefill_cap, int64_t *counts,
                              char *msg, size_t msg_cap)
{
    char err[512] = "";
    ooco_status st = OOCO_OK;
    HostPlan pl;
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads || (head_dim != 64 && head_dim != 128) ||
        block_size != kBlockSize || max_blocks_per_seq <= 0 || num_cus <= 0) {
        snprintf(err, sizeof err, "ooco_plan_dry_run: bad geometry");
        st = OOCO_ESHAPE;
    } else {
        PlanGeometry geo;
        geo.Hq = num_q_heads;
        geo.Hkv = num_kv_heads;
        geo.hd = head_dim;
        geo.BS = block_size;
        geo.max_blocks_per_seq = max_blocks_per_seq;
        geo.num_cus = num_cus;
        geo.ws_bytes = workspace_bytes;
        geo.split_blocks = split_blocks;
        geo.target_items = target_items;
        geo.force_splits = force_splits;
        st = build_plan(geo, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens, pl, err);
    }
    if (msg && msg_cap) snprintf(msg, msg_cap, "%s", err);
    if (st != OOCO_OK) return st;
    if (counts) {
        counts[0] = (int64_t)pl.d.size();
        counts[1] = (int64_t)pl.p.size();
        counts[2] = (int64_t)pl.m.size();
        counts[3] = pl.parts;
    }
    if (decode_items_out)
        for (int64_t i = 0; i < std::min<int64_t>(decode_cap, (int64_t)pl.d.size()); ++i) {
            const DecodeItem &d = pl.d[(size_t)i];
            int32_t *o = decode_items_out + 6 * i;
            o[0] = d.seq, o[1] = d.q_row, o[2] = d.blk_begin, o[3] = d.blk_end, o[4] = d.seq_len, o[5] = d.part;
        }
    if (prefill_tiles_out)
        for (int64_t i = 0; i < std::min<int64_t>(prefill_cap, (int64_t)pl.p.size()); ++i) {
            const PrefillTile &t = pl.p[(size_t)i];
            int32_t *o = prefill_tiles_out + 5 * i;
            o[0] = t.seq, o[1] = t.q_row0, o[2] = t.rows, o[3] = t.pos0, o[4] = t.seq_len;
        }
    return OOCO_OK;
}

ooco_status ooco_plan_info(const ooco_ctx *ctx, int64_t *decode_items, int64_t *prefill_tiles, int64_t *merged_seqs,
                           int64_t *workspace_used)
{
    if (!ctx) return OOCO_EINVAL;
    if (!ctx->plan_valid) return fail(ctx, OOCO_EINVAL, "ooco_plan_info: no current plan");
    if (decode_items) *decode_items = ctx->n_ditems;
    if (prefill_tiles) *prefill_tiles = ctx->n_ptiles;
    if (merged_seqs) *merged_seqs = ctx->n_mitems;
    if (workspace_used) *workspace_used = (int64_t)ctx->ws_used;
    return OOCO_OK;
}

ooco_status ooco_attn_mixed(ooco_ctx *ctx, const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *block_tables, const int32_t *seq_lens, const int32_t *query_start_loc,
                            const int32_t *ctx_lens, void *out, int num_seqs, int total_q_tokens, void *stream)
{
    if (!ctx) return OOCO_EINVAL;
    if (num_seqs < 0 || total_q_tokens < 0)
        return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: negative size (num_seqs=%d, total_q_tokens=%d)", num_seqs,
                    total_q_tokens);
    if (num_seqs == 0 || total_q_tokens == 0) return OOCO_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !seq_lens || !query_start_loc || !ctx_lens || !out)
        return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: NULL pointer argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    if (!ctx->plan_valid) {
        // No host plan for this batch: fetch the lengths and plan here (costs one stream sync).
        ctx->h_len_scratch.resize((size_t)3 * num_seqs + 1);
        int32_t *h_seq = ctx->h_len_scratch.data();
        int32_t *h_ctx = h_seq + num_seqs;
        int32_t *h_qsl = h_ctx + num_seqs;
        hipError_t e = hipMemcpyAsync(h_seq, seq_lens, sizeof(int32_t) * num_seqs, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipMemcpyAsync(h_ctx, ctx_lens, sizeof(int32_t) * num_seqs, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(h_qsl, query_start_loc, sizeof(int32_t) * (num_seqs + 1), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: reading lengths: %s", hipGetErrorString(e));
        ooco_status st = ooco_plan(ctx, num_seqs, h_seq, h_qsl, h_ctx);
        if (st != OOCO_OK) return st;
        ctx->plan_one_shot = true;
    }
    if (ctx->plan_num_seqs != num_seqs || ctx->plan_total_q != total_q_tokens)
        return fail(ctx, OOCO_ESHAPE, "ooco_attn_mixed: plan was made for %d sequences / %d query tokens, call has %d / %d",
                    ctx->plan_num_seqs, ctx->plan_total_q, num_seqs, total_q_tokens);

    if (ctx->plan_dirty && ctx->plan_used > 0) {
        hipError_t e = hipMemcpyAsync(ctx->plan_d, ctx->plan_h, ctx->plan_used, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipEventRecord(ctx->upload_done, s);
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: plan upload: %s", hipGetErrorString(e));
        ctx->upload_pending = true;
        ctx->plan_dirty = false;
    }

    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.block_tables = block_tables;
    p.out = static_cast<uint16_t *>(out);
    p.part_acc = static_cast<float *>(ctx->ws);
    p.part_ml = p.part_acc + (size_t)ctx->n_parts * ctx->Hq * ctx->hd;
    p.ditems = reinterpret_cast<const DecodeItem *>(ctx->plan_d + ctx->off_d);
    p.ptiles = reinterpret_cast<const PrefillTile *>(ctx->plan_d + ctx->off_p);
    p.mitems = reinterpret_cast<const MergeItem *>(ctx->plan_d + ctx->off_m);
    p.Hq = ctx->Hq;
    p.Hkv = ctx->Hkv;
    p.g = ctx->g;
    p.hd = ctx->hd;
    p.max_blocks_per_seq = ctx->max_blocks_per_seq;
    p.scale_log2e = ctx->scale * 1.4426950408889634f;
    p.n_ditems = (int32_t)ctx->n_ditems;
    p.n_ptiles = (int32_t)ctx->n_ptiles;
    p.n_mitems = (int32_t)ctx->n_mitems;

    hipEvent_t *ev = nullptr;
    hipError_t e = hipSuccess;
    if (ctx->opt_profile) {
        if (ctx->prof_calls >= kProfSlots)
            return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: more than %d profiled calls without ooco_profile_read",
                        kProfSlots);
        if (ctx->prof_ev.empty()) {
            ctx->prof_ev.assign((size_t)4 * kProfSlots, nullptr);
            for (auto &x : ctx->prof_ev)
                if (e == hipSuccess) e = hipEventCreate(&x);
            if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: %s", hipGetErrorString(e));
        }
        ev = ctx->prof_ev.data() + 4 * ctx->prof_calls++;
    }
    if (ev) e = hipEventRecord(ev[0], s);
    if (e == hipSuccess) e = launch_prefill(p, s);
    if (ev && e == hipSuccess) e = hipEventRecord(ev[1], s);
    if (e == hipSuccess) e = launch_decode(p, s);
    if (ev && e == hipSuccess) e = hipEventRecord(ev[2], s);
    if (e == hipSuccess) e = launch_merge(p, s);
    if (ev && e == hipSuccess) e = hipEventRecord(ev[3], s);
    if (ctx->plan_one_shot) {
        ctx->plan_one_shot = false;
        ctx->plan_valid = false;
    }
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

ooco_status ooco_kv_block_copy(ooco_ctx *ctx, const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                               const int64_t *src_block_ids, const int64_t *dst_block_ids, int64_t num_pairs,
                               void *stream)
{
    if (!ctx) return OOCO_EINVAL;
    if (num_pairs < 0) return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: num_pairs=%lld", (long long)num_pairs);
    if (num_pairs == 0) return OOCO_OK;
    if (!k_src || !v_src || !k_dst || !v_dst || !src_block_ids || !dst_block_ids)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: NULL pointer argument");
    if (num_pairs > (int64_t)1 << 26)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: num_pairs=%lld too large", (long long)num_pairs);
    const int64_t block_bytes = (int64_t)ctx->Hkv * ctx->BS * ctx->hd * 2;
    hipError_t e = launch_block_copy(k_src, v_src, k_dst, v_dst, src_block_ids, dst_block_ids, num_pairs, block_bytes,
                                     reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_kv_block_copy: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

}  // extern "C"
