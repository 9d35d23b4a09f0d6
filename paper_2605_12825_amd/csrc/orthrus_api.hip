// Host side of the C ABI declared in orthrus.h: argument validation, launch planning and
// workspace carving.  Nothing here computes; every step of the path runs in the kernels.
#include "../../include/orthrus.h"
#include "orthrus_internal.h"

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

struct orthrus_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

struct orthrus_ctx {
    int device;
    int num_cus;
    int32_t *err_word;  // device
    // optional per-kernel timing of the attention launches (orthrus_attn_timing*)
    bool timing = false;
    std::vector<hipEvent_t> free_events;
    struct Pending { hipEvent_t start, stop; int kind; };
    std::vector<Pending> pending;
    double sum_us[2] = {0.0, 0.0};
    int64_t launches[2] = {0, 0};
    // takes a pair of events from the free list (or creates them); false on a HIP error, nothing taken
    bool take_events(hipEvent_t *start, hipEvent_t *stop)
    {
        hipEvent_t got[2] = {nullptr, nullptr};
        for (int k = 0; k < 2; ++k) {
            if (!free_events.empty()) {
                got[k] = free_events.back();
                free_events.pop_back();
            } else if (hipEventCreate(&got[k]) != hipSuccess) {
                if (k == 1) free_events.push_back(got[0]);
                return false;
            }
        }
        *start = got[0];
        *stop = got[1];
        return true;
    }
};

namespace {
constexpr size_t kCtxWords = 64;
}

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int log2_exact(int x)
{
    if (x <= 0 || (x & (x - 1))) return -1;
    int s = 0;
    while ((1 << s) < x) ++s;
    return s;
}

// Checks shared by every entry point.  `need_attn` / `need_consensus` select the field groups.
orthrus_status check_params(const orthrus_params *p, bool need_attn, bool need_consensus, bool need_pool)
{
    if (!p) return ORTHRUS_EINVAL;
    if (p->batch < 0 || p->block_k <= 0) return ORTHRUS_EINVAL;
    if (p->batch > 65535) return ORTHRUS_EUNSUPPORTED;
    if (need_attn || need_pool) {
        if (p->num_kv_heads <= 0 || p->head_dim <= 0 || p->page_size <= 0 || p->max_pages_per_seq <= 0 ||
            p->num_pages <= 0)
            return ORTHRUS_EINVAL;
        if (p->pool_stride_page <= 0 || p->pool_stride_head <= 0 || p->pool_stride_tok <= 0) return ORTHRUS_EINVAL;
        if (p->head_dim != 64 && p->head_dim != 128) return ORTHRUS_EUNSUPPORTED;
        if (log2_exact(p->page_size) < 4) return ORTHRUS_EUNSUPPORTED;
        if (p->num_kv_heads > 65535) return ORTHRUS_EUNSUPPORTED;
        if ((p->pool_stride_page | p->pool_stride_head | p->pool_stride_tok | p->pool_stride_layer) & 7)
            return ORTHRUS_EUNSUPPORTED;
        if (p->pool_stride_tok < p->head_dim) return ORTHRUS_EINVAL;
        // block-input strides: 0 = dense, else 16-byte multiples that keep rows and heads apart
        if ((p->q_stride_row | p->q_stride_head | p->blk_stride_row | p->blk_stride_head | p->blk_stride_layer) & 7)
            return ORTHRUS_EUNSUPPORTED;
        if (p->q_stride_row < 0 || p->q_stride_head < 0 || p->blk_stride_row < 0 || p->blk_stride_head < 0 ||
            p->blk_stride_layer < 0)
            return ORTHRUS_EINVAL;
        if ((p->q_stride_head && p->q_stride_head < p->head_dim) || (p->blk_stride_head && p->blk_stride_head < p->head_dim))
            return ORTHRUS_EINVAL;
    }
    if (p->block_k > 32) return ORTHRUS_EUNSUPPORTED;
    if (need_attn) {
        if (p->num_q_heads <= 0 || p->num_q_heads % p->num_kv_heads != 0) return ORTHRUS_EINVAL;
        if (p->max_seq_len < 0 || p->num_splits < ORTHRUS_SPLITS_BALANCED) return ORTHRUS_EINVAL;
        if ((int64_t)p->max_seq_len > (int64_t)p->max_pages_per_seq * p->page_size) return ORTHRUS_EINVAL;
        if (!(p->sm_scale > 0.f) || !std::isfinite(p->sm_scale)) return ORTHRUS_EINVAL;
        if ((int64_t)(p->num_q_heads / p->num_kv_heads) * p->block_k > 256) return ORTHRUS_EUNSUPPORTED;
    }
    if (need_consensus) {
        if (p->vocab <= 0) return ORTHRUS_EINVAL;
    }
    return ORTHRUS_OK;
}

orthrus_status make_plan(const orthrus_params *p, int num_cus, orthrus::AttnPlan *plan)
{
    orthrus::plan_attn(p->head_dim, p->num_q_heads / p->num_kv_heads, p->block_k, p->batch, p->num_kv_heads,
                       p->max_seq_len, p->num_splits, num_cus, p->num_layers, plan);
    if (plan->num_splits > 65535 * 16) return ORTHRUS_EUNSUPPORTED;
    // the balanced partition counts one head's tiles in a 32-bit int
    if (plan->bal_wgs > 0 && (int64_t)p->batch * (p->max_seq_len / 32 + 2) > 0x7fffffff) return ORTHRUS_EUNSUPPORTED;
    return ORTHRUS_OK;
}

int consensus_chunks(const orthrus_params *p)
{
    const int ce = orthrus::consensus_chunk_elems();
    return (p->vocab + ce - 1) / ce;
}

constexpr int kDefaultCUs = 256;  // MI355X; used when sizing without a context

// CU count the launch plan of a context's device is made for
int plan_cus(const orthrus_ctx *ctx) { return ctx && ctx->num_cus > 0 ? ctx->num_cus : kDefaultCUs; }

int64_t attn_workspace_for(const orthrus_params *p, int num_cus)
{
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return (int64_t)s;
    orthrus::AttnPlan plan;
    s = make_plan(p, num_cus, &plan);
    if (s != ORTHRUS_OK) return (int64_t)s;
    return (int64_t)(align_up(plan.part_o_bytes, 256) + align_up(plan.part_ml_bytes, 256));
}

int32_t attn_splits_for(const orthrus_params *p, int num_cus)
{
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return (int32_t)s;
    orthrus::AttnPlan plan;
    s = make_plan(p, num_cus, &plan);
    if (s != ORTHRUS_OK) return (int32_t)s;
    return plan.bal_wgs > 0 ? 0 : plan.num_splits;
}

}  // namespace

// Kernel arguments of a decode-mode attention launch for `plan`.
orthrus::AttnArgs decode_attn_args(const orthrus_ctx *ctx, const orthrus_params *p, const orthrus::AttnPlan &plan,
                                   int view, const void *q, const void *k_blk, const void *v_blk,
                                   const void *k_pool, const void *v_pool, const int32_t *page_table,
                                   const int32_t *seq_lens, void *out, float *lse, void *workspace)
{
    orthrus::AttnArgs a;
    a.q = (const uint16_t *)q; a.k_blk = (const uint16_t *)k_blk; a.v_blk = (const uint16_t *)v_blk;
    a.k_pool = (const uint16_t *)k_pool; a.v_pool = (const uint16_t *)v_pool;
    a.page_table = page_table; a.seq_lens = seq_lens;
    a.out = (uint16_t *)out; a.lse = lse;
    a.part_o = (float *)workspace;
    a.part_ml = workspace ? (float *)((char *)workspace + align_up(plan.part_o_bytes, 256)) : nullptr;
    a.err_word = ctx->err_word;
    a.old_lens = nullptr; a.new_lens = nullptr; a.max_new = 0;
    a.stride_page = p->pool_stride_page; a.stride_head = p->pool_stride_head; a.stride_tok = p->pool_stride_tok;
    a.num_pages = p->num_pages;
    a.q_stride_head = p->q_stride_head ? p->q_stride_head : p->head_dim;
    a.q_stride_row = p->q_stride_row ? p->q_stride_row : (int64_t)p->num_q_heads * p->head_dim;
    a.blk_stride_head = p->blk_stride_head ? p->blk_stride_head : p->head_dim;
    a.blk_stride_row = p->blk_stride_row ? p->blk_stride_row : (int64_t)p->num_kv_heads * p->head_dim;
    a.batch = p->batch; a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads;
    a.group = p->num_q_heads / p->num_kv_heads; a.block_k = p->block_k; a.rows = plan.rows;
    a.page_shift = log2_exact(p->page_size); a.max_pages_per_seq = p->max_pages_per_seq;
    a.max_seq_len = p->max_seq_len; a.chunk_tokens = plan.chunk_tokens; a.num_splits = plan.num_splits;
    a.bal_wgs = plan.bal_wgs;
    a.kv_nt = plan.kv_nt;
    a.view = view;
    a.scale_log2e = p->sm_scale * 1.4426950408889634f;
    return a;
}

static orthrus_status consensus_commit_impl(orthrus_ctx *ctx, const orthrus_params *p,
                                        const float *ar_logits, const int32_t *draft_tokens,
                                        const void *k_blk_ar, const void *v_blk_ar,
                                        void *k_pool, void *v_pool,
                                        const int32_t *page_table, int32_t *seq_lens,
                                        int32_t *accept_len, int32_t *num_committed,
                                        int32_t *out_tokens, int32_t *next_anchor,
                                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    if ((k_blk_ar == nullptr) != (v_blk_ar == nullptr)) return ORTHRUS_EINVAL;
    const bool do_commit = k_blk_ar != nullptr;
    orthrus_status s = check_params(p, false, true, do_commit);
    if (s != ORTHRUS_OK) return s;
    if (!ar_logits || !draft_tokens || !accept_len || !num_committed || !out_tokens || !next_anchor)
        return ORTHRUS_EINVAL;
    if (((uintptr_t)ar_logits) & 3) return ORTHRUS_EINVAL;
    if (do_commit) {
        if (!k_pool || !v_pool || !page_table || !seq_lens || p->num_layers <= 0) return ORTHRUS_EINVAL;
        if (p->num_layers > 65535) return ORTHRUS_EUNSUPPORTED;
        const uintptr_t al = (uintptr_t)k_blk_ar | (uintptr_t)v_blk_ar | (uintptr_t)k_pool | (uintptr_t)v_pool;
        if (al & 15) return ORTHRUS_EINVAL;
    }
    if (p->batch == 0) return ORTHRUS_OK;
    const size_t rows = (size_t)p->batch * p->block_k;
    const size_t chunks = (size_t)consensus_chunks(p);
    if (rows * chunks > 0x7fffffffull) return ORTHRUS_EUNSUPPORTED;
    const size_t o1 = align_up(rows * chunks * sizeof(float), 256);
    const size_t o2 = o1 + align_up(rows * chunks * sizeof(int32_t), 256);
    const size_t need = o2 + align_up((size_t)p->batch * 2 * sizeof(int32_t), 256);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return ORTHRUS_EWORKSPACE;

    orthrus::ConsensusArgs a;
    a.ar_logits = ar_logits; a.draft_tokens = draft_tokens;
    a.k_blk_ar = (const uint16_t *)k_blk_ar; a.v_blk_ar = (const uint16_t *)v_blk_ar;
    a.k_pool = (uint16_t *)k_pool; a.v_pool = (uint16_t *)v_pool;
    a.page_table = page_table; a.seq_lens = seq_lens;
    a.accept_len = accept_len; a.num_committed = num_committed; a.out_tokens = out_tokens; a.next_anchor = next_anchor;
    a.part_val = (float *)workspace;
    a.part_idx = (int32_t *)((char *)workspace + o1);
    a.commit_info = (int32_t *)((char *)workspace + o2);
    a.err_word = ctx->err_word;
    a.stride_layer = p->pool_stride_layer; a.stride_page = p->pool_stride_page;
    a.stride_head = p->pool_stride_head; a.stride_tok = p->pool_stride_tok; a.num_pages = p->num_pages;
    a.blk_stride_head = p->blk_stride_head ? p->blk_stride_head : p->head_dim;
    a.blk_stride_row = p->blk_stride_row ? p->blk_stride_row : (int64_t)p->num_kv_heads * p->head_dim;
    a.blk_stride_layer = p->blk_stride_layer ? p->blk_stride_layer : (int64_t)p->batch * p->block_k * a.blk_stride_row;
    a.batch = p->batch; a.block_k = p->block_k; a.vocab = p->vocab; a.num_layers = p->num_layers;
    a.num_kv_heads = p->num_kv_heads; a.head_dim = p->head_dim;
    a.page_shift = do_commit ? log2_exact(p->page_size) : 0; a.max_pages_per_seq = p->max_pages_per_seq;
    a.chunks = (int)chunks; a.chunk_elems = orthrus::consensus_chunk_elems(); a.do_commit = do_commit ? 1 : 0;
    hipError_t e = orthrus::launch_consensus(a, (hipStream_t)stream);
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}


extern "C" {

const char *orthrus_status_string(orthrus_status s)
{
    switch (s) {
    case ORTHRUS_OK: return "ok";
    case ORTHRUS_EINVAL: return "invalid argument";
    case ORTHRUS_EUNSUPPORTED: return "shape not supported by the gfx950 kernels";
    case ORTHRUS_EWORKSPACE: return "workspace missing, misaligned or too small";
    case ORTHRUS_ECAPACITY: return "a needed cache page is not mapped";
    case ORTHRUS_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

orthrus_status orthrus_create(orthrus_ctx **out, int device)
{
    if (!out) return ORTHRUS_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return ORTHRUS_EHIP;
    if (hipSetDevice(device) != hipSuccess) return ORTHRUS_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return ORTHRUS_EHIP;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return ORTHRUS_EUNSUPPORTED;
    orthrus_ctx *c = new (std::nothrow) orthrus_ctx;
    if (!c) return ORTHRUS_EINVAL;
    c->device = device;
    c->num_cus = prop.multiProcessorCount;
    c->err_word = nullptr;
    if (hipMalloc((void **)&c->err_word, kCtxWords * sizeof(int32_t)) != hipSuccess) { delete c; return ORTHRUS_EHIP; }
    if (hipMemset(c->err_word, 0, kCtxWords * sizeof(int32_t)) != hipSuccess) { hipFree(c->err_word); delete c; return ORTHRUS_EHIP; }
    // address of this device's copy of the static scratch array (allocation-free entry point)
    if (orthrus::consensus_scratch_init(device) != hipSuccess) { hipFree(c->err_word); delete c; return ORTHRUS_EHIP; }
    *out = c;
    return ORTHRUS_OK;
}

orthrus_status orthrus_destroy(orthrus_ctx *ctx)
{
    if (!ctx) return ORTHRUS_EINVAL;
    hipError_t e = hipFree(ctx->err_word);
    for (auto &pd : ctx->pending) { hipEventDestroy(pd.start); hipEventDestroy(pd.stop); }
    for (auto ev : ctx->free_events) hipEventDestroy(ev);
    delete ctx;
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

int32_t orthrus_attn_num_splits(const orthrus_params *p) { return attn_splits_for(p, kDefaultCUs); }
int64_t orthrus_attn_workspace_bytes(const orthrus_params *p) { return attn_workspace_for(p, kDefaultCUs); }
int32_t orthrus_attn_num_splits_on(const orthrus_ctx *ctx, const orthrus_params *p)
{
    return ctx ? attn_splits_for(p, plan_cus(ctx)) : (int32_t)ORTHRUS_EINVAL;
}
int64_t orthrus_attn_workspace_bytes_on(const orthrus_ctx *ctx, const orthrus_params *p)
{
    return ctx ? attn_workspace_for(p, plan_cus(ctx)) : (int64_t)ORTHRUS_EINVAL;
}

int64_t orthrus_consensus_workspace_bytes(const orthrus_params *p)
{
    orthrus_status s = check_params(p, false, true, false);
    if (s != ORTHRUS_OK) return (int64_t)s;
    const size_t rows = (size_t)p->batch * p->block_k;
    const size_t chunks = (size_t)consensus_chunks(p);
    return (int64_t)(align_up(rows * chunks * sizeof(float), 256) + align_up(rows * chunks * sizeof(int32_t), 256) +
                     align_up((size_t)p->batch * 2 * sizeof(int32_t), 256));
}

orthrus_status orthrus_dual_view_attn(orthrus_ctx *ctx, const orthrus_params *p, orthrus_view view,
                                      const void *q, const void *k_blk, const void *v_blk,
                                      const void *k_pool, const void *v_pool,
                                      const int32_t *page_table, const int32_t *seq_lens,
                                      void *out, float *lse,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return s;
    if (view != ORTHRUS_VIEW_DIFFUSION && view != ORTHRUS_VIEW_AR_VERIFY) return ORTHRUS_EINVAL;
    if (!q || !k_blk || !v_blk || !k_pool || !v_pool || !page_table || !seq_lens || !out) return ORTHRUS_EINVAL;
    const uintptr_t al = (uintptr_t)q | (uintptr_t)k_blk | (uintptr_t)v_blk | (uintptr_t)k_pool | (uintptr_t)v_pool |
                         (uintptr_t)out;
    if (al & 15) return ORTHRUS_EINVAL;
    if (p->batch == 0) return ORTHRUS_OK;
    orthrus::AttnPlan plan;
    // planned for the device the context was created on (orthrus_attn_workspace_bytes_on gives the size
    // for exactly this plan; the context-free query assumes the full 256-CU part)
    s = make_plan(p, plan_cus(ctx), &plan);
    if (s != ORTHRUS_OK) return s;
    const size_t need = align_up(plan.part_o_bytes, 256) + align_up(plan.part_ml_bytes, 256);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return ORTHRUS_EWORKSPACE;

    orthrus::AttnArgs a = decode_attn_args(ctx, p, plan, view, q, k_blk, v_blk, k_pool, v_pool, page_table, seq_lens, out,
                                           lse, workspace);
    orthrus::AttnLaunchEvents ev;
    if (ctx->timing) {
        ev.on = true;
        if (!ctx->take_events(&ev.start[0], &ev.stop[0])) return ORTHRUS_EHIP;
        if (!ctx->take_events(&ev.start[1], &ev.stop[1])) {  // hand back what was taken; nothing has been launched
            ctx->free_events.push_back(ev.start[0]);
            ctx->free_events.push_back(ev.stop[0]);
            return ORTHRUS_EHIP;
        }
    }
    hipError_t e = orthrus::launch_attn(a, plan, p->head_dim, (hipStream_t)stream, &ev);
    if (ev.on) {
        for (int k = 0; k < 2; ++k) {
            if (ev.used[k] && e == hipSuccess) {
                ctx->pending.push_back({ev.start[k], ev.stop[k], k});
            } else {
                ctx->free_events.push_back(ev.start[k]);
                ctx->free_events.push_back(ev.stop[k]);
            }
        }
    }
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

int64_t orthrus_prefill_workspace_bytes(const orthrus_params *p, int32_t max_new_tokens)
{
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return (int64_t)s;
    if (max_new_tokens < 0) return (int64_t)ORTHRUS_EINVAL;
    return (int64_t)(2 * align_up((size_t)p->batch * sizeof(int32_t), 256));
}

orthrus_status orthrus_prefill_attn(orthrus_ctx *ctx, const orthrus_params *p, int32_t max_new_tokens,
                                    const void *q, const void *k_new, const void *v_new, const int32_t *new_lens,
                                    void *k_pool, void *v_pool,
                                    const int32_t *page_table, int32_t *seq_lens, void *out,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return s;
    if (max_new_tokens < 0) return ORTHRUS_EINVAL;
    const int group = p->num_q_heads / p->num_kv_heads;
    if (group > 8) return ORTHRUS_EUNSUPPORTED;  // 32 * group rows per work item, at most 256
    if (!q || !k_new || !v_new || !new_lens || !k_pool || !v_pool || !page_table || !seq_lens || !out)
        return ORTHRUS_EINVAL;
    const uintptr_t al = (uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_pool | (uintptr_t)v_pool |
                         (uintptr_t)out;
    if (al & 15) return ORTHRUS_EINVAL;
    if (p->batch == 0 || max_new_tokens == 0) return ORTHRUS_OK;
    const int64_t chunks = ((int64_t)max_new_tokens + 31) / 32;
    if (chunks * p->num_kv_heads * p->batch > 0x3fffffff) return ORTHRUS_EUNSUPPORTED;
    const size_t o1 = align_up((size_t)p->batch * sizeof(int32_t), 256);
    if (!workspace || workspace_bytes < 2 * o1 || ((uintptr_t)workspace & 255)) return ORTHRUS_EWORKSPACE;

    orthrus::PrefillArgs f;
    f.k_new = (const uint16_t *)k_new; f.v_new = (const uint16_t *)v_new; f.new_lens_in = new_lens;
    f.k_pool = (uint16_t *)k_pool; f.v_pool = (uint16_t *)v_pool;
    f.page_table = page_table; f.seq_lens = seq_lens;
    f.old_lens = (int32_t *)workspace; f.new_lens = (int32_t *)((char *)workspace + o1);
    f.err_word = ctx->err_word;
    f.stride_page = p->pool_stride_page; f.stride_head = p->pool_stride_head; f.stride_tok = p->pool_stride_tok;
    f.num_pages = p->num_pages;
    f.batch = p->batch; f.max_new = max_new_tokens; f.num_kv_heads = p->num_kv_heads; f.head_dim = p->head_dim;
    f.page_shift = log2_exact(p->page_size); f.max_pages_per_seq = p->max_pages_per_seq;
    f.max_seq_len = p->max_seq_len;
    hipError_t e = orthrus::launch_prefill_append(f, (hipStream_t)stream);
    if (e != hipSuccess) return ORTHRUS_EHIP;

    orthrus::AttnArgs a;
    a.q = (const uint16_t *)q; a.k_blk = nullptr; a.v_blk = nullptr;
    a.k_pool = (const uint16_t *)k_pool; a.v_pool = (const uint16_t *)v_pool;
    a.page_table = page_table; a.seq_lens = seq_lens;
    a.out = (uint16_t *)out; a.lse = nullptr; a.part_o = nullptr; a.part_ml = nullptr;
    a.err_word = ctx->err_word;
    a.old_lens = f.old_lens; a.new_lens = f.new_lens; a.max_new = max_new_tokens;
    a.stride_page = p->pool_stride_page; a.stride_head = p->pool_stride_head; a.stride_tok = p->pool_stride_tok;
    a.num_pages = p->num_pages;
    a.q_stride_head = p->head_dim; a.q_stride_row = (int64_t)p->num_q_heads * p->head_dim;
    a.blk_stride_head = p->head_dim; a.blk_stride_row = (int64_t)p->num_kv_heads * p->head_dim;
    a.batch = p->batch; a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads;
    a.group = group; a.block_k = 32; a.rows = 32 * group;
    a.page_shift = f.page_shift; a.max_pages_per_seq = p->max_pages_per_seq;
    a.max_seq_len = p->max_seq_len; a.chunk_tokens = 0; a.num_splits = (int)chunks;
    a.bal_wgs = 0;
    a.kv_nt = 0;  // every chunk of a sequence re-reads the same cache rows: keep them cached
    a.view = (int)ORTHRUS_VIEW_AR_VERIFY;
    a.scale_log2e = p->sm_scale * 1.4426950408889634f;
    e = orthrus::launch_prefill_attn(a, p->head_dim, (hipStream_t)stream);
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

orthrus_status orthrus_graph_begin(orthrus_ctx *ctx, void *stream)
{
    if (!ctx || !stream) return ORTHRUS_EINVAL;  // the NULL stream cannot be captured
    if (ctx->timing) return ORTHRUS_EINVAL;      // timed launches create events: not under capture
    return hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal) == hipSuccess ? ORTHRUS_OK
                                                                                                     : ORTHRUS_EHIP;
}

orthrus_status orthrus_graph_end(orthrus_ctx *ctx, void *stream, orthrus_graph **out)
{
    if (!ctx || !stream || !out) return ORTHRUS_EINVAL;
    *out = nullptr;
    hipGraph_t graph = nullptr;
    if (hipStreamEndCapture((hipStream_t)stream, &graph) != hipSuccess || !graph) return ORTHRUS_EHIP;
    hipGraphExec_t exec = nullptr;
    if (hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) {
        hipGraphDestroy(graph);
        return ORTHRUS_EHIP;
    }
    orthrus_graph *g = new (std::nothrow) orthrus_graph;
    if (!g) {
        hipGraphExecDestroy(exec);
        hipGraphDestroy(graph);
        return ORTHRUS_EINVAL;
    }
    g->graph = graph;
    g->exec = exec;
    *out = g;
    return ORTHRUS_OK;
}

orthrus_status orthrus_graph_launch(orthrus_graph *graph, void *stream)
{
    if (!graph || !graph->exec) return ORTHRUS_EINVAL;
    return hipGraphLaunch(graph->exec, (hipStream_t)stream) == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

orthrus_status orthrus_graph_destroy(orthrus_graph *graph)
{
    if (!graph) return ORTHRUS_EINVAL;
    hipError_t e1 = graph->exec ? hipGraphExecDestroy(graph->exec) : hipSuccess;
    hipError_t e2 = graph->graph ? hipGraphDestroy(graph->graph) : hipSuccess;
    delete graph;
    return (e1 == hipSuccess && e2 == hipSuccess) ? ORTHRUS_OK : ORTHRUS_EHIP;
}

orthrus_status orthrus_attn_timing(orthrus_ctx *ctx, int enable)
{
    if (!ctx) return ORTHRUS_EINVAL;
    ctx->timing = enable != 0;
    return ORTHRUS_OK;
}

orthrus_status orthrus_attn_timing_read(orthrus_ctx *ctx, double *split_us, int64_t *split_launches,
                                        double *combine_us, int64_t *combine_launches)
{
    if (!ctx || !split_us || !split_launches || !combine_us || !combine_launches) return ORTHRUS_EINVAL;
    orthrus_status st = ORTHRUS_OK;
    for (auto &pd : ctx->pending) {
        float ms = 0.f;
        if (hipEventSynchronize(pd.stop) != hipSuccess || hipEventElapsedTime(&ms, pd.start, pd.stop) != hipSuccess) {
            st = ORTHRUS_EHIP;
        } else {
            ctx->sum_us[pd.kind] += (double)ms * 1000.0;
            ctx->launches[pd.kind] += 1;
        }
        ctx->free_events.push_back(pd.start);
        ctx->free_events.push_back(pd.stop);
    }
    ctx->pending.clear();
    *split_us = ctx->sum_us[0]; *split_launches = ctx->launches[0];
    *combine_us = ctx->sum_us[1]; *combine_launches = ctx->launches[1];
    ctx->sum_us[0] = ctx->sum_us[1] = 0.0;
    ctx->launches[0] = ctx->launches[1] = 0;
    return st;
}

orthrus_status orthrus_attn_timing_samples(orthrus_ctx *ctx, double *split_us, double *combine_us, int64_t capacity,
                                          int64_t *count)
{
    if (!ctx || !split_us || !combine_us || !count || capacity < 0) return ORTHRUS_EINVAL;
    orthrus_status st = ORTHRUS_OK;
    int64_t n = 0;
    // pending holds the timed kernels in launch order: a split-kernel record opens a call's sample, the
    // combine record that follows it (if the call had one) completes it
    for (auto &pd : ctx->pending) {
        float ms = 0.f;
        if (hipEventSynchronize(pd.stop) != hipSuccess || hipEventElapsedTime(&ms, pd.start, pd.stop) != hipSuccess)
            st = ORTHRUS_EHIP;
        if (pd.kind == 0) {
            if (n < capacity) { split_us[n] = (double)ms * 1000.0; combine_us[n] = 0.0; }
            ++n;
        } else if (n > 0 && n <= capacity) {
            combine_us[n - 1] = (double)ms * 1000.0;
        }
        ctx->free_events.push_back(pd.start);
        ctx->free_events.push_back(pd.stop);
    }
    ctx->pending.clear();
    ctx->sum_us[0] = ctx->sum_us[1] = 0.0;
    ctx->launches[0] = ctx->launches[1] = 0;
    *count = n;
    return st;
}

orthrus_status orthrus_kv_stream_probe(orthrus_ctx *ctx, const orthrus_params *p, const void *k_pool,
                                       const void *v_pool, const int32_t *page_table, const int32_t *seq_lens,
                                       void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    orthrus_status s = check_params(p, true, false, true);
    if (s != ORTHRUS_OK) return s;
    if (!k_pool || !v_pool || !page_table || !seq_lens) return ORTHRUS_EINVAL;
    if (((uintptr_t)k_pool | (uintptr_t)v_pool) & 15) return ORTHRUS_EINVAL;
    if (p->batch == 0) return ORTHRUS_OK;
    orthrus::AttnPlan plan;
    s = make_plan(p, plan_cus(ctx), &plan);  // the partition the attention call would use
    if (s != ORTHRUS_OK) return s;
    const orthrus::AttnArgs a = decode_attn_args(ctx, p, plan, (int)ORTHRUS_VIEW_DIFFUSION, nullptr, nullptr, nullptr,
                                                 k_pool, v_pool, page_table, seq_lens, nullptr, nullptr, nullptr);
    hipEvent_t start = nullptr, stop = nullptr;
    if (ctx->timing && !ctx->take_events(&start, &stop)) return ORTHRUS_EHIP;
    hipError_t e = orthrus::launch_kv_stream_probe(a, plan, p->head_dim, (hipStream_t)stream, start, stop);
    if (start) {
        if (e == hipSuccess) ctx->pending.push_back({start, stop, 0});
        else { ctx->free_events.push_back(start); ctx->free_events.push_back(stop); }
    }
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

#ifndef ORTHRUS_BUILD_ID
#define ORTHRUS_BUILD_ID "unknown"
#endif
const char *orthrus_build_id(void) { return ORTHRUS_BUILD_ID; }

orthrus_status orthrus_consensus_commit(orthrus_ctx *ctx, const orthrus_params *p,
                                        const float *ar_logits, const int32_t *draft_tokens,
                                        const void *k_blk_ar, const void *v_blk_ar,
                                        void *k_pool, void *v_pool,
                                        const int32_t *page_table, int32_t *seq_lens,
                                        int32_t *accept_len, int32_t *num_committed,
                                        int32_t *out_tokens, int32_t *next_anchor,
                                        void *workspace, size_t workspace_bytes, void *stream)
{
    return consensus_commit_impl(ctx, p, ar_logits, draft_tokens, k_blk_ar, v_blk_ar, k_pool, v_pool, page_table,
                                 seq_lens, accept_len, num_committed, out_tokens, next_anchor, workspace,
                                 workspace_bytes, stream);
}

int64_t orthrus_noalloc_scratch_bytes(void) { return (int64_t)orthrus::consensus_scratch_bytes(); }

orthrus_status orthrus_consensus_commit_noalloc(orthrus_ctx *ctx, const orthrus_params *p,
                                                const float *ar_logits, const int32_t *draft_tokens,
                                                const void *k_blk_ar, const void *v_blk_ar,
                                                void *k_pool, void *v_pool,
                                                const int32_t *page_table, int32_t *seq_lens,
                                                int32_t *accept_len, int32_t *num_committed,
                                                int32_t *out_tokens, int32_t *next_anchor, void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    // the device address of this GPU's static scratch array, looked up when the context was created
    void *ws = orthrus::consensus_scratch(ctx->device);
    if (!ws) return ORTHRUS_EHIP;
    // a problem whose workspace does not fit the fixed array comes back as ORTHRUS_EWORKSPACE from the
    // shared size check, before anything is launched
    return consensus_commit_impl(ctx, p, ar_logits, draft_tokens, k_blk_ar, v_blk_ar, k_pool, v_pool, page_table,
                                 seq_lens, accept_len, num_committed, out_tokens, next_anchor, ws,
                                 orthrus::consensus_scratch_bytes(), stream);
}

int64_t orthrus_sampling_workspace_bytes(const orthrus_params *p)
{
    orthrus_status s = check_params(p, false, true, false);
    if (s != ORTHRUS_OK) return (int64_t)s;
    const size_t rows = (size_t)p->batch * p->block_k;
    const size_t chunks = (size_t)consensus_chunks(p);
    return (int64_t)(align_up(rows * chunks * 16, 256) + align_up((size_t)p->batch * chunks * 16, 256) +
                     align_up((size_t)p->batch * 2 * sizeof(int32_t), 256));
}

orthrus_status orthrus_sampling_consensus_commit(orthrus_ctx *ctx, const orthrus_params *p, float temperature,
                                                 const float *ar_logits, const float *diff_logits,
                                                 const int32_t *draft_tokens, const float *accept_u,
                                                 const float *gumbel,
                                                 const void *k_blk_ar, const void *v_blk_ar,
                                                 void *k_pool, void *v_pool,
                                                 const int32_t *page_table, int32_t *seq_lens,
                                                 int32_t *accept_len, int32_t *num_committed,
                                                 int32_t *out_tokens, int32_t *next_anchor,
                                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx) return ORTHRUS_EINVAL;
    if ((k_blk_ar == nullptr) != (v_blk_ar == nullptr)) return ORTHRUS_EINVAL;
    const bool do_commit = k_blk_ar != nullptr;
    orthrus_status s = check_params(p, false, true, do_commit);
    if (s != ORTHRUS_OK) return s;
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return ORTHRUS_EINVAL;
    if (!ar_logits || !diff_logits || !draft_tokens || !accept_u || !gumbel || !accept_len || !num_committed ||
        !out_tokens || !next_anchor)
        return ORTHRUS_EINVAL;
    if ((((uintptr_t)ar_logits) | ((uintptr_t)diff_logits) | ((uintptr_t)gumbel) | ((uintptr_t)accept_u)) & 3)
        return ORTHRUS_EINVAL;
    if (do_commit) {
        if (!k_pool || !v_pool || !page_table || !seq_lens || p->num_layers <= 0) return ORTHRUS_EINVAL;
        if (p->num_layers > 65535) return ORTHRUS_EUNSUPPORTED;
        const uintptr_t al = (uintptr_t)k_blk_ar | (uintptr_t)v_blk_ar | (uintptr_t)k_pool | (uintptr_t)v_pool;
        if (al & 15) return ORTHRUS_EINVAL;
    }
    if (p->batch == 0) return ORTHRUS_OK;
    const size_t rows = (size_t)p->batch * p->block_k;
    const size_t chunks = (size_t)consensus_chunks(p);
    if (rows * chunks > 0x7fffffffull || chunks > 65535) return ORTHRUS_EUNSUPPORTED;
    const size_t o1 = align_up(rows * chunks * 16, 256);
    const size_t o2 = o1 + align_up((size_t)p->batch * chunks * 16, 256);
    const size_t need = o2 + align_up((size_t)p->batch * 2 * sizeof(int32_t), 256);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return ORTHRUS_EWORKSPACE;

    orthrus::SamplingArgs a;
    orthrus::ConsensusArgs &c = a.c;
    c.ar_logits = ar_logits; c.draft_tokens = draft_tokens;
    c.k_blk_ar = (const uint16_t *)k_blk_ar; c.v_blk_ar = (const uint16_t *)v_blk_ar;
    c.k_pool = (uint16_t *)k_pool; c.v_pool = (uint16_t *)v_pool;
    c.page_table = page_table; c.seq_lens = seq_lens;
    c.accept_len = accept_len; c.num_committed = num_committed; c.out_tokens = out_tokens; c.next_anchor = next_anchor;
    c.part_val = nullptr; c.part_idx = nullptr;
    c.commit_info = (int32_t *)((char *)workspace + o2);
    c.err_word = ctx->err_word;
    c.stride_layer = p->pool_stride_layer; c.stride_page = p->pool_stride_page;
    c.stride_head = p->pool_stride_head; c.stride_tok = p->pool_stride_tok; c.num_pages = p->num_pages;
    c.blk_stride_head = p->blk_stride_head ? p->blk_stride_head : p->head_dim;
    c.blk_stride_row = p->blk_stride_row ? p->blk_stride_row : (int64_t)p->num_kv_heads * p->head_dim;
    c.blk_stride_layer = p->blk_stride_layer ? p->blk_stride_layer : (int64_t)p->batch * p->block_k * c.blk_stride_row;
    c.batch = p->batch; c.block_k = p->block_k; c.vocab = p->vocab; c.num_layers = p->num_layers;
    c.num_kv_heads = p->num_kv_heads; c.head_dim = p->head_dim;
    c.page_shift = do_commit ? log2_exact(p->page_size) : 0; c.max_pages_per_seq = p->max_pages_per_seq;
    c.chunks = (int)chunks; c.chunk_elems = orthrus::consensus_chunk_elems(); c.do_commit = do_commit ? 1 : 0;
    a.diff_logits = diff_logits; a.accept_u = accept_u; a.gumbel = gumbel;
    a.lse_part = (float4 *)workspace;
    a.draw_part = (float4 *)((char *)workspace + o1);
    a.inv_temperature = 1.0f / temperature;
    hipError_t e = orthrus::launch_sampling_consensus(a, (hipStream_t)stream);
    return e == hipSuccess ? ORTHRUS_OK : ORTHRUS_EHIP;
}

orthrus_status orthrus_last_device_error(orthrus_ctx *ctx, void *stream, int32_t *code)
{
    if (!ctx || !code) return ORTHRUS_EINVAL;
    int32_t v = 0;
    if (hipMemcpyAsync(&v, ctx->err_word, sizeof v, hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return ORTHRUS_EHIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ORTHRUS_EHIP;
    if (v != 0) {
        if (hipMemsetAsync(ctx->err_word, 0, sizeof v, (hipStream_t)stream) != hipSuccess) return ORTHRUS_EHIP;
        if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ORTHRUS_EHIP;
    }
    *code = v;
    return ORTHRUS_OK;
}

}  // extern "C"
