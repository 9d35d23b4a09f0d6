// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace orthrus {

// Finite stand-in for "no score seen yet" (keeps exp2(m_old - m_new) free of inf - inf).
constexpr float kNegBig = -1.0e30f;

struct AttnPlan {
    int rows;          // R = G * K query rows per KV head
    int waves;         // compute waves per workgroup = 32-row blocks (1 .. 8)
    int rows_padded;   // waves * 32
    int chunk_tokens;  // cache tokens per split at the host bound (the kernels cut each sequence by its own length)
    int num_splits;    // splits per (sequence, KV head)
    int bal_wgs;       // > 0: balanced partition over this many workgroups instead of fixed splits
    int kv_nt;         // 1: the call streams more K/V than the last-level cache holds: non-temporal tile loads
    size_t lds_bytes;  // dynamic LDS per workgroup
    size_t part_o_bytes, part_ml_bytes;  // workspace pieces (0 when nothing is merged)
};

struct AttnArgs {
    const uint16_t *q, *k_blk, *v_blk, *k_pool, *v_pool;
    const int32_t *page_table, *seq_lens;
    uint16_t *out;
    float *lse;
    // partial p = (unit, split), or workgroup slot 2w / 2w+1 of the balanced partition
    float *part_o;   // [p][wave][d block][4][lane] float4: unnormalised partial outputs, register order
    float *part_ml;  // [p][wave][32 rows] float2: running max (log2 domain) and sum
    int32_t *err_word;
    // prefill only: lengths before the call and validated new-token counts [B] (workspace), row stride T
    const int32_t *old_lens, *new_lens;
    int max_new;
    int64_t stride_page, stride_head, stride_tok, num_pages;
    // block inputs: elements between consecutive rows (b*K + i) and heads of q, and of k_blk / v_blk
    // (prefill: of q and of the new K/V rows, always dense)
    int64_t q_stride_row, q_stride_head, blk_stride_row, blk_stride_head;
    int batch, num_q_heads, num_kv_heads, group, block_k, rows;
    int page_shift, max_pages_per_seq, max_seq_len, chunk_tokens, num_splits, view;
    int bal_wgs;  // balanced partition: workgroups of the split launch (0 otherwise)
    int kv_nt;    // non-temporal K/V tile loads (see AttnPlan)
    float scale_log2e;  // sm_scale * log2(e)
};

struct ConsensusArgs {
    const float *ar_logits;
    const int32_t *draft_tokens;
    const uint16_t *k_blk_ar, *v_blk_ar;
    uint16_t *k_pool, *v_pool;
    const int32_t *page_table;
    int32_t *seq_lens, *accept_len, *num_committed, *out_tokens, *next_anchor;
    float *part_val;     // [B*K][chunks]
    int32_t *part_idx;   // [B*K][chunks]
    int32_t *commit_info;  // [B][2]: length before the step, rows to append (0 = none)
    int32_t *err_word;
    int64_t stride_layer, stride_page, stride_head, stride_tok, num_pages;
    int64_t blk_stride_layer, blk_stride_row, blk_stride_head;  // of k_blk_ar / v_blk_ar
    int batch, block_k, vocab, num_layers, num_kv_heads, head_dim;
    int page_shift, max_pages_per_seq, chunks, chunk_elems, do_commit;
};

struct SamplingArgs {
    ConsensusArgs c;          // shared fields (ar_logits, drafts, pools, outputs, commit_info, err_word, shapes)
    const float *diff_logits; // [B][K][V]
    const float *accept_u;    // [B][K]
    const float *gumbel;      // [B][V]
    float4 *lse_part;         // [B*K][chunks]: (max_p, sum_p, max_q, sum_q) of logits / T over the chunk
    float4 *draw_part;        // [B][chunks]: (best score among p>q, its index, best score of log p + g, its index)
    float inv_temperature;
};

// ---- commit helpers shared by the greedy and the sampling consensus kernels (device code)
#if defined(__HIPCC__)
// Copy rows 0..m-1 of the AR view's block K/V of (sequence b, layer) to token positions L..L+m-1 of the
// pools (Fig. 2(b): only the accepted tokens' K/V enters the shared cache), as 16-byte chunks.  `pages`
// (LDS or NULL) holds the page id of position L+k at index k when the caller has fetched them already.
__device__ __forceinline__ void append_rows(const ConsensusArgs &a, int b, int layer, int L, int m, int tid, int nthreads,
                                            const int *pages = nullptr)
{
    const int K = a.block_k, H = a.num_kv_heads, d = a.head_dim;
    const int cpr = d / 8;  // 16-byte chunks per row
    const int per_tok = H * cpr;
    const int total = m * per_tok;
    const int P = 1 << a.page_shift;
    // four chunks of each pool per thread are in flight before the first store (the compiler may not move
    // a load above a store to the pools): the copy costs a memory round trip per four chunks, not per chunk
    constexpr int kBatch = 4;
    auto src_of = [&](int e) __attribute__((always_inline)) {
        const int k = e / per_tok, rem = e - k * per_tok;
        const int g = rem / cpr, ch = rem - g * cpr;
        return (int64_t)layer * a.blk_stride_layer + ((int64_t)b * K + k) * a.blk_stride_row + (int64_t)g * a.blk_stride_head + ch * 8;
    };
    auto dst_of = [&](int e) __attribute__((always_inline)) {
        const int k = e / per_tok, rem = e - k * per_tok;
        const int g = rem / cpr, ch = rem - g * cpr;
        const int pos = L + k;
        const int pg = pages ? pages[k] : a.page_table[(int64_t)b * a.max_pages_per_seq + (pos >> a.page_shift)];
        return (int64_t)layer * a.stride_layer + (int64_t)pg * a.stride_page + (int64_t)g * a.stride_head +
               (int64_t)(pos & (P - 1)) * a.stride_tok + ch * 8;
    };
    for (int e0 = tid; e0 < total; e0 += nthreads * kBatch) {
        const int e1 = e0 + nthreads, e2 = e0 + 2 * nthreads, e3 = e0 + 3 * nthreads;
        uint4 k0, v0, k1, v1, k2, v2, k3, v3;
        k0 = *(const uint4 *)(a.k_blk_ar + src_of(e0)); v0 = *(const uint4 *)(a.v_blk_ar + src_of(e0));
        k1 = v1 = k2 = v2 = k3 = v3 = make_uint4(0, 0, 0, 0);
        if (e1 < total) { k1 = *(const uint4 *)(a.k_blk_ar + src_of(e1)); v1 = *(const uint4 *)(a.v_blk_ar + src_of(e1)); }
        if (e2 < total) { k2 = *(const uint4 *)(a.k_blk_ar + src_of(e2)); v2 = *(const uint4 *)(a.v_blk_ar + src_of(e2)); }
        if (e3 < total) { k3 = *(const uint4 *)(a.k_blk_ar + src_of(e3)); v3 = *(const uint4 *)(a.v_blk_ar + src_of(e3)); }
        { const int64_t t = dst_of(e0); *(uint4 *)(a.k_pool + t) = k0; *(uint4 *)(a.v_pool + t) = v0; }
        if (e1 < total) { const int64_t t = dst_of(e1); *(uint4 *)(a.k_pool + t) = k1; *(uint4 *)(a.v_pool + t) = v1; }
        if (e2 < total) { const int64_t t = dst_of(e2); *(uint4 *)(a.k_pool + t) = k2; *(uint4 *)(a.v_pool + t) = v2; }
        if (e3 < total) { const int64_t t = dst_of(e3); *(uint4 *)(a.k_pool + t) = k3; *(uint4 *)(a.v_pool + t) = v3; }
    }
    static_assert(kBatch == 4, "the loop body above is written out for four chunks");
}

// What lane k < K of a sequence's first wave learns about token position L + k (L = seq_lens[b]) before
// the number of rows to append is known: fetched at the start of the kernel, so that these dependent
// loads (length, then page id) run next to the argmax reductions instead of after them.
struct CommitProbe {
    int L;    // length before the step (same in every lane)
    int pg;   // page id of position L + lane, -1 if the slot lies beyond the page table
};
__device__ __forceinline__ CommitProbe commit_probe(const ConsensusArgs &a, int b, int lane)
{
    CommitProbe p;
    p.L = a.seq_lens[b];
    p.pg = -1;
    if (lane < a.block_k && p.L >= 0) {
        const int slot = (p.L + lane) >> a.page_shift;
        if (slot < a.max_pages_per_seq) p.pg = a.page_table[(int64_t)b * a.max_pages_per_seq + slot];
    }
    return p;
}

// Run by the first wave once it knows m, the number of rows to append: positions L..L+m-1 must be mapped;
// then the length is bumped, else the capacity error is flagged and the sequence left alone.  Records
// (L, rows to append) for a later copy launch.  Returns the rows that will be appended (m or 0).  Every
// lane of the wave must call it.
__device__ __forceinline__ int commit_decide(const ConsensusArgs &a, int b, int lane, int m, const CommitProbe &p)
{
    const bool bad = lane < m && (p.pg < 0 || p.pg >= a.num_pages);
    const bool any_bad = __ballot(bad) != 0ull;
    const int committed = any_bad ? 0 : m;
    if (lane == 0) {
        a.commit_info[b * 2] = p.L;
        a.commit_info[b * 2 + 1] = committed;
        if (any_bad) atomicExch(a.err_word, -4);
        else a.seq_lens[b] = p.L + m;
    }
    return committed;
}
#endif

// Optional start/stop events of the two attention kernels of one call (index 0 = split kernel,
// 1 = combine kernel).  When `on`, the launcher attaches them to the dispatches themselves, so that
// hipEventElapsedTime(start, stop) is the kernel's own execution time without any marker in between.
struct AttnLaunchEvents {
    bool on = false;
    hipEvent_t start[2] = {nullptr, nullptr}, stop[2] = {nullptr, nullptr};
    bool used[2] = {false, false};
};

// Host-side launchers (defined next to the kernels).  Return hipSuccess or the launch error.
hipError_t plan_attn(int head_dim, int group, int block_k, int batch, int num_kv_heads, int max_seq_len,
                     int requested_splits, int num_cus, int num_layers, AttnPlan *plan);
hipError_t launch_attn(const AttnArgs &a, const AttnPlan &plan, int head_dim, hipStream_t stream,
                       AttnLaunchEvents *events = nullptr);
hipError_t launch_prefill_attn(const AttnArgs &a, int head_dim, hipStream_t stream);
hipError_t launch_consensus(const ConsensusArgs &a, hipStream_t stream);
hipError_t launch_sampling_consensus(const SamplingArgs &a, hipStream_t stream);
int consensus_chunk_elems();
// Static device scratch of the allocation-free consensus entry point: looked up once per device (with
// that device current), then used through the returned device address only.
hipError_t consensus_scratch_init(int device);
void *consensus_scratch(int device);
size_t consensus_scratch_bytes();
// Measurement helper: the attention call's own K/V stream with idle compute waves (same grid, same
// partition, same loader, no arithmetic, nothing written).
hipError_t launch_kv_stream_probe(const AttnArgs &a, const AttnPlan &plan, int head_dim, hipStream_t stream,
                                  hipEvent_t start, hipEvent_t stop);

// Prefill front end (defined with the commit kernels): validates lengths and pages, records the lengths
// before the call and the accepted new-token counts, bumps seq_lens, then copies the new K/V rows in.
struct PrefillArgs {
    const uint16_t *k_new, *v_new;   // [B][T][H_kv][d]
    const int32_t *new_lens_in;      // [B] requested new tokens
    uint16_t *k_pool, *v_pool;
    const int32_t *page_table;
    int32_t *seq_lens;
    int32_t *old_lens, *new_lens;    // [B] outputs (workspace)
    int32_t *err_word;
    int64_t stride_page, stride_head, stride_tok, num_pages;
    int batch, max_new, num_kv_heads, head_dim, page_shift, max_pages_per_seq, max_seq_len;
};
hipError_t launch_prefill_append(const PrefillArgs &a, hipStream_t stream);

}  // namespace orthrus
