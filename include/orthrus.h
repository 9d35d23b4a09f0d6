/*
 * orthrus.h — C ABI of the MI355X (gfx950) library for the hot path of the Orthrus
 * dual-view decode step: block attention of the diffusion view and of the AR verification
 * view over one shared paged KV cache, greedy consensus, and in-place commit of the accepted
 * tokens' K/V.
 *
 * Conventions that hold for every entry point
 *   - Pointers marked [dev] are DEVICE pointers owned by the caller (for instance torch
 *     allocations); pointers marked [host] are host pointers.  The library never frees a
 *     caller's pointer and never keeps one after the call returns.
 *   - The compute entry points are asynchronous on the caller's HIP stream (`stream` is a
 *     hipStream_t passed as void*; NULL = the default stream), do not synchronise with the
 *     host and do not allocate.  Sequence lengths live on the device and are read by the
 *     kernels, so consecutive decode steps can be queued without a host round trip.
 *     (While per-kernel timing is enabled an attention call creates or reuses HIP events on the host;
 *     that is the one exception to "does not allocate", see orthrus_attn_timing.)
 *   - The context holds one device error word shared by every call made with it, and the host-side
 *     list of timing events.  A context is not thread-safe: calls that share one must not overlap in
 *     time on the host; use one context per host thread.
 *   - Every function returns an orthrus_status.  Argument errors are found on the host before
 *     anything is launched; on such an error nothing has been written.
 *   - Layouts are row-major with the last index contiguous.  bf16 means the upper 16 bits of
 *     an IEEE fp32 value.
 *   - Indices are 0-based: draft_tokens[b][k] is the paper's y-hat_{k+1}.
 */
#ifndef ORTHRUS_H
#define ORTHRUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orthrus_ctx orthrus_ctx; /* opaque: device id, cached device properties, a device error word */
typedef struct orthrus_graph orthrus_graph; /* opaque: a captured sequence of compute calls, ready to replay */

typedef enum {
    ORTHRUS_OK = 0,
    ORTHRUS_EINVAL = -1,       /* NULL pointer, non-positive size, inconsistent shape */
    ORTHRUS_EUNSUPPORTED = -2, /* legal shape outside what the kernels are built for (see orthrus_params) */
    ORTHRUS_EWORKSPACE = -3,   /* workspace missing, misaligned or smaller than the *_workspace_bytes value */
    ORTHRUS_ECAPACITY = -4,    /* device side: a needed page was not mapped (reported by orthrus_last_device_error) */
    ORTHRUS_EHIP = -5          /* a HIP runtime call failed */
} orthrus_status;

typedef enum {
    ORTHRUS_VIEW_DIFFUSION = 0, /* in-block keys visible to every block row (bidirectional) */
    ORTHRUS_VIEW_AR_VERIFY = 1  /* in-block keys causal: row i sees in-block rows 0..i */
} orthrus_view;

/*
 * num_splits value that asks for the balanced partition.  A fixed split count cuts every
 * sequence into the same number of pieces (each sequence by its own length, read on the device;
 * the host bound max_seq_len only sizes the grid): when the lengths of a batch differ widely,
 * the pieces of short sequences end early and the call lasts as long as the longest sequence's
 * pieces.  The balanced partition instead gives every resident workgroup the same number of
 * 32-token tiles, cutting sequences wherever the shares end; results are merged exactly as with
 * fixed splits and are equally deterministic.  Meant for batches with ragged lengths; with equal
 * lengths a fixed split count is as fast or faster.
 */
#define ORTHRUS_SPLITS_BALANCED (-1)

/*
 * Problem description shared by all entry points (plain data, filled by the caller).
 *
 * Supported by the kernels: head_dim in {64, 128}; page_size a power of two >= 16;
 * 1 <= block_k <= 32; num_q_heads a multiple of num_kv_heads with
 * (num_q_heads / num_kv_heads) * block_k <= 256; sm_scale > 0; every pool stride and every block-input
 * stride a multiple of 8 elements (16-byte rows), head strides >= d.  Anything else that is otherwise consistent returns
 * ORTHRUS_EUNSUPPORTED.
 */
typedef struct {
    int32_t batch;             /* B: sequences in the step */
    int32_t num_q_heads;       /* H_q */
    int32_t num_kv_heads;      /* H_kv; query head h reads KV head h / (H_q / H_kv) */
    int32_t head_dim;          /* d */
    int32_t block_k;           /* K: positions in the block (anchor + K-1 drafts) */
    int32_t page_size;         /* P: tokens per cache page */
    int32_t max_pages_per_seq; /* row length of page_table */
    int32_t max_seq_len;       /* HOST upper bound on every seq_lens[b] during the call (sizes the grid) */
    int32_t num_splits;        /* attention: KV splits per (sequence, KV head); 0 = library chooses;
                                  ORTHRUS_SPLITS_BALANCED = even partition of the whole batch (below) */
    int32_t num_layers;        /* layers of the model.  commit: layers written per call (block K/V and pools
                                  carry a layer axis).  attention: how many caches of this size the model
                                  streams between two passes over the same layer (with batch and max_seq_len
                                  it decides whether the K/V loads bypass the caches); <= 1 counts as 1 */
    int32_t vocab;             /* consensus: V */
    float sm_scale;            /* score scale of Eq. 4, normally 1/sqrt(d) */
    int64_t num_pages;         /* pages in each pool; page ids outside [0, num_pages) count as unmapped */
    /* element strides of k_pool / v_pool (both pools share them):
       element (layer, page, kv head g, slot s, c) is at
       layer*pool_stride_layer + page*pool_stride_page + g*pool_stride_head + s*pool_stride_tok + c */
    int64_t pool_stride_layer;
    int64_t pool_stride_page;
    int64_t pool_stride_head;
    int64_t pool_stride_tok;
    /* element strides of the block inputs, so that they can be read where the projections left them (for
       instance inside the output of one fused Q/K/V projection, [B*K, (H_q + 2 H_kv) * d], with the three
       pointers set to its Q, K and V column ranges) instead of being copied into dense tensors first.
       0 means dense: q_stride_row = H_q * d, q_stride_head = d, blk_stride_row = H_kv * d,
       blk_stride_head = d, blk_stride_layer = B * K * blk_stride_row.
       q element (b, i, h, c) is at (b*K + i) * q_stride_row + h * q_stride_head + c;
       k_blk / v_blk element (layer, b, i, g, c) is at
       layer * blk_stride_layer + (b*K + i) * blk_stride_row + g * blk_stride_head + c
       (attention reads layer 0 of the pointer it is given; the commit reads every layer).
       Outputs are always dense.  orthrus_prefill_attn ignores these fields (its inputs are dense). */
    int64_t q_stride_row;
    int64_t q_stride_head;
    int64_t blk_stride_row;
    int64_t blk_stride_head;
    int64_t blk_stride_layer;
} orthrus_params;

/* Creates a context on HIP device `device` (allocates one small device error word).  [host] out. */
orthrus_status orthrus_create(orthrus_ctx **out, int device);
/* Frees the context.  The caller must have synchronised every stream that used it. */
orthrus_status orthrus_destroy(orthrus_ctx *ctx);
/* Static description of a status code (never NULL). */
const char *orthrus_status_string(orthrus_status s);

/*
 * Workspace sizes in bytes for the given params (0 is a valid answer).  Workspaces are
 * [dev], 256-byte aligned, owned by the caller, and may be reused by the next call on the
 * same stream.  A negative return is an orthrus_status.
 */
int64_t orthrus_attn_workspace_bytes(const orthrus_params *p);
int64_t orthrus_consensus_workspace_bytes(const orthrus_params *p);
int64_t orthrus_sampling_workspace_bytes(const orthrus_params *p);
/* Number of KV splits the attention call will use for these params (>= 1; 0 for the balanced
   partition, which has no fixed split count), or a negative status. */
int32_t orthrus_attn_num_splits(const orthrus_params *p);
/*
 * The attention launch plan (split count, workgroups of the balanced partition, hence the workspace)
 * follows the compute-unit count of the context's device.  The two queries above assume the full
 * 256-CU part; these two answer for the device `ctx` was created on and are the ones to use when that
 * device exposes fewer CUs (a partitioned GPU).  orthrus_dual_view_attn checks the workspace against
 * the plan it actually uses and returns ORTHRUS_EWORKSPACE if it is too small.
 */
int32_t orthrus_attn_num_splits_on(const orthrus_ctx *ctx, const orthrus_params *p);
int64_t orthrus_attn_workspace_bytes_on(const orthrus_ctx *ctx, const orthrus_params *p);
/* Identifier of the sources and compiler flags this library was built from (a hex digest chosen by the
   build script; "unknown" if built by hand).  Lets a binding detect a library that is older than the
   sources next to it. */
const char *orthrus_build_id(void);

/*
 * Block attention of one view over the shared cache — Section 3.1, Eq. 4 of the paper:
 *   O = Softmax(Q [K_AR || K_blk]^T * sm_scale) [V_AR || V_blk]
 * for every sequence b, block row i < K and query head h.  The key axis is the sequence's
 * cached tokens 0..seq_lens[b]-1 (the cache built by the AR view, Section 3.3: tokens before
 * the anchor) followed by the block's own K rows.  In-block visibility depends on `view`:
 * ORTHRUS_VIEW_DIFFUSION lets every row see all K in-block keys (Section 3.2, rule (ii) of
 * the block mask, Eq. 6 second term); ORTHRUS_VIEW_AR_VERIFY is causal inside the block
 * (Section 3.2 "standard causal masking"; Section 3.3, verification pass).  The cache is
 * read-only here and is the same for both views.
 *
 *   q        [dev] bf16 [B, K, H_q, d]      queries of the block (post-projection, post-RoPE)
 *   k_blk    [dev] bf16 [B, K, H_kv, d]     the block's own keys for this view
 *   v_blk    [dev] bf16 [B, K, H_kv, d]     the block's own values for this view
 *            (these three dense by default, or strided views: q_stride_* / blk_stride_* in params; the
 *            block of Section 3.1, anchor + K-1 mask positions for the diffusion view, anchor + drafts
 *            for the AR view, is read where its projections were written)
 *   k_pool   [dev] bf16 paged cache, strides in params (layer 0 is used)
 *   v_pool   [dev] bf16 same strides
 *   page_table [dev] int32 [B, max_pages_per_seq]; entry j maps tokens j*P .. j*P+P-1
 *   seq_lens [dev] int32 [B]; 0 <= seq_lens[b] <= max_seq_len
 *   out      [dev] bf16 [B, K, H_q, d]      written
 *   lse      [dev] fp32 [B, H_q, K] or NULL natural-log sum of exp(scaled scores), written if given
 *   workspace/workspace_bytes: at least orthrus_attn_workspace_bytes(p)
 *
 * Arithmetic: bf16 inputs, fp32 scores/softmax/accumulation, probabilities rounded to bf16
 * for the value product, bf16 output.
 * Device-side errors: a page id outside [0, num_pages) for a token below seq_lens[b], or
 * seq_lens[b] outside [0, max_seq_len], sets the context's error word (ORTHRUS_ECAPACITY);
 * tokens behind a bad page id are read from page 0 instead (that sequence's output is then
 * meaningless), nothing is read out of bounds.
 */
orthrus_status orthrus_dual_view_attn(orthrus_ctx *ctx, const orthrus_params *p, orthrus_view view,
                                      const void *q, const void *k_blk, const void *v_blk,
                                      const void *k_pool, const void *v_pool,
                                      const int32_t *page_table, const int32_t *seq_lens,
                                      void *out, float *lse,
                                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Greedy consensus and commit — Section 3.3 "Architectural Consensus Mechanism", Eq. 8, and
 * Fig. 2(b): a draft is kept iff it equals the AR view's greedy token, left to right;
 * verification stops at the first divergence, the AR token there is emitted as the
 * correction, and only the K/V of the tokens now in the sequence is appended to the cache.
 * Per sequence b (L = seq_lens[b] on entry):
 *   am[k]  = argmax_v ar_logits[b][k][v]  (smallest index on ties; NaN ranks above all numbers)
 *   accept_len[b]    = number of leading k with draft_tokens[b][k] == am[k]          (0..K)
 *   num_committed[b] = m = min(accept_len[b] + 1, K)                                  (1..K)
 *   out_tokens[b][0..m-1] = am[0..m-1], out_tokens[b][m..K-1] = -1, next_anchor[b] = am[m-1]
 *   rows 0..m-1 of k_blk_ar / v_blk_ar (the AR view's K/V of the anchor and the accepted
 *   drafts) are copied to token positions L..L+m-1 of every layer's pool; seq_lens[b] = L+m.
 *
 *   ar_logits    [dev] fp32 [B, K, V]      row k is conditioned on the anchor and drafts 0..k-1
 *   draft_tokens [dev] int32 [B, K]        values outside [0, V) never match
 *   k_blk_ar, v_blk_ar [dev] bf16 [num_layers, B, K, H_kv, d] (dense, or strided by blk_stride_* in
 *                                           params), or both NULL: consensus only
 *                                           (pools, page_table and seq_lens are then not touched)
 *   k_pool, v_pool [dev] bf16, updated in place; page_table [dev] as above
 *   seq_lens     [dev] int32 [B], updated in place
 *   accept_len, num_committed, next_anchor [dev] int32 [B]; out_tokens [dev] int32 [B, K]
 *   workspace/workspace_bytes: at least orthrus_consensus_workspace_bytes(p)
 *
 * Device-side errors: if a position L..L+m-1 is not mapped (beyond max_pages_per_seq or page
 * id outside [0, num_pages)) the sequence's pools and length are left untouched,
 * num_committed[b] is 0 and the context's error word is set (ORTHRUS_ECAPACITY).
 * Integer and byte results are exact.
 */
orthrus_status orthrus_consensus_commit(orthrus_ctx *ctx, const orthrus_params *p,
                                        const float *ar_logits, const int32_t *draft_tokens,
                                        const void *k_blk_ar, const void *v_blk_ar,
                                        void *k_pool, void *v_pool,
                                        const int32_t *page_table, int32_t *seq_lens,
                                        int32_t *accept_len, int32_t *num_committed,
                                        int32_t *out_tokens, int32_t *next_anchor,
                                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * orthrus_consensus_commit for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results, errors and
 * kernels as orthrus_consensus_commit, minus the workspace: the chunk argmax pairs and the per-sequence
 * commit record go to a fixed array of orthrus_noalloc_scratch_bytes() bytes (1 MiB) that is part of the
 * library's device image, one copy per GPU, held until the process ends.  The call allocates nothing and
 * frees nothing.  A problem that needs more than the array holds (orthrus_consensus_workspace_bytes(p) >
 * orthrus_noalloc_scratch_bytes(): roughly batch * block_k * ceil(vocab / 8192) > 130000) returns
 * ORTHRUS_EWORKSPACE and launches nothing.  Every call on one GPU shares that GPU's array: calls that
 * overlap in time on one GPU (two streams, two contexts, two threads) race on it; calls queued on one
 * stream do not.  Nothing in the array has to be cleared between calls: each call writes every entry
 * it later reads.
 */
int64_t orthrus_noalloc_scratch_bytes(void);
orthrus_status orthrus_consensus_commit_noalloc(orthrus_ctx *ctx, const orthrus_params *p,
                                                const float *ar_logits, const int32_t *draft_tokens,
                                                const void *k_blk_ar, const void *v_blk_ar,
                                                void *k_pool, void *v_pool,
                                                const int32_t *page_table, int32_t *seq_lens,
                                                int32_t *accept_len, int32_t *num_committed,
                                                int32_t *out_tokens, int32_t *next_anchor, void *stream);

/*
 * Lossless consensus for temperature T > 0 and commit — Section 3.3, the sentence on diverse
 * generation: exact rejection sampling that aligns the diffusion view's drafts with the AR
 * distribution.  The accept/replace rule is the published speculative-sampling rule the paper cites:
 * with p_k = softmax(ar_logits[b][k] / T) and q_k = softmax(diff_logits[b][k] / T), the draft x of row
 * k (drawn from q_k by the caller) is kept iff accept_u[b][k] * q_k(x) < p_k(x), rows are examined left
 * to right, and at the first row j that is not kept the emitted token is
 *   argmax_v [ log max(0, p_j(v) - q_j(v)) + gumbel[b][v] ]   (smallest index on ties),
 * i.e. a draw from the normalised positive part of p_j - q_j when gumbel holds independent standard
 * Gumbel noise (from p_j itself if that part is empty).  accept_len[b] = j (K if every draft is kept),
 * num_committed[b] = m = min(j + 1, K); out_tokens[b] = the kept drafts, then the replacement when
 * j < K, then -1; next_anchor[b] = the last emitted token.  Cache commit, length update and the
 * device-side capacity error are exactly those of orthrus_consensus_commit.
 * Every random number is an argument, so the call is a deterministic function of its inputs.
 *
 *   temperature  [host value] T > 0, applied to both logit sets
 *   ar_logits, diff_logits [dev] fp32 [B, K, V]
 *   draft_tokens [dev] int32 [B, K]        a value outside [0, V) is never kept
 *   accept_u     [dev] fp32 [B, K]         uniforms in [0, 1)
 *   gumbel       [dev] fp32 [B, V]         standard Gumbel noise for the replacement draw
 *   remaining arguments as in orthrus_consensus_commit; workspace at least
 *   orthrus_sampling_workspace_bytes(p)
 *
 * Arithmetic is fp32 (log-sum-exp per 8192-element chunk, merged in chunk order); a decision whose
 * two sides differ by less than fp32 rounding of the log-sum-exp may fall either way.
 */
orthrus_status orthrus_sampling_consensus_commit(orthrus_ctx *ctx, const orthrus_params *p, float temperature,
                                                 const float *ar_logits, const float *diff_logits,
                                                 const int32_t *draft_tokens, const float *accept_u,
                                                 const float *gumbel,
                                                 const void *k_blk_ar, const void *v_blk_ar,
                                                 void *k_pool, void *v_pool,
                                                 const int32_t *page_table, int32_t *seq_lens,
                                                 int32_t *accept_len, int32_t *num_committed,
                                                 int32_t *out_tokens, int32_t *next_anchor,
                                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * AR-view prefill attention of one layer — Section 3.1 (first paragraph) and Section 3.3: the frozen AR
 * view processes the context with its ordinary causal self-attention, and the K/V it produces is the
 * cache both views share afterwards.  Per sequence b with L = seq_lens[b] cached tokens and
 * n = new_lens[b] new tokens (0 <= n <= max_new_tokens; L > 0 continues an earlier prefill or decode):
 *   rows i < n of k_new / v_new are written to token positions L+i of the pools,
 *   out[b][i][h][:] = softmax over cache tokens j = 0 .. L+i of (sm_scale * <q[b][i][h], K_j>) applied to V_j
 *                     (token L+i sees everything before it and itself), for i < n,
 *   seq_lens[b] = L + n.
 * Rows i >= n of out are not written.
 *
 *   max_new_tokens [host value] T: row stride of q, k_new, v_new, out along the token axis
 *   q, out         [dev] bf16 [B, T, H_q, d]
 *   k_new, v_new   [dev] bf16 [B, T, H_kv, d]
 *   new_lens       [dev] int32 [B]
 *   k_pool, v_pool [dev] bf16, updated in place; page_table [dev]; seq_lens [dev] int32 [B], updated
 *   p->max_seq_len [host] must bound L + n of every sequence; p->block_k, p->num_splits, p->vocab unused
 *   workspace      at least orthrus_prefill_workspace_bytes(p, T)
 * Supported: H_q / H_kv <= 8 (and the head sizes / page sizes of orthrus_params).
 * Device-side errors: a sequence whose lengths are out of range or whose new positions are not all
 * mapped is left untouched (cache, length, output) and the context's error word is set
 * (ORTHRUS_ECAPACITY).  Output within the tolerance of orthrus_dual_view_attn; cache rows bit-exact.
 */
int64_t orthrus_prefill_workspace_bytes(const orthrus_params *p, int32_t max_new_tokens);
orthrus_status orthrus_prefill_attn(orthrus_ctx *ctx, const orthrus_params *p, int32_t max_new_tokens,
                                    const void *q, const void *k_new, const void *v_new, const int32_t *new_lens,
                                    void *k_pool, void *v_pool,
                                    const int32_t *page_table, int32_t *seq_lens, void *out,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Replay of a fixed sequence of compute calls as one HIP graph.  A decode cycle is two passes of the
 * whole layer stack plus the consensus (Section 3.2-3.3; Section 4 counts "forward passes"), i.e. tens
 * of short launches whose arguments do not change from cycle to cycle when the caller reuses its
 * buffers; replaying them as a graph removes the per-launch host cost and most of the gaps between
 * kernels.  Usage: orthrus_graph_begin(ctx, stream); any number of orthrus_dual_view_attn /
 * orthrus_consensus_commit / orthrus_sampling_consensus_commit calls on that same stream (nothing
 * runs, the launches are recorded; the entry points launch kernels only, so all of them may be
 * recorded); orthrus_graph_end(ctx, stream, &g); then orthrus_graph_launch(g, stream) once per cycle.
 *   - `stream` must be a created stream (not NULL).  The calling thread must not allocate or free
 *     device memory between begin and end.
 *   - Every pointer and every orthrus_params field is frozen into the graph: new inputs are written
 *     into the same buffers before each launch, and max_seq_len must bound the lengths of every
 *     replay.  Sequence lengths and caches live on the device and keep evolving across replays.
 *   - Per-kernel timing must be off while recording.
 * The graph is independent of the context afterwards, except that its kernels report device errors
 * into the context's error word: destroy the graph before the context.
 */
orthrus_status orthrus_graph_begin(orthrus_ctx *ctx, void *stream);
orthrus_status orthrus_graph_end(orthrus_ctx *ctx, void *stream, orthrus_graph **out);
orthrus_status orthrus_graph_launch(orthrus_graph *graph, void *stream);
orthrus_status orthrus_graph_destroy(orthrus_graph *graph);

/*
 * Per-kernel timing of orthrus_dual_view_attn, for measurement (Section 4 reports throughput; this is
 * how this library's own kernels are timed).  While enabled (enable != 0), every attention call made
 * with `ctx` attaches a pair of HIP events to each kernel it launches (the split kernel and, when the
 * plan has more than one split, the combine kernel): the events belong to the dispatches themselves, so
 * the elapsed time between them is the kernel's execution time and nothing is inserted between
 * kernels.  Events are created on first use and recycled (host-side allocation only; do not enable
 * under stream capture).  orthrus_attn_timing_read waits for the recorded kernels to finish, returns
 * the sums of kernel times in microseconds and the launch counts accumulated since the last read
 * (all [host] pointers), and resets them.  Events stay queued in the context until they are read: read
 * after a bounded number of timed calls.
 */
orthrus_status orthrus_attn_timing(orthrus_ctx *ctx, int enable);
orthrus_status orthrus_attn_timing_read(orthrus_ctx *ctx, double *split_us, int64_t *split_launches,
                                        double *combine_us, int64_t *combine_launches);
/*
 * The same records one by one instead of summed: for the i-th timed call since the last read, in launch
 * order, split_us[i] is its split kernel's time and combine_us[i] its combine kernel's (0 when the call
 * had none), both in microseconds.  At most `capacity` entries are written to the two [host] arrays;
 * *count receives the number of timed calls (it may exceed capacity: the rest are dropped).  Resets the
 * records like orthrus_attn_timing_read.
 */
orthrus_status orthrus_attn_timing_samples(orthrus_ctx *ctx, double *split_us, double *combine_us, int64_t capacity,
                                          int64_t *count);

/*
 * Measurement helper: the K/V stream of one attention call with no arithmetic.  Sections 1, 2.1 and 3.1
 * name the repeated loading of the KV cache as the memory-bandwidth bottleneck of decoding; this call
 * launches the attention kernel of orthrus_dual_view_attn for these params in a form whose compute
 * waves do nothing: same grid, same partition of the sequences, the same loads of the cached K and V
 * rows through the page table, no queries, no arithmetic, nothing written (the block's own K/V tile
 * is not read either).  Its duration is the time this library's access pattern needs for the call's
 * K/V bytes on the machine at hand: a measured ceiling to hold the attention kernels against, next to
 * the published peak.  Asynchronous on `stream`, allocates nothing.  While per-kernel timing is
 * enabled the launch is recorded like an attention call without a combine kernel.
 *   k_pool, v_pool, page_table, seq_lens [dev] as in orthrus_dual_view_attn (read only)
 * Page ids outside [0, num_pages) are read as page 0 and lengths are clamped to [0, max_seq_len], with
 * the context's error word set as in orthrus_dual_view_attn.
 */
orthrus_status orthrus_kv_stream_probe(orthrus_ctx *ctx, const orthrus_params *p, const void *k_pool,
                                       const void *v_pool, const int32_t *page_table, const int32_t *seq_lens,
                                       void *stream);

/*
 * Synchronises `stream`, copies the context's device error word to *code [host] (ORTHRUS_OK or
 * ORTHRUS_ECAPACITY) and clears it.  This is the only entry point that blocks.
 */
orthrus_status orthrus_last_device_error(orthrus_ctx *ctx, void *stream, int32_t *code);

#ifdef __cplusplus
}
#endif
#endif /* ORTHRUS_H */
