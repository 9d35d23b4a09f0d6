/*
 * CPU oracle for the Orthrus dual-view decode step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the hot path computes, written from the
 * paper's definitions.  It exists so that the GPU library can be checked against something
 * that shares no code with it; only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  Nothing here is tuned: every output element is evaluated from the
 * definition (all scores, then a two-pass softmax, then the weighted sum), and the only
 * parallelism is an OpenMP loop over independent (sequence, query head) outputs.
 *
 * What follows what:
 *   orthrus_oracle_dual_view_attn     Section 3.1, Eq. 4 (softmax attention over the shared
 *                                     AR cache concatenated with the block's own keys);
 *                                     in-block visibility: bidirectional for the diffusion
 *                                     view (Section 3.2, rule (ii) of the block mask, Eq. 6
 *                                     second term), causal for the AR view (Section 3.2,
 *                                     "standard causal masking"; Section 3.3 "Intra-Model
 *                                     Distribution Matching").
 *   orthrus_oracle_consensus_commit   Section 3.3 "Architectural Consensus Mechanism", Eq. 8
 *                                     (keep a draft iff it equals the greedy AR token, left
 *                                     to right, stop at the first divergence, emit the AR
 *                                     correction, cache ends at step t+j); Fig. 2(b)
 *                                     (accepted tokens' KV appended to the shared cache).
 *
 *   orthrus_oracle_sampling_consensus Section 3.3, the sentence on temperature T > 0: exact rejection
 *                                     sampling after the cited speculative-sampling rule (a draft x
 *                                     drawn from q is kept with probability min(1, p(x)/q(x)); a
 *                                     rejected one is replaced by a draw from the normalised positive
 *                                     part of p - q), applied left to right over the block.
 *
 *   orthrus_oracle_prefill_attn       Section 3.1, first paragraph, and Section 3.3: the frozen AR view's
 *                                     ordinary causal self-attention over the context ("pre-filling"),
 *                                     which is what builds the shared K/V cache: token t attends tokens
 *                                     0..t (textbook causal softmax attention, Section 2.1), and its K/V
 *                                     row is appended to the cache.
 *
 * Readings taken where the paper is silent (each is a stated reading, not a derivation):
 *   - the cache holds tokens strictly before the anchor x_t (Section 3.3: K_AR^{<t}); the
 *     anchor's own K/V is in-block row 0;
 *   - GQA: query head h reads KV head h / (H_q / H_kv);
 *   - argmax ties go to the smallest index; a NaN logit ranks above every number and the
 *     first NaN wins;
 *   - a draft token outside [0, V) never matches;
 *   - no bonus (K+1)-th token: the verify pass has K rows, so at most K tokens are emitted.
 *
 * All pointers are host pointers.  bf16 values arrive as 16-bit patterns and are widened
 * exactly to fp64; nothing in the attention oracle rounds.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_VIEW_DIFFUSION 0
#define ORACLE_VIEW_AR_VERIFY 1

static double bf16_to_f64(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int orthrus_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Eq. 4 for every (sequence b, block row i, query head h):
 *   keys   = cache keys 0..L_b-1 of KV head g = h/G, then the in-block keys visible to row i
 *   s_n    = sm_scale * <q, key_n>
 *   p      = softmax(s)            (two passes: max, then exp and sum)
 *   out    = sum_n p_n value_n
 * Visible in-block keys: all K rows (diffusion view) or rows 0..i (AR verify view).
 *
 * q [B,K,H_q,d], k_blk/v_blk [B,K,H_kv,d], pools addressed as
 *   pool[page*stride_page + g*stride_head + slot*stride_tok + c], c < d,
 * page_table [B,max_pages], seq_lens [B]; out [B,K,H_q,d] fp64; lse [B,H_q,K] fp64 or NULL
 * (natural-log-sum-exp of the scaled scores).
 * Returns 0, or -1 on an argument error, -4 if a needed page is not mapped.
 */
int orthrus_oracle_dual_view_attn(
    int batch, int num_q_heads, int num_kv_heads, int head_dim, int block_k,
    int page_size, int max_pages_per_seq, int64_t num_pages, int view, double sm_scale,
    const uint16_t *q, const uint16_t *k_blk, const uint16_t *v_blk,
    const uint16_t *k_pool, const uint16_t *v_pool,
    int64_t stride_page, int64_t stride_head, int64_t stride_tok,
    const int32_t *page_table, const int32_t *seq_lens,
    double *out, double *lse)
{
    if (batch < 0 || num_q_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || block_k <= 0 ||
        page_size <= 0 || num_q_heads % num_kv_heads != 0)
        return -1;
    if (view != ORACLE_VIEW_DIFFUSION && view != ORACLE_VIEW_AR_VERIFY)
        return -1;
    const int G = num_q_heads / num_kv_heads;
    const int d = head_dim, K = block_k;
    int status = 0;

    /* page checks first, so the parallel loop below never dereferences a bad page */
    for (int b = 0; b < batch; ++b) {
        int L = seq_lens[b];
        if (L < 0) return -1;
        for (int j = 0; j < L; j += page_size) {
            int slot = j / page_size;
            if (slot >= max_pages_per_seq) return -4;
            int32_t pg = page_table[(int64_t)b * max_pages_per_seq + slot];
            if (pg < 0 || pg >= num_pages) return -4;
        }
    }

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b) {
        for (int h = 0; h < num_q_heads; ++h) {
            const int g = h / G;
            const int L = seq_lens[b];
            double *s = (double *)malloc(sizeof(double) * (size_t)(L + K));
            if (!s) {
#pragma omp atomic write
                status = -1;
                continue;
            }
            for (int i = 0; i < K; ++i) {
                const uint16_t *qv = q + (((int64_t)b * K + i) * num_q_heads + h) * d;
                const int n_blk = (view == ORACLE_VIEW_DIFFUSION) ? K : i + 1;
                const int n = L + n_blk;
                /* scores over the cache */
                for (int j = 0; j < L; ++j) {
                    int32_t pg = page_table[(int64_t)b * max_pages_per_seq + j / page_size];
                    const uint16_t *kv = k_pool + (int64_t)pg * stride_page + (int64_t)g * stride_head +
                                         (int64_t)(j % page_size) * stride_tok;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(qv[c]) * bf16_to_f64(kv[c]);
                    s[j] = sm_scale * acc;
                }
                /* scores over the visible in-block keys */
                for (int r = 0; r < n_blk; ++r) {
                    const uint16_t *kv = k_blk + (((int64_t)b * K + r) * num_kv_heads + g) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(qv[c]) * bf16_to_f64(kv[c]);
                    s[L + r] = sm_scale * acc;
                }
                double mx = s[0];
                for (int j = 1; j < n; ++j) if (s[j] > mx) mx = s[j];
                double denom = 0.0;
                for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - mx); denom += s[j]; }
                double *o = out + (((int64_t)b * K + i) * num_q_heads + h) * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int j = 0; j < L; ++j) {
                    int32_t pg = page_table[(int64_t)b * max_pages_per_seq + j / page_size];
                    const uint16_t *vv = v_pool + (int64_t)pg * stride_page + (int64_t)g * stride_head +
                                         (int64_t)(j % page_size) * stride_tok;
                    double p = s[j] / denom;
                    for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f64(vv[c]);
                }
                for (int r = 0; r < n_blk; ++r) {
                    const uint16_t *vv = v_blk + (((int64_t)b * K + r) * num_kv_heads + g) * d;
                    double p = s[L + r] / denom;
                    for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f64(vv[c]);
                }
                if (lse) lse[((int64_t)b * num_q_heads + h) * K + i] = mx + log(denom);
            }
            free(s);
        }
    }
    return status;
}

/*
 * AR prefill of one attention layer (Section 3.1: the AR view processes the context with standard causal
 * self-attention and leaves its K/V in the cache).  Per sequence b with L = seq_lens[b] cached tokens
 * and n = new_lens[b] new tokens (0 <= n <= T):
 *   cache rows L..L+n-1 of KV head g  <-  k_new[b,i,g,:], v_new[b,i,g,:]      i = 0..n-1
 *   out[b,i,h,:] = sum_j softmax_j( sm_scale * <q[b,i,h,:], K_j> ) V_j  over cache tokens j = 0..L+i
 *   seq_lens[b] = L + n
 * i.e. the new token at position L+i sees everything before it and itself.  Rows i >= n of out are left
 * untouched.  q, out [B,T,H_q,d]; k_new, v_new [B,T,H_kv,d]; pools and page table as above (updated in
 * place).  If a needed page of sequence b is not mapped, that sequence's cache, length and output are left
 * untouched and -4 is returned after the other sequences were processed.  Returns 0, -1 or -4.
 */
int orthrus_oracle_prefill_attn(
    int batch, int max_new, int num_q_heads, int num_kv_heads, int head_dim,
    int page_size, int max_pages_per_seq, int64_t num_pages, double sm_scale,
    const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, const int32_t *new_lens,
    uint16_t *k_pool, uint16_t *v_pool,
    int64_t stride_page, int64_t stride_head, int64_t stride_tok,
    const int32_t *page_table, int32_t *seq_lens, double *out)
{
    if (batch < 0 || max_new < 0 || num_q_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 ||
        page_size <= 0 || num_q_heads % num_kv_heads != 0)
        return -1;
    const int G = num_q_heads / num_kv_heads, d = head_dim, T = max_new;
    int status = 0;
    for (int b = 0; b < batch; ++b) {
        const int L = seq_lens[b], n = new_lens[b];
        if (L < 0 || n < 0 || n > T) return -1;
    }
    for (int b = 0; b < batch; ++b) {
        const int L = seq_lens[b], n = new_lens[b];
        const int32_t *pt = page_table + (int64_t)b * max_pages_per_seq;
        int ok = 1;
        for (int j = 0; j < L + n && ok; j += page_size) {
            const int slot = j / page_size;
            if (slot >= max_pages_per_seq || pt[slot] < 0 || pt[slot] >= num_pages) ok = 0;
        }
        if (!ok) { status = -4; continue; }
        /* append the new tokens' K/V rows */
        for (int i = 0; i < n; ++i) {
            const int pos = L + i;
            const int64_t base = (int64_t)pt[pos / page_size] * stride_page + (int64_t)(pos % page_size) * stride_tok;
            for (int g = 0; g < num_kv_heads; ++g) {
                const uint16_t *ks = k_new + (((int64_t)b * T + i) * num_kv_heads + g) * d;
                const uint16_t *vs = v_new + (((int64_t)b * T + i) * num_kv_heads + g) * d;
                memcpy(k_pool + base + (int64_t)g * stride_head, ks, sizeof(uint16_t) * (size_t)d);
                memcpy(v_pool + base + (int64_t)g * stride_head, vs, sizeof(uint16_t) * (size_t)d);
            }
        }
        /* causal attention of every new token over the cache as it now stands */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int i = 0; i < n; ++i) {
            for (int h = 0; h < num_q_heads; ++h) {
                const int g = h / G, vis = L + i + 1;
                double *s = (double *)malloc(sizeof(double) * (size_t)vis);
                if (!s) {
#pragma omp atomic write
                    status = -1;
                    continue;
                }
                const uint16_t *qv = q + (((int64_t)b * T + i) * num_q_heads + h) * d;
                for (int j = 0; j < vis; ++j) {
                    const uint16_t *kv = k_pool + (int64_t)pt[j / page_size] * stride_page + (int64_t)g * stride_head +
                                         (int64_t)(j % page_size) * stride_tok;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(qv[c]) * bf16_to_f64(kv[c]);
                    s[j] = sm_scale * acc;
                }
                double mx = s[0];
                for (int j = 1; j < vis; ++j) if (s[j] > mx) mx = s[j];
                double denom = 0.0;
                for (int j = 0; j < vis; ++j) { s[j] = exp(s[j] - mx); denom += s[j]; }
                double *o = out + (((int64_t)b * T + i) * num_q_heads + h) * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int j = 0; j < vis; ++j) {
                    const uint16_t *vv = v_pool + (int64_t)pt[j / page_size] * stride_page + (int64_t)g * stride_head +
                                         (int64_t)(j % page_size) * stride_tok;
                    const double p = s[j] / denom;
                    for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f64(vv[c]);
                }
                free(s);
            }
        }
        seq_lens[b] = L + n;
    }
    return status;
}

/* 1 if logit a (at a lower index) must be replaced by logit b (at a higher index). */
static int later_is_better(float a, float b)
{
    if (isnan(a)) return 0;      /* first NaN wins, and a NaN beats every number */
    if (isnan(b)) return 1;
    return b > a;                /* strict: ties keep the smaller index */
}

/*
 * Greedy consensus (Eq. 8) and commit, per sequence b with L = seq_lens[b]:
 *   am[k]   = argmax_v ar_logits[b,k,v]                                   k = 0..K-1
 *   n_acc   = number of leading k with draft[b,k] == am[k]                (0..K)
 *   m       = min(n_acc + 1, K)       tokens emitted = am[0..m-1]
 *             (accepted drafts, then the AR correction at the first divergence; when all K
 *              drafts match there is no further logits row, so m = K)
 *   out_tokens[b,0..m-1] = am[0..m-1], the rest -1; next_anchor[b] = am[m-1]
 *   cache: rows 0..m-1 of the AR view's block K/V (the anchor and the accepted drafts that
 *          were fed to the verify pass) are written at token positions L..L+m-1; seq_lens[b]=L+m.
 * ar_logits [B,K,V] fp32; draft_tokens [B,K]; k_blk_ar/v_blk_ar [layers,B,K,H_kv,d] bf16 bits
 * or both NULL (consensus only: lengths and pools untouched); pools as in the attention
 * oracle plus stride_layer between layers.
 * If a position L..L+m-1 of some sequence is not mapped (slot >= max_pages_per_seq or page id
 * outside [0,num_pages)), that sequence's cache and length are left untouched, its
 * num_committed is 0, and the function returns -4 after finishing the other sequences.
 */
int orthrus_oracle_consensus_commit(
    int batch, int block_k, int vocab, int num_layers, int num_kv_heads, int head_dim,
    int page_size, int max_pages_per_seq, int64_t num_pages,
    const float *ar_logits, const int32_t *draft_tokens,
    const uint16_t *k_blk_ar, const uint16_t *v_blk_ar,
    uint16_t *k_pool, uint16_t *v_pool,
    int64_t stride_layer, int64_t stride_page, int64_t stride_head, int64_t stride_tok,
    const int32_t *page_table, int32_t *seq_lens,
    int32_t *accept_len, int32_t *num_committed, int32_t *out_tokens, int32_t *next_anchor)
{
    if (batch < 0 || block_k <= 0 || vocab <= 0) return -1;
    const int K = block_k;
    const int do_commit = (k_blk_ar != NULL && v_blk_ar != NULL);
    if (do_commit && (num_layers <= 0 || num_kv_heads <= 0 || head_dim <= 0 || page_size <= 0)) return -1;
    int status = 0;
    int32_t *am = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    if (!am) return -1;

    for (int b = 0; b < batch; ++b) {
        for (int k = 0; k < K; ++k) {
            const float *row = ar_logits + ((int64_t)b * K + k) * vocab;
            int best = 0;
            for (int v = 1; v < vocab; ++v)
                if (later_is_better(row[best], row[v])) best = v;
            am[k] = best;
        }
        int n_acc = 0;
        while (n_acc < K && draft_tokens[(int64_t)b * K + n_acc] == am[n_acc]) ++n_acc;
        const int m = (n_acc + 1 < K) ? n_acc + 1 : K;
        accept_len[b] = n_acc;
        for (int k = 0; k < K; ++k) out_tokens[(int64_t)b * K + k] = (k < m) ? am[k] : -1;
        next_anchor[b] = am[m - 1];
        num_committed[b] = m;
        if (!do_commit) continue;

        const int L = seq_lens[b];
        int mapped = (L >= 0);
        for (int k = 0; k < m && mapped; ++k) {
            int slot = (L + k) / page_size;
            if (slot >= max_pages_per_seq) { mapped = 0; break; }
            int32_t pg = page_table[(int64_t)b * max_pages_per_seq + slot];
            if (pg < 0 || pg >= num_pages) mapped = 0;
        }
        if (!mapped) { num_committed[b] = 0; status = -4; continue; }

        /* one appended row per emitted token, in order */
        for (int k = 0; k < m; ++k) {
            const int pos = L + k;
            const int32_t pg = page_table[(int64_t)b * max_pages_per_seq + pos / page_size];
            for (int layer = 0; layer < num_layers; ++layer) {
                for (int g = 0; g < num_kv_heads; ++g) {
                    int64_t dst = (int64_t)layer * stride_layer + (int64_t)pg * stride_page +
                                  (int64_t)g * stride_head + (int64_t)(pos % page_size) * stride_tok;
                    int64_t src = ((((int64_t)layer * batch + b) * K + k) * num_kv_heads + g) * head_dim;
                    memcpy(k_pool + dst, k_blk_ar + src, sizeof(uint16_t) * (size_t)head_dim);
                    memcpy(v_pool + dst, v_blk_ar + src, sizeof(uint16_t) * (size_t)head_dim);
                }
            }
        }
        seq_lens[b] = L + m;
    }
    free(am);
    return status;
}

/*
 * Lossless sampling consensus for temperature T > 0 (Section 3.3; the accept/replace rule is the
 * published speculative-sampling rule the paper cites, restated here):
 *   p_k = softmax(ar_logits[b,k,:] / T)     target distribution of block row k (AR view)
 *   q_k = softmax(diff_logits[b,k,:] / T)   distribution the draft token of row k was drawn from
 *   for k = 0, 1, ...: x = draft[b,k]; keep x iff  accept_u[b,k] * q_k(x) < p_k(x)
 *                      (probability min(1, p/q) for a uniform accept_u in [0,1); an x outside [0,V)
 *                      is never kept)
 *   at the first row j that is not kept, the emitted token is a draw from r = max(0, p_j - q_j)
 *   normalised, taken as  argmax_v [ log r(v) + gumbel[b,v] ]  (exact categorical sampling when
 *   gumbel holds independent standard Gumbel noise; smallest index on ties); if r is zero
 *   everywhere the draw is from p_j instead.
 *   n_acc = j (K if every draft is kept), m = min(n_acc + 1, K) tokens are emitted: the kept drafts,
 *   then the replacement when j < K.  Outputs and the commit are as in the greedy oracle.
 * All random numbers are inputs (accept_u [B,K], gumbel [B,V]); nothing is drawn here.
 * margin_accept [B,K] / margin_draw [B] (optional, may be NULL) report how far each decision was from
 * flipping: |log(u q(x)) - log p(x)| for the rows that were examined (0 for an out-of-range x, -1 for
 * rows not examined), and the gap between the best and second-best score of the draw (-1 if none).
 */
int orthrus_oracle_sampling_consensus_commit(
    int batch, int block_k, int vocab, double temperature, int num_layers, int num_kv_heads, int head_dim,
    int page_size, int max_pages_per_seq, int64_t num_pages,
    const float *ar_logits, const float *diff_logits, const int32_t *draft_tokens,
    const float *accept_u, const float *gumbel,
    const uint16_t *k_blk_ar, const uint16_t *v_blk_ar,
    uint16_t *k_pool, uint16_t *v_pool,
    int64_t stride_layer, int64_t stride_page, int64_t stride_head, int64_t stride_tok,
    const int32_t *page_table, int32_t *seq_lens,
    int32_t *accept_len, int32_t *num_committed, int32_t *out_tokens, int32_t *next_anchor,
    double *margin_accept, double *margin_draw)
{
    if (batch < 0 || block_k <= 0 || vocab <= 0 || !(temperature > 0.0)) return -1;
    const int K = block_k, V = vocab;
    const int do_commit = (k_blk_ar != NULL && v_blk_ar != NULL);
    if (do_commit && (num_layers <= 0 || num_kv_heads <= 0 || head_dim <= 0 || page_size <= 0)) return -1;
    int status = 0;
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    if (!lp || !lq) { free(lp); free(lq); return -1; }

    for (int b = 0; b < batch; ++b) {
        int n_acc = K;
        int replacement = -1;
        if (margin_draw) margin_draw[b] = -1.0;
        for (int k = 0; k < K; ++k)
            if (margin_accept) margin_accept[(int64_t)b * K + k] = -1.0;
        for (int k = 0; k < K; ++k) {
            const float *pr = ar_logits + ((int64_t)b * K + k) * V;
            const float *qr = diff_logits + ((int64_t)b * K + k) * V;
            /* log-softmax of both rows at temperature T (two passes: max, then log-sum-exp) */
            double mp = -INFINITY, mq = -INFINITY;
            for (int v = 0; v < V; ++v) {
                lp[v] = (double)pr[v] / temperature;
                lq[v] = (double)qr[v] / temperature;
                if (lp[v] > mp) mp = lp[v];
                if (lq[v] > mq) mq = lq[v];
            }
            double sp = 0.0, sq = 0.0;
            for (int v = 0; v < V; ++v) { sp += exp(lp[v] - mp); sq += exp(lq[v] - mq); }
            const double lsep = mp + log(sp), lseq = mq + log(sq);
            const int32_t x = draft_tokens[(int64_t)b * K + k];
            int keep = 0;
            if (x >= 0 && x < V) {
                const double px = exp(lp[x] - lsep), qx = exp(lq[x] - lseq);
                const double u = (double)accept_u[(int64_t)b * K + k];
                keep = (u * qx < px);
                if (margin_accept) {
                    const double a = log(u * qx), c = log(px);   /* -inf when a factor is zero */
                    margin_accept[(int64_t)b * K + k] = (isinf(a) && isinf(c)) ? 0.0 : fabs(a - c);
                }
            } else if (margin_accept) {
                margin_accept[(int64_t)b * K + k] = 0.0;
            }
            if (keep) continue;
            /* first rejection: draw the replacement from the positive part of p - q */
            n_acc = k;
            double best = -INFINITY, second = -INFINITY;
            int best_v = -1, any = 0;
            for (int v = 0; v < V; ++v) {
                const double r = exp(lp[v] - lsep) - exp(lq[v] - lseq);
                if (r > 0.0) any = 1;
            }
            for (int v = 0; v < V; ++v) {
                double w;
                if (any) {
                    const double r = exp(lp[v] - lsep) - exp(lq[v] - lseq);
                    if (!(r > 0.0)) continue;
                    w = log(r);
                } else {
                    w = lp[v] - lsep;
                }
                const double score = w + (double)gumbel[(int64_t)b * V + v];
                if (score > best) { second = best; best = score; best_v = v; }
                else if (score > second) second = score;
            }
            replacement = best_v;
            if (margin_draw) margin_draw[b] = isinf(second) ? INFINITY : best - second;
            break;
        }
        const int m = (n_acc + 1 < K) ? n_acc + 1 : K;
        accept_len[b] = n_acc;
        for (int k = 0; k < K; ++k) {
            int32_t t = -1;
            if (k < n_acc) t = draft_tokens[(int64_t)b * K + k];
            else if (k == n_acc && k < m) t = replacement;
            out_tokens[(int64_t)b * K + k] = (k < m) ? t : -1;
        }
        next_anchor[b] = out_tokens[(int64_t)b * K + m - 1];
        num_committed[b] = m;
        if (!do_commit) continue;

        const int L = seq_lens[b];
        int mapped = (L >= 0);
        for (int k = 0; k < m && mapped; ++k) {
            int slot = (L + k) / page_size;
            if (slot >= max_pages_per_seq) { mapped = 0; break; }
            int32_t pg = page_table[(int64_t)b * max_pages_per_seq + slot];
            if (pg < 0 || pg >= num_pages) mapped = 0;
        }
        if (!mapped) { num_committed[b] = 0; status = -4; continue; }
        for (int k = 0; k < m; ++k) {
            const int pos = L + k;
            const int32_t pg = page_table[(int64_t)b * max_pages_per_seq + pos / page_size];
            for (int layer = 0; layer < num_layers; ++layer) {
                for (int g = 0; g < num_kv_heads; ++g) {
                    int64_t dst = (int64_t)layer * stride_layer + (int64_t)pg * stride_page +
                                  (int64_t)g * stride_head + (int64_t)(pos % page_size) * stride_tok;
                    int64_t src = ((((int64_t)layer * batch + b) * K + k) * num_kv_heads + g) * head_dim;
                    memcpy(k_pool + dst, k_blk_ar + src, sizeof(uint16_t) * (size_t)head_dim);
                    memcpy(v_pool + dst, v_blk_ar + src, sizeof(uint16_t) * (size_t)head_dim);
                }
            }
        }
        seq_lens[b] = L + m;
    }
    free(lp);
    free(lq);
    return status;
}
