/*
 * Sanitizer driver of the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Built together with orthrus_oracle.c under -fsanitize=address,undefined and run by the CPU test suite:
 * every oracle entry point is called on small seeded problems whose buffers are heap blocks of exactly
 * the documented sizes, so that a read or write one element outside any of them, a signed overflow or
 * a misaligned access ends the process with a report.  Ragged lengths, an empty sequence, a page size
 * above the block size, several layers and the capacity-error path are included.  No result is checked
 * here (the pins in tests/ do that); the exit status is 0 when every call returned what was expected.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orthrus_oracle_dual_view_attn(int, int, int, int, int, int, int, int64_t, int, double, const uint16_t *,
                                  const uint16_t *, const uint16_t *, const uint16_t *, const uint16_t *, int64_t,
                                  int64_t, int64_t, const int32_t *, const int32_t *, double *, double *);
int orthrus_oracle_prefill_attn(int, int, int, int, int, int, int, int64_t, double, const uint16_t *, const uint16_t *,
                                const uint16_t *, const int32_t *, uint16_t *, uint16_t *, int64_t, int64_t, int64_t,
                                const int32_t *, int32_t *, double *);
int orthrus_oracle_consensus_commit(int, int, int, int, int, int, int, int, int64_t, const float *, const int32_t *,
                                    const uint16_t *, const uint16_t *, uint16_t *, uint16_t *, int64_t, int64_t,
                                    int64_t, int64_t, const int32_t *, int32_t *, int32_t *, int32_t *, int32_t *,
                                    int32_t *);
int orthrus_oracle_sampling_consensus_commit(int, int, int, double, int, int, int, int, int, int64_t, const float *,
                                             const float *, const int32_t *, const float *, const float *,
                                             const uint16_t *, const uint16_t *, uint16_t *, uint16_t *, int64_t,
                                             int64_t, int64_t, int64_t, const int32_t *, int32_t *, int32_t *,
                                             int32_t *, int32_t *, int32_t *, double *, double *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float unit(void) { return (float)(rnd() & 0xFFFFFF) / 16777216.0f; }
static uint16_t bf16_small(void)
{ /* a finite bf16 in about [-2, 2): sign, exponent 125..127, 7 mantissa bits */
    return (uint16_t)(((rnd() & 1u) << 15) | ((125u + rnd() % 3u) << 7) | (rnd() & 0x7Fu));
}
static uint16_t *bf16_block(size_t n)
{
    uint16_t *p = (uint16_t *)malloc(n * sizeof *p + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = bf16_small();
    return p;
}
static float *f32_block(size_t n, float scale)
{
    float *p = (float *)malloc(n * sizeof *p + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = (unit() - 0.5f) * scale;
    return p;
}

static int fails = 0;
#define EXPECT(call, want)                                                         \
    do {                                                                           \
        int rc_ = (call);                                                          \
        if (rc_ != (want)) { printf("line %d: returned %d, expected %d\n", __LINE__, rc_, (want)); ++fails; } \
    } while (0)

static void one_shape(int B, int Hq, int Hkv, int d, int K, int P, int layers, int V, const int *lens, int starve)
{
    int max_len = 0;
    for (int b = 0; b < B; ++b) if (lens[b] > max_len) max_len = lens[b];
    const int T = 5;                                       /* new tokens per sequence in the prefill call */
    const int max_pages = (max_len + K + T + P - 1) / P;   /* room for one commit and one prefill */
    const int64_t pages = (int64_t)B * max_pages;
    const int64_t s_tok = d, s_head = (int64_t)P * d, s_page = (int64_t)Hkv * P * d, s_layer = pages * s_page;
    uint16_t *kp = bf16_block((size_t)(layers * s_layer)), *vp = bf16_block((size_t)(layers * s_layer));
    int32_t *pt = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * max_pages));
    for (int i = 0; i < B * max_pages; ++i) pt[i] = (int32_t)((i * 7 + 3) % pages);   /* a permutation-like map */
    for (int i = 0; i < B * max_pages; ++i) pt[i] = (int32_t)i;
    for (int i = B * max_pages - 1; i > 0; --i) { int j = (int)(rnd() % (uint32_t)(i + 1)); int32_t t = pt[i]; pt[i] = pt[j]; pt[j] = t; }
    int32_t *sl = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    memcpy(sl, lens, sizeof(int32_t) * (size_t)B);
    uint16_t *q = bf16_block((size_t)B * K * Hq * d), *kb = bf16_block((size_t)layers * B * K * Hkv * d),
             *vb = bf16_block((size_t)layers * B * K * Hkv * d);
    double *out = (double *)malloc(sizeof(double) * (size_t)B * K * Hq * d), *lse = (double *)malloc(sizeof(double) * (size_t)B * Hq * K);
    for (int view = 0; view < 2; ++view) {
        EXPECT(orthrus_oracle_dual_view_attn(B, Hq, Hkv, d, K, P, max_pages, pages, view, 0.125, q, kb, vb, kp, vp, s_page,
                                             s_head, s_tok, pt, sl, out, lse), 0);
        EXPECT(orthrus_oracle_dual_view_attn(B, Hq, Hkv, d, K, P, max_pages, pages, view, 0.125, q, kb, vb, kp, vp, s_page,
                                             s_head, s_tok, pt, sl, out, NULL), 0);
    }
    /* greedy consensus: consensus only, then with commit into every layer */
    float *logits = f32_block((size_t)B * K * V, 8.0f), *dlogits = f32_block((size_t)B * K * V, 8.0f);
    int32_t *draft = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * K);
    for (int i = 0; i < B * K; ++i) draft[i] = (int32_t)(rnd() % (uint32_t)(V + 2)) - 1;   /* includes -1 and V */
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)B), *ncm = (int32_t *)malloc(sizeof(int32_t) * (size_t)B),
            *anc = (int32_t *)malloc(sizeof(int32_t) * (size_t)B), *toks = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * K);
    EXPECT(orthrus_oracle_consensus_commit(B, K, V, 0, 0, 0, 0, 0, 0, logits, draft, NULL, NULL, NULL, NULL, 0, 0, 0, 0, NULL,
                                           NULL, acc, ncm, toks, anc), 0);
    if (starve) pt[0 * max_pages + (lens[0] / P)] = -1;   /* the first sequence cannot grow: capacity error */
    EXPECT(orthrus_oracle_consensus_commit(B, K, V, layers, Hkv, d, P, max_pages, pages, logits, draft, kb, vb, kp, vp, s_layer,
                                           s_page, s_head, s_tok, pt, sl, acc, ncm, toks, anc), starve ? -4 : 0);
    /* sampling consensus with commit */
    float *u = f32_block((size_t)B * K, 1.0f), *gum = f32_block((size_t)B * V, 6.0f);
    for (int i = 0; i < B * K; ++i) u[i] = unit();
    double *ma = (double *)malloc(sizeof(double) * (size_t)B * K), *md = (double *)malloc(sizeof(double) * (size_t)B);
    EXPECT(orthrus_oracle_sampling_consensus_commit(B, K, V, 0.7, layers, Hkv, d, P, max_pages, pages, logits, dlogits, draft, u,
                                                    gum, kb, vb, kp, vp, s_layer, s_page, s_head, s_tok, pt, sl, acc, ncm, toks,
                                                    anc, ma, md), starve ? -4 : 0);
    EXPECT(orthrus_oracle_sampling_consensus_commit(B, K, V, 1.3, 0, 0, 0, 0, 0, 0, logits, dlogits, draft, u, gum, NULL, NULL, NULL,
                                                    NULL, 0, 0, 0, 0, NULL, NULL, acc, ncm, toks, anc, NULL, NULL), 0);
    /* prefill of up to T new tokens per sequence on top of the (grown) cache, layer 0 */
    if (!starve) {
        uint16_t *qn = bf16_block((size_t)B * T * Hq * d), *kn = bf16_block((size_t)B * T * Hkv * d), *vn = bf16_block((size_t)B * T * Hkv * d);
        int32_t *nl = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
        for (int b = 0; b < B; ++b) {
            const int room = max_pages * P - sl[b];
            nl[b] = (int32_t)(rnd() % (uint32_t)(T + 1));
            if (nl[b] > room) nl[b] = room;
        }
        double *po = (double *)malloc(sizeof(double) * (size_t)B * T * Hq * d);
        EXPECT(orthrus_oracle_prefill_attn(B, T, Hq, Hkv, d, P, max_pages, pages, 0.125, qn, kn, vn, nl, kp, vp, s_page, s_head, s_tok,
                                           pt, sl, po), 0);
        free(qn); free(kn); free(vn); free(nl); free(po);
    }
    free(kp); free(vp); free(pt); free(sl); free(q); free(kb); free(vb); free(out); free(lse); free(logits); free(dlogits);
    free(draft); free(acc); free(ncm); free(anc); free(toks); free(u); free(gum); free(ma); free(md);
}

int main(void)
{
    const int a[] = {0, 1, 31, 70};
    one_shape(4, 4, 2, 64, 4, 16, 1, 97, a, 0);
    const int b[] = {17, 33};
    one_shape(2, 6, 2, 32, 7, 32, 3, 513, b, 0);
    const int c[] = {15, 40, 5};
    one_shape(3, 2, 2, 16, 5, 16, 2, 64, c, 1);
    const int e[] = {0};
    one_shape(1, 1, 1, 8, 1, 16, 1, 3, e, 0);
    if (fails) { printf("%d unexpected return codes\n", fails); return 1; }
    printf("oracle sanitizer self-test ok\n");
    return 0;
}
