/* Exercises every entry point of the CPU oracle on a tiny seeded model; built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py, so that an out-of-bounds access, a
 * use-after-free, a leak or undefined integer / pointer arithmetic anywhere in the oracle fails the CPU
 * test run.  Exit status 0 = every check held. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/st_oracle.h"

static uint32_t rng_state = 12345u;
static float rnd(void) { /* uniform in [-0.05, 0.05) */
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) / 16777216.0f - 0.5f) * 0.1f;
}
static float *tensor(size_t n, float offset) {
    float *p = (float *)malloc(sizeof(float) * n);
    if (!p) exit(2);
    for (size_t i = 0; i < n; ++i) p[i] = offset + rnd();
    return p;
}
#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); \
            return 1;                                                   \
        }                                                               \
    } while (0)

enum { L = 2, H = 48, NQ = 4, NKV = 2, D = 12, I = 40, V = 37, MAXSEQ = 24 };

int main(void) {
    orc_config c = {L, H, NQ, NKV, D, I, V, 1e-6f, 1e6f, 1, MAXSEQ};
    float *embed = tensor((size_t)V * H, 0.f), *head = tensor((size_t)V * H, 0.f), *fnorm = tensor(H, 1.f);
    const float *wq[L], *wk[L], *wv[L], *bq[L], *bk[L], *bv[L], *wo[L], *wg[L], *wu[L], *wd[L], *na[L], *nm[L];
    for (int l = 0; l < L; ++l) {
        wq[l] = tensor((size_t)NQ * D * H, 0.f), wk[l] = tensor((size_t)NKV * D * H, 0.f);
        wv[l] = tensor((size_t)NKV * D * H, 0.f), bq[l] = tensor(NQ * D, 0.f), bk[l] = tensor(NKV * D, 0.f);
        bv[l] = tensor(NKV * D, 0.f), wo[l] = tensor((size_t)H * NQ * D, 0.f), wg[l] = tensor((size_t)I * H, 0.f);
        wu[l] = tensor((size_t)I * H, 0.f), wd[l] = tensor((size_t)H * I, 0.f);
        na[l] = tensor(H, 1.f), nm[l] = tensor(H, 1.f);
    }
    orc_weights w = {embed, head, fnorm, wq, wk, wv, bq, bk, bv, wo, wg, wu, wd, na, nm};
    CHECK(orc_create(NULL, &w) == NULL);
    orc_config bad = c;
    bad.n_q_heads = 3; /* not a multiple of the kv heads */
    CHECK(orc_create(&bad, &w) == NULL);
    orc_model *a = orc_create(&c, &w), *b = orc_create(&c, &w);
    CHECK(a && b);
    CHECK(orc_threads() >= 1);

    int32_t toks[MAXSEQ];
    for (int i = 0; i < MAXSEQ; ++i) toks[i] = (i * 7 + 3) % V;
    float *la = (float *)malloc(sizeof(float) * V), *lb = (float *)malloc(sizeof(float) * V);
    float *all = (float *)malloc(sizeof(float) * (size_t)MAXSEQ * V);
    CHECK(la && lb && all);
    /* token by token against block-wise, ragged splits, up to the very last cache position */
    CHECK(orc_feed(a, toks, 9, la, all) == 0);
    CHECK(orc_feed_block(b, toks, 4, NULL, NULL) == 0 && orc_feed_block(b, toks + 4, 5, lb, NULL) == 0);
    for (int i = 0; i < V; ++i) CHECK(fabsf(la[i] - lb[i]) <= 1e-5f && la[i] == all[8 * V + i]);
    CHECK(orc_feed(a, toks + 9, MAXSEQ - 9, la, NULL) == 0 && orc_kv_len(a) == MAXSEQ);
    CHECK(orc_feed(a, toks, 1, la, NULL) == -1);             /* cache full */
    CHECK(orc_feed_block(b, toks + 9, MAXSEQ - 9, lb, all) == 0);
    for (int i = 0; i < V; ++i) CHECK(fabsf(la[i] - lb[i]) <= 1e-5f);
    CHECK(orc_feed_block(b, toks, 1, NULL, NULL) == -1);
    /* rollback and refeed reproduces the logits exactly */
    CHECK(orc_kv_truncate(a, MAXSEQ + 1) == -1 && orc_kv_truncate(a, -1) == -1);
    CHECK(orc_kv_truncate(a, 11) == 0 && orc_feed(a, toks + 11, MAXSEQ - 11, lb, NULL) == 0);
    for (int i = 0; i < V; ++i) CHECK(la[i] == lb[i]);
    int32_t bad_tok = V;
    CHECK(orc_kv_truncate(a, 0) == 0 && orc_feed(a, &bad_tok, 1, la, NULL) == -1 && orc_feed(a, toks, 0, la, NULL) == -1);

    /* primitives at their smallest sizes */
    float one[2] = {3.f, -4.f}, g2[2] = {1.f, 1.f}, out2[2];
    orc_rmsnorm(one, g2, 2, 0.f, out2);
    CHECK(fabsf(out2[0] * out2[0] + out2[1] * out2[1] - 2.f) < 1e-5f);
    orc_rope(one, 2, 5, 1e6f);
    CHECK(fabsf(one[0] * one[0] + one[1] * one[1] - 25.f) < 1e-4f);
    float s1[1] = {123.f};
    orc_softmax(s1, 1);
    CHECK(s1[0] == 1.f && orc_argmax(s1, 1) == 0 && orc_argmax(s1, 0) == -1);
    CHECK(fabsf(orc_silu(1.f) - 0.7310586f) < 1e-6f);
    float q[NQ * D], K[3 * NKV * D], Vv[3 * NKV * D], o[NQ * D];
    for (int i = 0; i < NQ * D; ++i) q[i] = rnd();
    for (int i = 0; i < 3 * NKV * D; ++i) K[i] = rnd(), Vv[i] = rnd();
    orc_attention(q, K, Vv, 1, NQ, NKV, D, o);
    for (int h = 0; h < NQ; ++h)
        for (int i = 0; i < D; ++i) CHECK(fabsf(o[h * D + i] - Vv[(h / (NQ / NKV)) * D + i]) < 1e-6f);
    orc_attention(q, K, Vv, 3, NQ, NKV, D, o);

    /* trigger scan: ranges touching both ends, every window up to the range length, cap below the count */
    uint32_t kw[2] = {0, 0}, dl[2] = {0, 0};
    for (int id = 0; id < V; id += 3) kw[id >> 5] |= 1u << (id & 31);
    for (int id = 1; id < V; id += 4) dl[id >> 5] |= 1u << (id & 31);
    int32_t pos[MAXSEQ];
    for (int win = 1; win <= MAXSEQ + 1; ++win)
        for (int lo = 0; lo <= MAXSEQ; lo += 5) {
            int32_t n = orc_trigger_scan(toks, lo, MAXSEQ, V, kw, dl, win, pos, MAXSEQ);
            CHECK(n >= 0 && n <= MAXSEQ - lo);
            int32_t n2 = orc_trigger_scan(toks, lo, MAXSEQ, V, kw, dl, win, pos, 1);
            CHECK(n2 == n && orc_trigger_scan(toks, lo, lo, V, kw, dl, win, NULL, 0) == 0);
        }
    toks[3] = V + 5;
    CHECK(orc_trigger_scan(toks, 0, MAXSEQ, V, kw, dl, 1, pos, MAXSEQ) == -1);

    orc_destroy(a);
    orc_destroy(b);
    orc_destroy(NULL);
    free(la), free(lb), free(all);
    free(embed), free(head), free(fnorm);
    for (int l = 0; l < L; ++l) {
        free((void *)wq[l]), free((void *)wk[l]), free((void *)wv[l]), free((void *)bq[l]), free((void *)bk[l]);
        free((void *)bv[l]), free((void *)wo[l]), free((void *)wg[l]), free((void *)wu[l]), free((void *)wd[l]);
        free((void *)na[l]), free((void *)nm[l]);
    }
    puts("oracle sanitizer driver: ok");
    return 0;
}
