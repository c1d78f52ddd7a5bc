/*
 * CPU oracle for the Speculative Thinking hot path (test infrastructure only).
 *
 * This is the slow, plain definition of what the GPU library computes: the
 * autoregressive step of a Qwen2.5-architecture decoder with a KV cache (the
 * paper's "decode" and "prefix" passes, Section 4 / Table 3 / Eq. 1) and the
 * integer trigger predicate of the takeover rule (Section 3 (1), Appendix C).
 * Storage is fp32, every reduction (dot product, sum of squares, softmax
 * normaliser, weighted value sum) accumulates in fp64.
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * link or load this file.  It shares nothing with the HIP library: no header,
 * no table, no helper.
 */
#ifndef ST_ORACLE_H
#define ST_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
    float rms_eps, rope_theta;
    int32_t qkv_bias; /* 1: q/k/v projections carry a bias */
    int32_t max_seq;  /* KV cache capacity in positions */
} orc_config;

/* All tensors are host fp32, row-major [out][in]; per-layer arrays have
 * n_layers entries.  The oracle borrows the pointers (no copy). */
typedef struct {
    const float *embed;      /* [vocab][hidden] */
    const float *lm_head;    /* [vocab][hidden]; may alias embed (tied) */
    const float *final_norm; /* [hidden] */
    const float *const *wq;  /* [n_q_heads*head_dim][hidden] */
    const float *const *wk;  /* [n_kv_heads*head_dim][hidden] */
    const float *const *wv;  /* [n_kv_heads*head_dim][hidden] */
    const float *const *bq;  /* [n_q_heads*head_dim] (ignored if !qkv_bias) */
    const float *const *bk;
    const float *const *bv;
    const float *const *wo;  /* [hidden][n_q_heads*head_dim] */
    const float *const *wg;  /* [intermediate][hidden] */
    const float *const *wu;  /* [intermediate][hidden] */
    const float *const *wd;  /* [hidden][intermediate] */
    const float *const *norm_attn; /* [hidden] */
    const float *const *norm_mlp;  /* [hidden] */
} orc_weights;

typedef struct orc_model orc_model;

/* Returns NULL on bad config or allocation failure. */
orc_model *orc_create(const orc_config *cfg, const orc_weights *w);
void orc_destroy(orc_model *m);
int32_t orc_kv_len(const orc_model *m);
/* 0 on success, -1 if new_len is outside [0, kv_len]. */
int orc_kv_truncate(orc_model *m, int32_t new_len);

/* Feed n tokens at positions [kv_len, kv_len+n) as n successive single-token
 * steps (position-outer, layer-inner).  logits_last (fp32[vocab], may be NULL)
 * receives the logits of the last position; logits_all (fp32[n][vocab], may be
 * NULL) those of every fed position.  Returns 0, or -1 on overflow / bad id. */
int orc_feed(orc_model *m, const int32_t *tokens, int32_t n, float *logits_last, float *logits_all);

/* Same function of the same inputs, evaluated layer-outer over the whole
 * block (a causal pass over n rows on top of the existing cache). */
int orc_feed_block(orc_model *m, const int32_t *tokens, int32_t n, float *logits_last, float *logits_all);

/* Number of threads the matvec loops actually use. */
int orc_threads(void);

/* --- primitives, exported so that each can be pinned on its own --- */
void orc_rmsnorm(const float *x, const float *g, int32_t n, float eps, float *out);
/* rotate-half RoPE of one head vector (length d) at absolute position pos. */
void orc_rope(float *v, int32_t d, int32_t pos, float theta);
/* in-place softmax of n scores. */
void orc_softmax(float *s, int32_t n);
float orc_silu(float z);
/* lowest index of the maximum; NaN entries never win; -1 if n <= 0 or all NaN. */
int32_t orc_argmax(const float *v, int32_t n);
/* GQA attention of one query token over t cached keys.
 * q [nq][d]; K, V [t][nkv][d]; out [nq][d].  Query head h uses kv head h/(nq/nkv). */
void orc_attention(const float *q, const float *K, const float *V, int32_t t,
                   int32_t nq, int32_t nkv, int32_t d, float *out);
/* Positions p in [lo,hi) where the token-level takeover rule holds (Section 3 (1)).  window == 1: tokens[p] is in
 * the keyword set.  window == w + 1 >= 2: the w tokens ending at p are the sentence that follows a delimiter
 * (tokens[p-w] is in the delimiter set, none of tokens[p-w+1 .. p-1] is) and at least one of them is a keyword; the
 * look-back may reach before lo but not before position 0.  Bitmaps: bit (id&31) of word id>>5.  Writes the first
 * min(count,cap) positions ascending; returns the total count, or -1 on a token id outside [0, vocab). */
int32_t orc_trigger_scan(const int32_t *tokens, int32_t lo, int32_t hi, int32_t vocab,
                         const uint32_t *kw, const uint32_t *delim, int32_t window,
                         int32_t *positions, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif
