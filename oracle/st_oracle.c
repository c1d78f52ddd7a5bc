/*
 * CPU oracle for the Speculative Thinking hot path (test infrastructure only;
 * see st_oracle.h).  Plain C, fp32 storage, fp64 reductions, OpenMP over the
 * output rows of each matrix-vector product and nothing cleverer than that.
 *
 * What is computed, per fed position p (the paper's decode / prefix pass with
 * the key-value cache enabled, Section 4, Table 3 and Eq. 1, on the Qwen-2.5
 * decoder its experiments use):
 *
 *   x = E[tok]
 *   for each layer:
 *     y = rmsnorm(x, g_attn);  q,k,v = Wq y + bq, Wk y + bk, Wv y + bv
 *     rotate-half RoPE on every q and k head at position p; append k,v to the cache
 *     o_h = sum_{j<=p} softmax_j(q_h . k_{g(h),j} / sqrt(d)) v_{g(h),j},  g(h) = h / (nq/nkv)
 *     x += Wo o;  y = rmsnorm(x, g_mlp);  x += Wd (silu(Wg y) * (Wu y))
 *   logits = W_lm rmsnorm(x, g_final)
 */
#include "st_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

struct orc_model {
    orc_config c;
    orc_weights w;
    int32_t kv_len;
    float *kcache; /* [L][max_seq][nkv*d] */
    float *vcache;
};

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* out[r] = W[r,:] . x (+ b[r]) */
static void matvec(const float *W, const float *b, const float *x, int32_t rows, int32_t cols, float *out) {
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < rows; ++r) {
        const float *wr = W + (size_t)r * cols;
        double acc = 0.0;
        for (int32_t c = 0; c < cols; ++c) acc += (double)wr[c] * (double)x[c];
        if (b) acc += (double)b[r];
        out[r] = (float)acc;
    }
}

void orc_rmsnorm(const float *x, const float *g, int32_t n, float eps, float *out) {
    double ss = 0.0;
    for (int32_t i = 0; i < n; ++i) ss += (double)x[i] * (double)x[i];
    double inv = 1.0 / sqrt(ss / (double)n + (double)eps);
    for (int32_t i = 0; i < n; ++i) out[i] = (float)((double)x[i] * inv * (double)g[i]);
}

void orc_rope(float *v, int32_t d, int32_t pos, float theta) {
    int32_t half = d / 2;
    for (int32_t i = 0; i < half; ++i) {
        double freq = pow((double)theta, -2.0 * (double)i / (double)d);
        double a = (double)pos * freq;
        double c = cos(a), s = sin(a);
        double lo = v[i], hi = v[i + half];
        v[i] = (float)(lo * c - hi * s);
        v[i + half] = (float)(hi * c + lo * s);
    }
}

void orc_softmax(float *s, int32_t n) {
    if (n <= 0) return;
    double mx = s[0];
    for (int32_t i = 1; i < n; ++i)
        if (s[i] > mx) mx = s[i];
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += exp((double)s[i] - mx);
    for (int32_t i = 0; i < n; ++i) s[i] = (float)(exp((double)s[i] - mx) / sum);
}

float orc_silu(float z) { return (float)((double)z / (1.0 + exp(-(double)z))); }

int32_t orc_argmax(const float *v, int32_t n) {
    int32_t best = -1;
    for (int32_t i = 0; i < n; ++i) {
        if (v[i] != v[i]) continue; /* NaN never wins */
        if (best < 0 || v[i] > v[best]) best = i;
    }
    return best;
}

/* Attention of one query token; K and V rows have stride `stride` floats per position. */
static void attention_strided(const float *q, const float *K, const float *V, int32_t t, int32_t stride,
                              int32_t nq, int32_t nkv, int32_t d, float *out) {
    int32_t group = nq / nkv;
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(static)
    for (int32_t h = 0; h < nq; ++h) {
        int32_t g = h / group;
        const float *qh = q + (size_t)h * d;
        float *p = (float *)malloc(sizeof(float) * (size_t)(t > 0 ? t : 1));
        for (int32_t j = 0; j < t; ++j) {
            const float *kj = K + (size_t)j * stride + (size_t)g * d;
            double acc = 0.0;
            for (int32_t i = 0; i < d; ++i) acc += (double)qh[i] * (double)kj[i];
            p[j] = (float)(acc * scale);
        }
        orc_softmax(p, t);
        for (int32_t i = 0; i < d; ++i) {
            double acc = 0.0;
            for (int32_t j = 0; j < t; ++j) acc += (double)p[j] * (double)V[(size_t)j * stride + (size_t)g * d + i];
            out[(size_t)h * d + i] = (float)acc;
        }
        free(p);
    }
}

void orc_attention(const float *q, const float *K, const float *V, int32_t t,
                   int32_t nq, int32_t nkv, int32_t d, float *out) {
    attention_strided(q, K, V, t, nkv * d, nq, nkv, d, out);
}

int32_t orc_trigger_scan(const int32_t *tokens, int32_t lo, int32_t hi, int32_t vocab,
                         const uint32_t *kw, const uint32_t *delim, int32_t window,
                         int32_t *positions, int32_t cap) {
    int32_t count = 0;
    for (int32_t p = lo; p < hi; ++p) {
        int32_t id = tokens[p];
        if (id < 0 || id >= vocab) return -1;
        int fire;
        if (window == 1) {
            fire = (kw[id >> 5] >> (id & 31)) & 1u;
        } else {
            /* the sentence of w = window - 1 tokens that ends at p: a delimiter right before it, no
             * delimiter inside it before its last token, and a keyword somewhere in it */
            int32_t w = window - 1, first = p - w + 1;
            fire = 0;
            if (first >= 1) {
                int32_t d = tokens[first - 1];
                if (d < 0 || d >= vocab) return -1;
                int ok = (delim[d >> 5] >> (d & 31)) & 1u, any = 0;
                for (int32_t q = first; q <= p; ++q) {
                    int32_t t = tokens[q];
                    if (t < 0 || t >= vocab) return -1;
                    if (q < p && ((delim[t >> 5] >> (t & 31)) & 1u)) ok = 0;
                    if ((kw[t >> 5] >> (t & 31)) & 1u) any = 1;
                }
                fire = ok && any;
            }
        }
        if (fire) {
            if (count < cap && positions) positions[count] = p;
            ++count;
        }
    }
    return count;
}

orc_model *orc_create(const orc_config *cfg, const orc_weights *w) {
    if (!cfg || !w) return NULL;
    if (cfg->n_layers <= 0 || cfg->hidden <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 ||
        cfg->head_dim <= 0 || (cfg->head_dim & 1) || cfg->intermediate <= 0 || cfg->vocab <= 0 ||
        cfg->max_seq <= 0 || cfg->n_q_heads % cfg->n_kv_heads != 0)
        return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    if (!m) return NULL;
    m->c = *cfg;
    m->w = *w;
    size_t n = (size_t)cfg->n_layers * cfg->max_seq * cfg->n_kv_heads * cfg->head_dim;
    m->kcache = (float *)calloc(n, sizeof(float));
    m->vcache = (float *)calloc(n, sizeof(float));
    if (!m->kcache || !m->vcache) {
        orc_destroy(m);
        return NULL;
    }
    return m;
}

void orc_destroy(orc_model *m) {
    if (!m) return;
    free(m->kcache);
    free(m->vcache);
    free(m);
}

int32_t orc_kv_len(const orc_model *m) { return m ? m->kv_len : -1; }

int orc_kv_truncate(orc_model *m, int32_t new_len) {
    if (!m || new_len < 0 || new_len > m->kv_len) return -1;
    m->kv_len = new_len;
    return 0;
}

static int check_feed(const orc_model *m, const int32_t *tokens, int32_t n) {
    if (!m || !tokens || n <= 0) return -1;
    if ((int64_t)m->kv_len + n > m->c.max_seq) return -1;
    for (int32_t i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->c.vocab) return -1;
    return 0;
}

/* One layer applied to the residual x of the token at position pos (cache rows < pos are valid). */
static void layer_step(orc_model *m, int32_t l, int32_t pos, float *x, float *y, float *q, float *o, float *gate,
                       float *up, float *tmp) {
    const orc_config *c = &m->c;
    const orc_weights *w = &m->w;
    int32_t h = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, I = c->intermediate;
    int32_t kvw = nkv * d;
    float *Kl = m->kcache + (size_t)l * c->max_seq * kvw;
    float *Vl = m->vcache + (size_t)l * c->max_seq * kvw;
    float *kp = Kl + (size_t)pos * kvw;
    float *vp = Vl + (size_t)pos * kvw;

    orc_rmsnorm(x, w->norm_attn[l], h, c->rms_eps, y);
    matvec(w->wq[l], c->qkv_bias ? w->bq[l] : NULL, y, nq * d, h, q);
    matvec(w->wk[l], c->qkv_bias ? w->bk[l] : NULL, y, kvw, h, kp);
    matvec(w->wv[l], c->qkv_bias ? w->bv[l] : NULL, y, kvw, h, vp);
    for (int32_t hq = 0; hq < nq; ++hq) orc_rope(q + (size_t)hq * d, d, pos, c->rope_theta);
    for (int32_t hk = 0; hk < nkv; ++hk) orc_rope(kp + (size_t)hk * d, d, pos, c->rope_theta);
    attention_strided(q, Kl, Vl, pos + 1, kvw, nq, nkv, d, o);
    matvec(w->wo[l], NULL, o, h, nq * d, tmp);
    for (int32_t i = 0; i < h; ++i) x[i] += tmp[i];

    orc_rmsnorm(x, w->norm_mlp[l], h, c->rms_eps, y);
    matvec(w->wg[l], NULL, y, I, h, gate);
    matvec(w->wu[l], NULL, y, I, h, up);
    for (int32_t i = 0; i < I; ++i) gate[i] = orc_silu(gate[i]) * up[i];
    matvec(w->wd[l], NULL, gate, h, I, tmp);
    for (int32_t i = 0; i < h; ++i) x[i] += tmp[i];
}

static void head(const orc_model *m, const float *x, float *y, float *logits) {
    orc_rmsnorm(x, m->w.final_norm, m->c.hidden, m->c.rms_eps, y);
    matvec(m->w.lm_head, NULL, y, m->c.vocab, m->c.hidden, logits);
}

typedef struct {
    float *x, *y, *q, *o, *gate, *up, *tmp, *logits;
} scratch;

static int scratch_alloc(const orc_config *c, int32_t rows, scratch *s) {
    size_t h = c->hidden, qd = (size_t)c->n_q_heads * c->head_dim, I = c->intermediate;
    s->x = (float *)malloc(sizeof(float) * h * rows);
    s->y = (float *)malloc(sizeof(float) * h);
    s->q = (float *)malloc(sizeof(float) * qd);
    s->o = (float *)malloc(sizeof(float) * qd);
    s->gate = (float *)malloc(sizeof(float) * I);
    s->up = (float *)malloc(sizeof(float) * I);
    s->tmp = (float *)malloc(sizeof(float) * h);
    s->logits = (float *)malloc(sizeof(float) * c->vocab);
    return (s->x && s->y && s->q && s->o && s->gate && s->up && s->tmp && s->logits) ? 0 : -1;
}

static void scratch_free(scratch *s) {
    free(s->x); free(s->y); free(s->q); free(s->o);
    free(s->gate); free(s->up); free(s->tmp); free(s->logits);
}

int orc_feed(orc_model *m, const int32_t *tokens, int32_t n, float *logits_last, float *logits_all) {
    if (check_feed(m, tokens, n)) return -1;
    const orc_config *c = &m->c;
    scratch s;
    if (scratch_alloc(c, 1, &s)) { scratch_free(&s); return -1; }
    for (int32_t t = 0; t < n; ++t) {
        int32_t pos = m->kv_len;
        memcpy(s.x, m->w.embed + (size_t)tokens[t] * c->hidden, sizeof(float) * c->hidden);
        for (int32_t l = 0; l < c->n_layers; ++l)
            layer_step(m, l, pos, s.x, s.y, s.q, s.o, s.gate, s.up, s.tmp);
        m->kv_len = pos + 1;
        int want = logits_all != NULL || (t == n - 1 && logits_last != NULL);
        if (want) {
            head(m, s.x, s.y, s.logits);
            if (logits_all) memcpy(logits_all + (size_t)t * c->vocab, s.logits, sizeof(float) * c->vocab);
            if (t == n - 1 && logits_last) memcpy(logits_last, s.logits, sizeof(float) * c->vocab);
        }
    }
    scratch_free(&s);
    return 0;
}

int orc_feed_block(orc_model *m, const int32_t *tokens, int32_t n, float *logits_last, float *logits_all) {
    if (check_feed(m, tokens, n)) return -1;
    const orc_config *c = &m->c;
    scratch s;
    if (scratch_alloc(c, n, &s)) { scratch_free(&s); return -1; }
    int32_t base = m->kv_len;
    for (int32_t t = 0; t < n; ++t)
        memcpy(s.x + (size_t)t * c->hidden, m->w.embed + (size_t)tokens[t] * c->hidden, sizeof(float) * c->hidden);
    /* layer-outer: within a layer the rows go in order, so row t sees the keys of rows <= t. */
    for (int32_t l = 0; l < c->n_layers; ++l)
        for (int32_t t = 0; t < n; ++t)
            layer_step(m, l, base + t, s.x + (size_t)t * c->hidden, s.y, s.q, s.o, s.gate, s.up, s.tmp);
    m->kv_len = base + n;
    for (int32_t t = 0; t < n; ++t) {
        int want = logits_all != NULL || (t == n - 1 && logits_last != NULL);
        if (!want) continue;
        head(m, s.x + (size_t)t * c->hidden, s.y, s.logits);
        if (logits_all) memcpy(logits_all + (size_t)t * c->vocab, s.logits, sizeof(float) * c->vocab);
        if (t == n - 1 && logits_last) memcpy(logits_last, s.logits, sizeof(float) * c->vocab);
    }
    scratch_free(&s);
    return 0;
}
