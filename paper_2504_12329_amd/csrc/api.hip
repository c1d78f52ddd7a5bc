// The C ABI: argument validation, model records, workspace carving, and the host-side
// orchestration of prefill, decode, hand-over (paper Section 3 (1)) and the whole loop.
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>

#include <hip/hip_ext.h>

#include "st_device.h"
#include "st_internal.h"

namespace st {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define ST_HIP(expr)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(ST_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

static int check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ST_EHIP, "%s: %s", what, hipGetErrorString(e));
    return ST_OK;
}

static int validate_config(const st_config *c) {
    if (!c) return fail(ST_EINVAL, "config is NULL");
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->intermediate <= 0 ||
        c->vocab <= 0 || c->max_seq <= 0 || c->max_chunk <= 0)
        return fail(ST_EINVAL, "config has a non-positive dimension");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(ST_EINVAL, "head_dim must be 64 or 128");
    if (c->hidden % 8 || c->intermediate % 8) return fail(ST_EINVAL, "hidden and intermediate must be multiples of 8");
    if (c->hidden > 8192) return fail(ST_EINVAL, "hidden must be <= 8192");
    if (c->n_q_heads % c->n_kv_heads) return fail(ST_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (c->n_q_heads / c->n_kv_heads > 8) return fail(ST_EINVAL, "at most 8 query heads per kv head");
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(ST_EINVAL, "bad rms_eps or rope_theta");
    if ((c->tie_embeddings != 0 && c->tie_embeddings != 1) || (c->qkv_bias != 0 && c->qkv_bias != 1))
        return fail(ST_EINVAL, "tie_embeddings and qkv_bias must be 0 or 1");
    return ST_OK;
}

static size_t kv_bytes_of(const st_config &c) {
    return (size_t)2 * c.n_layers * c.n_kv_heads * (size_t)c.max_seq * c.head_dim * sizeof(bf16_t);
}

int persist_cu_count() {
    static std::once_flag once;
    static int n_cu = 0;
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
            n_cu = n;
        else
            (void)hipGetLastError();
    });
    return n_cu;
}

void carve_workspace(const st_config &c, char *base, Workspace *ws) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    const size_t mc = c.max_chunk, h = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim;
    const size_t I = c.intermediate;
    ws->state = (int32_t *)take(sizeof(int32_t) * kStateInts);
    ws->counters = (int32_t *)take(sizeof(int32_t) * c.n_kv_heads);
    ws->rope = (float2 *)take(sizeof(float2) * (size_t)c.max_seq * (c.head_dim / 2));
    ws->tokens = (int32_t *)take(sizeof(int32_t) * mc);
    ws->out_tokens = (int32_t *)take(sizeof(int32_t) * (size_t)c.max_seq);
    ws->x = (float *)take(sizeof(float) * mc * h);
    ws->xn = (bf16_t *)take(sizeof(bf16_t) * mc * h);
    ws->qkv = (float *)take(sizeof(float) * partial_floats(c));
    ws->qb = (bf16_t *)take(sizeof(bf16_t) * mc * qd);
    ws->attn = (bf16_t *)take(sizeof(bf16_t) * mc * qd);
    ws->act = (bf16_t *)take(sizeof(bf16_t) * mc * I);
    ws->xn_lo = (bf16_t *)take(sizeof(bf16_t) * mc * h);
    ws->attn_lo = (bf16_t *)take(sizeof(bf16_t) * mc * qd);
    ws->act_lo = (bf16_t *)take(sizeof(bf16_t) * mc * I);
    ws->qb_lo = (bf16_t *)take(sizeof(bf16_t) * mc * qd);
    ws->q1 = (float *)take(sizeof(float) * qd);
    ws->o1 = (float *)take(sizeof(float) * qd);
    ws->a1 = (float *)take(sizeof(float) * I);
    ws->part_ml = (float *)take(sizeof(float) * c.n_q_heads * kAttnSplits * 2);
    ws->part_acc = (float *)take(sizeof(float) * c.n_q_heads * kAttnSplits * c.head_dim);
    ws->logits = (float *)take(sizeof(float) * (size_t)c.vocab);
    ws->amax_val = (float *)take(sizeof(float) * kLmBlocks);
    ws->amax_idx = (int32_t *)take(sizeof(int32_t) * kLmBlocks);
    PersistPlan plan;
    const bool planned = persist_plan(c, persist_cu_count(), &plan);
    ws->ll = (unsigned long long *)take(planned ? sizeof(unsigned long long) * plan.ll_words : 0);
    ws->ptab = (PersistLayer *)take(planned ? sizeof(PersistLayer) * (size_t)c.n_layers : 0);
    ws->pargs = (PersistArgs *)take(planned ? sizeof(PersistArgs) : 0);
    ws->bytes = off;
}

// Enqueues the catch-up pass over `n` tokens (host or device ids); the last row's logits and greedy
// token (with the trigger predicate when a rule is given) end up in ws.logits / state.
enum PrefillMode { kPassDefault, kPassTwoTerm, kPassFast };
// Precision and kernel regime of the passes enqueued next (read by pass_terms / gemm in prefill.hip).
static void set_pass_mode(Model *m, PrefillMode mode) {
    m->long_terms = mode == kPassFast ? 0 : kDefaultLongTerms;
    m->f16_pass = mode == kPassDefault && m->f16_on;
    m->ring_min_rows = (mode == kPassFast || m->f16_pass) ? kRingMinRowsFast : kRingMinRows;
}
static int prefill_impl(Model *m, const int32_t *tokens, int32_t n, bool tokens_dev, const st_trigger_rule *rule,
                        PrefillMode mode = kPassDefault) {
    const st_config &c = m->c;
    if (!tokens) return fail(ST_EINVAL, "tokens is NULL");
    if (n <= 0) return fail(ST_ERANGE, "n must be positive (got %d)", n);
    if ((int64_t)m->kv_len + n > c.max_seq)
        return fail(ST_ERANGE, "KV overflow: kv_len %d + n %d > max_seq %d", m->kv_len, n, c.max_seq);
    if (!tokens_dev)
        for (int32_t i = 0; i < n; ++i)
            if (tokens[i] < 0 || tokens[i] >= c.vocab)
                return fail(ST_ERANGE, "token id %d at index %d is outside the vocabulary [0,%d)", tokens[i], i, c.vocab);
    // passes of at most max_chunk rows; 256 rows on request: the longest pass that keeps every GEMM input in two terms
    const int32_t step = mode == kPassTwoTerm && c.max_chunk > 256 ? 256 : c.max_chunk;
    set_pass_mode(m, mode);
    for (int32_t done = 0; done < n; done += step) {
        int32_t cn = n - done < step ? n - done : step;
        ST_HIP(hipMemcpyAsync(m->ws.tokens, tokens + done, sizeof(int32_t) * cn,
                              tokens_dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, m->stream));
        bool last_chunk = done + cn == n;
        launch_prefill_layers(*m, m->kv_len + done, cn);
        if (last_chunk) launch_head(*m, m->ws.x + (size_t)(cn - 1) * c.hidden, rule, cn, nullptr, m->stream);
        else launch_set_state(*m, kPos, m->kv_len + done + cn);
        if (int rc = check_launch("prefill")) return rc;
    }
    m->kv_len += n;
    return ST_OK;
}

// The captured graph of one decode step for this rule / output buffer, or nullptr when graphs are off.
// Every kernel of a step reads the position and token from the device state block, so one graph
// serves every step.  Capture happens on a private stream (the caller's may be the legacy default
// stream, which cannot be captured); the graph is then launched on the model's stream.
static hipGraphExec_t step_graph(Model *m, const st_trigger_rule *rule, int32_t *out_seq_dev) {
    if (m->graphs_off || m->timers) return nullptr;
    const void *kw = rule ? rule->kw_bitmap : nullptr, *dl = rule ? rule->delim_bitmap : nullptr;
    int window = rule ? rule->window : 0, vocab = rule ? rule->vocab : 0;
    // the single-kernel step sizes its attention split on the device: one graph serves every context length
    const int bucket = m->persist_on ? 0 : attn_bucket(m->kv_len + 1);
    for (const StepGraph &g : m->graphs)
        if (g.kw == kw && g.delim == dl && g.out_seq == out_seq_dev && g.window == window && g.vocab == vocab &&
            g.attn_blocks == bucket)
            return g.exec;
    if (m->graphs.size() >= 64) return nullptr;  // unusual caller: many distinct rules; launch directly
    // A failure here is not fatal -- the step is launched kernel by kernel instead, about a tenth slower -- but it is
    // not silent either: the HIP message goes to st_last_error() and st_decode_graph_state() reports mode 2.
    auto give_up = [&](const char *what, hipError_t e) -> hipGraphExec_t {
        m->graphs_off = true;
        m->graph_failed = true;
        (void)fail(ST_EHIP, "decode-step graph: %s failed (%s); steps are launched kernel by kernel from now on", what,
                   hipGetErrorString(e));
        (void)hipGetLastError();
        return nullptr;
    };
    if (!m->capture_stream) {
        hipError_t e = hipStreamCreateWithFlags(&m->capture_stream, hipStreamNonBlocking);
        if (e != hipSuccess) {
            m->capture_stream = nullptr;
            return give_up("hipStreamCreateWithFlags", e);
        }
    }
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipError_t e = hipStreamBeginCapture(m->capture_stream, hipStreamCaptureModeRelaxed);
    if (e != hipSuccess) return give_up("hipStreamBeginCapture", e);
    launch_decode_step(*m, rule, out_seq_dev, m->capture_stream, bucket);
    e = hipStreamEndCapture(m->capture_stream, &graph);
    if (e != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        return give_up("hipStreamEndCapture", e);
    }
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return give_up("hipGraphInstantiate", e);
    m->graphs.push_back(StepGraph{kw, dl, out_seq_dev, window, vocab, bucket, exec});
    return exec;
}

static int decode_impl(Model *m, const st_trigger_rule *rule, int32_t *out_seq_dev) {
    if (m->kv_len + 1 > m->c.max_seq)
        return fail(ST_ERANGE, "KV overflow: kv_len %d + 1 > max_seq %d", m->kv_len, m->c.max_seq);
    if (m->persist_on && ++m->persist_launches >= (1L << 24)) {  // long before the 32-bit epochs could repeat
        launch_persist_reset(*m);
        m->persist_launches = 0;
    }
    if (hipGraphExec_t exec = step_graph(m, rule, out_seq_dev)) {
        ST_HIP(hipGraphLaunch(exec, m->stream));
    } else {
        launch_decode_step(*m, rule, out_seq_dev, m->stream, attn_bucket(m->kv_len + 1));
        if (int rc = check_launch("decode step")) return rc;
    }
    m->kv_len += 1;
    return ST_OK;
}

static int persist_failed() {
    return fail(ST_EHIP, "a wait inside the single-kernel decode step timed out (another kernel holding compute units "
                         "for too long, or a lost block); results since the last successful call are invalid");
}

// Copies logits / greedy token out; host destinations synchronise the stream.
static int deliver(Model *m, float *logits, int32_t *next_tok, bool out_dev) {
    hipMemcpyKind kind = out_dev ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
    if (logits) ST_HIP(hipMemcpyAsync(logits, m->ws.logits, sizeof(float) * (size_t)m->c.vocab, kind, m->stream));
    if (next_tok) ST_HIP(hipMemcpyAsync(next_tok, m->ws.state + kTok, sizeof(int32_t), kind, m->stream));
    if (!out_dev) {
        int32_t perr = 0;
        if (m->persist_on)
            ST_HIP(hipMemcpyAsync(&perr, m->ws.state + kPersistErr, sizeof(int32_t), hipMemcpyDeviceToHost, m->stream));
        ST_HIP(hipStreamSynchronize(m->stream));
        if (perr) return persist_failed();
    }
    return ST_OK;
}

// Reads (greedy token, fired) back to the host.
static int fetch_token(Model *m, int32_t *tok, int32_t *fired) {
    int32_t st[kPersistErr + 1];
    static_assert(kTok == 1 && kFired == 2, "slots read back together");
    ST_HIP(hipMemcpyAsync(st, m->ws.state, sizeof(st), hipMemcpyDeviceToHost, m->stream));
    ST_HIP(hipStreamSynchronize(m->stream));
    if (m->persist_on && st[kPersistErr]) return persist_failed();
    *tok = st[kTok];
    if (fired) *fired = st[kFired];
    return ST_OK;
}

static int handoff_impl(Model *small, Model *large, int32_t *seq, int32_t *T, int32_t n_large, int32_t budget,
                        const st_trigger_rule *rule, float *small_logits, int32_t *small_next, int32_t *small_fired,
                        st_spans *spans, double *ms_large_prefill, double *ms_large_decode, double *ms_small_prefill) {
    using clk = std::chrono::steady_clock;
    auto ms = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); };
    int32_t t0 = *T;
    if (t0 <= 0) return fail(ST_ERANGE, "sequence is empty");
    if (n_large <= 0 || budget <= 0) return fail(ST_ERANGE, "n_large and budget must be positive");
    if (large->kv_len >= t0 || small->kv_len >= t0)
        return fail(ST_ERANGE, "a model has already been fed the whole sequence (kv_len %d / %d, T %d)", small->kv_len,
                    large->kv_len, t0);
    int32_t n = n_large < budget ? n_large : budget;
    if ((int64_t)t0 + n - 1 > large->c.max_seq || (int64_t)t0 + n > small->c.max_seq)
        return fail(ST_ERANGE, "KV overflow during hand-over (T %d, segment %d)", t0, n);
    st_spans sp = {large->kv_len, t0, t0, t0, small->kv_len, small->kv_len};
    auto a = clk::now();
    if (int rc = prefill_impl(large, seq + large->kv_len, t0 - large->kv_len, false, nullptr)) return rc;
    int32_t tok;
    if (int rc = fetch_token(large, &tok, nullptr)) return rc;
    auto b = clk::now();
    int32_t t = t0;
    for (int32_t j = 0; j < n; ++j) {
        seq[t++] = tok;
        if (j < n - 1) {  // the segment's last token is not fed to the target yet
            if (int rc = decode_impl(large, nullptr, nullptr)) return rc;   // feeds state[kTok] == tok
            if (int rc = fetch_token(large, &tok, nullptr)) return rc;
        }
    }
    auto c = clk::now();
    sp.large_decode_hi = t;
    bool ended = budget <= n_large;
    if (!ended) {
        sp.small_prefill_hi = t;
        if (int rc = prefill_impl(small, seq + small->kv_len, t - small->kv_len, false, rule)) return rc;
        int32_t stok, sfired;
        if (small_logits)
            ST_HIP(hipMemcpyAsync(small_logits, small->ws.logits, sizeof(float) * (size_t)small->c.vocab,
                                  hipMemcpyDeviceToHost, small->stream));
        if (int rc = fetch_token(small, &stok, &sfired)) return rc;
        if (small_next) *small_next = stok;
        if (small_fired) *small_fired = sfired;
    }
    auto d = clk::now();
    *T = t;
    if (spans) *spans = sp;
    if (ms_large_prefill) *ms_large_prefill += ms(a, b);
    if (ms_large_decode) *ms_large_decode += ms(b, c);
    if (ms_small_prefill) *ms_small_prefill += ms(c, d);
    return ST_OK;
}

}  // namespace st

using namespace st;

extern "C" {

const char *st_last_error(void) { return g_err; }

int st_query_sizes(const st_config *cfg, size_t *kv_bytes, size_t *workspace_bytes) {
    if (int rc = validate_config(cfg)) return rc;
    if (kv_bytes) *kv_bytes = kv_bytes_of(*cfg);
    if (workspace_bytes) {
        Workspace ws;
        carve_workspace(*cfg, nullptr, &ws);
        *workspace_bytes = ws.bytes;
    }
    return ST_OK;
}

int st_prefill_plan_check(const st_config *cfg, int32_t rows, int32_t *launches, int32_t *blocks) {
    if (int rc = validate_config(cfg)) return rc;
    if (rows <= 0 || rows > cfg->max_chunk) return fail(ST_ERANGE, "rows %d outside 1..max_chunk", rows);
    if (launches) *launches = 0;
    if (blocks) *blocks = 0;
    if (rows < kRingMinRowsFast) return ST_OK;  // shorter chunks take the streaming kernel: one tile list, no leftovers
    const int h = cfg->hidden, I = cfg->intermediate, qd = cfg->n_q_heads * cfg->head_dim;
    const int qkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
    const long long cap = (long long)partial_floats(*cfg);
    const struct {
        const char *name;
        int dual, N, K;
        bool def_two;
    } g[4] = {{"QKV", 0, qkv, h, (kDefaultLongTerms & kTermQKV) != 0},
              {"O", 0, h, qd, (kDefaultLongTerms & kTermO) != 0},
              {"gate/up", 1, I, h, (kDefaultLongTerms & kTermGateUp) != 0},
              {"down", 0, h, I, (kDefaultLongTerms & kTermDown) != 0}};
    for (const auto &e : g) {
        if (e.K % 64 || e.K < 128) continue;  // the general-shape kernel serves such a K
        // a projection whose input carries two bf16 terms runs the doubled contraction [A | Alo] x [B | B]: the
        // plans of both forms are walked
        for (int terms = 1; terms <= 2; ++terms) {
            int nl = 0, nb = 0, ni = 0;
            const int rc = ring_plan_check(e.dual, rows, e.N, terms * e.K, cap, 1, &nl, &nb, &ni);
            if (rc)
                return fail(ST_EINVAL, "block plan of the %s projection at %d rows (%d-term input) fails check %d",
                            e.name, rows, terms, rc);
            if (terms != (e.def_two ? 2 : 1)) continue;  // the counts reported are the default pass's
            if (launches) *launches += nl;
            if (blocks) *blocks += nb;
        }
    }
    return ST_OK;
}

// Checks the weights and fills a model record over the given cache and workspace (sizes checked by the caller).
static int build_model(const st_config *cfg, const st_weights *w, void *kv, void *workspace, void *stream, Model *m) {
    if (!w) return fail(ST_EINVAL, "weights is NULL");
    if (!w->embed || !w->final_norm || (!cfg->tie_embeddings && !w->lm_head))
        return fail(ST_EINVAL, "embed, final_norm or lm_head is NULL");
    if (!w->wqkv || !w->wo || !w->w_gate_up || !w->w_down || !w->norm_attn || !w->norm_mlp ||
        (cfg->qkv_bias && !w->bqkv))
        return fail(ST_EINVAL, "a per-layer weight array is NULL");
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->wqkv[l] || !w->wo[l] || !w->w_gate_up[l] || !w->w_down[l] || !w->norm_attn[l] || !w->norm_mlp[l] ||
            (cfg->qkv_bias && !w->bqkv[l]))
            return fail(ST_EINVAL, "a weight pointer of layer %d is NULL", l);
    if (!kv || !workspace) return fail(ST_EINVAL, "kv or workspace is NULL");
    if (((uintptr_t)kv & 255) || ((uintptr_t)workspace & 255))
        return fail(ST_EINVAL, "kv and workspace must be 256-byte aligned");
    m->c = *cfg;
    m->qkv_dim = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
    auto cp = [&](std::vector<const bf16_t *> &dst, const void *const *src) {
        dst.resize(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers; ++l) dst[l] = src ? (const bf16_t *)src[l] : nullptr;
    };
    cp(m->wqkv, w->wqkv);
    cp(m->bqkv, cfg->qkv_bias ? w->bqkv : nullptr);
    cp(m->wo, w->wo);
    cp(m->wgu, w->w_gate_up);
    cp(m->wdown, w->w_down);
    cp(m->norm_attn, w->norm_attn);
    cp(m->norm_mlp, w->norm_mlp);
    m->embed = (const bf16_t *)w->embed;
    m->lm_head = cfg->tie_embeddings ? m->embed : (const bf16_t *)w->lm_head;
    m->final_norm = (const bf16_t *)w->final_norm;
    m->kcache = (bf16_t *)kv;
    m->vcache = m->kcache + (size_t)cfg->n_layers * cfg->n_kv_heads * (size_t)cfg->max_seq * cfg->head_dim;
    carve_workspace(*cfg, (char *)workspace, &m->ws);
    m->stream = (hipStream_t)stream;
    m->kv_len = 0;
    m->timers = nullptr;
    m->capture_stream = nullptr;
    m->graphs_off = getenv("ST_NO_GRAPH") != nullptr;
    m->graph_failed = false;
    m->long_terms = kDefaultLongTerms;
    m->ring_min_rows = kRingMinRows;
    m->f16_on = m->f16_pass = false;
    static std::once_flag lds_once;
    static hipError_t lds_rc = hipSuccess;
    std::call_once(lds_once, [] { lds_rc = raise_lds_limits(); });
    if (lds_rc != hipSuccess) return fail(ST_EHIP, "raising the kernels' LDS limit: %s", hipGetErrorString(lds_rc));
    launch_init(*m);
    if (int rc = check_launch("workspace initialisation")) return rc;
    // the single-kernel decode step: on request (ST_DECODE_PERSIST=1), where the shape fits it.  Measured on the
    // 1.5B / 7B / 32B shapes it is 5-10 % slower than the kernel-per-stage step, so it is not the default.
    m->persist_on = false;
    m->persist_launches = 0;
    const char *pe = getenv("ST_DECODE_PERSIST");
    if (pe && pe[0] == '1' && persist_plan(*cfg, persist_cu_count(), &m->persist)) {
        const char *sl = getenv("ST_PERSIST_SPIN");
        m->persist_spin_limit = sl ? atoi(sl) : (1 << 20);
        if (m->persist_spin_limit < 1) m->persist_spin_limit = 1;
        m->ptab_host.resize(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers; ++l)
            m->ptab_host[l] = PersistLayer{m->wqkv[l], m->bqkv[l], m->wo[l], m->wgu[l], m->wdown[l], m->norm_attn[l],
                                           m->norm_mlp[l], nullptr};
        ST_HIP(hipMemcpyAsync(m->ws.ptab, m->ptab_host.data(), sizeof(PersistLayer) * (size_t)cfg->n_layers,
                              hipMemcpyHostToDevice, m->stream));
        m->pargs_host = persist_args(*m);
        ST_HIP(hipMemcpyAsync(m->ws.pargs, &m->pargs_host, sizeof(PersistArgs), hipMemcpyHostToDevice, m->stream));
        ST_HIP(persist_prepare(*m));
        launch_persist_reset(*m);
        if (int rc = check_launch("hand-over words")) return rc;
        m->persist_on = true;
    }
    return ST_OK;
}

int st_model_create(const st_config *cfg, const st_weights *w, void *kv, size_t kv_bytes, void *workspace,
                    size_t workspace_bytes, void *stream, st_model **out) {
    if (!out) return fail(ST_EINVAL, "out is NULL");
    *out = nullptr;
    if (int rc = validate_config(cfg)) return rc;
    Workspace sized;
    carve_workspace(*cfg, nullptr, &sized);
    if (kv && kv_bytes < kv_bytes_of(*cfg))
        return fail(ST_ENOMEM, "kv buffer has %zu bytes, %zu needed", kv_bytes, kv_bytes_of(*cfg));
    if (workspace && workspace_bytes < sized.bytes)
        return fail(ST_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, sized.bytes);
    Model *m = new (std::nothrow) Model();
    if (!m) return fail(ST_ENOMEM, "out of host memory");
    if (int rc = build_model(cfg, w, kv, workspace, stream, m)) {
        delete m;
        return rc;
    }
    *out = reinterpret_cast<st_model *>(m);
    return ST_OK;
}

void st_model_destroy(st_model *h) {
    Model *m = reinterpret_cast<Model *>(h);
    if (!m) return;
    for (StepGraph &g : m->graphs) (void)hipGraphExecDestroy(g.exec);
    if (m->capture_stream) (void)hipStreamDestroy(m->capture_stream);
    delete m;
}

static size_t f16_elems(const st_config &c) {  // elements of one layer's O, gate/up and down projection matrices
    const size_t h = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, I = c.intermediate;
    return h * qd + 2 * I * h + h * I;
}

int st_query_f16_bytes(const st_config *cfg, size_t *bytes) {
    if (int rc = validate_config(cfg)) return rc;
    if (!bytes) return fail(ST_EINVAL, "bytes is NULL");
    if (!f16_shape_ok(*cfg))
        return fail(ST_EINVAL, "the fp16 operand mode needs hidden, n_q_heads*head_dim and intermediate to be multiples of 64");
    *bytes = f16_elems(*cfg) * cfg->n_layers * sizeof(bf16_t);
    return ST_OK;
}

static int attach_f16(Model *m, void *buf, size_t bytes) {
    m->f16_on = m->f16_pass = false;
    m->wo16.clear(), m->wgu16.clear(), m->wdown16.clear();
    if (!buf) return ST_OK;  // detach
    const st_config &c = m->c;
    if (!f16_shape_ok(c))
        return fail(ST_EINVAL, "the fp16 operand mode needs hidden, n_q_heads*head_dim and intermediate to be multiples of 64");
    const size_t need = f16_elems(c) * c.n_layers * sizeof(bf16_t);
    if (bytes < need) return fail(ST_ENOMEM, "fp16 weight buffer has %zu bytes, %zu needed", bytes, need);
    if ((uintptr_t)buf & 255) return fail(ST_EINVAL, "the fp16 weight buffer must be 256-byte aligned");
    const size_t h = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, I = c.intermediate;
    const size_t n_o = h * qd, n_gu = 2 * I * h, n_d = h * I;
    launch_set_state(*m, kCount, 0);
    bf16_t *p = static_cast<bf16_t *>(buf);
    int32_t *bad = m->ws.state + kCount;
    for (int l = 0; l < c.n_layers; ++l) {
        launch_f16_copy(*m, m->wo[l], p, n_o, bad), m->wo16.push_back(p), p += n_o;
        launch_f16_copy(*m, m->wgu[l], p, n_gu, bad), m->wgu16.push_back(p), p += n_gu;
        launch_f16_copy(*m, m->wdown[l], p, n_d, bad), m->wdown16.push_back(p), p += n_d;
    }
    if (int rc = check_launch("fp16 weight copy")) return rc;
    int32_t n_bad = 0;
    ST_HIP(hipMemcpyAsync(&n_bad, bad, sizeof(int32_t), hipMemcpyDeviceToHost, m->stream));
    ST_HIP(hipStreamSynchronize(m->stream));
    if (n_bad) {
        m->wo16.clear(), m->wgu16.clear(), m->wdown16.clear();
        return fail(ST_ERANGE, "%d weights are NaN or exceed the largest fp16 number: fp16 operand mode not enabled", n_bad);
    }
    m->f16_on = true;
    return ST_OK;
}

int st_model_attach_f16(st_model *hm, void *buf, size_t bytes) {
    if (!hm) return fail(ST_EINVAL, "model is NULL");
    return attach_f16(reinterpret_cast<Model *>(hm), buf, bytes);
}

int st_kv_len(const st_model *h, int32_t *out) {
    if (!h || !out) return fail(ST_EINVAL, "model or out is NULL");
    *out = reinterpret_cast<const Model *>(h)->kv_len;
    return ST_OK;
}

int st_decode_graph_state(const st_model *h, int32_t *graphs, int32_t *mode) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    const Model *m = reinterpret_cast<const Model *>(h);
    if (graphs) *graphs = (int32_t)m->graphs.size();
    if (mode) *mode = m->graph_failed ? 2 : (m->graphs_off ? 1 : 0);
    return ST_OK;
}

int st_decode_step_kind(const st_model *h, int32_t *kind) {
    if (!h || !kind) return fail(ST_EINVAL, "model or kind is NULL");
    *kind = reinterpret_cast<const Model *>(h)->persist_on ? 1 : 0;
    return ST_OK;
}

int st_decode_persist_plan(const st_config *cfg, int32_t n_cu, size_t *lds_bytes, size_t *handover_words,
                           int32_t *regions, int32_t *parts) {
    if (int rc = validate_config(cfg)) return rc;
    PersistPlan p;
    if (!persist_plan(*cfg, n_cu, &p))
        return fail(ST_EINVAL, "the shape does not fit the single-kernel decode step on %d compute units", n_cu);
    if (lds_bytes) *lds_bytes = p.lds_bytes;
    if (handover_words) *handover_words = p.ll_words;
    if (regions) {
        const int r[7] = {p.off_x, p.off_qkv, p.off_part, p.off_attn, p.off_x2, p.off_act, p.off_cand};
        for (int i = 0; i < 7; ++i) regions[i] = r[i];
    }
    if (parts) {
        const int lp[5] = {p.lp_qkv, p.lp_o, p.lp_gu, p.lp_dn, p.lp_lm};
        for (int i = 0; i < 5; ++i) parts[i] = 1 << lp[i];
    }
    return ST_OK;
}

int st_kv_truncate(st_model *h, int32_t new_len) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    Model *m = reinterpret_cast<Model *>(h);
    if (new_len < 0 || new_len > m->kv_len)
        return fail(ST_ERANGE, "new_len %d outside [0, %d]", new_len, m->kv_len);
    launch_set_state(*m, kPos, new_len);
    if (m->persist_on) {  // also the way back from a step that gave up waiting: clears its error flag
        launch_persist_reset(*m);
        m->persist_launches = 0;
    }
    if (int rc = check_launch("truncate")) return rc;
    m->kv_len = new_len;
    return ST_OK;
}

static int check_flags(uint32_t flags, uint32_t allowed) {
    if (flags & ~allowed) return fail(ST_EINVAL, "unsupported flag bits 0x%x", flags & ~allowed);
    return ST_OK;
}

int st_prefill(st_model *h, const int32_t *tokens, int32_t n, float *logits, int32_t *next_tok, uint32_t flags) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    if (int rc = check_flags(flags, ST_TOKENS_DEVICE | ST_OUT_DEVICE | ST_PREFILL_TWO_TERM | ST_PREFILL_FAST)) return rc;
    if ((flags & ST_PREFILL_TWO_TERM) && (flags & ST_PREFILL_FAST))
        return fail(ST_EINVAL, "ST_PREFILL_TWO_TERM and ST_PREFILL_FAST exclude each other");
    Model *m = reinterpret_cast<Model *>(h);
    const PrefillMode mode = (flags & ST_PREFILL_TWO_TERM) ? kPassTwoTerm : (flags & ST_PREFILL_FAST) ? kPassFast : kPassDefault;
    if (int rc = prefill_impl(m, tokens, n, flags & ST_TOKENS_DEVICE, nullptr, mode)) return rc;
    return deliver(m, logits, next_tok, flags & ST_OUT_DEVICE);
}

int st_decode_step(st_model *h, int32_t token, float *logits, int32_t *next_tok, uint32_t flags) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    if (int rc = check_flags(flags, ST_OUT_DEVICE | ST_TOKEN_CHAINED)) return rc;
    Model *m = reinterpret_cast<Model *>(h);
    if (!(flags & ST_TOKEN_CHAINED)) {
        if (token < 0 || token >= m->c.vocab)
            return fail(ST_ERANGE, "token id %d is outside the vocabulary [0,%d)", token, m->c.vocab);
        if (m->kv_len + 1 > m->c.max_seq)
            return fail(ST_ERANGE, "KV overflow: kv_len %d + 1 > max_seq %d", m->kv_len, m->c.max_seq);
        launch_set_token(*m, token);
    }
    if (int rc = decode_impl(m, nullptr, nullptr)) return rc;
    return deliver(m, logits, next_tok, flags & ST_OUT_DEVICE);
}

int st_decode_greedy(st_model *h, int32_t first_token, int32_t n, int32_t *out_tokens, uint32_t flags) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    if (int rc = check_flags(flags, ST_OUT_DEVICE | ST_TOKEN_CHAINED)) return rc;
    Model *m = reinterpret_cast<Model *>(h);
    if (n <= 0) return fail(ST_ERANGE, "n must be positive (got %d)", n);
    if ((int64_t)m->kv_len + n > m->c.max_seq)
        return fail(ST_ERANGE, "KV overflow: kv_len %d + n %d > max_seq %d", m->kv_len, n, m->c.max_seq);
    if (!(flags & ST_TOKEN_CHAINED)) {
        if (first_token < 0 || first_token >= m->c.vocab)
            return fail(ST_ERANGE, "token id %d is outside the vocabulary [0,%d)", first_token, m->c.vocab);
        launch_set_token(*m, first_token);
    }
    launch_set_state(*m, kStep, 0);
    for (int32_t i = 0; i < n; ++i)
        if (int rc = decode_impl(m, nullptr, m->ws.out_tokens)) return rc;
    if (out_tokens) {
        bool dev = flags & ST_OUT_DEVICE;
        ST_HIP(hipMemcpyAsync(out_tokens, m->ws.out_tokens, sizeof(int32_t) * n,
                              dev ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, m->stream));
        if (!dev) ST_HIP(hipStreamSynchronize(m->stream));
    }
    return ST_OK;
}

int st_decode_step_timed(st_model *h, double *gateup_mean_us, double *step_us) {
    if (!h) return fail(ST_EINVAL, "model is NULL");
    Model *m = reinterpret_cast<Model *>(h);
    if (m->kv_len + 1 > m->c.max_seq)
        return fail(ST_ERANGE, "KV overflow: kv_len %d + 1 > max_seq %d", m->kv_len, m->c.max_seq);
    StepTimers t;
    t.ev.resize(2 + 2 * (size_t)m->c.n_layers);
    int rc = ST_OK;
    for (auto &e : t.ev) {
        e = nullptr;
        if (rc == ST_OK && hipEventCreate(&e) != hipSuccess) rc = fail(ST_EHIP, "hipEventCreate failed");
    }
    if (rc == ST_OK) {
        m->timers = &t;
        (void)hipEventRecord(t.ev[0], m->stream);
        rc = decode_impl(m, nullptr, nullptr);
        (void)hipEventRecord(t.ev[1], m->stream);
        m->timers = nullptr;
        if (rc == ST_OK && hipStreamSynchronize(m->stream) != hipSuccess) rc = fail(ST_EHIP, "synchronise failed");
    }
    if (rc == ST_OK) {
        float ms = 0.f;
        double sum = 0.0;
        for (int l = 0; l < m->c.n_layers && rc == ST_OK; ++l) {
            if (hipEventElapsedTime(&ms, t.ev[2 + 2 * l], t.ev[3 + 2 * l]) != hipSuccess)
                rc = fail(ST_EHIP, "hipEventElapsedTime failed");
            sum += ms;
        }
        if (rc == ST_OK && gateup_mean_us) *gateup_mean_us = sum * 1e3 / m->c.n_layers;
        if (rc == ST_OK && hipEventElapsedTime(&ms, t.ev[0], t.ev[1]) != hipSuccess)
            rc = fail(ST_EHIP, "hipEventElapsedTime failed");
        if (rc == ST_OK && step_us) *step_us = ms * 1e3;
    }
    for (auto &e : t.ev)
        if (e) (void)hipEventDestroy(e);
    return rc;
}

int st_trigger_scan(const st_trigger_rule *rule, const int32_t *tokens, int32_t lo, int32_t hi, int32_t *positions,
                    int32_t cap, int32_t *n_found, int32_t *scratch, void *stream, uint32_t flags) {
    if (!rule || !rule->kw_bitmap || !tokens || !n_found) return fail(ST_EINVAL, "rule, bitmap, tokens or n_found is NULL");
    if (rule->window < 1 || rule->window > ST_MAX_SCAN_WINDOW) return fail(ST_EINVAL, "window must be in [1, %d]", ST_MAX_SCAN_WINDOW);
    if (rule->window >= 2 && !rule->delim_bitmap) return fail(ST_EINVAL, "a window above 1 needs a delimiter bitmap");
    if (rule->vocab <= 0) return fail(ST_EINVAL, "rule vocab must be positive");
    if (int rc = check_flags(flags, ST_OUT_DEVICE)) return rc;
    if (cap < 0 || (cap > 0 && !positions)) return fail(ST_EINVAL, "cap < 0, or positions is NULL with cap > 0");
    if (lo < 0 || hi < lo) return fail(ST_ERANGE, "bad range [%d,%d)", lo, hi);
    hipStream_t s = (hipStream_t)stream;
    if (flags & ST_OUT_DEVICE) {
        launch_trigger_scan(*rule, tokens, lo, hi, positions, cap, n_found, s);
        return check_launch("trigger scan");
    }
    if (!scratch) return fail(ST_EINVAL, "host outputs need a device scratch of cap+1 int32");
    launch_trigger_scan(*rule, tokens, lo, hi, scratch + 1, cap, scratch, s);
    if (int rc = check_launch("trigger scan")) return rc;
    ST_HIP(hipMemcpyAsync(n_found, scratch, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ST_HIP(hipStreamSynchronize(s));
    int32_t k = *n_found < cap ? *n_found : cap;
    if (k > 0) {
        ST_HIP(hipMemcpyAsync(positions, scratch + 1, sizeof(int32_t) * k, hipMemcpyDeviceToHost, s));
        ST_HIP(hipStreamSynchronize(s));
    }
    return ST_OK;
}

int st_handoff(st_model *small, st_model *large, int32_t *seq, int32_t *T, int32_t n_large, int32_t budget,
               float *small_logits, int32_t *small_next_tok, st_spans *spans, uint32_t flags) {
    if (!small || !large || !seq || !T) return fail(ST_EINVAL, "small, large, seq or T is NULL");
    if (small == large) return fail(ST_EINVAL, "small and large must be different models");
    if (int rc = check_flags(flags, 0)) return rc;
    return handoff_impl(reinterpret_cast<Model *>(small), reinterpret_cast<Model *>(large), seq, T, n_large, budget,
                        nullptr, small_logits, small_next_tok, nullptr, spans, nullptr, nullptr, nullptr);
}

int st_generate(st_model *hs, st_model *hl, const st_trigger_rule *rule, int32_t forced_period, const int32_t *prompt,
                int32_t P, int32_t n_out, int32_t n_seg, int32_t *seq, uint8_t *src, st_spans *spans, int32_t span_cap,
                st_gen_stats *stats) {
    using clk = std::chrono::steady_clock;
    auto ms = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); };
    if (!hs || !hl || !prompt || !seq) return fail(ST_EINVAL, "small, large, prompt or seq is NULL");
    if (hs == hl) return fail(ST_EINVAL, "small and large must be different models");
    if (forced_period < 0) return fail(ST_EINVAL, "forced_period must be >= 0");
    if (forced_period == 0) {
        if (!rule || !rule->kw_bitmap) return fail(ST_EINVAL, "a trigger rule (or forced_period > 0) is required");
        if (rule->window != 1 && rule->window != 2) return fail(ST_EINVAL, "window must be 1 or 2");
        if (rule->window == 2 && !rule->delim_bitmap) return fail(ST_EINVAL, "window 2 needs a delimiter bitmap");
    }
    if (P <= 0 || n_out < 0 || n_seg <= 0) return fail(ST_ERANGE, "P, n_seg must be positive and n_out non-negative");
    if (span_cap < 0 || (span_cap > 0 && !spans)) return fail(ST_EINVAL, "bad span buffer");
    Model *S = reinterpret_cast<Model *>(hs), *L = reinterpret_cast<Model *>(hl);
    if (S->kv_len != 0 || L->kv_len != 0) return fail(ST_EINVAL, "both models must start with an empty KV cache");
    if ((int64_t)P + n_out > S->c.max_seq || (int64_t)P + n_out > L->c.max_seq)
        return fail(ST_ERANGE, "P + n_out = %d exceeds a model's max_seq", P + n_out);
    const st_trigger_rule *use_rule = forced_period > 0 ? nullptr : rule;
    st_gen_stats st = {};
    memcpy(seq, prompt, sizeof(int32_t) * P);
    int32_t T = P, tok = 0, fired = 0;
    if (n_out > 0) {
        auto a = clk::now();
        if (int rc = prefill_impl(S, seq, P, false, use_rule)) return rc;
        if (int rc = fetch_token(S, &tok, &fired)) return rc;
        auto b = clk::now();
        if (int rc = prefill_impl(L, seq, P, false, nullptr)) return rc;
        ST_HIP(hipStreamSynchronize(L->stream));
        auto c = clk::now();
        st.ms_small_prefill += ms(a, b);
        st.ms_large_prefill += ms(b, c);
    }
    int32_t small_count = 0;
    while (T - P < n_out) {
        seq[T++] = tok;
        if (src) src[T - 1 - P] = 0;
        ++small_count;
        if (T - P == n_out) break;
        bool fire = forced_period > 0 ? (small_count % forced_period == 0) : fired != 0;
        if (fire) {
            st_spans sp;
            if (int rc = handoff_impl(S, L, seq, &T, n_seg, n_out - (T - P), use_rule, nullptr, &tok, &fired, &sp,
                                      &st.ms_large_prefill, &st.ms_large_decode, &st.ms_small_prefill))
                return rc;
            if (src)
                for (int32_t p = sp.large_decode_lo; p < sp.large_decode_hi; ++p) src[p - P] = 1;
            st.n_large += sp.large_decode_hi - sp.large_decode_lo;
            if (st.n_spans < span_cap) spans[st.n_spans++] = sp;
            ++st.n_handoffs;
        } else {
            auto a = clk::now();
            if (int rc = decode_impl(S, use_rule, nullptr)) return rc;   // feeds state[kTok] == tok
            if (int rc = fetch_token(S, &tok, &fired)) return rc;
            st.ms_small_decode += ms(a, clk::now());
        }
    }
    st.n_out = T - P;
    if (stats) *stats = st;
    return ST_OK;
}

int st_generate_policy(st_model *hs, st_model *hl, const st_policy *pol, const int32_t *prompt, int32_t P,
                       int32_t n_out, int32_t *seq, uint8_t *src, st_action *actions, int32_t action_cap,
                       st_gen_stats *stats) {
    using clk = std::chrono::steady_clock;
    if (!hs || !hl || !pol || !prompt || !seq) return fail(ST_EINVAL, "small, large, policy, prompt or seq is NULL");
    if (hs == hl) return fail(ST_EINVAL, "small and large must be different models");
    if (!pol->delim_bitmap || pol->vocab <= 0) return fail(ST_EINVAL, "the policy needs a delimiter bitmap and a vocabulary size");
    if (pol->sentence_len < 1) return fail(ST_EINVAL, "sentence_len must be >= 1");
    if ((pol->ar_bitmap || pol->unconditional) && pol->n1 < 1) return fail(ST_EINVAL, "n1 must be positive");
    if (pol->verify_bitmap && pol->n2 < 1) return fail(ST_EINVAL, "n2 must be positive");
    if (pol->neg_bitmap && (pol->n3 < 1 || pol->neg_threshold < 0 || pol->n_aux < 0 || (pol->n_aux > 0 && !pol->aux_tokens)))
        return fail(ST_EINVAL, "malformed excessive-reflection settings");
    if (pol->initial_target < 0) return fail(ST_EINVAL, "initial_target must be >= 0");
    if (P <= 0 || n_out < 0) return fail(ST_ERANGE, "P must be positive and n_out non-negative");
    if (action_cap < 0 || (action_cap > 0 && !actions)) return fail(ST_EINVAL, "bad action buffer");
    Model *M[2] = {reinterpret_cast<Model *>(hs), reinterpret_cast<Model *>(hl)};
    if (M[0]->kv_len != 0 || M[1]->kv_len != 0) return fail(ST_EINVAL, "both models must start with an empty KV cache");
    if ((int64_t)P + n_out > M[0]->c.max_seq || (int64_t)P + n_out > M[1]->c.max_seq)
        return fail(ST_ERANGE, "P + n_out = %d exceeds a model's max_seq", P + n_out);
    for (int32_t i = 0; i < pol->n_aux; ++i)
        if (pol->aux_tokens[i] < 0 || pol->aux_tokens[i] >= pol->vocab) return fail(ST_ERANGE, "auxiliary token outside the vocabulary");

    auto in_class = [&](const uint32_t *bm, int32_t t) {
        return bm && t >= 0 && t < pol->vocab && ((bm[t >> 5] >> (t & 31)) & 1u);
    };
    st_gen_stats st = {};
    memcpy(seq, prompt, sizeof(int32_t) * P);
    int32_t T = P;                       // tokens in seq
    int32_t pred_pos[2] = {-1, -1};      // position the model's last feed predicted, and that token
    int32_t pred_tok[2] = {0, 0};
    double *ms_prefill[2] = {&st.ms_small_prefill, &st.ms_large_prefill};
    double *ms_decode[2] = {&st.ms_small_decode, &st.ms_large_decode};
    int rc_out = ST_OK;

    // feeds model w every token of seq it has not seen; its greedy prediction becomes pred_tok[w]
    auto feed = [&](int w) -> bool {
        Model *m = M[w];
        const int32_t lo = m->kv_len, n = T - lo;
        if (n == 0 && pred_pos[w] == T) return true;  // nothing new (a replaced sentence right after the prompt)
        auto a = clk::now();
        int rc;
        const bool own = n == 1 && pred_pos[w] == lo && pred_tok[w] == seq[lo];  // its own last token: decode step
        if (own)
            rc = decode_impl(m, nullptr, nullptr);
        else
            rc = prefill_impl(m, seq + lo, n, false, nullptr);
        if (!rc) rc = fetch_token(m, &pred_tok[w], nullptr);
        if (rc) {
            rc_out = rc;
            return false;
        }
        pred_pos[w] = T;
        *(own ? ms_decode[w] : ms_prefill[w]) += std::chrono::duration<double, std::milli>(clk::now() - a).count();
        return true;
    };
    auto done = [&]() { return T - P >= n_out; };
    if (n_out == 0) {
        if (stats) *stats = st;
        return ST_OK;
    }

    int32_t start = -1, counter = 0;     // armed sentence start (or -1) and the negativity counter
    bool all_small = true;
    int pend_kind = -1, pend_s = 0, pend_e = 0;
    // appends one output token, does the sentence bookkeeping; true when the budget is spent
    auto emit = [&](int32_t tok, int source) {
        seq[T] = tok;
        if (src) src[T - P] = (uint8_t)source;
        const int32_t pos = T++;
        if (source == ST_SRC_LARGE) ++st.n_large;
        pend_kind = -1;
        if (start >= 0) {
            if (source != ST_SRC_SMALL) all_small = false;
            if (pos == start + pol->sentence_len - 1) {
                bool neg = false, ver = false, ar = false;
                for (int32_t q = start; q <= pos; ++q) {
                    neg |= in_class(pol->neg_bitmap, seq[q]);
                    ver |= in_class(pol->verify_bitmap, seq[q]);
                    ar |= in_class(pol->ar_bitmap, seq[q]);
                }
                int kind = -1;
                if (neg && ++counter > pol->neg_threshold) {
                    counter = 0;
                    kind = ST_KIND_EXCESS;
                }
                if (kind < 0 && ver) kind = ST_KIND_VERIFY;
                if (kind < 0 && all_small && (pol->unconditional || ar)) kind = ST_KIND_AR;
                if (kind >= 0) pend_kind = kind, pend_s = start, pend_e = pos;
                start = -1;
            }
        }
        if (in_class(pol->delim_bitmap, tok)) start = pos + 1, all_small = true;
        return done();
    };
    auto log_action = [&](int kind, int32_t e, int32_t dropped, int32_t aux_lo, int32_t aux_hi, int32_t granted) {
        if (st.n_spans < action_cap) actions[st.n_spans++] = st_action{kind, e, dropped, aux_lo, aux_hi, granted};
        ++st.n_handoffs;
    };
    auto insert_aux = [&](int32_t *lo, int32_t *hi) {
        *lo = T;
        for (int32_t i = 0; i < pol->n_aux; ++i)
            if (emit(pol->aux_tokens[i], ST_SRC_AUX)) break;
        pend_kind = -1;  // the inserted sentence triggers nothing itself
        *hi = T;
    };
    // the target writes n tokens (the count restarts when (2) or (3) fires on its own text), then the speculative
    // model catches up; returns 1 when the budget ran out, 0 to continue, negative on error
    auto target_segment = [&](int32_t n, bool have_pred) -> int {
        int32_t remaining = n;
        if (!have_pred && !feed(1)) return -1;
        while (remaining > 0) {
            if (emit(pred_tok[1], ST_SRC_LARGE)) return 1;
            --remaining;
            if (pend_kind == ST_KIND_EXCESS) {
                int32_t lo, hi, e = pend_e;
                insert_aux(&lo, &hi);
                log_action(ST_KIND_EXCESS, e, 0, lo, hi, pol->n3);
                if (done()) return 1;
                remaining = pol->n3;
            } else if (pend_kind == ST_KIND_VERIFY) {
                log_action(ST_KIND_VERIFY, pend_e, 0, T, T, pol->n2);
                remaining = pol->n2;
            }
            if (remaining > 0 && !feed(1)) return -1;  // the segment's last token is not fed to the target
        }
        return feed(0) ? 0 : -1;
    };

    if (!feed(0) || !feed(1)) return rc_out;
    if (in_class(pol->delim_bitmap, seq[P - 1])) start = P, all_small = true;
    if (pol->initial_target > 0) {
        log_action(ST_KIND_INITIAL, -1, 0, P, P, pol->initial_target);
        int r = target_segment(pol->initial_target, true);
        if (r < 0) return rc_out;
        if (r > 0) goto finished;
    }
    while (true) {
        if (emit(pred_tok[0], ST_SRC_SMALL)) break;
        if (pend_kind < 0) {
            if (!feed(0)) return rc_out;
            continue;
        }
        int32_t n;
        if (pend_kind == ST_KIND_AR) {
            int32_t dropped = 0;
            if (pol->replace) {  // the drafted sentence goes; the target writes in its place
                dropped = pend_e - pend_s + 1;
                T = pend_s;
                for (int w = 0; w < 2; ++w)
                    if (M[w]->kv_len > pend_s) {
                        launch_set_state(*M[w], kPos, pend_s);
                        if (int rc = check_launch("truncate")) return rc;
                        M[w]->kv_len = pend_s;
                    }
            }
            log_action(ST_KIND_AR, pend_e, dropped, T, T, pol->n1);
            n = pol->n1;
        } else if (pend_kind == ST_KIND_VERIFY) {
            log_action(ST_KIND_VERIFY, pend_e, 0, T, T, pol->n2);
            n = pol->n2;
        } else {
            int32_t lo, hi, e = pend_e;
            insert_aux(&lo, &hi);
            log_action(ST_KIND_EXCESS, e, 0, lo, hi, pol->n3);
            if (done()) break;
            n = pol->n3;
        }
        int r = target_segment(n, false);
        if (r < 0) return rc_out;
        if (r > 0) break;
    }
finished:
    st.n_out = T - P;
    if (stats) *stats = st;
    return ST_OK;
}

// ---- a batch of independent sequences sharing one set of weights ----
namespace {
struct Batch {
    Model base;                    // sequence 0's caches; the workspace is shared by all sequences
    int32_t n_seq;
    std::vector<int32_t> kv_len;
    size_t seq_stride;             // elements between consecutive sequences' caches
    int32_t *row_ints;             // device: tok | pos | seq (row_cap each), next (n_seq)
    size_t row_cap;                // max(max_chunk, n_seq)
    float *q_rows, *o_rows, *part_ml, *part_acc, *logits;
    FlashSeg *seg_tab;             // device: kMaxBatch entries, the segment table of a ragged catch-up pass
};
constexpr int kMaxBatch = 64;

size_t batch_extra(const st_config &c, int32_t n, char *base, Batch *b) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    size_t qd = (size_t)c.n_q_heads * c.head_dim;
    if ((size_t)c.hidden > qd) qd = c.hidden;  // o_rows also holds gathered residual rows
    const size_t rows = c.max_chunk > n ? c.max_chunk : n;  // a ragged catch-up pass has up to max_chunk rows
    int32_t *ri = (int32_t *)take(sizeof(int32_t) * (3 * rows + n));
    float *q = (float *)take(sizeof(float) * n * qd), *o = (float *)take(sizeof(float) * n * qd);
    float *ml = (float *)take(sizeof(float) * (size_t)n * c.n_q_heads * kAttnSplits * 2);
    float *acc = (float *)take(sizeof(float) * (size_t)n * c.n_q_heads * kAttnSplits * c.head_dim);
    float *lg = (float *)take(sizeof(float) * (size_t)n * c.vocab);
    FlashSeg *st = (FlashSeg *)take(sizeof(FlashSeg) * kMaxBatch);
    if (b) b->row_ints = ri, b->q_rows = q, b->o_rows = o, b->part_ml = ml, b->part_acc = acc, b->logits = lg, b->seg_tab = st;
    return off;
}
int check_batch(const st_config *cfg, int32_t n_seq) {
    if (int rc = validate_config(cfg)) return rc;
    if (n_seq < 1 || n_seq > kMaxBatch) return fail(ST_ERANGE, "n_seq must be in [1, %d]", kMaxBatch);
    if (cfg->max_chunk < n_seq) return fail(ST_ERANGE, "max_chunk (%d) must be at least n_seq (%d)", cfg->max_chunk, n_seq);
    return ST_OK;
}
}  // namespace

int st_batch_query_sizes(const st_config *cfg, int32_t n_seq, size_t *kv_bytes, size_t *workspace_bytes) {
    if (int rc = check_batch(cfg, n_seq)) return rc;
    if (kv_bytes) *kv_bytes = kv_bytes_of(*cfg) * (size_t)n_seq;
    if (workspace_bytes) {
        Workspace ws;
        carve_workspace(*cfg, nullptr, &ws);
        *workspace_bytes = ws.bytes + batch_extra(*cfg, n_seq, nullptr, nullptr);
    }
    return ST_OK;
}

int st_batch_create(const st_config *cfg, const st_weights *w, int32_t n_seq, void *kv, size_t kv_bytes,
                    void *workspace, size_t workspace_bytes, void *stream, st_batch **out) {
    if (!out) return fail(ST_EINVAL, "out is NULL");
    *out = nullptr;
    if (int rc = check_batch(cfg, n_seq)) return rc;
    Workspace sized;
    carve_workspace(*cfg, nullptr, &sized);
    const size_t need_kv = kv_bytes_of(*cfg) * (size_t)n_seq, need_ws = sized.bytes + batch_extra(*cfg, n_seq, nullptr, nullptr);
    if (kv && kv_bytes < need_kv) return fail(ST_ENOMEM, "kv buffer has %zu bytes, %zu needed", kv_bytes, need_kv);
    if (workspace && workspace_bytes < need_ws)
        return fail(ST_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, need_ws);
    Batch *b = new (std::nothrow) Batch();
    if (!b) return fail(ST_ENOMEM, "out of host memory");
    if (int rc = build_model(cfg, w, kv, workspace, stream, &b->base)) {
        delete b;
        return rc;
    }
    b->base.graphs_off = true;  // the batched step is launched kernel by kernel
    b->base.persist_on = false;
    b->n_seq = n_seq;
    b->kv_len.assign(n_seq, 0);
    b->seq_stride = kv_bytes_of(*cfg) / sizeof(bf16_t);
    batch_extra(*cfg, n_seq, (char *)workspace + sized.bytes, b);
    b->row_cap = cfg->max_chunk > n_seq ? cfg->max_chunk : n_seq;
    *out = reinterpret_cast<st_batch *>(b);
    return ST_OK;
}

void st_batch_destroy(st_batch *h) { delete reinterpret_cast<Batch *>(h); }

int st_batch_attach_f16(st_batch *h, void *buf, size_t bytes) {
    if (!h) return fail(ST_EINVAL, "batch is NULL");
    return attach_f16(&reinterpret_cast<Batch *>(h)->base, buf, bytes);
}

int st_batch_kv_len(const st_batch *h, int32_t seq, int32_t *out) {
    const Batch *b = reinterpret_cast<const Batch *>(h);
    if (!b || !out) return fail(ST_EINVAL, "batch or out is NULL");
    if (seq < 0 || seq >= b->n_seq) return fail(ST_ERANGE, "sequence %d outside [0, %d)", seq, b->n_seq);
    *out = b->kv_len[seq];
    return ST_OK;
}

int st_batch_truncate(st_batch *h, int32_t seq, int32_t new_len) {
    Batch *b = reinterpret_cast<Batch *>(h);
    if (!b) return fail(ST_EINVAL, "batch is NULL");
    if (seq < 0 || seq >= b->n_seq) return fail(ST_ERANGE, "sequence %d outside [0, %d)", seq, b->n_seq);
    if (new_len < 0 || new_len > b->kv_len[seq])
        return fail(ST_ERANGE, "new_len %d outside [0, %d]", new_len, b->kv_len[seq]);
    b->kv_len[seq] = new_len;
    return ST_OK;
}

int st_batch_prefill(st_batch *h, int32_t seq, const int32_t *tokens, int32_t n, float *logits, int32_t *next_tok) {
    Batch *b = reinterpret_cast<Batch *>(h);
    if (!b) return fail(ST_EINVAL, "batch is NULL");
    if (seq < 0 || seq >= b->n_seq) return fail(ST_ERANGE, "sequence %d outside [0, %d)", seq, b->n_seq);
    Model view = b->base;  // same weights and workspace, this sequence's caches
    view.kcache = b->base.kcache + (size_t)seq * b->seq_stride;
    view.vcache = b->base.vcache + (size_t)seq * b->seq_stride;
    view.kv_len = b->kv_len[seq];
    if (int rc = prefill_impl(&view, tokens, n, false, nullptr)) return rc;
    b->kv_len[seq] = view.kv_len;
    return deliver(&view, logits, next_tok, false);
}

int st_batch_decode_step(st_batch *h, int32_t n_rows, const int32_t *seqs, const int32_t *tokens, float *logits,
                         int32_t *next_tokens) {
    Batch *b = reinterpret_cast<Batch *>(h);
    if (!b || !seqs || !tokens) return fail(ST_EINVAL, "batch, seqs or tokens is NULL");
    if (n_rows < 1 || n_rows > b->n_seq) return fail(ST_ERANGE, "n_rows must be in [1, %d]", b->n_seq);
    const st_config &c = b->base.c;
    std::vector<int32_t> host(3 * (size_t)n_rows);
    uint64_t seen = 0;
    int32_t max_pos = 0;
    for (int32_t r = 0; r < n_rows; ++r) {
        const int32_t s = seqs[r];
        if (s < 0 || s >= b->n_seq) return fail(ST_ERANGE, "sequence %d outside [0, %d)", s, b->n_seq);
        if (seen >> s & 1) return fail(ST_EINVAL, "sequence %d appears twice in one step", s);
        seen |= (uint64_t)1 << s;
        if (tokens[r] < 0 || tokens[r] >= c.vocab)
            return fail(ST_ERANGE, "token id %d of row %d is outside the vocabulary [0,%d)", tokens[r], r, c.vocab);
        if (b->kv_len[s] + 1 > c.max_seq) return fail(ST_ERANGE, "KV overflow in sequence %d", s);
        host[r] = tokens[r];
        host[n_rows + r] = b->kv_len[s];
        host[2 * (size_t)n_rows + r] = s;
        if (b->kv_len[s] > max_pos) max_pos = b->kv_len[s];
    }
    int32_t *dev = b->row_ints;
    ST_HIP(hipMemcpyAsync(dev, host.data(), sizeof(int32_t) * host.size(), hipMemcpyHostToDevice, b->base.stream));
    ST_HIP(hipStreamSynchronize(b->base.stream));  // `host` leaves scope before the copy would otherwise be read
    BatchRows rows = {dev, dev + n_rows, dev + 2 * (size_t)n_rows, dev + 3 * b->row_cap, b->seq_stride,
                      b->q_rows, b->o_rows, b->part_ml, b->part_acc, logits ? b->logits : nullptr, nullptr};
    launch_batch_step(b->base, rows, n_rows, attn_bucket(max_pos + 1));
    if (int rc = check_launch("batched decode step")) return rc;
    if (logits)
        ST_HIP(hipMemcpyAsync(logits, b->logits, sizeof(float) * (size_t)n_rows * c.vocab, hipMemcpyDeviceToHost,
                              b->base.stream));
    if (next_tokens)
        ST_HIP(hipMemcpyAsync(next_tokens, rows.row_next, sizeof(int32_t) * n_rows, hipMemcpyDeviceToHost,
                              b->base.stream));
    ST_HIP(hipStreamSynchronize(b->base.stream));
    for (int32_t r = 0; r < n_rows; ++r) b->kv_len[seqs[r]] += 1;
    return ST_OK;
}

int st_batch_prefill_many(st_batch *h, int32_t n, const int32_t *seqs, const int32_t *const *tokens,
                          const int32_t *lens, float *logits, int32_t *next_tokens) {
    Batch *b = reinterpret_cast<Batch *>(h);
    if (!b || !seqs || !tokens || !lens) return fail(ST_EINVAL, "batch, seqs, tokens or lens is NULL");
    if (n < 1 || n > b->n_seq) return fail(ST_ERANGE, "n must be in [1, %d]", b->n_seq);
    const st_config &c = b->base.c;
    int64_t R = 0;
    uint64_t seen = 0;
    for (int32_t j = 0; j < n; ++j) {
        const int32_t s = seqs[j];
        if (s < 0 || s >= b->n_seq) return fail(ST_ERANGE, "sequence %d outside [0, %d)", s, b->n_seq);
        if (seen >> s & 1) return fail(ST_EINVAL, "sequence %d appears twice", s);
        seen |= (uint64_t)1 << s;
        if (!tokens[j] || lens[j] <= 0) return fail(ST_EINVAL, "bad tokens or length of entry %d", j);
        if ((int64_t)b->kv_len[s] + lens[j] > c.max_seq) return fail(ST_ERANGE, "KV overflow in sequence %d", s);
        for (int32_t i = 0; i < lens[j]; ++i)
            if (tokens[j][i] < 0 || tokens[j][i] >= c.vocab)
                return fail(ST_ERANGE, "token id %d of entry %d is outside the vocabulary [0,%d)", tokens[j][i], j, c.vocab);
        R += lens[j];
    }
    if (R > c.max_chunk) return fail(ST_ERANGE, "%lld rows in all exceed max_chunk %d", (long long)R, c.max_chunk);
    std::vector<int32_t> host(3 * (size_t)R + n);
    std::vector<FlashSeg> segs(n);
    int32_t row = 0, blk = 0;
    for (int32_t j = 0; j < n; ++j) {
        const int32_t s = seqs[j];
        segs[j] = FlashSeg{row, lens[j], b->kv_len[s], s, blk, flash_row_blocks(c, lens[j])};
        blk += segs[j].nblk;
        for (int32_t i = 0; i < lens[j]; ++i, ++row) {
            host[row] = tokens[j][i];
            host[R + row] = b->kv_len[s] + i;
            host[2 * (size_t)R + row] = s;
        }
        host[3 * (size_t)R + j] = row - 1;  // the segment's last row
    }
    int32_t *dev = b->row_ints, *next = dev + 3 * b->row_cap;
    hipStream_t st = b->base.stream;
    ST_HIP(hipMemcpyAsync(dev, host.data(), sizeof(int32_t) * 3 * (size_t)R, hipMemcpyHostToDevice, st));
    ST_HIP(hipMemcpyAsync(next, host.data() + 3 * (size_t)R, sizeof(int32_t) * n, hipMemcpyHostToDevice, st));
    ST_HIP(hipMemcpyAsync(b->seg_tab, segs.data(), sizeof(FlashSeg) * n, hipMemcpyHostToDevice, st));
    ST_HIP(hipStreamSynchronize(st));
    BatchRows rows = {dev, dev + R, dev + 2 * (size_t)R, next, b->seq_stride, b->q_rows, b->o_rows, b->part_ml,
                      b->part_acc, logits ? b->logits : nullptr, b->seg_tab};
    set_pass_mode(&b->base, kPassDefault);
    launch_prefill_varlen(b->base, rows, segs.data(), n, (int)R);
    if (int rc = check_launch("ragged catch-up pass")) return rc;
    if (logits) ST_HIP(hipMemcpyAsync(logits, b->logits, sizeof(float) * (size_t)n * c.vocab, hipMemcpyDeviceToHost, st));
    if (next_tokens) ST_HIP(hipMemcpyAsync(next_tokens, next, sizeof(int32_t) * n, hipMemcpyDeviceToHost, st));
    ST_HIP(hipStreamSynchronize(st));
    for (int32_t j = 0; j < n; ++j) b->kv_len[seqs[j]] += lens[j];
    return ST_OK;
}

int st_generate_batch(st_batch *hs, st_batch *hl, const st_host_rule *rule, int32_t forced_period,
                      const int32_t *forced_phase, int32_t gather, int32_t n_seq,
                      const int32_t *const *prompts, const int32_t *prompt_lens, int32_t n_out, int32_t n_seg,
                      int32_t *const *seqs, uint8_t *const *srcs, st_gen_stats *stats) {
    using clk = std::chrono::steady_clock;
    auto ms_since = [](clk::time_point a) { return std::chrono::duration<double, std::milli>(clk::now() - a).count(); };
    Batch *S = reinterpret_cast<Batch *>(hs), *L = reinterpret_cast<Batch *>(hl);
    if (!S || !L || !prompts || !prompt_lens || !seqs) return fail(ST_EINVAL, "a batch, prompts, prompt_lens or seqs is NULL");
    if (S == L) return fail(ST_EINVAL, "small and large must be different batches");
    if (forced_period < 0) return fail(ST_EINVAL, "forced_period must be >= 0");
    if (forced_period == 0) {
        if (!rule || !rule->kw_bitmap || rule->vocab <= 0) return fail(ST_EINVAL, "a trigger rule (or forced_period > 0) is required");
        if (rule->window != 1 && rule->window != 2) return fail(ST_EINVAL, "window must be 1 or 2");
        if (rule->window == 2 && !rule->delim_bitmap) return fail(ST_EINVAL, "window 2 needs a delimiter bitmap");
    }
    if (n_seq < 1 || n_seq > S->n_seq || n_seq > L->n_seq) return fail(ST_ERANGE, "n_seq %d exceeds a batch", n_seq);
    if (n_out < 0 || n_seg <= 0) return fail(ST_ERANGE, "n_seg must be positive and n_out non-negative");
    if (gather < 0 || gather > n_seq) return fail(ST_ERANGE, "gather must be in [0, n_seq]");
    for (int32_t i = 0; i < n_seq; ++i) {
        if (!prompts[i] || !seqs[i] || prompt_lens[i] <= 0) return fail(ST_EINVAL, "bad prompt or output buffer of sequence %d", i);
        if (S->kv_len[i] != 0 || L->kv_len[i] != 0) return fail(ST_EINVAL, "sequence %d does not start with empty caches", i);
        if ((int64_t)prompt_lens[i] + n_out > S->base.c.max_seq || (int64_t)prompt_lens[i] + n_out > L->base.c.max_seq)
            return fail(ST_ERANGE, "sequence %d: prompt + n_out exceeds a model's max_seq", i);
    }
    auto in_class = [&](const uint32_t *bm, int32_t t) {
        return bm && t >= 0 && t < rule->vocab && ((bm[t >> 5] >> (t & 31)) & 1u);
    };
    // Per sequence: *_READY = the model's prediction (pend) is there and can be emitted; *_FEED = the emitted token
    // waits to be fed to that model by a decode step; *_CATCH = the model has to catch up on tokens it has not seen.
    enum { S_READY, S_FEED, S_CATCH, L_READY, L_FEED, L_CATCH, DONE };
    std::vector<int> who(n_seq, S_READY);
    std::vector<int32_t> T(n_seq), pend(n_seq), rem(n_seq, 0), small_count(n_seq, 0);
    if (forced_phase)
        for (int32_t i = 0; i < n_seq; ++i) {
            if (forced_phase[i] < 0) return fail(ST_EINVAL, "forced_phase[%d] is negative", i);
            small_count[i] = forced_phase[i];
        }
    st_gen_stats st = {};
    // catches the listed sequences of one batch up on every token they have not seen, as few ragged passes as
    // max_chunk allows (a span longer than max_chunk goes through the chunked single-sequence pass); pend[] gets
    // each sequence's next token
    auto catch_up = [&](st_batch *hb, Batch *B_, const std::vector<int32_t> &list, double *ms) -> int {
        auto a = clk::now();
        const int32_t cap = B_->base.c.max_chunk;
        std::vector<int32_t> ids, lens, next;
        std::vector<const int32_t *> ptrs;
        int64_t rows = 0;
        auto flush = [&]() -> int {
            if (ids.empty()) return ST_OK;
            next.resize(ids.size());
            if (int rc = st_batch_prefill_many(hb, (int32_t)ids.size(), ids.data(), ptrs.data(), lens.data(), nullptr, next.data()))
                return rc;
            for (size_t j = 0; j < ids.size(); ++j) pend[ids[j]] = next[j];
            ids.clear(), lens.clear(), ptrs.clear();
            rows = 0;
            return ST_OK;
        };
        for (int32_t i : list) {
            const int32_t lo = B_->kv_len[i], len = T[i] - lo;
            if (len > cap) {
                if (int rc = st_batch_prefill(hb, i, seqs[i] + lo, len, nullptr, &pend[i])) return rc;
                continue;
            }
            if (rows + len > cap)
                if (int rc = flush()) return rc;
            ids.push_back(i), lens.push_back(len), ptrs.push_back(seqs[i] + lo);
            rows += len;
        }
        if (int rc = flush()) return rc;
        *ms += ms_since(a);
        return ST_OK;
    };
    std::vector<int32_t> list;
    for (int32_t i = 0; i < n_seq; ++i) {
        memcpy(seqs[i], prompts[i], sizeof(int32_t) * prompt_lens[i]);
        T[i] = prompt_lens[i];
        if (n_out == 0)
            who[i] = DONE;
        else
            list.push_back(i);
    }
    if (int rc = catch_up(hl, L, list, &st.ms_large_prefill)) return rc;   // its predictions are not used
    if (int rc = catch_up(hs, S, list, &st.ms_small_prefill)) return rc;
    // One batched decode step of `b` for the listed rows; pend[] gets each row's next token.
    auto step = [&](st_batch *b, const std::vector<int32_t> &rows, const std::vector<int32_t> &toks, double *ms) -> int {
        if (rows.empty()) return ST_OK;
        std::vector<int32_t> next(rows.size());
        auto a = clk::now();
        if (int rc = st_batch_decode_step(b, (int32_t)rows.size(), rows.data(), toks.data(), nullptr, next.data())) return rc;
        *ms += ms_since(a);
        for (size_t r = 0; r < rows.size(); ++r) pend[rows[r]] = next[r];
        return ST_OK;
    };
    // The two models work on disjoint sets of sequences in every round, so their passes run side by side: the
    // target's on a stream of its own (default priority) from a second host thread, the speculative model's on the
    // calling thread.  Every call below ends with its stream idle, so the streams only have to be ordered once, here.
    hipStream_t caller_stream = L->base.stream, side_stream = nullptr;
    int device = 0;
    ST_HIP(hipGetDevice(&device));
    ST_HIP(hipStreamSynchronize(caller_stream));
    ST_HIP(hipStreamCreateWithFlags(&side_stream, hipStreamNonBlocking));
    L->base.stream = side_stream;
    struct Restore {
        Batch *L;
        hipStream_t caller, side;
        ~Restore() {
            (void)hipStreamSynchronize(side);
            L->base.stream = caller;
            (void)hipStreamDestroy(side);
        }
    } restore{L, caller_stream, side_stream};

    std::vector<int32_t> rows_s, toks_s, list_s, rows_l, toks_l, list_l, fed(n_seq, 0);
    while (true) {
        // emit what is ready and decide what each sequence needs next
        for (int32_t i = 0; i < n_seq; ++i) {
            const int32_t P = prompt_lens[i];
            if (who[i] == S_READY) {
                const int32_t tok = pend[i];
                seqs[i][T[i]++] = tok;
                if (srcs && srcs[i]) srcs[i][T[i] - 1 - P] = 0;
                ++small_count[i];
                if (T[i] - P == n_out) {
                    who[i] = DONE;
                    continue;
                }
                bool fire;
                if (forced_period > 0)
                    fire = small_count[i] % forced_period == 0;
                else
                    fire = in_class(rule->kw_bitmap, tok) &&
                           (rule->window == 1 || (T[i] >= 2 && in_class(rule->delim_bitmap, seqs[i][T[i] - 2])));
                if (fire) {
                    who[i] = L_CATCH;  // the target reads everything it has not seen, the trigger token included
                    rem[i] = n_seg;
                    ++st.n_handoffs;
                } else {
                    who[i] = S_FEED;
                    fed[i] = tok;
                }
            } else if (who[i] == L_READY) {
                const int32_t tok = pend[i];
                seqs[i][T[i]++] = tok;
                if (srcs && srcs[i]) srcs[i][T[i] - 1 - P] = 1;
                ++st.n_large;
                if (T[i] - P == n_out) {
                    who[i] = DONE;
                } else if (--rem[i] == 0) {
                    who[i] = S_CATCH;  // the segment's last token is not fed to the target
                } else {
                    who[i] = L_FEED;
                    fed[i] = tok;
                }
            }
        }
        rows_s.clear(), toks_s.clear(), list_s.clear(), rows_l.clear(), toks_l.clear(), list_l.clear();
        for (int32_t i = 0; i < n_seq; ++i) {
            if (who[i] == S_FEED) rows_s.push_back(i), toks_s.push_back(fed[i]);
            if (who[i] == S_CATCH) list_s.push_back(i);
            if (who[i] == L_FEED) rows_l.push_back(i), toks_l.push_back(fed[i]);
            if (who[i] == L_CATCH) list_l.push_back(i);
        }
        const bool small_work = !rows_s.empty() || !list_s.empty();
        bool large_work = !rows_l.empty() || !list_l.empty();
        if (!small_work && !large_work) break;
        // A pass of the target costs about the same for one sequence as for sixteen (it streams the weights
        // either way), so sequences may be held until `gather` of them wait for it -- unless nothing else can run.
        if (large_work && small_work && (int32_t)(rows_l.size() + list_l.size()) < gather) large_work = false;
        // target: the waiting hand-overs together, then its decode step; speculative model: its decode step, then
        // the segments that ended, together.  (Each model's own passes share its workspace and stay in order.)
        int rc_l = ST_OK;
        std::string err_l;
        std::thread side;
        if (large_work)
            side = std::thread([&]() {
                (void)hipSetDevice(device);
                rc_l = step(hl, rows_l, toks_l, &st.ms_large_decode);
                if (rc_l == ST_OK) rc_l = catch_up(hl, L, list_l, &st.ms_large_prefill);
                if (rc_l != ST_OK) err_l = st_last_error();
            });
        int rc_s = step(hs, rows_s, toks_s, &st.ms_small_decode);
        if (rc_s == ST_OK) rc_s = catch_up(hs, S, list_s, &st.ms_small_prefill);
        if (large_work) side.join();
        if (rc_s != ST_OK) return rc_s;
        if (rc_l != ST_OK) return fail(rc_l, "%s", err_l.c_str());
        for (int32_t i : rows_s) who[i] = S_READY;
        for (int32_t i : list_s) who[i] = S_READY;
        if (large_work) {
            for (int32_t i : rows_l) who[i] = L_READY;
            for (int32_t i : list_l) who[i] = L_READY;
        }
    }
    for (int32_t i = 0; i < n_seq; ++i) st.n_out += T[i] - prompt_lens[i];
    if (stats) *stats = st;
    return ST_OK;
}

}  // extern "C"
