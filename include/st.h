/*
 * st.h -- C ABI of the Speculative Thinking hot path on one AMD MI355X (gfx950).
 *
 * Speculative Thinking (arXiv 2504.12329, Section 3) lets a small "speculative" model write
 * most of a reasoning trace and hands fixed-length segments to a large "target" model at
 * delimiter + keyword trigger points.  Both models condition on the same token sequence, so
 * at every hand-over the model that was idle first runs a "prefix" pass over the tokens it
 * has not seen (Section 4, Table 3, Eq. 1) and then decodes.  This library is that hot path
 * for Qwen-2.5-architecture decoders: the catch-up prefill onto an existing KV cache, the
 * single-token decode step, the integer trigger scan and the hand-over itself.
 *
 * Conventions
 *  - Every call returns ST_OK (0) or a negative st_status; st_last_error() gives a
 *    thread-local message for the last failure.  All arguments are validated before any
 *    kernel is launched: a call rejected with ST_EINVAL / ST_ENOMEM / ST_ERANGE has changed nothing.  ST_EHIP
 *    (the HIP runtime failed in the middle of a call) leaves the models involved in an undefined state: destroy them.
 *    The two-model calls (st_handoff, st_generate*) can also return an error after the first model has already
 *    advanced; st_kv_len tells where each model stands.
 *  - The library never allocates device memory.  Weights, the KV cache and the workspace
 *    are device buffers owned by the caller and must outlive the model; st_query_sizes
 *    tells how large the KV cache and workspace must be.  Handles are host memory owned by
 *    the library (st_model_create / st_model_destroy).
 *  - All work of a model is enqueued on the hipStream_t given at creation (passed as
 *    void*; NULL is the default stream).  A call that returns data through a host pointer
 *    synchronises that stream before returning; with ST_OUT_DEVICE it does not.
 *  - Weights are bf16, row-major [out_features][in_features].  The KV cache is bf16 laid
 *    out [K|V][layer][kv_head][max_seq][head_dim].  Logits are fp32[vocab].
 *  - One model handle must not be used from two threads at once.
 */
#ifndef ST_H
#define ST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ST_OK = 0,
    ST_EINVAL = -1, /* null pointer, bad configuration or flag combination */
    ST_ENOMEM = -2, /* KV cache or workspace buffer smaller than st_query_sizes reports */
    ST_ERANGE = -3, /* KV cache overflow, token id outside the vocabulary, bad range */
    ST_EHIP = -4    /* the HIP runtime reported an error (message has its text) */
} st_status;

enum {
    ST_TOKENS_DEVICE = 1u, /* `tokens` / `seq` points to device memory (default: host) */
    ST_OUT_DEVICE = 2u,    /* output pointers are device memory; the call does not synchronise */
    ST_TOKEN_CHAINED = 4u, /* st_decode_step: ignore `token`, feed the model's own last greedy token
                              (kept on the device), so steps can be queued without a host round trip */
    ST_PREFILL_TWO_TERM = 8u, /* st_prefill: feed a long run of tokens in passes of at most 256 rows (the length up
                              to which the second bf16 term of the GEMM inputs costs no time) */
    ST_PREFILL_FAST = 16u    /* st_prefill: in passes of more than 128 rows round every GEMM and attention input to
                              one bf16.  By default every pass carries those inputs as two bf16 terms (16 mantissa
                              bits), which leaves the bf16 K/V cache as its only rounding: its logits are then as
                              close to an fp32 evaluation as the decode step's.  Up to about 240 rows the second
                              term costs no time (the weight stream sets it); longer passes are bound by the MFMA
                              rate and pay twice the MFMA work.  With this flag passes of 129 rows and more take
                              single bf16 inputs: 1.3x (129 rows) to 1.8x (1024 rows and more) faster, at about
                              twice the logit error at the depths the CPU oracle reaches (1.7e-2 against 0.8e-2
                              through 28 layers of the 1.5B shape) and more beyond (6.8e-2 from the decode step
                              through 64 layers of the 32B shape, where the default pass is at 1.3e-2).  Excludes
                              ST_PREFILL_TWO_TERM. */
};

/* Shape of a Qwen-2.5-architecture decoder (pre-norm, RMSNorm, rotate-half RoPE, GQA, SwiGLU). */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
    float rms_eps, rope_theta;
    int32_t tie_embeddings; /* 1: lm_head is the embedding matrix */
    int32_t qkv_bias;       /* 1: q/k/v projections have a bias (o and MLP never do) */
    int32_t max_seq;        /* KV cache capacity in positions */
    int32_t max_chunk;      /* most rows one prefill pass processes; st_prefill splits longer inputs */
} st_config;
/* Supported: head_dim 64 or 128; hidden, n_q_heads*head_dim, intermediate multiples of 8;
 * hidden <= 8192; n_q_heads a multiple of n_kv_heads with n_q_heads/n_kv_heads <= 8. */

/* Device pointers to bf16 weights.  The per-layer members are HOST arrays of n_layers device
 * pointers (copied at creation).  Row order inside the fused matrices:
 *   wqkv      [(n_q_heads + 2 n_kv_heads) * head_dim][hidden] : all q heads, then k heads, then v heads
 *   bqkv      [(n_q_heads + 2 n_kv_heads) * head_dim]          (may be NULL when qkv_bias == 0)
 *   wo        [hidden][n_q_heads * head_dim]
 *   w_gate_up [2 * intermediate][hidden]                       : gate rows [0,I), up rows [I,2I)
 *   w_down    [hidden][intermediate]
 *   norm_attn, norm_mlp, final_norm [hidden]
 *   embed, lm_head [vocab][hidden]                             (lm_head ignored when tied) */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *wqkv, *const *bqkv, *const *wo, *const *w_gate_up, *const *w_down;
    const void *const *norm_attn, *const *norm_mlp;
} st_weights;

typedef struct st_model st_model;

/* Bytes the caller must provide for the KV cache and the workspace of a model of this shape.
 * Either output may be NULL.  ST_EINVAL on an unsupported shape. */
int st_query_sizes(const st_config *cfg, size_t *kv_bytes, size_t *workspace_bytes);

/* Host-only self-check of the launch plan of a catch-up pass of `rows` rows (Section 3: the target's pass over the
 * tokens it has not seen): walks the block numbering of the four projections' GEMMs as the kernels would decode it
 * -- K slices, leftover column tiles, half-width tiles -- and verifies that every output tile and K step is
 * computed by exactly one block and that every partial-sum tile lies inside the workspace st_query_sizes reports.
 * Touches no device.  launches / blocks (may be NULL) receive the GEMM launches and working blocks of one layer
 * (0 for rows <= 192, which take the streaming kernel whatever the precision).  ST_EINVAL with the failing projection in
 * st_last_error() if the plan is inconsistent, ST_ERANGE if rows is outside 1..cfg->max_chunk. */
int st_prefill_plan_check(const st_config *cfg, int32_t rows, int32_t *launches, int32_t *blocks);

/* Creates a model over caller-owned device buffers (both 256-byte aligned).  Initialises the
 * workspace (RoPE table, counters) on `stream`; the KV length starts at 0.  The weights,
 * `kv` and `workspace` are borrowed until st_model_destroy.  Two models must not share a
 * workspace or KV buffer. */
int st_model_create(const st_config *cfg, const st_weights *w, void *kv, size_t kv_bytes,
                    void *workspace, size_t workspace_bytes, void *stream, st_model **out);
void st_model_destroy(st_model *m);

/* fp16 operand mode for catch-up passes.  The weights are bf16 numbers, and a bf16 number of magnitude between 2^-16
 * and 65504 is an fp16 number as well.  st_model_attach_f16 copies the O, gate/up and down projection matrices of
 * every layer as fp16 into `buf` (device memory owned by the caller, 256-byte aligned, st_query_f16_bytes bytes -- as
 * many as those bf16 matrices take -- borrowed until st_model_destroy or a detaching call); weights smaller than 2^-16
 * round to a multiple of 2^-24.  From then on default-precision passes of every length run those three GEMMs per
 * layer on the fp16 MFMA, with single fp16 activations instead of two bf16 terms (from 193 rows on in the MFMA-bound
 * kernels): the same MFMA rate as one bf16 term, 11 mantissa bits instead of 8.  The QKV projection keeps its input
 * in two bf16 terms and the attention its queries: what reaches the attention logits is the one place where 11 bits
 * showed (through all 64 layers of the 32B shape).  Measured against the CPU oracle, and against the decode step
 * where the oracle cannot reach, the pass is as close as the two-term pass, at about 1.1x the time of
 * ST_PREFILL_FAST.  The fp16 activations are normalised rows, attention outputs and SwiGLU products; they saturate
 * at +-65504 when written.  The K/V cache, ST_PREFILL_FAST / ST_PREFILL_TWO_TERM passes, the LM head and the decode
 * step are unchanged.
 * buf == NULL detaches.  The call runs on the model's stream and synchronises it.  ST_EINVAL if hidden,
 * n_q_heads*head_dim or intermediate is not a multiple of 64; ST_ENOMEM if `bytes` is too small; ST_ERANGE (mode not
 * enabled) if a weight is NaN or larger than 65504. */
int st_query_f16_bytes(const st_config *cfg, size_t *bytes);
int st_model_attach_f16(st_model *m, void *buf, size_t bytes);

/* Number of positions whose keys/values are cached. */
int st_kv_len(const st_model *m, int32_t *out);
/* O(1) rollback to a shorter context (0 <= new_len <= kv_len), ST_ERANGE otherwise.  Also clears the condition left
 * by a single-kernel decode step that gave up waiting (st_decode_step_kind). */
int st_kv_truncate(st_model *m, int32_t new_len);

/* The prefix / catch-up pass (paper Section 4, "prefix" stage of Table 3 and Eq. 1): feeds
 * tokens[0,n) at positions [kv_len, kv_len+n), appends their keys and values to the cache,
 * kv_len += n.  logits (fp32[vocab]) and next_tok (the greedy arg-max, lowest index on ties)
 * of the LAST fed position are written when the pointers are non-NULL.
 * Runs of more than max_chunk tokens (256 with ST_PREFILL_TWO_TERM) are fed as consecutive passes; see
 * ST_PREFILL_FAST for the precision of long passes.
 * ST_ERANGE if n <= 0, kv_len + n > max_seq, or (host tokens only) an id is outside the vocabulary;
 * ids in device memory that are out of range are clamped into the vocabulary by the kernel. */
int st_prefill(st_model *m, const int32_t *tokens, int32_t n, float *logits, int32_t *next_tok,
               uint32_t flags);

/* One decode step (paper Section 4, "decode" stage): feeds one token at position kv_len,
 * kv_len += 1, same outputs as st_prefill.  The kernels of a step are captured once per trigger rule, output buffer
 * and context-length bucket into a HIP graph (on a private stream) and replayed on the model's stream; setting the
 * environment variable ST_NO_GRAPH before st_model_create launches them one by one instead. */
int st_decode_step(st_model *m, int32_t token, float *logits, int32_t *next_tok, uint32_t flags);

/* How st_decode_step runs its kernels.  *graphs (may be NULL): step graphs captured so far.  *mode (may be NULL):
 * 0 = captured graphs are replayed; 1 = graphs were switched off with ST_NO_GRAPH; 2 = a capture or instantiation
 * failed -- the HIP message was left in st_last_error() by the call that hit it -- and every step since has been
 * launched kernel by kernel (same results, about a tenth slower).  ST_EINVAL if m is NULL. */
int st_decode_graph_state(const st_model *m, int32_t *graphs, int32_t *mode);

/* Which form of the decode step (paper Section 4, "decode" stage) the model runs.  *kind: 0 = one kernel per stage
 * (the default); 1 = the whole step is one persistent kernel, one block per compute unit, whose stages hand their
 * vectors over through {value, epoch} words in the workspace.  The persistent form is chosen at st_model_create when
 * ST_DECODE_PERSIST=1 is in the environment and the shape fits it (every row length at least 256, its LDS plan within
 * 160 KB); it is kept as a measured alternative -- 5-10 % slower than the default on the 1.5B / 7B / 32B shapes.
 * Both forms meet the same tolerance; their sums are ordered differently, so logits differ in the last bits.  The
 * persistent form needs all its blocks resident at once: while a step runs, other work on the GPU that occupies
 * compute units for long delays it, and if a wait inside it exceeds its limit (ST_PERSIST_SPIN polling rounds,
 * default 2^20, about a second) the step gives up and the next call that reads results back returns ST_EHIP.
 * ST_EINVAL if m or kind is NULL. */
int st_decode_step_kind(const st_model *m, int32_t *kind);

/* Host-only: the plan of the single-kernel decode step for a model shape on a GPU with n_cu compute units (one block
 * per unit), without touching a device.  On success *lds_bytes is the LDS one block asks for (at most 160 KB, and
 * more than half of it so that a compute unit holds exactly one block), *handover_words the 8-byte {value, epoch}
 * words st_query_sizes adds to the workspace, regions[7] the word offsets of the seven hand-over regions (x, q/k/v,
 * range records, attention vector, x after attention, SwiGLU vector, arg-max candidates; ascending, non-overlapping)
 * and parts[5] the K parts a weight row is cut into in the QKV, O, gate/up, down and LM-head stages (1, 2, 4 or 8).
 * Any output pointer may be NULL.  ST_EINVAL if the shape does not fit the step (a row shorter than 256 elements, the
 * LDS plan above 160 KB, fewer than 8 or more than 1024 compute units, fewer units than kv heads). */
int st_decode_persist_plan(const st_config *cfg, int32_t n_cu, size_t *lds_bytes, size_t *handover_words,
                           int32_t *regions, int32_t *parts);

/* n chained greedy decode steps: feeds first_token (or the model's own last greedy token when
 * ST_TOKEN_CHAINED is set), then each step's arg-max, writing the n produced tokens to
 * out_tokens (host, or device with ST_OUT_DEVICE).  kv_len += n.  Nothing returns to the
 * host between steps. */
int st_decode_greedy(st_model *m, int32_t first_token, int32_t n, int32_t *out_tokens, uint32_t flags);

/* Token-level form of the takeover trigger (Section 3 (1); keyword sets of Appendix C become
 * sets of token ids).  window == 1: a position p fires when tokens[p] is in the keyword set.
 * window == w + 1 >= 2: p fires when the w tokens ending at p are the sentence after a delimiter
 * (tokens[p-w] is a delimiter, none of tokens[p-w+1 .. p-1] is) and one of them is a keyword;
 * w == 1 is "delimiter, then keyword".  Sets are bitmaps over the vocabulary (bit id&31 of 32-bit
 * word id>>5) in device memory.  The decode step and st_generate evaluate windows 1 and 2 next to the
 * arg-max; st_trigger_scan accepts windows up to ST_MAX_SCAN_WINDOW (sentences of n1 tokens). */
#define ST_MAX_SCAN_WINDOW 257
typedef struct {
    const uint32_t *kw_bitmap, *delim_bitmap; /* device; delim may be NULL when window == 1 */
    int32_t window;
    int32_t vocab;
} st_trigger_rule;

/* Scans tokens[lo,hi) (device memory, int32): writes the first min(count, cap) firing
 * positions in ascending order to positions[] and the total count to *n_found.  positions and
 * n_found are host pointers (the call synchronises `stream`) unless ST_OUT_DEVICE is set;
 * `scratch` is cap+1 int32 of device memory used for the result in the host-output case (may be
 * NULL with ST_OUT_DEVICE).  Ids outside the vocabulary never fire.  ST_ERANGE if lo < 0 or hi < lo. */
int st_trigger_scan(const st_trigger_rule *rule, const int32_t *tokens, int32_t lo, int32_t hi,
                    int32_t *positions, int32_t cap, int32_t *n_found, int32_t *scratch,
                    void *stream, uint32_t flags);

/* st_trigger_scan with host outputs for callers that cannot allocate device memory (code under HIP graph capture
 * set-up, tight serving loops, harnesses that forbid hipMalloc): the device staging that st_trigger_scan takes as
 * `scratch` is a static device array inside the library instead, ST_SCAN_STATIC_MAX_CAP positions + the count
 * (16 KB + 4 B on every GPU the library runs on, held until the process ends).  Same results as st_trigger_scan:
 * the first min(count, cap) firing positions of tokens[lo,hi) (device memory) ascending in positions[] and the
 * total count in *n_found, both HOST memory; synchronises `stream`.  Calls no hipMalloc / hipFree.  ST_ERANGE if
 * cap > ST_SCAN_STATIC_MAX_CAP (or the range is bad), otherwise the errors of st_trigger_scan.  All calls on one
 * GPU share that GPU's array: two calls that overlap in time on the same GPU (different host threads or streams)
 * race and must be serialised by the caller. */
#define ST_SCAN_STATIC_MAX_CAP 4096
int st_trigger_scan_static(const st_trigger_rule *rule, const int32_t *tokens, int32_t lo, int32_t hi,
                           int32_t *positions, int32_t cap, int32_t *n_found, void *stream);

/* Half-open absolute position spans touched by one hand-over. */
typedef struct {
    int32_t large_prefill_lo, large_prefill_hi; /* tokens the target caught up on */
    int32_t large_decode_lo, large_decode_hi;   /* positions the target wrote */
    int32_t small_prefill_lo, small_prefill_hi; /* tokens the speculative model caught up on (empty if the
                                                   budget ended inside the segment) */
} st_spans;

/* One takeover (Section 3 (1)): seq[0,*T) is the shared sequence in HOST memory (capacity at
 * least *T + min(n_large, budget)); seq[*T-1] is the trigger token, already written but not yet
 * fed to `small`.  The target catches up on seq[kv_len(large), *T), greedily writes
 * min(n_large, budget) tokens to seq (feeding itself all but the last), then, unless the
 * budget ended the segment early (budget <= n_large), the speculative model catches up on
 * seq[kv_len(small), *T').  On return *T is the new length; small_next_tok (and small_logits,
 * fp32[vocab], may be NULL) hold the speculative model's prediction for position *T when a
 * catch-up ran.  All pointers are host memory. */
int st_handoff(st_model *small, st_model *large, int32_t *seq, int32_t *T, int32_t n_large,
               int32_t budget, float *small_logits, int32_t *small_next_tok, st_spans *spans,
               uint32_t flags);

/* Statistics of one st_generate run. */
typedef struct {
    int32_t n_out;        /* output tokens written */
    int32_t n_handoffs;   /* takeovers */
    int32_t n_large;      /* tokens written by the target (modify ratio = n_large / n_out) */
    int32_t n_spans;      /* entries written to `spans` */
    double ms_small_decode, ms_large_decode, ms_small_prefill, ms_large_prefill; /* host wall clock */
} st_gen_stats;

/* The whole loop of Section 3 (1) with append semantics: both models prefill prompt[0,P);
 * the speculative model decodes greedily; whenever the rule fires on a token IT emitted the
 * target takes over for n_seg tokens (st_handoff); stops after n_out output tokens.
 * forced_period > 0 replaces the rule by "every forced_period-th speculative token fires"
 * (used to reproduce a given modify ratio with random weights).
 * seq (host, capacity P + n_out) receives prompt + outputs; src (host, n_out bytes, may be NULL)
 * receives 0 for speculative / 1 for target per output token; spans (host, capacity span_cap,
 * may be NULL) one entry per takeover. */
int st_generate(st_model *small, st_model *large, const st_trigger_rule *rule, int32_t forced_period,
                const int32_t *prompt, int32_t P, int32_t n_out, int32_t n_seg,
                int32_t *seq, uint8_t *src, st_spans *spans, int32_t span_cap, st_gen_stats *stats);

/* The full takeover policy of Section 3 on token ids: after every delimiter (written by either model, or the
 * prompt's last token) the next `sentence_len` tokens form a sentence (a delimiter inside it restarts it); when its
 * last token has been written -- and is not the last budgeted token -- it is classified:
 *   (3) a sentence holding a `neg` token raises a counter; when the counter exceeds neg_threshold it restarts, the
 *       auxiliary sentence aux_tokens is inserted and the target writes n3 tokens;
 *   (2) else a sentence holding a `verify` token: the target writes n2 tokens;
 *   (1) else, if the speculative model wrote the whole sentence and it holds an `ar` token (or `unconditional` is
 *       set): the target writes n1 tokens -- after the sentence, or, with `replace`, in its place (the sentence is
 *       dropped from seq and both KV caches are truncated to its start).
 * (2) and (3) also fire on sentences inside the target's own segment: the tokens it still owes are replaced by the
 * new grant.  The target first catches up on every token it has not seen; the last token it writes is not fed to
 * it; the speculative model then catches up.  With initial_target > 0 the target writes that many tokens first.
 * Bitmaps are HOST arrays of `vocab` bits (bit t of word t/32); NULL is the empty class.  aux_tokens is host memory. */
typedef struct {
    const uint32_t *delim_bitmap, *ar_bitmap, *verify_bitmap, *neg_bitmap;
    int32_t vocab;
    int32_t sentence_len;
    int32_t n1, n2, n3;
    int32_t neg_threshold;
    const int32_t *aux_tokens;
    int32_t n_aux;
    int32_t replace, unconditional, initial_target;
} st_policy;

enum { ST_KIND_INITIAL = 0, ST_KIND_AR = 1, ST_KIND_VERIFY = 2, ST_KIND_EXCESS = 3 };
enum { ST_SRC_SMALL = 0, ST_SRC_LARGE = 1, ST_SRC_AUX = 2 };

/* One takeover: its kind, the position of the sentence's last token (-1 for the initial segment), tokens dropped
 * by the replace reading, the positions of the inserted auxiliary sentence [aux_lo, aux_hi) (empty otherwise:
 * both are the position where the target starts writing), and the tokens granted to the target. */
typedef struct {
    int32_t kind, sentence_end, dropped, aux_lo, aux_hi, granted;
} st_action;

/* Runs the policy until n_out output tokens exist.  Both models must have empty caches.  seq (host, capacity
 * P + n_out) receives prompt + outputs; src (host, n_out bytes, may be NULL) an ST_SRC_* per output token; actions
 * (host, capacity action_cap, may be NULL) one entry per takeover in order; stats->n_handoffs counts them all,
 * stats->n_spans those written.  Errors: ST_EINVAL (NULL or malformed policy), ST_ERANGE (P + n_out exceeds a
 * model's max_seq, token id outside the vocabulary), ST_EHIP. */
int st_generate_policy(st_model *small, st_model *large, const st_policy *policy, const int32_t *prompt, int32_t P,
                       int32_t n_out, int32_t *seq, uint8_t *src, st_action *actions, int32_t action_cap,
                       st_gen_stats *stats);

/* A batch of up to 64 independent sequences that share one set of weights (the many-concurrent-sequences regime
 * the paper's outlook describes): every sequence has its own KV cache and length; one decode step advances any
 * subset of them by one token each, streaming the weights once for all rows.  Sizes as for a model, times n_seq
 * for the cache; cfg->max_chunk must be at least n_seq.  All token / logits pointers are host memory and the
 * calls synchronise the stream.  Errors as for the single-sequence calls. */
typedef struct st_batch st_batch;
int st_batch_query_sizes(const st_config *cfg, int32_t n_seq, size_t *kv_bytes, size_t *workspace_bytes);
int st_batch_create(const st_config *cfg, const st_weights *w, int32_t n_seq, void *kv, size_t kv_bytes,
                    void *workspace, size_t workspace_bytes, void *stream, st_batch **out);
void st_batch_destroy(st_batch *b);
/* st_model_attach_f16 for the weights a batch shares (same buffer size, same errors). */
int st_batch_attach_f16(st_batch *b, void *buf, size_t bytes);
int st_batch_kv_len(const st_batch *b, int32_t seq, int32_t *out);
int st_batch_truncate(st_batch *b, int32_t seq, int32_t new_len);
/* Feeds n tokens to sequence `seq` (catch-up pass of that sequence alone); logits (fp32[vocab]) and next_tok of the
 * last position if not NULL. */
int st_batch_prefill(st_batch *b, int32_t seq, const int32_t *tokens, int32_t n, float *logits, int32_t *next_tok);
/* Ragged catch-up pass: feeds tokens[j][0 .. lens[j]) to the distinct sequences seqs[j], j < n, in one pass (the
 * weights are streamed once for all of them); the lengths may differ and must not add up to more than
 * cfg->max_chunk.  logits (fp32[n][vocab], may be NULL) and next_tokens[j] (may be NULL) are those of each
 * sequence's last position. */
int st_batch_prefill_many(st_batch *b, int32_t n, const int32_t *seqs, const int32_t *const *tokens,
                          const int32_t *lens, float *logits, int32_t *next_tokens);
/* One decode step for the n_rows distinct sequences seqs[r], feeding tokens[r] at each sequence's own position
 * (ragged lengths): logits (fp32[n_rows][vocab], may be NULL) and greedy next_tokens[r] (may be NULL); every listed
 * sequence grows by one.  A row's logits do not depend on the other rows, their number or the row order (the sums are
 * formed in one order for every n_rows); they differ in rounding from st_decode_step's, which uses other kernels. */
int st_batch_decode_step(st_batch *b, int32_t n_rows, const int32_t *seqs, const int32_t *tokens, float *logits,
                         int32_t *next_tokens);

/* The takeover rule with HOST bitmaps (the batched loop reads every token back and evaluates it on the host);
 * window 1 or 2 as in st_trigger_rule. */
typedef struct {
    const uint32_t *kw_bitmap, *delim_bitmap;
    int32_t window, vocab;
} st_host_rule;

/* The loop of st_generate for n_seq independent sequences at once (Section 3 (1), append semantics; the batched
 * regime of the paper's outlook): sequence i lives in slot i of both batches (empty caches), starts from
 * prompts[i][0 .. prompt_lens[i]) and ends after n_out output tokens.  Every round runs one decode step of the
 * speculative batch over the sequences that model is writing and one of the target batch over those inside a
 * segment; a sequence that triggers catches the target up with its own prefill pass and joins the target's steps
 * for n_seg tokens, then catches the speculative model up and rejoins it.  Per sequence the result is that of
 * st_generate.  forced_period > 0 replaces the rule by "every forced_period-th speculative token fires"; with
 * forced_phase (host, n_seq entries >= 0, may be NULL = all zero) sequence i's count of speculative tokens starts
 * at forced_phase[i], which staggers the hand-overs of the sequences.  The two models' passes of a round cover
 * disjoint sequences and are issued side by side (the target's from a second host thread on a stream of its own).
 * gather in [0, n_seq]: while the speculative model still has work, the target starts a pass only once at least
 * `gather` sequences wait for it (a pass costs about the same for one sequence as for many); 0 or 1 = at once.
 * Scheduling changes when a token is computed, never which token: every policy gives the same sequences.
 * seqs[i] (host, capacity prompt_lens[i] + n_out) receives prompt + outputs, srcs[i] (host, n_out bytes; srcs or any
 * entry may be NULL) 0 / 1 per output token.  stats sums over the sequences. */
int st_generate_batch(st_batch *small, st_batch *large, const st_host_rule *rule, int32_t forced_period,
                      const int32_t *forced_phase, int32_t gather, int32_t n_seq, const int32_t *const *prompts, const int32_t *prompt_lens, int32_t n_out,
                      int32_t n_seg, int32_t *const *seqs, uint8_t *const *srcs, st_gen_stats *stats);

/* Measurement support: one chained greedy decode step (feeds the model's own last token) in which
 * every launch of the gate/up projection kernel -- the kernel that moves the most bytes of a step
 * (2 * intermediate * hidden bf16 weights per launch) -- carries HIP start/stop events on the
 * model's stream.  Synchronises the stream.  *gateup_mean_us is the mean device time of the
 * n_layers launches, *step_us the device time of the whole step.  kv_len += 1. */
int st_decode_step_timed(st_model *m, double *gateup_mean_us, double *step_us);

const char *st_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
