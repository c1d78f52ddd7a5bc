// Host-side internals of the library: the model record, workspace carving and the launchers
// the API layer calls.  Nothing here is part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/st.h"

namespace st {

typedef uint16_t bf16_t;

// ---- the persistent single-kernel decode step (persist.hip) ----
constexpr int kPersistThreads = 512;  // threads of its blocks (one block per compute unit)
struct PersistLayer {                 // device table: weights of one layer
    const bf16_t *wqkv, *bqkv, *wo, *wgu, *wdown, *norm_attn, *norm_mlp, *pad;
};
// Geometry of the step for a model shape on a device with nb compute units: regions of the hand-over words (offsets
// in 8-byte words), attention split, LDS size.
struct PersistPlan {
    int nb;        // blocks
    int s_cap;     // most key ranges per kv head
    int dsl;       // output elements per work item of the range merge
    int kmax;      // longest GEMV input (floats of LDS for it)
    int lp_qkv, lp_o, lp_gu, lp_dn, lp_lm;  // log2 of the K parts a row is cut into, per stage
    size_t lds_bytes;
    int off_x, off_qkv, off_part, off_attn, off_x2, off_act, off_cand;
    size_t ll_words;
};
struct PersistArgs {
    const PersistLayer *layers;
    const bf16_t *embed, *lm_head, *final_norm;
    bf16_t *kc, *vc;
    int32_t *state;
    const float2 *rope;
    unsigned long long *ll;
    float *logits;
    int L, h, nq, nkv, I, V, max_seq;
    float eps;
    int s_cap, dsl, kmax;
    int lp_qkv, lp_o, lp_gu, lp_dn, lp_lm;
    int off_x, off_qkv, off_part, off_attn, off_x2, off_act, off_cand;
    int spin_limit;
};

struct PersistRule {  // what changes from launch to launch: trigger rule and output buffer
    const uint32_t *kw, *delim;
    int32_t *out_seq;
    int window, rule_vocab;
};

struct Workspace {
    int32_t *state;        // kStateInts
    int32_t *counters;     // n_kv_heads arrival counters of the split attention
    float2 *rope;          // [max_seq][head_dim/2] (cos, sin)
    int32_t *tokens;       // [max_chunk] staged ids
    int32_t *out_tokens;   // [max_seq] tokens produced by chained steps
    float *x;              // [max_chunk][hidden] residual stream
    bf16_t *xn;            // [max_chunk][hidden] normalised rows (GEMM input)
    float *qkv;            // partial_floats(cfg) floats: split-K partial results of the prefill GEMMs
    bf16_t *qb;            // [max_chunk][n_q*d] rotated queries
    bf16_t *attn;          // [max_chunk][n_q*d] attention output (GEMM input)
    bf16_t *act;           // [max_chunk][intermediate] SwiGLU output
    bf16_t *xn_lo, *attn_lo, *act_lo;  // [max_chunk][...] second bf16 terms of the three above
    bf16_t *qb_lo;         // [max_chunk][n_q*d] second bf16 term of the rotated queries
    float *q1;             // [n_q*d] decode query
    float *o1;             // [n_q*d] decode attention output
    float *a1;             // [intermediate] decode SwiGLU output
    float *part_ml;        // [n_q][splits][2]
    float *part_acc;       // [n_q][splits][d]
    float *logits;         // [vocab]
    float *amax_val;       // [kLmBlocks]
    int32_t *amax_idx;     // [kLmBlocks]
    unsigned long long *ll;  // hand-over words of the persistent decode step (PersistPlan::ll_words; may be empty)
    PersistLayer *ptab;      // [n_layers] its table of weight pointers
    PersistArgs *pargs;      // its per-model arguments
    size_t bytes;
};

// Rows of the decode attention: row z attends with its new token at position pos[z] to the cache of sequence
// seq[z] (seq == nullptr: sequence 0), caches seq_stride elements apart; q / out rows q_stride floats apart and
// the per-row partial buffers ml_stride / acc_stride floats apart.  With out_hi / out_lo the result is written as two
// bf16 terms (rows q_stride elements apart: the input of the O projection GEMM) instead of fp32.
struct AttnRows {
    const int32_t *pos, *seq;
    size_t seq_stride;
    int q_stride;
    size_t ml_stride, acc_stride;
    bf16_t *out_hi, *out_lo;
};

// Inputs that may carry a second bf16 term in a pass of more than 256 rows (Model::long_terms): the activations of
// the four projections and the rotated queries of the attention
enum LongTerms { kTermQKV = 1, kTermO = 2, kTermGateUp = 4, kTermDown = 8, kTermQuery = 16, kTermAll = 31 };
constexpr int kDefaultLongTerms = kTermAll;
// Passes of at least this many rows take the 256 x 256 ring GEMMs, shorter ones the weight-streaming kernel.  Measured
// per layer of the 32B shape on 4096 cached keys, streaming against ring kernel -- two bf16 terms: 129 rows 0.50 / 0.60,
// 224 rows 0.63 / 0.64, 256 rows 0.69 / 0.64 ms; one term (fp16 operands): 129 rows 0.36 / 0.40, 160 rows 0.38 / 0.41,
// 192 rows 0.41 / 0.42, 224 rows 0.47 / 0.43, 256 rows 0.50 / 0.44 ms (single bf16: 0.02-0.03 ms less on both sides).
constexpr int kRingMinRows = 241;      // two bf16 terms
constexpr int kRingMinRowsFast = 193;  // one term: ST_PREFILL_FAST, or the fp16 operand mode

constexpr int kLmBlocks = 1024;   // blocks (and arg-max partials) of the LM-head kernel
constexpr int kAttnSplits = 128;  // most key ranges one kv head is split into at decode

// Events recorded by a timed step: [0] step start, [1] step stop, then one (start, stop) pair per layer.
struct StepTimers {
    std::vector<hipEvent_t> ev;
};

// One captured decode step (all kernels of a token) for a given trigger rule / output buffer.
struct StepGraph {
    const void *kw, *delim, *out_seq;
    int window, vocab;
    int attn_blocks;  // key ranges the attention grid provides (context-length bucket)
    hipGraphExec_t exec;
};

struct Model {
    st_config c;
    std::vector<const bf16_t *> wqkv, bqkv, wo, wgu, wdown, norm_attn, norm_mlp;
    const bf16_t *embed, *lm_head, *final_norm;
    bf16_t *kcache, *vcache;   // [layer][kv_head][max_seq][d]
    Workspace ws;
    hipStream_t stream;
    int32_t kv_len;
    int qkv_dim;
    StepTimers *timers;  // non-null only inside st_decode_step_timed
    hipStream_t capture_stream;      // private stream the step graphs are captured on (lazily created)
    std::vector<StepGraph> graphs;
    bool graphs_off;                 // capture failed or was disabled: steps are launched kernel by kernel
    bool graph_failed;               // graphs_off because a capture or instantiation failed (reported, not silent)
    int long_terms;                  // LongTerms mask of the pass being enqueued (see pass_terms in prefill.hip)
    int ring_min_rows;               // passes of at least this many rows take the 256 x 256 ring GEMMs
    // fp16 copies of the O, gate/up and down projection matrices of every layer (st_model_attach_f16), empty until
    // attached
    std::vector<const bf16_t *> wo16, wgu16, wdown16;
    bool f16_on;                     // the copies exist
    bool f16_pass;                   // the pass being enqueued uses them (default precision only)
    // persistent single-kernel decode step: on when the shape fits (persist_plan) and ST_DECODE_PERSIST is not 0
    bool persist_on;
    PersistPlan persist;
    int persist_spin_limit;          // polling rounds a wait may take before the step gives up
    long persist_launches;           // since the hand-over words were last cleared
    std::vector<PersistLayer> ptab_host;
    PersistArgs pargs_host;
};

// Records the thread's error message (st_last_error) and returns `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// Carves the workspace; with base == nullptr only sizes it.
void carve_workspace(const st_config &c, char *base, Workspace *ws);
// Compute units the persistent decode step is planned for (those of the current device; 0 if it cannot be read).
int persist_cu_count();

// ---- launchers (decode.hip) ----
void launch_init(const Model &m);
void launch_set_token(const Model &m, int32_t token);
void launch_set_token_from(const Model &m, const int32_t *tokens_dev, int32_t index);
void launch_set_state(const Model &m, int slot, int32_t value);
// Runs one whole single-token step on the model's stream: embeds state[kTok] at state[kPos],
// all layers, LM head, arg-max; leaves state[kTok] = greedy token and state[kPos] += 1.
// rule may be null (state[kFired] is then 0).  out_seq (device, may be null) receives the token at
// index state[kStep]++.
void launch_decode_step(const Model &m, const st_trigger_rule *rule, int32_t *out_seq_dev, hipStream_t stream,
                        int attn_blocks);
// Key ranges the decode attention needs for a context of t keys, rounded up to a bucket (the grid of
// a captured step is fixed, so steps are captured per bucket).
int attn_bucket(int t);
// Decode attention of layer `layer` for n_rows rows of a batch (see AttnRows); m.kcache / m.vcache are the caches of
// sequence 0.
void launch_attn_rows(const Model &m, int layer, hipStream_t stream, int attn_blocks, const AttnRows &rows, int n_rows,
                      const float *q, float *part_ml, float *part_acc, float *out);
// Embedding of state[kTok] and all layers at position state[kPos], on the residual row x (fp32[hidden]).
void launch_decode_layers(const Model &m, float *x, hipStream_t stream, int attn_blocks);
// LM head + arg-max over the residual row x_row (fp32[hidden]); advances state[kPos] by `advance`.
void launch_head(const Model &m, const float *x_row, const st_trigger_rule *rule, int32_t advance,
                 int32_t *out_seq_dev, hipStream_t stream);

// ---- launchers (persist.hip) ----
// Plans the persistent step for a shape on n_cu compute units; false if the shape does not fit it.
bool persist_plan(const st_config &c, int n_cu, PersistPlan *out);
hipError_t persist_prepare(const Model &m);  // raises the kernel's LDS limit (once per model)
void launch_persist_reset(const Model &m);   // clears the hand-over words, the launch counter and the error flag
PersistArgs persist_args(const Model &m);    // the per-model arguments (to be copied to Workspace::pargs)
// The whole single-token step as one kernel: same contract as launch_decode_step.
void launch_decode_persist(const Model &m, const st_trigger_rule *rule, int32_t *out_seq_dev, hipStream_t stream);

// ---- launchers (prefill.hip) ----
// Feeds ws.tokens[0,n) at positions [pos0, pos0+n) through all layers; leaves the residual rows in ws.x.
// Host walk over the block numbering of the long-chunk GEMM (0 = every tile and K step covered exactly once and
// every partial-sum tile inside cap_floats; negative = which check failed).
int ring_plan_check(int dual, int M, int N, int K, long long cap_floats, int allow_tail, int *launches_out,
                    int *blocks_out, int *ids_out);
size_t partial_floats(const st_config &c);  // floats of Workspace::qkv (the split-K / split-key partial results)
hipError_t raise_lds_limits();              // once per process, before the first ring / streaming GEMM launch
// fp16 operand mode: element-wise copy of n bf16 numbers as fp16 (counts the ones no half can hold in *bad), and
// whether a model shape can run in that mode
void launch_f16_copy(const Model &m, const bf16_t *src, bf16_t *dst, size_t n, int32_t *bad);
bool f16_shape_ok(const st_config &c);
void launch_prefill_layers(const Model &m, int32_t pos0, int32_t n);

// Device arrays of one batched decode step (n rows = n sequences, each at its own position).
struct BatchRows {
    const int32_t *row_tok, *row_pos, *row_seq;  // [n] token fed, its position, sequence index
    int32_t *row_next;                           // [n] greedy next token
    size_t seq_stride;                           // elements between the caches of consecutive sequences
    float *q_rows, *o_rows;                      // [n][n_q*d]
    float *part_ml, *part_acc;                   // [n][n_q][kAttnSplits][2 | d]
    float *logits;                               // [n][vocab] or nullptr
    const struct FlashSeg *seg_tab;              // device: segment table of a ragged catch-up pass (else nullptr)
};
// All layers, LM head and arg-max for n rows (n <= 64); m.kcache / m.vcache are the caches of sequence 0.
void launch_batch_step(const Model &m, const BatchRows &b, int n, int attn_blocks);
// One segment of a ragged catch-up pass: query rows [row0, row0 + len) of the pass are positions kv0 .. kv0 + len - 1
// of sequence `seq`; the attention launch gives it the row blocks [blk0, blk0 + nblk) of grid.x
// (nblk = flash_row_blocks(cfg, len)).
struct FlashSeg {
    int32_t row0, len, kv0, seq, blk0, nblk;
};
int flash_row_blocks(const st_config &c, int len);
// Ragged catch-up over R rows of n_seg sequences (R <= max_chunk); b.row_next holds the row index of every
// segment's last row on entry and the greedy next tokens on return; b.o_rows needs n_seg * hidden floats; segs is
// the host copy of the segment table already uploaded to b.seg_tab.
void launch_prefill_varlen(const Model &m, const BatchRows &b, const FlashSeg *segs, int n_seg, int R);

// ---- launchers (trigger.hip) ----
void launch_trigger_scan(const st_trigger_rule &rule, const int32_t *tokens, int32_t lo, int32_t hi,
                         int32_t *positions, int32_t cap, int32_t *n_found, hipStream_t stream);

}  // namespace st
