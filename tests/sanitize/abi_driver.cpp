// Host-side walk over the C ABI's argument validation and launch planning -- everything the library does before
// its first kernel launch -- for a build of the library sources with -fsanitize=address,undefined on the host
// pass (tests/test_sanitizers.py).  Needs no GPU: every call here returns before touching a device.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/st.h"

#define CHECK(c)                                                                                   \
    do {                                                                                           \
        if (!(c)) {                                                                                \
            std::fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #c, st_last_error()); \
            return 1;                                                                              \
        }                                                                                          \
    } while (0)

static st_config shape(int layers, int h, int nq, int nkv, int d, int I, int V, int tie, int max_seq, int max_chunk) {
    st_config c;
    std::memset(&c, 0, sizeof c);
    c.n_layers = layers, c.hidden = h, c.n_q_heads = nq, c.n_kv_heads = nkv, c.head_dim = d, c.intermediate = I;
    c.vocab = V, c.rms_eps = 1e-6f, c.rope_theta = 1e6f, c.tie_embeddings = tie, c.qkv_bias = 1;
    c.max_seq = max_seq, c.max_chunk = max_chunk;
    return c;
}

int main() {
    const st_config shapes[] = {
        shape(2, 256, 4, 2, 64, 688, 1024, 0, 256, 64),
        shape(28, 1536, 12, 2, 128, 8960, 151936, 1, 8192, 4096),
        shape(28, 3584, 28, 4, 128, 18944, 152064, 0, 8192, 4096),
        shape(64, 5120, 40, 8, 128, 27648, 152064, 0, 8256, 4096),
        shape(1, 4288, 6, 1, 128, 2240, 2048, 0, 4200, 4096),
    };
    for (const st_config &c : shapes) {
        size_t kv = 0, ws = 0;
        CHECK(st_query_sizes(&c, &kv, &ws) == ST_OK && kv > 0 && ws > 0);
        CHECK(st_query_sizes(&c, nullptr, nullptr) == ST_OK);
        for (int rows = 1; rows <= c.max_chunk; rows += (rows < 300 ? 37 : 211)) {
            int32_t launches = -1, blocks = -1;
            CHECK(st_prefill_plan_check(&c, rows, &launches, &blocks) == ST_OK);
            CHECK(launches >= 0 && blocks >= 0 && (rows <= 256 || c.hidden % 64 || launches >= 4));
        }
        CHECK(st_prefill_plan_check(&c, c.max_chunk, nullptr, nullptr) == ST_OK);
        CHECK(st_prefill_plan_check(&c, 0, nullptr, nullptr) == ST_ERANGE);
        CHECK(st_prefill_plan_check(&c, c.max_chunk + 1, nullptr, nullptr) == ST_ERANGE);
        size_t bkv = 0, bws = 0;
        if (c.max_chunk >= 16) {
            CHECK(st_batch_query_sizes(&c, 16, &bkv, &bws) == ST_OK && bkv == 16 * kv && bws > ws);
        }
        CHECK(st_batch_query_sizes(&c, 0, &bkv, &bws) == ST_ERANGE && st_batch_query_sizes(&c, 65, &bkv, &bws) == ST_ERANGE);
        // the fp16 weight copy: as many bytes as the bf16 O, gate/up and down matrices, only where every K is a multiple of 64
        size_t f16 = 0;
        const int rc16 = st_query_f16_bytes(&c, &f16);
        if (c.hidden % 64 == 0 && c.intermediate % 64 == 0 && (c.n_q_heads * c.head_dim) % 64 == 0) {
            const size_t qd = (size_t)c.n_q_heads * c.head_dim, h = c.hidden;
            CHECK(rc16 == ST_OK && f16 == 2 * (size_t)c.n_layers * (h * qd + 3 * h * (size_t)c.intermediate));
        } else {
            CHECK(rc16 == ST_EINVAL);
        }
        CHECK(st_query_f16_bytes(&c, nullptr) == ST_EINVAL);
    }
    // rejected shapes
    st_config bad = shapes[0];
    bad.head_dim = 96;
    CHECK(st_query_sizes(&bad, nullptr, nullptr) == ST_EINVAL);
    bad = shapes[0], bad.hidden = 257;
    CHECK(st_query_sizes(&bad, nullptr, nullptr) == ST_EINVAL);
    bad = shapes[0], bad.n_q_heads = 3;
    CHECK(st_query_sizes(&bad, nullptr, nullptr) == ST_EINVAL);
    bad = shapes[0], bad.n_q_heads = 18, bad.n_kv_heads = 2;
    CHECK(st_query_sizes(&bad, nullptr, nullptr) == ST_EINVAL);
    bad = shapes[0], bad.rope_theta = 0.f;
    CHECK(st_query_sizes(&bad, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_query_sizes(nullptr, nullptr, nullptr) == ST_EINVAL && std::strlen(st_last_error()) > 0);

    // creation: every rejection comes before the first device call
    st_model *m = reinterpret_cast<st_model *>(1);
    st_weights w;
    std::memset(&w, 0, sizeof w);
    CHECK(st_model_create(&shapes[0], &w, nullptr, 0, nullptr, 0, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_model_create(&shapes[0], nullptr, nullptr, 0, nullptr, 0, nullptr, &m) == ST_EINVAL && m == nullptr);
    CHECK(st_model_create(&shapes[0], &w, nullptr, 0, nullptr, 0, nullptr, &m) == ST_EINVAL && m == nullptr);
    alignas(256) static char fake[512];
    CHECK(st_model_create(&shapes[0], &w, fake, 16, fake + 256, 16, nullptr, &m) == ST_ENOMEM && m == nullptr);
    st_batch *b = nullptr;
    CHECK(st_batch_create(&shapes[0], &w, 65, nullptr, 0, nullptr, 0, nullptr, &b) == ST_ERANGE && b == nullptr);
    st_model_destroy(nullptr);
    st_batch_destroy(nullptr);

    // calls on a NULL handle or with malformed arguments
    int32_t n = 0, tok = 0;
    float lg = 0.f;
    CHECK(st_kv_len(nullptr, &n) == ST_EINVAL && st_kv_truncate(nullptr, 0) == ST_EINVAL);
    CHECK(st_prefill(nullptr, &tok, 1, &lg, &tok, 0) == ST_EINVAL && st_decode_step(nullptr, 0, &lg, &tok, 0) == ST_EINVAL);
    CHECK(st_decode_greedy(nullptr, 0, 1, &tok, 0) == ST_EINVAL && st_decode_step_timed(nullptr, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_decode_graph_state(nullptr, &n, &n) == ST_EINVAL);
    CHECK(st_model_attach_f16(nullptr, fake, 256) == ST_EINVAL && st_batch_attach_f16(nullptr, fake, 256) == ST_EINVAL);
    CHECK(st_handoff(nullptr, nullptr, &tok, &n, 1, 1, nullptr, &tok, nullptr, 0) == ST_EINVAL);
    CHECK(st_generate(nullptr, nullptr, nullptr, 0, &tok, 1, 1, 1, &tok, nullptr, nullptr, 0, nullptr) == ST_EINVAL);
    CHECK(st_generate_policy(nullptr, nullptr, nullptr, &tok, 1, 1, &tok, nullptr, nullptr, 0, nullptr) == ST_EINVAL);
    CHECK(st_batch_kv_len(nullptr, 0, &n) == ST_EINVAL && st_batch_truncate(nullptr, 0, 0) == ST_EINVAL);
    CHECK(st_batch_prefill(nullptr, 0, &tok, 1, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_batch_decode_step(nullptr, 1, &tok, &tok, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_batch_prefill_many(nullptr, 1, &tok, nullptr, &tok, nullptr, nullptr) == ST_EINVAL);
    CHECK(st_generate_batch(nullptr, nullptr, nullptr, 1, nullptr, 0, 1, nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == ST_EINVAL);
    uint32_t bits[4] = {1, 0, 0, 0};
    st_trigger_rule rule = {bits, nullptr, 2, 100};
    int32_t pos[4];
    CHECK(st_trigger_scan(nullptr, &tok, 0, 1, pos, 4, &n, nullptr, nullptr, 0) == ST_EINVAL);
    CHECK(st_trigger_scan(&rule, &tok, 0, 1, pos, 4, &n, nullptr, nullptr, 0) == ST_EINVAL);  // window 2 without delimiters
    rule.window = 1;
    CHECK(st_trigger_scan(&rule, &tok, 0, 1, pos, 4, &n, nullptr, nullptr, 0) == ST_EINVAL);  // host outputs, no scratch
    CHECK(st_trigger_scan(&rule, &tok, 2, 1, pos, 4, &n, pos, nullptr, 0) == ST_ERANGE);
    CHECK(st_trigger_scan(&rule, &tok, 0, 1, pos, -1, &n, pos, nullptr, 0) == ST_EINVAL);
    rule.window = ST_MAX_SCAN_WINDOW + 1;
    CHECK(st_trigger_scan(&rule, &tok, 0, 1, pos, 4, &n, pos, nullptr, 0) == ST_EINVAL);
    std::puts("abi sanitizer driver: ok");
    return 0;
}
