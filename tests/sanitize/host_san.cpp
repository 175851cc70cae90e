// Host-side self-test, built with -fsanitize=address,undefined (tests/test_host_sanitizers.py).
// It runs, without a GPU, every piece of the build that executes on the host: the sizing and launch
// planning behind the C ABI (swept over every (B, k) of several configurations), the drafter, and
// the C oracle on a small model.  Any sanitizer report or failed check makes the run fail.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/sssd_draft.h"
#include "../../include/sssd_ops.h"
#include "../../include/sssd_verify.h"

extern "C" {
// oracle/sssd_oracle.c (test infrastructure; linked here only to run it under the sanitizers)
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rms_eps, rope_base;
    int32_t max_seq;
} orc_config;
typedef struct {
    const uint16_t *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down, *attn_norm, *mlp_norm;
} orc_layer_weights;
void orc_embed(const orc_config *c, const uint16_t *embed, const int32_t *tokens, int M, float *x);
void orc_layer_verify(const orc_config *c, const orc_layer_weights *w, float *x, uint16_t *Kc, uint16_t *Vc,
                      const int32_t *lens, int B, int k);
void orc_lm_head(const orc_config *c, const uint16_t *final_norm, const uint16_t *lm_head, const float *x, int M,
                 float *logits);
void orc_accept(const int32_t *tokens, const int32_t *that, int k, int32_t *accepted_len, int32_t *next_token);
}

static int failures = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "CHECK failed at line %d: %s\n", __LINE__, #cond); \
            ++failures;                                                      \
        }                                                                    \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static uint16_t rnd_bf16(float scale)
{
    const float v = ((float)(rnd() % 2001) - 1000.f) / 1000.f * scale;
    uint32_t u;
    std::memcpy(&u, &v, 4);
    return (uint16_t)(u >> 16);
}

static void sweep_plans()
{
    struct Case { sssd_model_config c; const char *name; };
    const Case cases[] = {
        {{4, 256, 8, 2, 64, 688, 1024, 1e-5f, 10000.f, 8, 31, 260}, "tiny"},
        {{32, 4096, 32, 8, 128, 14336, 128256, 1e-5f, 500000.f, 32, 16, 4113}, "8b"},
        {{80, 8192, 64, 8, 128, 28672, 128256, 1e-5f, 500000.f, 16, 8, 2057}, "70b"},
        {{2, 1040, 5, 5, 64, 2064, 4112, 1e-5f, 10000.f, 3, 7, 77}, "odd widths"},
        {{1, 64, 1, 1, 64, 16, 16, 1e-5f, 10000.f, 1, 0, 1}, "smallest"},
        {{2, 4096, 32, 8, 128, 14336, 128256, 1e-5f, 500000.f, 4, 8, 32777}, "long context"},
    };
    for (const Case &cs : cases) {
        size_t kv = 0, ws = 0, pk = 0;
        CHECK(sssd_verify_sizes(&cs.c, &kv, &ws, &pk) == SSSD_OK);
        CHECK(kv > 0 && ws > 0 && pk > 0);
        int32_t rows = 0, bps = 0, pages = 0;
        CHECK(sssd_kv_geometry(&cs.c, &rows, &bps, &pages) == SSSD_OK);
        CHECK(rows == 32 && (int64_t)bps * 32 >= cs.c.max_seq && pages == bps * cs.c.max_batch);
        for (int B = 1; B <= cs.c.max_batch; ++B)
            for (int k = 0; k <= cs.c.max_k; ++k) {
                const int rc = sssd_verify_plan_check(&cs.c, B, k);
                if (rc != SSSD_OK) {
                    std::fprintf(stderr, "%s: plan check B=%d k=%d -> %d\n", cs.name, B, k, rc);
                    ++failures;
                }
            }
        CHECK(sssd_verify_plan_check(&cs.c, cs.c.max_batch + 1, 0) == SSSD_ECAPACITY);
        CHECK(sssd_verify_plan_check(&cs.c, 1, cs.c.max_k + 1) == SSSD_ECAPACITY);
        std::printf("plans %-12s kv %zu ws %zu packed %zu: every (B, k) fits\n", cs.name, kv, ws, pk);
    }
    sssd_model_config bad = cases[0].c;
    bad.head_dim = 96;
    CHECK(sssd_verify_sizes(&bad, nullptr, nullptr, nullptr) == SSSD_EINVAL);
    CHECK(sssd_verify_sizes(nullptr, nullptr, nullptr, nullptr) == SSSD_EINVAL);
    // kernel-level GEMM sizing over a grid of shapes
    for (int M : {1, 16, 17, 32, 33, 64, 100, 160, 161, 320})
        for (int N : {16, 256, 4096, 28672, 128256})
            for (int K : {32, 256, 688, 4096, 14336, 28672}) {
                const size_t sc = sssd_op_gemm_scratch_bytes(M, N, K);
                CHECK(sc % 4 == 0);
                CHECK(sssd_op_packed_weight_bytes(N, K) >= (size_t)N * K * 2);
                CHECK(sssd_op_packed_act_bytes(M, K) >= (size_t)M * K * 2);
            }
    CHECK(sssd_op_gemm_static_scratch_limit() == SSSD_OP_GEMM_STATIC_SCRATCH_BYTES);
    CHECK(sssd_op_gemm_small_step_rows() == 32);
}

static void run_drafter()
{
    sssd_draft_params p;
    sssd_draft_default_params(&p);
    sssd_drafter *d = nullptr;
    CHECK(sssd_draft_create(&p, 3, &d) == SSSD_OK && d);
    if (!d) return;
    const int vocab = 50;
    std::vector<int32_t> text(20000);
    for (size_t i = 0; i < text.size(); ++i) text[i] = (int32_t)((i % 97 < 60) ? (i % 13) : rnd() % vocab);
    CHECK(sssd_draft_datastore_add(d, text.data(), (int64_t)text.size()) == SSSD_OK);
    CHECK(sssd_draft_datastore_add(d, text.data(), 0) == SSSD_OK);          // empty sub-index
    CHECK(sssd_draft_datastore_add(d, text.data() + 5000, 3000) == SSSD_OK);
    std::vector<int32_t> tokens(64), parents(64);
    for (int seq = 0; seq < 3; ++seq) {
        for (int round = 0; round < 40; ++round) {
            std::vector<int32_t> more(1 + rnd() % 9);
            for (auto &t : more) t = (int32_t)(rnd() % 13);
            CHECK(sssd_draft_input_append(d, seq, more.data(), (int32_t)more.size()) == SSSD_OK);
            for (int dec_len : {1, 2, 9, 32, 64}) {
                int32_t n = 0;
                CHECK(sssd_draft_propose(d, seq, dec_len, tokens.data(), parents.data(), &n) == SSSD_OK);
                CHECK(n >= 1 && n <= dec_len);
                for (int i = 1; i < n; ++i) CHECK(parents[i] >= 0 && parents[i] < i);
            }
            int32_t ml[64];
            const int32_t found = sssd_draft_match_input(d, seq, ml);
            CHECK(found >= 0 && found <= p.prefix_len);
            for (int i = 1; i < found; ++i) CHECK(ml[i] < ml[i - 1]);
        }
        CHECK(sssd_draft_input_count(d, seq, tokens.data(), 0) > 0);
        CHECK(sssd_draft_input_reset(d, seq) == SSSD_OK);
        int32_t n = 0;
        CHECK(sssd_draft_propose(d, seq, 8, tokens.data(), parents.data(), &n) != SSSD_OK || n >= 0);   // empty input: an error code, no crash
    }
    int64_t total = 0, pos[8];
    const int32_t probe[3] = {1, 2, 3};
    CHECK(sssd_draft_datastore_lookup(d, 0, probe, 3, pos, 8, &total) == SSSD_OK && total >= 0);
    CHECK(sssd_draft_datastore_lookup(d, 7, probe, 3, pos, 8, &total) == SSSD_EINVAL);
    CHECK(sssd_draft_propose(d, 9, 8, tokens.data(), parents.data(), nullptr) == SSSD_EINVAL);
    CHECK(sssd_draft_speculation_length(2.5e15, 8e12, 8, 32) == 32);
    CHECK(sssd_draft_speculation_length(312e12, 2e12, 8, 64) == 20);
    CHECK(sssd_draft_destroy(d) == SSSD_OK);
    std::printf("drafter: 3 sequences x 40 rounds of append / propose / match, lookups, error paths\n");
}

static void run_oracle()
{
    const orc_config c = {2, 64, 4, 2, 16, 96, 80, 1e-5f, 10000.f, 24};
    const int B = 2, k = 3, M = B * (k + 1), qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim;
    auto mat = [&](size_t n, float scale) {
        std::vector<uint16_t> v(n);
        for (auto &x : v) x = rnd_bf16(scale);
        return v;
    };
    std::vector<std::vector<uint16_t>> keep;
    std::vector<orc_layer_weights> lw(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        auto add = [&](size_t n, float s) { keep.push_back(mat(n, s)); return keep.back().data(); };
        lw[l] = {add((size_t)qd * c.hidden, 0.1f), add((size_t)kd * c.hidden, 0.1f), add((size_t)kd * c.hidden, 0.1f),
                 add((size_t)c.hidden * qd, 0.1f), add((size_t)c.ffn * c.hidden, 0.1f), add((size_t)c.ffn * c.hidden, 0.1f),
                 add((size_t)c.hidden * c.ffn, 0.1f), add(c.hidden, 1.f), add(c.hidden, 1.f)};
    }
    const auto embed = mat((size_t)c.vocab * c.hidden, 1.f), lm = mat((size_t)c.vocab * c.hidden, 0.1f), fn = mat(c.hidden, 1.f);
    const size_t cache = (size_t)B * c.n_kv_heads * c.max_seq * c.head_dim;
    std::vector<std::vector<uint16_t>> Kc(c.n_layers, std::vector<uint16_t>(cache, 0)), Vc = Kc;
    std::vector<int32_t> tokens(M), lens = {0, c.max_seq - (k + 1)};     // an empty cache and a full one
    for (auto &t : tokens) t = (int32_t)(rnd() % c.vocab);
    std::vector<float> x((size_t)M * c.hidden), logits((size_t)M * c.vocab);
    orc_embed(&c, embed.data(), tokens.data(), M, x.data());
    for (int l = 0; l < c.n_layers; ++l) orc_layer_verify(&c, &lw[l], x.data(), Kc[l].data(), Vc[l].data(), lens.data(), B, k);
    orc_lm_head(&c, fn.data(), lm.data(), x.data(), M, logits.data());
    for (float v : logits) CHECK(std::isfinite(v));
    std::vector<int32_t> that(k + 1);
    for (int j = 0; j <= k; ++j) {
        int best = 0;
        for (int n = 1; n < c.vocab; ++n)
            if (logits[(size_t)j * c.vocab + n] > logits[(size_t)j * c.vocab + best]) best = n;
        that[j] = best;
    }
    int32_t acc = -1, nxt = -1;
    orc_accept(tokens.data(), that.data(), k, &acc, &nxt);
    CHECK(acc >= 0 && acc <= k && nxt == that[acc]);
    std::printf("oracle: %d-layer verify pass over %d rows, cache rows up to max_seq\n", c.n_layers, M);
}

int main()
{
    sweep_plans();
    run_drafter();
    run_oracle();
    if (failures) {
        std::fprintf(stderr, "%d check(s) failed\n", failures);
        return 1;
    }
    std::printf("host self-test passed\n");
    return 0;
}
