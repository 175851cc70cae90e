/*
 * CPU oracle for the SSSD verification step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, obviously-correct statement of what the GPU
 * library must compute.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may call it; the product never does, and the
 * two share no code.
 *
 * What it computes: one forward pass of a Llama-style decoder over
 * b sequences x s_q = k+1 tokens (the last accepted token followed by k
 * drafts) against a per-sequence KV cache, i.e. the operations listed row by
 * row in the paper's Table 2 (App. B, the table of decode-phase operations)
 * with tensor parallelism p = 1, followed by greedy acceptance (Sec. 2: one
 * pass of the target model checks all drafts, and what is emitted is exactly
 * what the target model alone would emit).
 *
 * Arithmetic: values are fp32; every reduction (dot product, sum of squares,
 * softmax denominator) accumulates in fp64 and is rounded to fp32 once.
 * Weights and the KV cache are stored as bf16 (Table 2 caption: 2 bytes per
 * weight and per KV-cache element) and upcast exactly.  New K/V rows are
 * rounded to bf16 (nearest-even) when appended, and attention reads the
 * rounded rows, so a (k+1)-row pass and k+1 single-row passes see the same
 * cache.
 *
 * No tiling, no online softmax, no fusion: each function is the definition
 * written out.  OpenMP only parallelises independent output elements, so the
 * result does not depend on the thread count.
 *
 * Parity pins (tests/test_oracle_*.py): linear vs fp64 matmul; RMSNorm and
 * attention closed forms and library routines; attention vs dense masked
 * softmax; RoPE identities; verify pass == sequential single-token decode;
 * acceptance special cases and brute force; speculative loop == greedy loop.
 * Tree verification (second half of the file): masked attention vs dense
 * fp64 softmax with the explicit mask; a chain given as a tree == the chain
 * functions bit for bit; every root-to-node path == sequential decode of that
 * path; tree acceptance vs enumeration of all root paths; tree speculative
 * loop == greedy loop including the compacted cache.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rms_eps, rope_base;
    int32_t max_seq; /* rows per (sequence, kv head) in the oracle's cache */
} orc_config;

/* bf16 weights of one layer, each matrix row-major [out][in]. */
typedef struct {
    const uint16_t *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down, *attn_norm, *mlp_norm;
} orc_layer_weights;

/* Multiply-accumulate counters (GEMM MACs only), for checking the cost model
 * of Table 2 against what is actually executed. */
static double g_linear_macs = 0.0, g_attn_macs = 0.0;
void orc_counters_reset(void) { g_linear_macs = 0.0; g_attn_macs = 0.0; }
void orc_counters_get(double *linear_macs, double *attn_macs)
{
    *linear_macs = g_linear_macs;
    *attn_macs = g_attn_macs;
}

float orc_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even (finite inputs). */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* y[m][n] = sum_k x[m][k] * W[n][k]   (Table 2: Q = X W_q etc., W stored [out][in]) */
void orc_linear(const float *x, int M, int K, const uint16_t *W, int N, float *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *w = W + (size_t)n * K;
        for (int m = 0; m < M; ++m) {
            const float *xr = x + (size_t)m * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)xr[k] * (double)orc_bf16_to_f32(w[k]);
            y[(size_t)m * N + n] = (float)acc;
        }
    }
    g_linear_macs += (double)M * (double)N * (double)K;
}

/* out[i] = x[i] / sqrt(mean(x^2) + eps) * gamma[i] */
void orc_rmsnorm(const float *x, const uint16_t *gamma, float eps, int n, float *out)
{
    double ss = 0.0;
    for (int i = 0; i < n; ++i)
        ss += (double)x[i] * (double)x[i];
    double r = 1.0 / sqrt(ss / (double)n + (double)eps);
    for (int i = 0; i < n; ++i)
        out[i] = (float)((double)x[i] * r * (double)orc_bf16_to_f32(gamma[i]));
}

/* Rotary embedding of one head vector of length d at position pos, pairing
 * element i with element i + d/2 and rotating the pair by pos * base^(-2i/d). */
void orc_rope(float *v, int d, int pos, float base)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double theta = (double)pos * pow((double)base, -2.0 * (double)i / (double)d);
        double c = cos(theta), s = sin(theta);
        double a = v[i], b = v[i + half];
        v[i] = (float)(a * c - b * s);
        v[i + half] = (float)(a * s + b * c);
    }
}

static float silu(float x) { return (float)((double)x / (1.0 + exp(-(double)x))); }

/* One query row of one head: softmax_t(q . k_t / sqrt(d)) V over cache rows
 * t = 0 .. n_keys-1 (Table 2, attention row; the mask M restricted to a causal
 * chain is "row j sees the old cache and new rows 0..j", which the caller
 * expresses through n_keys). */
void orc_attention_row(const float *q, const uint16_t *Kc, const uint16_t *Vc, int n_keys, int d,
                       float *out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double mx = -INFINITY;
    for (int t = 0; t < n_keys; ++t) {
        double s = 0.0;
        for (int i = 0; i < d; ++i)
            s += (double)q[i] * (double)orc_bf16_to_f32(Kc[(size_t)t * d + i]);
        float sf = (float)(s / sqrt((double)d));
        p[t] = sf;
        if (p[t] > mx) mx = p[t];
    }
    double den = 0.0;
    for (int t = 0; t < n_keys; ++t) {
        p[t] = exp(p[t] - mx);
        den += p[t];
    }
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int t = 0; t < n_keys; ++t)
            acc += p[t] * (double)orc_bf16_to_f32(Vc[(size_t)t * d + i]);
        out[i] = (float)(acc / den);
    }
    free(p);
}

/* Cache of one layer: K and V each [B][n_kv_heads][max_seq][head_dim] bf16. */
static size_t cache_off(const orc_config *c, int b, int kvh, int t)
{
    return (((size_t)b * c->n_kv_heads + kvh) * c->max_seq + t) * (size_t)c->head_dim;
}

/*
 * One decoder layer of the verify pass (Table 2 rows in order):
 *   a = RMSNorm(x); Q,K_new,V_new = a W_q, a W_k, a W_v; RoPE(Q, K_new) at
 *   position lens[b]+j; append K_new,V_new to the cache (bf16);
 *   A = softmax(Q K^T / sqrt(d) + mask) V; x += A W_o;
 *   m = RMSNorm(x); x += (silu(m W_gate) * (m W_up)) W_down.
 * x is [B][k+1][hidden], updated in place.
 */
void orc_layer_verify(const orc_config *c, const orc_layer_weights *w, float *x, uint16_t *Kc,
                      uint16_t *Vc, const int32_t *lens, int B, int k)
{
    const int sq = k + 1, M = B * sq, h = c->hidden, d = c->head_dim;
    const int qd = c->n_q_heads * d, kd = c->n_kv_heads * d, g = c->n_q_heads / c->n_kv_heads;
    float *a = malloc(sizeof(float) * (size_t)M * h);
    float *q = malloc(sizeof(float) * (size_t)M * qd);
    float *kn = malloc(sizeof(float) * (size_t)M * kd);
    float *vn = malloc(sizeof(float) * (size_t)M * kd);
    float *ao = malloc(sizeof(float) * (size_t)M * qd);
    float *y = malloc(sizeof(float) * (size_t)M * h);
    float *gt = malloc(sizeof(float) * (size_t)M * c->ffn);
    float *up = malloc(sizeof(float) * (size_t)M * c->ffn);

    for (int m = 0; m < M; ++m)
        orc_rmsnorm(x + (size_t)m * h, w->attn_norm, c->rms_eps, h, a + (size_t)m * h);
    orc_linear(a, M, h, w->wq, qd, q);
    orc_linear(a, M, h, w->wk, kd, kn);
    orc_linear(a, M, h, w->wv, kd, vn);

    for (int b = 0; b < B; ++b)
        for (int j = 0; j < sq; ++j) {
            const int m = b * sq + j, pos = lens[b] + j;
            for (int hq = 0; hq < c->n_q_heads; ++hq)
                orc_rope(q + (size_t)m * qd + (size_t)hq * d, d, pos, c->rope_base);
            for (int hk = 0; hk < c->n_kv_heads; ++hk) {
                orc_rope(kn + (size_t)m * kd + (size_t)hk * d, d, pos, c->rope_base);
                for (int i = 0; i < d; ++i) {
                    Kc[cache_off(c, b, hk, pos) + i] = orc_f32_to_bf16(kn[(size_t)m * kd + hk * d + i]);
                    Vc[cache_off(c, b, hk, pos) + i] = orc_f32_to_bf16(vn[(size_t)m * kd + hk * d + i]);
                }
            }
        }

#pragma omp parallel for schedule(dynamic)
    for (int mh = 0; mh < M * c->n_q_heads; ++mh) {
        const int m = mh / c->n_q_heads, hq = mh % c->n_q_heads;
        const int b = m / sq, j = m % sq, hk = hq / g;
        const int n_keys = lens[b] + j + 1; /* old cache plus new rows 0..j */
        orc_attention_row(q + (size_t)m * qd + (size_t)hq * d, Kc + cache_off(c, b, hk, 0),
                          Vc + cache_off(c, b, hk, 0), n_keys, d, ao + (size_t)m * qd + (size_t)hq * d);
    }
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < sq; ++j)
            g_attn_macs += 2.0 * (double)c->n_q_heads * (double)d * (double)(lens[b] + j + 1);

    orc_linear(ao, M, qd, w->wo, h, y);
    for (size_t i = 0; i < (size_t)M * h; ++i)
        x[i] += y[i];

    for (int m = 0; m < M; ++m)
        orc_rmsnorm(x + (size_t)m * h, w->mlp_norm, c->rms_eps, h, a + (size_t)m * h);
    orc_linear(a, M, h, w->w_gate, c->ffn, gt);
    orc_linear(a, M, h, w->w_up, c->ffn, up);
    for (size_t i = 0; i < (size_t)M * c->ffn; ++i)
        gt[i] = silu(gt[i]) * up[i];
    orc_linear(gt, M, c->ffn, w->w_down, h, y);
    for (size_t i = 0; i < (size_t)M * h; ++i)
        x[i] += y[i];

    free(a); free(q); free(kn); free(vn); free(ao); free(y); free(gt); free(up);
}

/* x[m][:] = E[tokens[m]][:] */
void orc_embed(const orc_config *c, const uint16_t *embed, const int32_t *tokens, int M, float *x)
{
    for (int m = 0; m < M; ++m)
        for (int i = 0; i < c->hidden; ++i)
            x[(size_t)m * c->hidden + i] = orc_bf16_to_f32(embed[(size_t)tokens[m] * c->hidden + i]);
}

/* logits[m][:] = RMSNorm(x[m]) W_lm^T */
void orc_lm_head(const orc_config *c, const uint16_t *final_norm, const uint16_t *lm_head,
                 const float *x, int M, float *logits)
{
    float *a = malloc(sizeof(float) * (size_t)M * c->hidden);
    for (int m = 0; m < M; ++m)
        orc_rmsnorm(x + (size_t)m * c->hidden, final_norm, c->rms_eps, c->hidden, a + (size_t)m * c->hidden);
    orc_linear(a, M, c->hidden, lm_head, c->vocab, logits);
    free(a);
}

/* Index of the largest element; the lowest index wins a tie. */
int32_t orc_argmax(const float *v, int n)
{
    int32_t best = 0;
    for (int i = 1; i < n; ++i)
        if (v[i] > v[best]) best = i;
    return best;
}

/* Largest and second-largest value of a row (for the parity tests' margin rule). */
void orc_top2(const float *v, int n, float *top1, float *top2)
{
    float a = -INFINITY, b = -INFINITY;
    for (int i = 0; i < n; ++i) {
        if (v[i] > a) { b = a; a = v[i]; }
        else if (v[i] > b) b = v[i];
    }
    *top1 = a; *top2 = b;
}

/*
 * Greedy acceptance for one sequence.  tokens[0] is the last accepted token,
 * tokens[1..k] the drafts; that[j] is the target's argmax after row j, i.e.
 * its own choice for position j+1.  Draft j+1 is accepted while it equals
 * that[j] and every earlier draft was accepted.  Returns the number of accepted
 * drafts n in 0..k and the bonus token that[n], so the emitted stream
 * (accepted drafts, then the bonus token) is what greedy decoding would emit.
 */
void orc_accept(const int32_t *tokens, const int32_t *that, int k, int32_t *accepted_len,
                int32_t *next_token)
{
    int n = 0;
    while (n < k && tokens[n + 1] == that[n])
        ++n;
    *accepted_len = n;
    *next_token = that[n];
}

/*
 * Plain single-token decode of one sequence through ONE layer, written
 * without any notion of drafts or masks: the new token sits at position pos,
 * its K/V are appended, and it attends to every cached row 0..pos.
 * The verify pass must reproduce k+1 of these in a row (Table 2 text: with
 * s_q = 1 the pass is standard autoregressive decoding).
 * Kc/Vc point at this sequence's rows of this layer: [n_kv_heads][max_seq][d].
 */
void orc_layer_decode_token(const orc_config *c, const orc_layer_weights *w, float *x, uint16_t *Kc,
                            uint16_t *Vc, int pos)
{
    const int h = c->hidden, d = c->head_dim, nq = c->n_q_heads, nk = c->n_kv_heads;
    const int qd = nq * d, kd = nk * d, g = nq / nk;
    float *a = malloc(sizeof(float) * h), *q = malloc(sizeof(float) * qd);
    float *kn = malloc(sizeof(float) * kd), *vn = malloc(sizeof(float) * kd);
    float *ao = malloc(sizeof(float) * qd), *y = malloc(sizeof(float) * h);
    float *gt = malloc(sizeof(float) * c->ffn), *up = malloc(sizeof(float) * c->ffn);

    orc_rmsnorm(x, w->attn_norm, c->rms_eps, h, a);
    orc_linear(a, 1, h, w->wq, qd, q);
    orc_linear(a, 1, h, w->wk, kd, kn);
    orc_linear(a, 1, h, w->wv, kd, vn);
    for (int hq = 0; hq < nq; ++hq)
        orc_rope(q + hq * d, d, pos, c->rope_base);
    for (int hk = 0; hk < nk; ++hk) {
        orc_rope(kn + hk * d, d, pos, c->rope_base);
        uint16_t *krow = Kc + ((size_t)hk * c->max_seq + pos) * d;
        uint16_t *vrow = Vc + ((size_t)hk * c->max_seq + pos) * d;
        for (int i = 0; i < d; ++i) {
            krow[i] = orc_f32_to_bf16(kn[hk * d + i]);
            vrow[i] = orc_f32_to_bf16(vn[hk * d + i]);
        }
    }
    for (int hq = 0; hq < nq; ++hq) {
        const int hk = hq / g;
        orc_attention_row(q + hq * d, Kc + (size_t)hk * c->max_seq * d, Vc + (size_t)hk * c->max_seq * d,
                          pos + 1, d, ao + hq * d);
    }
    orc_linear(ao, 1, qd, w->wo, h, y);
    for (int i = 0; i < h; ++i) x[i] += y[i];
    orc_rmsnorm(x, w->mlp_norm, c->rms_eps, h, a);
    orc_linear(a, 1, h, w->w_gate, c->ffn, gt);
    orc_linear(a, 1, h, w->w_up, c->ffn, up);
    for (int i = 0; i < c->ffn; ++i) gt[i] = silu(gt[i]) * up[i];
    orc_linear(gt, 1, c->ffn, w->w_down, h, y);
    for (int i = 0; i < h; ++i) x[i] += y[i];
    free(a); free(q); free(kn); free(vn); free(ao); free(y); free(gt); free(up);
}

/* ------------------------------------------------------------------------
 * Tree verification.  The paper verifies a draft TREE, not a chain (Sec. 3.1:
 * candidates from the input trie and the datastore are merged into a draft
 * tree, which yields the vector of candidate tokens to verify and the
 * attention mask that goes with it); Table 2's attention row carries
 * that mask explicitly, M of shape (b, s_q, s_kv + s_q), one byte per element.
 * Node 0 is the root (the last accepted token), parent[i] < i for i = 1..k.
 * A node sees the old cache, its ancestors and itself; its position is
 * lens + depth.  Every node's K/V is appended at cache row lens + node index.
 * ------------------------------------------------------------------------ */

/* depth[0] = 0, depth[i] = depth[parent[i]] + 1 */
void orc_tree_depths(const int32_t *parent, int k, int32_t *depth)
{
    depth[0] = 0;
    for (int i = 1; i <= k; ++i)
        depth[i] = depth[parent[i]] + 1;
}

/* mask[j][i] = 1 iff node i is node j itself or one of its ancestors; [k+1][k+1] */
void orc_tree_mask(const int32_t *parent, int k, uint8_t *mask)
{
    const int sq = k + 1;
    memset(mask, 0, (size_t)sq * sq);
    for (int j = 0; j <= k; ++j) {
        int i = j;
        for (;;) {
            mask[(size_t)j * sq + i] = 1;
            if (i == 0) break;
            i = parent[i];
        }
    }
}

/* softmax_t(q . k_t / sqrt(d) + M_t) V over rows t = 0 .. n_rows-1, where the
 * additive mask M_t is 0 for mask[t] != 0 and -infinity otherwise (Table 2,
 * attention row, with the mask given explicitly). */
void orc_attention_row_masked(const float *q, const uint16_t *Kc, const uint16_t *Vc,
                              const uint8_t *mask, int n_rows, int d, float *out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)n_rows);
    double mx = -INFINITY;
    for (int t = 0; t < n_rows; ++t) {
        if (!mask[t]) continue;
        double s = 0.0;
        for (int i = 0; i < d; ++i)
            s += (double)q[i] * (double)orc_bf16_to_f32(Kc[(size_t)t * d + i]);
        float sf = (float)(s / sqrt((double)d));
        p[t] = sf;
        if (p[t] > mx) mx = p[t];
    }
    double den = 0.0;
    for (int t = 0; t < n_rows; ++t) {
        if (!mask[t]) continue;
        p[t] = exp(p[t] - mx);
        den += p[t];
    }
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int t = 0; t < n_rows; ++t)
            if (mask[t]) acc += p[t] * (double)orc_bf16_to_f32(Vc[(size_t)t * d + i]);
        out[i] = (float)(acc / den);
    }
    free(p);
}

/* One decoder layer of the verify pass over draft trees; parents is [B][k+1]
 * (entry 0 of each sequence unused).  Same operations as orc_layer_verify;
 * only positions (lens + depth) and the attention mask differ. */
void orc_layer_verify_tree(const orc_config *c, const orc_layer_weights *w, float *x, uint16_t *Kc,
                           uint16_t *Vc, const int32_t *lens, const int32_t *parents, int B, int k)
{
    const int sq = k + 1, M = B * sq, h = c->hidden, d = c->head_dim;
    const int qd = c->n_q_heads * d, kd = c->n_kv_heads * d, g = c->n_q_heads / c->n_kv_heads;
    float *a = malloc(sizeof(float) * (size_t)M * h);
    float *q = malloc(sizeof(float) * (size_t)M * qd);
    float *kn = malloc(sizeof(float) * (size_t)M * kd);
    float *vn = malloc(sizeof(float) * (size_t)M * kd);
    float *ao = malloc(sizeof(float) * (size_t)M * qd);
    float *y = malloc(sizeof(float) * (size_t)M * h);
    float *gt = malloc(sizeof(float) * (size_t)M * c->ffn);
    float *up = malloc(sizeof(float) * (size_t)M * c->ffn);
    int32_t *depth = malloc(sizeof(int32_t) * (size_t)M);
    uint8_t *tmask = malloc((size_t)B * sq * sq);
    for (int b = 0; b < B; ++b) {
        orc_tree_depths(parents + (size_t)b * sq, k, depth + (size_t)b * sq);
        orc_tree_mask(parents + (size_t)b * sq, k, tmask + (size_t)b * sq * sq);
    }

    for (int m = 0; m < M; ++m)
        orc_rmsnorm(x + (size_t)m * h, w->attn_norm, c->rms_eps, h, a + (size_t)m * h);
    orc_linear(a, M, h, w->wq, qd, q);
    orc_linear(a, M, h, w->wk, kd, kn);
    orc_linear(a, M, h, w->wv, kd, vn);

    for (int b = 0; b < B; ++b)
        for (int j = 0; j < sq; ++j) {
            const int m = b * sq + j, pos = lens[b] + depth[m], row = lens[b] + j;
            for (int hq = 0; hq < c->n_q_heads; ++hq)
                orc_rope(q + (size_t)m * qd + (size_t)hq * d, d, pos, c->rope_base);
            for (int hk = 0; hk < c->n_kv_heads; ++hk) {
                orc_rope(kn + (size_t)m * kd + (size_t)hk * d, d, pos, c->rope_base);
                for (int i = 0; i < d; ++i) {
                    Kc[cache_off(c, b, hk, row) + i] = orc_f32_to_bf16(kn[(size_t)m * kd + hk * d + i]);
                    Vc[cache_off(c, b, hk, row) + i] = orc_f32_to_bf16(vn[(size_t)m * kd + hk * d + i]);
                }
            }
        }

#pragma omp parallel for schedule(dynamic)
    for (int mh = 0; mh < M * c->n_q_heads; ++mh) {
        const int m = mh / c->n_q_heads, hq = mh % c->n_q_heads;
        const int b = m / sq, j = m % sq, hk = hq / g;
        const int n_rows = lens[b] + sq;
        uint8_t *mask = malloc((size_t)n_rows);   /* row j of M: old cache visible, then the tree mask */
        memset(mask, 1, (size_t)lens[b]);
        memcpy(mask + lens[b], tmask + ((size_t)b * sq + j) * sq, (size_t)sq);
        orc_attention_row_masked(q + (size_t)m * qd + (size_t)hq * d, Kc + cache_off(c, b, hk, 0),
                                 Vc + cache_off(c, b, hk, 0), mask, n_rows, d,
                                 ao + (size_t)m * qd + (size_t)hq * d);
        free(mask);
    }

    orc_linear(ao, M, qd, w->wo, h, y);
    for (size_t i = 0; i < (size_t)M * h; ++i)
        x[i] += y[i];

    for (int m = 0; m < M; ++m)
        orc_rmsnorm(x + (size_t)m * h, w->mlp_norm, c->rms_eps, h, a + (size_t)m * h);
    orc_linear(a, M, h, w->w_gate, c->ffn, gt);
    orc_linear(a, M, h, w->w_up, c->ffn, up);
    for (size_t i = 0; i < (size_t)M * c->ffn; ++i)
        gt[i] = silu(gt[i]) * up[i];
    orc_linear(gt, M, c->ffn, w->w_down, h, y);
    for (size_t i = 0; i < (size_t)M * h; ++i)
        x[i] += y[i];

    free(a); free(q); free(kn); free(vn); free(ao); free(y); free(gt); free(up); free(depth); free(tmask);
}

/*
 * Greedy acceptance on a draft tree for one sequence.  that[i] is the target's
 * argmax after node i, i.e. its own choice for the token that follows node i.
 * Starting at the root, step to the child whose token equals that[current]
 * (children of a node carry distinct tokens in a trie; if not, the lowest node
 * index wins) until no child matches.  path[0..n] are the nodes walked (path[0]
 * = 0), n the number of accepted drafts, that[path[n]] the bonus token -- the
 * emitted stream equals greedy decoding (Sec. 2).
 */
void orc_accept_tree(const int32_t *tokens, const int32_t *parent, const int32_t *that, int k,
                     int32_t *accepted_len, int32_t *next_token, int32_t *path)
{
    int cur = 0, n = 0;
    path[0] = 0;
    for (;;) {
        int next = -1;
        for (int c2 = cur + 1; c2 <= k; ++c2)
            if (parent[c2] == cur && tokens[c2] == that[cur]) { next = c2; break; }
        if (next < 0) break;
        cur = next;
        path[++n] = cur;
    }
    *accepted_len = n;
    *next_token = that[cur];
}

/* After acceptance the cache rows of the accepted nodes path[1..n] (at rows
 * len + path[i]) move to rows len + i, so that the cache is again one
 * contiguous row per position.  Kc/Vc: one layer, all sequences. */
void orc_kv_compact(const orc_config *c, uint16_t *Kc, uint16_t *Vc, int b, int len,
                    const int32_t *path, int n)
{
    for (int i = 1; i <= n; ++i) {
        if (path[i] == i) continue;
        for (int hk = 0; hk < c->n_kv_heads; ++hk) {
            memcpy(Kc + cache_off(c, b, hk, len + i), Kc + cache_off(c, b, hk, len + path[i]),
                   sizeof(uint16_t) * (size_t)c->head_dim);
            memcpy(Vc + cache_off(c, b, hk, len + i), Vc + cache_off(c, b, hk, len + path[i]),
                   sizeof(uint16_t) * (size_t)c->head_dim);
        }
    }
}
