// C ABI of the SSSD verify library: context, buffer map, and the per-step launch sequence.
#include <mutex>
#include "../../include/sssd_ops.h"
#include "kernels.h"

#include <cmath>
#include <new>
#include <vector>

namespace {

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct LayerW {
    const uint16_t *wq, *wk, *wv, *wo, *wg, *wu, *wd;  // packed
    const uint16_t *attn_norm, *mlp_norm;
};

struct Buffers {
    float *X;
    uint16_t *Ah_hi, *Ah_lo, *Aq_hi, *Aq_lo, *Af_hi, *Af_lo;
    uint16_t *Ah2_hi, *Ah2_lo;   // normed stream after the attention block (O writes, gate/up reads); Ah_*: after the MLP block
    uint16_t *Qp, *Qp_lo;
    float *part_o, *part_ml, *part_val;
    int *part_idx;
    int32_t *pos_base, *err_flag, *that_dbg, *rope_pos;
    int *tail_count;   // TAIL_SLOTS split-K arrival counters, zero between launches
    uint32_t *anc;
    float *rope_cs, *ssq1;
    uint8_t *staging;
    size_t staging_bytes;
    float *partials;
    size_t partial_bytes;
    void *sample_scratch;         // sampled steps of few rows: the row sampler's cluster scratch
    size_t sample_scratch_bytes;
    size_t attn_slots;   // attention partial slots ([b][kv head][split]) the buffers behind part_o / part_ml hold
};

struct Sizes {
    size_t kv_bytes, ws_bytes, packed_bytes;
    size_t kv_layer_elems;  // bf16 elements of K (or V) of one layer
    int m_alloc, tiles_alloc, q_rows_pad;
};

struct ProfEvent {
    hipEvent_t a, b;
    int cls;
};

}  // namespace

struct sssd_ctx {
    uint32_t magic;
    Dims D;
    Sizes S;
    Buffers W;
    std::vector<LayerW> layers;
    const uint16_t *embed, *lm_head, *final_norm;
    uint16_t *Kc, *Vc;
    const int32_t *block_table;   // device [max_batch][blocks_per_seq] or nullptr (contiguous runs of pages)
    float *dbg_logits, *dbg_hidden;
    int32_t *dbg_that;
    bool prof_on;
    std::vector<ProfEvent> prof_pool;
    size_t prof_used;
    double prof_ms[SSSD_PROF_CLASSES];
    int64_t prof_n[SSSD_PROF_CLASSES];
    int device, n_cu;
};

namespace {

constexpr uint32_t MAGIC = 0x53535344u;

size_t packed_elems(int N, int K) { return (size_t)(N / 16) * ((K + 31) / 32) * 512; }

int check_config(const sssd_model_config *c)
{
    if (!c) return SSSD_EINVAL;
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->ffn <= 0 || c->vocab <= 0)
        return SSSD_EINVAL;
    if (c->head_dim != 64 && c->head_dim != 128) return SSSD_EINVAL;
    if (c->n_q_heads % c->n_kv_heads) return SSSD_EINVAL;
    const int qd = c->n_q_heads * c->head_dim, kd = c->n_kv_heads * c->head_dim;
    if (c->hidden % 16 || qd % 16 || kd % 16 || c->ffn % 16 || c->vocab % 16) return SSSD_EINVAL;
    if (c->max_batch <= 0 || c->max_k < 0 || c->max_k > 31 || c->max_seq <= c->max_k) return SSSD_EINVAL;
    if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return SSSD_EINVAL;
    return SSSD_OK;
}

Dims make_dims(const sssd_model_config *c)
{
    Dims D;
    D.L = c->n_layers; D.h = c->hidden; D.nq = c->n_q_heads; D.nkv = c->n_kv_heads; D.d = c->head_dim;
    D.f = c->ffn; D.V = c->vocab;
    D.qd = D.nq * D.d; D.kd = D.nkv * D.d; D.g = D.nq / D.nkv;
    D.max_batch = c->max_batch; D.max_k = c->max_k; D.max_seq = c->max_seq;
    D.seq_pad = round_up(c->max_seq, 32);
    D.blocks_per_seq = D.seq_pad / 32;
    D.n_pages = D.max_batch * D.blocks_per_seq;
    D.eps = c->rms_eps; D.rope_base = c->rope_base;
    return D;
}

// Lays the workspace out; with base == nullptr it only measures.
constexpr int TAIL_SLOTS = 256;

size_t layout(const Dims &D, Sizes &S, Buffers *B, uint8_t *base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) {
        uint8_t *p = base ? base + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    const int M = D.max_batch * (D.max_k + 1);
    S.tiles_alloc = ((M + 15) / 16 + 9) / 10 * 10;
    S.m_alloc = S.tiles_alloc * 16;
    S.q_rows_pad = round_up(D.g * (D.max_k + 1), 16);
    const size_t KTh = (D.h + 31) / 32, KTq = (D.qd + 31) / 32, KTf = (D.f + 31) / 32;
    const size_t NTv = D.V / 16;
    Buffers b{};
    b.X = (float *)take((size_t)S.m_alloc * D.h * 4);
    b.Ah_hi = (uint16_t *)take(S.tiles_alloc * KTh * 1024);
    b.Ah_lo = (uint16_t *)take(S.tiles_alloc * KTh * 1024);
    b.Ah2_hi = (uint16_t *)take(S.tiles_alloc * KTh * 1024);
    b.Ah2_lo = (uint16_t *)take(S.tiles_alloc * KTh * 1024);
    b.Aq_hi = (uint16_t *)take(S.tiles_alloc * KTq * 1024);
    b.Aq_lo = (uint16_t *)take(S.tiles_alloc * KTq * 1024);
    b.Af_hi = (uint16_t *)take(S.tiles_alloc * KTf * 1024);
    b.Af_lo = (uint16_t *)take(S.tiles_alloc * KTf * 1024);
    b.Qp = (uint16_t *)take((size_t)D.max_batch * D.nkv * S.q_rows_pad * D.d * 2);
    b.Qp_lo = (uint16_t *)take((size_t)D.max_batch * D.nkv * S.q_rows_pad * D.d * 2);
    size_t slots = 0;   // attention partial slots: the most any batch size needs
    for (int B = 1; B <= D.max_batch; ++B) {
        const size_t need = (size_t)B * D.nkv * attention_splits(D, B);
        if (need > slots) slots = need;
    }
    b.attn_slots = slots;
    const size_t prow = slots * S.q_rows_pad;
    b.part_o = (float *)take(prow * D.d * 4);
    b.part_ml = (float *)take(prow * 2 * 4);
    b.part_val = (float *)take((size_t)S.m_alloc * NTv * 4);
    b.part_idx = (int *)take((size_t)S.m_alloc * NTv * 4);
    b.pos_base = (int32_t *)take((size_t)D.max_batch * 4);
    b.rope_pos = (int32_t *)take((size_t)S.m_alloc * 4);
    b.anc = (uint32_t *)take((size_t)S.m_alloc * 4);
    b.err_flag = (int32_t *)take(4);
    b.tail_count = (int *)take(TAIL_SLOTS * sizeof(int));
    b.ssq1 = (float *)take((size_t)S.m_alloc * (D.h / 16) * 4);
    b.that_dbg = (int32_t *)take((size_t)S.m_alloc * 4);
    b.rope_cs = (float *)take((size_t)D.max_seq * (D.d / 2) * 2 * 4);
    b.staging_bytes = (size_t)64 << 20;
    b.staging = take(b.staging_bytes);
    b.sample_scratch_bytes = sample_scratch_bytes(M < 128 ? M : 128, 256);   // clusters form at up to half as many rows as compute units
    b.sample_scratch = take(b.sample_scratch_bytes);
    b.partial_bytes = stream_gemm_partial_bytes(D, M);
    b.partials = (float *)take(b.partial_bytes);
    if (B) *B = b;
    return off;
}

void compute_sizes(const Dims &D, Sizes &S)
{
    S.kv_layer_elems = (size_t)D.max_batch * D.nkv * D.seq_pad * D.d;
    S.kv_bytes = 2 * (size_t)D.L * S.kv_layer_elems * 2;
    S.ws_bytes = layout(D, S, nullptr, nullptr);
    const size_t per_layer = packed_elems(D.qd, D.h) + 2 * packed_elems(D.kd, D.h) + packed_elems(D.h, D.qd) +
                             2 * packed_elems(D.f, D.h) + packed_elems(D.h, D.f);
    S.packed_bytes = 2 * ((size_t)D.L * per_layer + packed_elems(D.V, D.h));
}

#define HIP_TRY(x)                          \
    do {                                    \
        if ((x) != hipSuccess) return SSSD_EHIP; \
    } while (0)

// Packs [N][K] into dst; in place (dst == src) it goes through the staging buffer in
// groups of whole 16-row tiles, whose packed bytes occupy exactly the rows' own bytes.
int pack_matrix(sssd_ctx *c, const uint16_t *src, uint16_t *dst, int N, int K, hipStream_t s)
{
    if ((const void *)src != (void *)dst) {
        HIP_TRY(launch_pack_weight(src, dst, N, K, s));
        return SSSD_OK;
    }
    if (K % 32) return SSSD_EINVAL;
    const size_t row_bytes = (size_t)K * 2;
    int rows_per = (int)(c->W.staging_bytes / row_bytes) / 16 * 16;
    if (rows_per < 16) return SSSD_ECAPACITY;
    for (int n0 = 0; n0 < N; n0 += rows_per) {
        const int rows = N - n0 < rows_per ? N - n0 : rows_per;
        HIP_TRY(hipMemcpyAsync(c->W.staging, src + (size_t)n0 * K, rows * row_bytes, hipMemcpyDeviceToDevice, s));
        HIP_TRY(launch_pack_weight((const uint16_t *)c->W.staging, dst + (size_t)n0 * K, rows, K, s));
    }
    return SSSD_OK;
}

struct Prof {
    sssd_ctx *c;
    hipStream_t s;
    int cls;
    ProfEvent *ev;
    bool own;   // true: the launch itself stamps the events (kernel start and end), nothing is recorded here
    Prof(sssd_ctx *ctx, hipStream_t st, int k, bool kernel_stamps = false) : c(ctx), s(st), cls(k), ev(nullptr), own(kernel_stamps)
    {
        if (!c->prof_on) return;
        if (c->prof_used == c->prof_pool.size()) {
            ProfEvent e;
            e.cls = k;
            if (hipEventCreate(&e.a) != hipSuccess) return;
            if (hipEventCreate(&e.b) != hipSuccess) { (void)hipEventDestroy(e.a); return; }
            c->prof_pool.push_back(e);
        }
        ev = &c->prof_pool[c->prof_used++];
        ev->cls = k;
        if (!own) (void)hipEventRecord(ev->a, s);
    }
    hipEvent_t start() const { return ev ? ev->a : nullptr; }
    hipEvent_t stop() const { return ev ? ev->b : nullptr; }
    ~Prof()
    {
        if (ev && !own) (void)hipEventRecord(ev->b, s);
    }
};

int drain_prof(sssd_ctx *c)
{
    for (size_t i = 0; i < c->prof_used; ++i) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->prof_pool[i].a, c->prof_pool[i].b));
        c->prof_ms[c->prof_pool[i].cls] += ms;
        c->prof_n[c->prof_pool[i].cls] += 1;
    }
    c->prof_used = 0;
    return SSSD_OK;
}

bool valid(const sssd_ctx *c) { return c && c->magic == MAGIC; }

KvGeom kv_geom(const sssd_ctx *c) { return KvGeom{c->block_table, c->D.blocks_per_seq, c->D.n_pages, c->D.nkv, c->D.d}; }

}  // namespace

extern "C" {

const char *sssd_strerror(int code)
{
    switch (code) {
    case SSSD_OK: return "ok";
    case SSSD_EINVAL: return "invalid argument (null pointer, bad handle or unsupported shape)";
    case SSSD_ECAPACITY: return "capacity exceeded (batch, draft count or buffer size)";
    case SSSD_ENOSPACE: return "a sequence does not fit its KV rows, or a token id is out of range";
    case SSSD_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

int sssd_verify_sizes(const sssd_model_config *cfg, size_t *kv_bytes, size_t *ws_bytes, size_t *packed_weight_bytes)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    Dims D = make_dims(cfg);
    Sizes S;
    compute_sizes(D, S);
    if (kv_bytes) *kv_bytes = S.kv_bytes;
    if (ws_bytes) *ws_bytes = S.ws_bytes;
    if (packed_weight_bytes) *packed_weight_bytes = S.packed_bytes;
    return SSSD_OK;
}

int sssd_verify_plan_check(const sssd_model_config *cfg, int32_t B, int32_t k)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    if (B <= 0 || k < 0) return SSSD_EINVAL;
    const Dims D = make_dims(cfg);
    if (B > D.max_batch || k > D.max_k) return SSSD_ECAPACITY;
    Sizes S;
    Buffers W;
    compute_sizes(D, S);
    const size_t end = layout(D, S, &W, nullptr);
    if (end != S.ws_bytes) return SSSD_ECAPACITY;
    const int M = B * (k + 1);
    if (M > S.m_alloc || D.g * (k + 1) > S.q_rows_pad) return SSSD_ECAPACITY;
    // what the GEMM launchers will ask of the split-K scratch at this row count
    const size_t ntot[5] = {(size_t)D.qd + 2 * D.kd, (size_t)D.h, 2 * (size_t)D.f, (size_t)D.h, (size_t)D.V};
    const int kin[5] = {D.h, D.qd, D.h, D.f, D.h};
    for (int i = 0; i < 5; ++i)
        if (stream_gemm_scratch_bytes(M, (int)ntot[i], kin[i]) > W.partial_bytes) return SSSD_ECAPACITY;
    // attention partial slots: [B][kv heads][splits] x q_rows_pad rows, laid out behind part_o / part_ml
    const size_t slots = (size_t)B * D.nkv * attention_splits(D, B);
    if (slots > W.attn_slots || attention_splits(D, B) > 64) return SSSD_ECAPACITY;
    return SSSD_OK;
}

int sssd_verify_init(const sssd_model_config *cfg, const sssd_weights *w, void *kv_cache, size_t kv_bytes,
                     void *workspace, size_t ws_bytes, void *packed, size_t packed_bytes, uint32_t flags,
                     sssd_ctx **out)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !kv_cache || !workspace || !out) return SSSD_EINVAL;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate ||
        !w->w_up || !w->w_down || !w->attn_norm || !w->mlp_norm)
        return SSSD_EINVAL;
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->w_gate[l] || !w->w_up[l] || !w->w_down[l] ||
            !w->attn_norm[l] || !w->mlp_norm[l])
            return SSSD_EINVAL;
    const bool in_place = flags & SSSD_PACK_IN_PLACE;
    if ((uintptr_t)workspace % ALIGN || (uintptr_t)kv_cache % ALIGN) return SSSD_EINVAL;
    if (!in_place && (!packed || (uintptr_t)packed % ALIGN)) return SSSD_EINVAL;

    sssd_ctx *c = new (std::nothrow) sssd_ctx();
    if (!c) return SSSD_EINVAL;
    c->D = make_dims(cfg);
    compute_sizes(c->D, c->S);
    const Dims &D = c->D;
    if (kv_bytes < c->S.kv_bytes || ws_bytes < c->S.ws_bytes || (!in_place && packed_bytes < c->S.packed_bytes)) {
        delete c;
        return SSSD_ECAPACITY;
    }
    if (in_place && (D.h % 32 || D.qd % 32 || D.f % 32)) {
        delete c;
        return SSSD_EINVAL;
    }
    layout(D, c->S, &c->W, (uint8_t *)workspace);
    c->Kc = (uint16_t *)kv_cache;
    c->Vc = c->Kc + (size_t)D.L * c->S.kv_layer_elems;
    c->embed = (const uint16_t *)w->embed;
    c->final_norm = (const uint16_t *)w->final_norm;
    c->dbg_logits = c->dbg_hidden = nullptr;
    c->dbg_that = nullptr;
    c->block_table = nullptr;
    c->prof_on = false;
    c->prof_used = 0;
    for (int i = 0; i < SSSD_PROF_CLASSES; ++i) { c->prof_ms[i] = 0; c->prof_n[i] = 0; }

#define INIT_TRY(x)                     \
    do {                                \
        if ((x) != hipSuccess) {        \
            delete c;                   \
            return SSSD_EHIP;           \
        }                               \
    } while (0)
#define INIT_RC(x)                      \
    do {                                \
        int rc__ = (x);                 \
        if (rc__) {                     \
            delete c;                   \
            return rc__;                \
        }                               \
    } while (0)

    INIT_TRY(hipGetDevice(&c->device));
    hipStream_t s = nullptr;
    INIT_TRY(hipMemsetAsync(kv_cache, 0, c->S.kv_bytes, s));
    INIT_TRY(hipMemsetAsync(workspace, 0, c->S.ws_bytes, s));

    // Rotary table in fp64 on the host: angle = pos * base^(-2i/d).
    {
        const int half = D.d / 2;
        std::vector<float> tab((size_t)D.max_seq * half * 2);
        std::vector<double> inv(half);
        for (int i = 0; i < half; ++i) inv[i] = std::pow((double)D.rope_base, -2.0 * i / (double)D.d);
        for (int p = 0; p < D.max_seq; ++p)
            for (int i = 0; i < half; ++i) {
                const double th = (double)p * inv[i];
                tab[((size_t)p * half + i) * 2] = (float)std::cos(th);
                tab[((size_t)p * half + i) * 2 + 1] = (float)std::sin(th);
            }
        INIT_TRY(hipMemcpy(c->W.rope_cs, tab.data(), tab.size() * 4, hipMemcpyHostToDevice));
    }

    uint16_t *pk = (uint16_t *)packed;
    auto place = [&](const void *src, int N, int K, const uint16_t **dst_out) -> int {
        uint16_t *dst = in_place ? (uint16_t *)src : pk;
        int r = pack_matrix(c, (const uint16_t *)src, dst, N, K, s);
        if (r) return r;
        if (!in_place) pk += packed_elems(N, K);
        *dst_out = dst;
        return SSSD_OK;
    };
    c->layers.resize(D.L);
    for (int l = 0; l < D.L; ++l) {
        LayerW &lw = c->layers[l];
        INIT_RC(place(w->wq[l], D.qd, D.h, &lw.wq));
        INIT_RC(place(w->wk[l], D.kd, D.h, &lw.wk));
        INIT_RC(place(w->wv[l], D.kd, D.h, &lw.wv));
        INIT_RC(place(w->wo[l], D.h, D.qd, &lw.wo));
        INIT_RC(place(w->w_gate[l], D.f, D.h, &lw.wg));
        INIT_RC(place(w->w_up[l], D.f, D.h, &lw.wu));
        INIT_RC(place(w->w_down[l], D.h, D.f, &lw.wd));
        lw.attn_norm = (const uint16_t *)w->attn_norm[l];
        lw.mlp_norm = (const uint16_t *)w->mlp_norm[l];
    }
    INIT_RC(place(w->lm_head, D.V, D.h, &c->lm_head));
    {
        hipDeviceProp_t prop;
        INIT_TRY(hipGetDeviceProperties(&prop, c->device));
        c->n_cu = prop.multiProcessorCount;
    }
    INIT_TRY(hipStreamSynchronize(s));
    c->magic = MAGIC;
    *out = c;
    return SSSD_OK;
}

int sssd_verify_destroy(sssd_ctx *c)
{
    if (!valid(c)) return SSSD_EINVAL;
    for (auto &e : c->prof_pool) {
        (void)hipEventDestroy(e.a);
        (void)hipEventDestroy(e.b);
    }
    c->magic = 0;
    delete c;
    return SSSD_OK;
}

int sssd_debug_outputs(sssd_ctx *c, float *logits, float *hidden)
{
    if (!valid(c)) return SSSD_EINVAL;
    c->dbg_logits = logits;
    c->dbg_hidden = hidden;
    return SSSD_OK;
}

int sssd_debug_logits(sssd_ctx *c, float *logits)
{
    if (!valid(c)) return SSSD_EINVAL;
    c->dbg_logits = logits;
    return SSSD_OK;
}

int sssd_debug_argmax(sssd_ctx *c, int32_t *that)
{
    if (!valid(c)) return SSSD_EINVAL;
    c->dbg_that = that;
    return SSSD_OK;
}

}  // extern "C"

namespace {

// The verify pass over chains (parents == nullptr) or draft trees.
struct Sampling {
    float temperature, top_p;
    int32_t top_k;
    const float *uniforms;   // device [B][k+1]
    float *logits;           // device scratch [B*(k+1)][vocab]
};

int run_step(sssd_ctx *c, int32_t B, int32_t k, const int32_t *tokens, const int32_t *parents, const int32_t *lens,
             int32_t *accepted_len, int32_t *next_token, int32_t *path, void *stream, const Sampling *smp = nullptr)
{
    if (!valid(c) || !tokens || !lens || !accepted_len || !next_token) return SSSD_EINVAL;
    const Dims &D = c->D;
    if (B <= 0 || k < 0) return SSSD_EINVAL;
    if (B > D.max_batch || k > D.max_k) return SSSD_ECAPACITY;
    hipStream_t s = (hipStream_t)stream;
    Buffers &W = c->W;
    const int M = B * (k + 1);
    StepIO io{tokens, lens, accepted_len, next_token, B, k, parents, path};

    // Six launches per layer (QKV, attention, merge, O, gate/up, down) plus an epilogue launch
    // after every GEMM whose K is split over workgroups.
    {
        Prof p(c, s, SSSD_PROF_ELEM);
        HIP_TRY(launch_fused_embed(D, io, kv_geom(c), c->embed, c->layers[0].attn_norm, W.X, W.Ah_hi, W.Ah_lo, W.ssq1, W.pos_base,
                                   W.rope_pos, W.anc, W.err_flag, s));
    }
    FusedGemmArgs f{};
    f.M = M; f.h = D.h; f.d = D.d; f.nq = D.nq; f.nkv = D.nkv; f.seq_pad = D.seq_pad; f.k = k;
    f.q_rows_pad = c->S.q_rows_pad; f.vocab = D.V; f.eps = D.eps; f.kv = kv_geom(c);
    f.X = W.X; f.rope_cs = W.rope_cs; f.pos_base = W.pos_base; f.rope_pos = W.rope_pos; f.Qp = W.Qp; f.Qp_lo = W.Qp_lo;
    f.logits = smp ? smp->logits : c->dbg_logits; f.part_val = W.part_val; f.part_idx = W.part_idx;
    const int KTh = (D.h + 31) / 32, KTq = (D.qd + 31) / 32, KTf = (D.f + 31) / 32;
    f.n_cu = c->n_cu; f.partials = W.partials; f.partial_bytes = W.partial_bytes;
    auto fgemm = [&](int epi) -> hipError_t {
        bool more = false;
        f.tail_count = W.tail_count; f.tail_slots = TAIL_SLOTS;   // the launcher clears it when it does not apply
        {
            Prof p(c, s, SSSD_PROF_GEMM, true);
            hipError_t e = launch_stream_gemm(f, epi, s, &more, p.start(), p.stop());
            if (e != hipSuccess || !more) return e;
        }
        Prof p(c, s, SSSD_PROF_ELEM);
        return launch_stream_epilogue(f, epi, s);
    };
    auto set_qkv = [&](FusedGemmArgs &g, int l) {
        const LayerW &lw = c->layers[l];
        g.A_hi = (const u32x4 *)W.Ah_hi; g.A_lo = (const u32x4 *)W.Ah_lo; g.KT = KTh; g.ssq_in = W.ssq1;
        g.W0 = (const u32x4 *)lw.wq; g.W1 = (const u32x4 *)lw.wk; g.W2 = (const u32x4 *)lw.wv;
        g.NT = D.qd / 16;
        g.Kc = c->Kc + (size_t)l * c->S.kv_layer_elems; g.Vc = c->Vc + (size_t)l * c->S.kv_layer_elems;
        g.n_units = (D.nq + 2 * D.nkv) * (D.d / 32); g.Ntot = D.qd + 2 * D.kd;
    };
    auto set_o = [&](FusedGemmArgs &g, int l) {
        const LayerW &lw = c->layers[l];
        g.A_hi = (const u32x4 *)W.Aq_hi; g.A_lo = (const u32x4 *)W.Aq_lo; g.KT = KTq;
        g.W0 = (const u32x4 *)lw.wo; g.NT = D.h / 16; g.gamma_next = lw.mlp_norm;
        g.n_units = g.NT; g.Ntot = D.h;
        g.out_hi = W.Ah2_hi; g.out_lo = W.Ah2_lo; g.ssq_out = W.ssq1;
    };
    auto set_gate_up = [&](FusedGemmArgs &g, int l) {
        const LayerW &lw = c->layers[l];
        g.A_hi = (const u32x4 *)W.Ah2_hi; g.A_lo = (const u32x4 *)W.Ah2_lo; g.KT = KTh; g.ssq_in = W.ssq1;
        g.W0 = (const u32x4 *)lw.wg; g.W1 = (const u32x4 *)lw.wu;
        g.NT = D.f / 16; g.n_units = g.NT; g.Ntot = 2 * D.f;
        g.out_hi = W.Af_hi; g.out_lo = W.Af_lo; g.KT_out = KTf;
    };
    auto set_down = [&](FusedGemmArgs &g, int l) {
        const LayerW &lw = c->layers[l];
        g.A_hi = (const u32x4 *)W.Af_hi; g.A_lo = (const u32x4 *)W.Af_lo; g.KT = KTf;
        g.W0 = (const u32x4 *)lw.wd; g.NT = D.h / 16;
        g.n_units = g.NT; g.Ntot = D.h;
        g.gamma_next = l + 1 < D.L ? c->layers[l + 1].attn_norm : c->final_norm;
        g.out_hi = W.Ah_hi; g.out_lo = W.Ah_lo; g.ssq_out = W.ssq1;
    };
    auto set_lm = [&](FusedGemmArgs &g) {
        g.A_hi = (const u32x4 *)W.Ah_hi; g.A_lo = (const u32x4 *)W.Ah_lo; g.KT = KTh; g.ssq_in = W.ssq1;
        g.W0 = (const u32x4 *)c->lm_head; g.NT = D.V / 16;
        g.n_units = g.NT; g.Ntot = D.V;
    };
    // Per layer: QKV, attention and its merge, O, gate/up, down; then the LM head.
    set_qkv(f, 0);
    HIP_TRY(fgemm(FEPI_QKV));
    for (int l = 0; l < D.L; ++l) {
        uint16_t *Kl = c->Kc + (size_t)l * c->S.kv_layer_elems, *Vl = c->Vc + (size_t)l * c->S.kv_layer_elems;
        {
            AttnArgs a{W.Qp, W.Qp_lo, Kl, Vl, kv_geom(c), W.pos_base, W.anc, W.part_o, W.part_ml, W.Aq_hi, W.Aq_lo, B, k, 0, 0};
            Prof p(c, s, SSSD_PROF_ATTN);
            HIP_TRY(launch_attention(D, a, s));
        }
        const bool last = l + 1 == D.L;
        set_o(f, l); HIP_TRY(fgemm(FEPI_RESID));
        set_gate_up(f, l); HIP_TRY(fgemm(FEPI_SWIGLU));
        set_down(f, l); HIP_TRY(fgemm(FEPI_RESID));
        if (last && c->dbg_hidden)
            HIP_TRY(hipMemcpyAsync(c->dbg_hidden, W.X, (size_t)M * D.h * 4, hipMemcpyDeviceToDevice, s));
        if (last) { set_lm(f); HIP_TRY(fgemm(FEPI_LM)); }
        else { set_qkv(f, l + 1); HIP_TRY(fgemm(FEPI_QKV)); }
    }
    if (smp) {
        if (c->dbg_logits)
            HIP_TRY(hipMemcpyAsync(c->dbg_logits, smp->logits, (size_t)M * D.V * 4, hipMemcpyDeviceToDevice, s));
        Prof p(c, s, SSSD_PROF_ACCEPT);
        HIP_TRY(launch_sample_rows(smp->logits, M, D.V, smp->temperature, smp->top_k, smp->top_p, smp->uniforms, W.that_dbg,
                                   W.sample_scratch, W.sample_scratch_bytes, true, c->n_cu, W.err_flag, s));
        HIP_TRY(launch_accept(D, io, nullptr, nullptr, D.V / 16, W.that_dbg, s));
    } else {
        Prof p(c, s, SSSD_PROF_ACCEPT);
        HIP_TRY(launch_accept(D, io, W.part_val, W.part_idx, D.V / 16, W.that_dbg, s));
    }
    if (c->dbg_that)
        HIP_TRY(hipMemcpyAsync(c->dbg_that, W.that_dbg, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
    return SSSD_OK;
}

}  // namespace

extern "C" {

int sssd_verify_step(sssd_ctx *c, int32_t B, int32_t k, const int32_t *tokens, const int32_t *lens,
                     int32_t *accepted_len, int32_t *next_token, void *stream)
{
    return run_step(c, B, k, tokens, nullptr, lens, accepted_len, next_token, nullptr, stream);
}

int sssd_verify_step_tree(sssd_ctx *c, int32_t B, int32_t k, const int32_t *tokens, const int32_t *parents,
                          const int32_t *lens, int32_t *accepted_len, int32_t *next_token, int32_t *accepted_path,
                          void *stream)
{
    if (!parents || !accepted_path) return SSSD_EINVAL;
    return run_step(c, B, k, tokens, parents, lens, accepted_len, next_token, accepted_path, stream);
}

int sssd_verify_step_tree_sampled(sssd_ctx *c, int32_t B, int32_t k, const int32_t *tokens, const int32_t *parents,
                                  const int32_t *lens, const sssd_sampling_params *sampling, const float *uniforms,
                                  float *logits_scratch, int32_t *accepted_len, int32_t *next_token,
                                  int32_t *accepted_path, void *stream)
{
    if (!parents || !accepted_path || !sampling || !uniforms || !logits_scratch) return SSSD_EINVAL;
    if (!(sampling->temperature > 0.f) || sampling->top_k < 0 || !(sampling->top_p > 0.f) || sampling->top_p > 1.f)
        return SSSD_EINVAL;
    Sampling smp{sampling->temperature, sampling->top_p, sampling->top_k, uniforms, logits_scratch};
    return run_step(c, B, k, tokens, parents, lens, accepted_len, next_token, accepted_path, stream, &smp);
}

int sssd_kv_commit_tree(sssd_ctx *c, int32_t B, int32_t k, int32_t *lens, const int32_t *accepted_len,
                        const int32_t *accepted_path, void *stream)
{
    if (!valid(c) || !lens || !accepted_len || !accepted_path) return SSSD_EINVAL;
    if (B <= 0 || k < 0) return SSSD_EINVAL;
    if (B > c->D.max_batch || k > c->D.max_k) return SSSD_ECAPACITY;
    HIP_TRY(launch_kv_compact(c->D, kv_geom(c), c->Kc, c->Vc, c->S.kv_layer_elems, B, k, lens, accepted_len, accepted_path,
                              c->W.err_flag, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_kv_geometry(const sssd_model_config *cfg, int32_t *rows_per_page, int32_t *blocks_per_seq, int32_t *n_pages)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    const Dims D = make_dims(cfg);
    if (rows_per_page) *rows_per_page = 32;
    if (blocks_per_seq) *blocks_per_seq = D.blocks_per_seq;
    if (n_pages) *n_pages = D.n_pages;
    return SSSD_OK;
}

int sssd_kv_set_block_table(sssd_ctx *c, const int32_t *block_table)
{
    if (!valid(c)) return SSSD_EINVAL;
    c->block_table = block_table;
    return SSSD_OK;
}

int sssd_kv_rollback(sssd_ctx *c, int32_t B, int32_t *lens, const int32_t *accepted_len, const int32_t *new_lens,
                     void *stream)
{
    if (!valid(c) || !lens || (!accepted_len && !new_lens)) return SSSD_EINVAL;
    if (B <= 0) return SSSD_EINVAL;
    if (B > c->D.max_batch) return SSSD_ECAPACITY;
    HIP_TRY(launch_rollback(B, lens, accepted_len, new_lens, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_verify_sync(sssd_ctx *c, void *stream)
{
    if (!valid(c)) return SSSD_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int32_t flag = 0;
    HIP_TRY(hipMemcpyAsync(&flag, c->W.err_flag, 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (flag) {
        HIP_TRY(hipMemsetAsync(c->W.err_flag, 0, 4, s));
        if ((flag & 2) && c->W.sample_scratch_bytes)   // the sampler's counters are left mid-count by a failed wait
            HIP_TRY(hipMemsetAsync(c->W.sample_scratch, 0, c->W.sample_scratch_bytes, s));
        HIP_TRY(hipStreamSynchronize(s));
        return (flag & 2) ? SSSD_EHIP : SSSD_ENOSPACE;   // bit 1: the row sampler's workgroups could not synchronise
    }
    return SSSD_OK;
}

static int kv_copy(sssd_ctx *c, int32_t layer, int32_t b, int32_t t0, int32_t n_rows, void *k_ext, void *v_ext,
                   bool import, void *stream)
{
    if (!valid(c) || !k_ext || !v_ext) return SSSD_EINVAL;
    const Dims &D = c->D;
    if (layer < 0 || layer >= D.L || b < 0 || b >= D.max_batch || t0 < 0 || n_rows < 0) return SSSD_EINVAL;
    if ((long)t0 + n_rows > D.max_seq) return SSSD_ECAPACITY;
    const size_t off = (size_t)layer * c->S.kv_layer_elems;
    HIP_TRY(launch_kv_copy(D, kv_geom(c), c->Kc + off, c->Vc + off, b, t0, n_rows, (uint16_t *)k_ext, (uint16_t *)v_ext, import,
                           c->W.err_flag, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_kv_import(sssd_ctx *c, int32_t layer, int32_t b, int32_t t0, int32_t n_rows, const void *k_src,
                   const void *v_src, void *stream)
{
    return kv_copy(c, layer, b, t0, n_rows, (void *)k_src, (void *)v_src, true, stream);
}

int sssd_kv_export(sssd_ctx *c, int32_t layer, int32_t b, int32_t t0, int32_t n_rows, void *k_dst, void *v_dst,
                   void *stream)
{
    return kv_copy(c, layer, b, t0, n_rows, k_dst, v_dst, false, stream);
}

int sssd_profile_enable(sssd_ctx *c, int32_t on)
{
    if (!valid(c)) return SSSD_EINVAL;
    c->prof_on = on != 0;
    c->prof_used = 0;
    for (int i = 0; i < SSSD_PROF_CLASSES; ++i) { c->prof_ms[i] = 0; c->prof_n[i] = 0; }
    return SSSD_OK;
}

int sssd_profile_read(sssd_ctx *c, void *stream, double *ms, int64_t *n)
{
    if (!valid(c) || !ms || !n) return SSSD_EINVAL;
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    int rc = drain_prof(c);
    if (rc) return rc;
    for (int i = 0; i < SSSD_PROF_CLASSES; ++i) {
        ms[i] = c->prof_ms[i]; n[i] = c->prof_n[i];
        c->prof_ms[i] = 0; c->prof_n[i] = 0;
    }
    return SSSD_OK;
}


// ---- kernel-level entry points ----

size_t sssd_op_packed_weight_bytes(int32_t N, int32_t K)
{
    if (N <= 0 || K <= 0 || N % 16) return 0;
    return packed_elems(N, K) * 2;
}

size_t sssd_op_packed_act_bytes(int32_t M, int32_t K)
{
    if (M <= 0 || K <= 0) return 0;
    const size_t tiles = (size_t)(((M + 15) / 16 + 9) / 10 * 10);  // whole GEMM passes of 10 row tiles
    return tiles * ((K + 31) / 32) * 1024;
}

int sssd_op_pack_weight(const void *w, void *packed, int32_t N, int32_t K, void *stream)
{
    if (!w || !packed || N <= 0 || K <= 0 || N % 16 || K % 8 || w == packed) return SSSD_EINVAL;
    HIP_TRY(launch_pack_weight((const uint16_t *)w, (uint16_t *)packed, N, K, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_op_pack_activation(const float *x, int32_t M, int32_t K, void *a_hi, void *a_lo, void *stream)
{
    if (!x || !a_hi || !a_lo || M <= 0 || K <= 0) return SSSD_EINVAL;
    HIP_TRY(launch_pack_act(x, M, K, (uint16_t *)a_hi, (uint16_t *)a_lo, (hipStream_t)stream));
    return SSSD_OK;
}

size_t sssd_op_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || N % 16) return 0;
    return stream_gemm_scratch_bytes(M, N, K);
}

int sssd_op_gemm(const void *a_hi, const void *a_lo, const void *w_packed, int32_t M, int32_t N, int32_t K, float *out,
                 void *scratch, size_t scratch_bytes, void *stream)
{
    if (!a_hi || !a_lo || !w_packed || !out || M <= 0 || N <= 0 || K <= 0 || N % 16) return SSSD_EINVAL;
    const size_t need = stream_gemm_scratch_bytes(M, N, K);
    if (need && (!scratch || scratch_bytes < need)) return SSSD_ECAPACITY;
    FusedGemmArgs a{};
    a.A_hi = (const u32x4 *)a_hi; a.A_lo = (const u32x4 *)a_lo; a.W0 = (const u32x4 *)w_packed;
    a.KT = (K + 31) / 32; a.NT = N / 16; a.n_units = a.NT; a.Ntot = N; a.M = M; a.out = out;
    a.partials = (float *)scratch; a.partial_bytes = scratch_bytes;
    bool more = false;
    HIP_TRY(launch_stream_gemm(a, FEPI_STORE, (hipStream_t)stream, &more, nullptr, nullptr));
    if (more) HIP_TRY(launch_stream_epilogue(a, FEPI_STORE, (hipStream_t)stream));
    return SSSD_OK;
}

int32_t sssd_op_gemm_small_step_rows(void) { return stream_gemm_max_rows(); }

const char *sssd_op_gemm_kernel_name(int32_t M) { return stream_gemm_kernel_name(M); }

}  // extern "C"

// Split-K partial sums of sssd_op_gemm_static.  One copy per device, held until the process ends.
// In host code the name is only a handle: static_scratch_ptr() asks the runtime for the address of
// the CURRENT device's copy, once per device, and everything else uses that address.
static __device__ __align__(256) unsigned char static_scratch[SSSD_OP_GEMM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex static_scratch_mu;
void *static_scratch_addr[MAX_DEVICES];   // per device, nullptr until resolved

int static_scratch_ptr(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return SSSD_EINVAL;
    std::lock_guard<std::mutex> lock(static_scratch_mu);
    if (!static_scratch_addr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return SSSD_EHIP;
        static_scratch_addr[dev] = p;
    }
    *out = static_scratch_addr[dev];
    return SSSD_OK;
}
}  // namespace

extern "C" {

size_t sssd_op_gemm_static_scratch_limit(void) { return SSSD_OP_GEMM_STATIC_SCRATCH_BYTES; }

int sssd_op_gemm_static(const void *a_hi, const void *a_lo, const void *w_packed, int32_t M, int32_t N, int32_t K,
                        float *out, void *stream)
{
    if (!a_hi || !a_lo || !w_packed || !out || M <= 0 || N <= 0 || K <= 0 || N % 16) return SSSD_EINVAL;
    if (stream_gemm_scratch_bytes(M, N, K) > (size_t)SSSD_OP_GEMM_STATIC_SCRATCH_BYTES) return SSSD_ECAPACITY;
    void *scratch = nullptr;
    const int rc = static_scratch_ptr(&scratch);
    if (rc) return rc;
    // every partial slice a launch reads was written by the same launch: nothing has to start at zero
    return sssd_op_gemm(a_hi, a_lo, w_packed, M, N, K, out, scratch, SSSD_OP_GEMM_STATIC_SCRATCH_BYTES, stream);
}

int sssd_op_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || (uintptr_t)src % 16) return SSSD_EINVAL;
    int dev = 0, n_cu = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    HIP_TRY(launch_stream_read(src, bytes, sink, n_cu, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_op_sample(const float *logits, int32_t rows, int32_t vocab, const sssd_sampling_params *sampling,
                   const float *uniforms, int32_t *sampled, void *stream)
{
    if (!logits || !sampling || !uniforms || !sampled || rows <= 0 || vocab <= 0) return SSSD_EINVAL;
    if (!(sampling->temperature > 0.f) || sampling->top_k < 0 || !(sampling->top_p > 0.f) || sampling->top_p > 1.f)
        return SSSD_EINVAL;
    HIP_TRY(launch_sample_rows(logits, rows, vocab, sampling->temperature, sampling->top_k, sampling->top_p, uniforms, sampled,
                               nullptr, 0, false, 0, nullptr, (hipStream_t)stream));
    return SSSD_OK;
}

static int device_cus(int *n_cu)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    return SSSD_OK;
}

size_t sssd_op_sample_scratch_bytes(int32_t rows)
{
    int n_cu = 0;
    if (rows <= 0 || device_cus(&n_cu) != SSSD_OK) return 0;
    return sample_scratch_bytes(rows, n_cu);
}

int sssd_op_sample_wide(const float *logits, int32_t rows, int32_t vocab, const sssd_sampling_params *sampling,
                        const float *uniforms, int32_t *sampled, void *scratch, size_t scratch_bytes, void *stream)
{
    if (!logits || !sampling || !uniforms || !sampled || rows <= 0 || vocab <= 0) return SSSD_EINVAL;
    if (!(sampling->temperature > 0.f) || sampling->top_k < 0 || !(sampling->top_p > 0.f) || sampling->top_p > 1.f)
        return SSSD_EINVAL;
    int n_cu = 0;
    const int rc = device_cus(&n_cu);
    if (rc) return rc;
    const size_t need = sample_scratch_bytes(rows, n_cu);
    if (need && (!scratch || scratch_bytes < need)) return SSSD_ECAPACITY;
    HIP_TRY(launch_sample_rows(logits, rows, vocab, sampling->temperature, sampling->top_k, sampling->top_p, uniforms, sampled,
                               need ? scratch : nullptr, scratch_bytes, false, n_cu, nullptr, (hipStream_t)stream));
    return SSSD_OK;
}

int sssd_op_attention(sssd_ctx *c, int32_t layer, int32_t B, int32_t k, const float *q, const int32_t *lens, float *out,
                      void *stream)
{
    if (!valid(c) || !q || !lens || !out) return SSSD_EINVAL;
    const Dims &D = c->D;
    if (layer < 0 || layer >= D.L || B <= 0 || k < 0) return SSSD_EINVAL;
    if (B > D.max_batch || k > D.max_k) return SSSD_ECAPACITY;
    hipStream_t s = (hipStream_t)stream;
    Buffers &W = c->W;
    HIP_TRY(launch_lens(D, B, k, lens, W.pos_base, W.rope_pos, W.anc, W.err_flag, s));
    HIP_TRY(launch_q_pack(D, q, B, k, W.Qp, W.Qp_lo, s));
    uint16_t *Kl = c->Kc + (size_t)layer * c->S.kv_layer_elems, *Vl = c->Vc + (size_t)layer * c->S.kv_layer_elems;
    AttnArgs a{W.Qp, W.Qp_lo, Kl, Vl, kv_geom(c), W.pos_base, W.anc, W.part_o, W.part_ml, W.Aq_hi, W.Aq_lo, B, k, 0, 0};
    HIP_TRY(launch_attention(D, a, s));
    HIP_TRY(launch_unpack_act(W.Aq_hi, W.Aq_lo, B * (k + 1), D.qd, out, s));
    return SSSD_OK;
}

}  // extern "C"
