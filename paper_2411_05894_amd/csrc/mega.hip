// The whole verify step as ONE persistent kernel for small M = B*(k+1) (at most 48 rows).
//
// At batch 1 the step streams ~15 GB of weights through ~230 short operations; run as
// separate launches, each pays its own ramp-up and drain, and the paper's premise --
// linear layers cost the same for s_q = k+1 tokens as for one (Sec. 3.2, App. B) --
// drowns in fixed overheads.  Here one workgroup per compute unit stays resident for
// the whole step and walks the phases
//     embed | per layer: QKV+RoPE+append, attention, combine, O+residual,
//                         gate/up+SwiGLU, down+residual | LM head+arg-max | acceptance
// separated by grid-wide barriers (a monotonic device-scope counter with a bounded
// spin, so a wave can never wait forever).  RMSNorm is folded away: the phase that
// updates the residual stream also writes x*gamma as packed bf16 hi/lo operands and
// per-16-column sums of squares; the consuming GEMM scales its fp32 results by
// rsqrt(mean(x^2)+eps), which commutes with the matrix product.
//
// The same kernel can run a single phase (phase_lo + 1 == phase_hi) as an ordinary
// launch; the library uses that when a cooperative launch is not possible.
#include "kernels.h"

namespace {

__device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// The kernel's argument block is read where it lies, in the constant kernarg segment
// (scalar loads), by every phase function.
typedef const __attribute__((address_space(4))) MegaArgs CArgs;

// Loads of data that OTHER workgroups wrote earlier in the same launch.  The barrier makes a
// writer's data visible device-wide (release); readers do not invalidate their caches (that
// costs ~17 us per barrier with 2048 waves) but bypass them with agent-scope loads instead.
__device__ __forceinline__ u32x4 ld_shared16(const u32x4 *p)
{
    const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
    const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
}
__device__ __forceinline__ float ld_shared(const float *p)
{
    return bits_f32(__hip_atomic_load(reinterpret_cast<const uint32_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ int ld_shared(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float2 ld_shared2(const float *p)
{
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return float2{bits_f32((uint32_t)v), bits_f32((uint32_t)(v >> 32))};
}

constexpr int WAVES = 8;
constexpr int THREADS = WAVES * 64;
constexpr float NEG_BIG = -1.0e30f;
constexpr unsigned SPIN_LIMIT = 4000000u;  // polls before a barrier gives up (seconds, not microseconds)

// ---------------------------------------------------------------- barrier ----
// All workgroups are co-resident (cooperative launch).  bar[0] counts arrivals and
// only grows during a launch; bar[1] is raised when some workgroup gave up.
__device__ bool grid_barrier(unsigned *bar, unsigned &epoch, unsigned n_wg)
{
    __shared__ int ok;
    __syncthreads();
    if (threadIdx.x == 0) {
        epoch += 1;
        const unsigned target = epoch * n_wg;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // the workgroup's writes (ordered by the barrier above) become visible device-wide
        __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        int good = 1;
        while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins > SPIN_LIMIT || __hip_atomic_load(bar + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                __hip_atomic_store(bar + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                good = 0;
                break;
            }
        }
        ok = good;
    }
    __syncthreads();
    return ok != 0;
}

// ------------------------------------------------------------------ phases ----
__device__ __noinline__ void phase_embed(CArgs &a)
{
    const auto &D = a.D;
    const int M = a.io.B * (a.io.k + 1);
    if (blockIdx.x == 0) {
        for (int b = threadIdx.x; b < a.io.B; b += THREADS) {
            int len = a.io.lens[b];
            if (len < 0 || len + a.io.k + 1 > D.max_seq) {
                *a.err_flag = 1;
                len = 0;
            }
            a.pos_base[b] = len;
        }
    }
    const uint16_t *gamma = a.layers[0].attn_norm;
    const int KT = (D.h + 31) >> 5, NSS = D.h >> 4;
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        int tok = a.io.tokens[m];
        if (tok < 0 || tok >= D.V) {
            if (threadIdx.x == 0) *a.err_flag = 1;
            tok = 0;
        }
        const uint16_t *row = a.embed + (size_t)tok * D.h;
        for (int i = threadIdx.x; i < D.h; i += THREADS) {
            const float x = bf16_to_f32(row[i]);
            a.X[(size_t)m * D.h + i] = x;
            uint16_t hi, lo;
            split_bf16(x * bf16_to_f32(gamma[i]), hi, lo);
            const size_t idx = packed_index(m, i, KT);
            a.A[AK_QKV][idx] = hi;
            a.A[AK_QKV][a.A_half[AK_QKV] + idx] = lo;
            float ss = x * x;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
            if ((i & 15) == 0) a.ssq[(size_t)m * NSS + (i >> 4)] = ss;
        }
    }
}

// Per-workgroup copies of small per-row facts, in LDS.
struct RowInfo {
    float rstd[48];  // rsqrt(mean(x^2) + eps) of the stream the current GEMM consumes
    int pos[48];     // cache position lens[b] + j of row m = b*(k+1) + j
};

// rstd[m] from the per-16-column partial sums.  All loads are issued before any is used
// (one memory round trip); the caller synchronises before reading ri.rstd.
template <int MT> __device__ __forceinline__ void load_rstd(CArgs &a, const float *ssq, int M, RowInfo &ri)
{
    const auto &D = a.D;
    const int NSS = D.h >> 4;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    constexpr int ROWS = MT * 16 / WAVES;  // rows per wave
    if (NSS <= 512) {
        float v[ROWS][8];
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int m = wave + r * WAVES, slot = lane + 64 * t;
                v[r][t] = (m < M && slot < NSS) ? ssq[(size_t)m * NSS + slot] : 0.f;
            }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) sum += v[r][t];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
            if (lane == 0) ri.rstd[wave + r * WAVES] = rsqrtf(sum / (float)D.h + D.eps);
        }
    } else {
        for (int m = wave; m < MT * 16; m += WAVES) {
            float sum = 0.f;
            if (m < M)
                for (int t = lane; t < NSS; t += 64) sum += ssq[(size_t)m * NSS + t];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
            if (lane == 0) ri.rstd[m] = rsqrtf(sum / (float)D.h + D.eps);
        }
    }
}

__device__ __forceinline__ void load_positions(CArgs &a, RowInfo &ri)
{
    const int M = a.io.B * (a.io.k + 1);
    for (int m = threadIdx.x; m < M && m < 48; m += THREADS) ri.pos[m] = ld_shared(a.pos_base + m / (a.io.k + 1)) + m % (a.io.k + 1);
    __syncthreads();
}

// Phases of the step, in execution order (per layer: QKV .. DOWN).
enum { PK_EMBED = 0, PK_QKV, PK_ATT, PK_COMB, PK_O, PK_GU, PK_DOWN, PK_LM, PK_ACCEPT, PK_NONE };

__device__ __forceinline__ void decode_phase(int ph, int L, int &kind, int &layer)
{
    layer = 0;
    if (ph == 0) kind = PK_EMBED;
    else if (ph == 1 + 6 * L) kind = PK_LM;
    else if (ph == 2 + 6 * L) kind = PK_ACCEPT;
    else if (ph > 2 + 6 * L) kind = PK_NONE;
    else { layer = (ph - 1) / 6; kind = PK_QKV + (ph - 1) % 6; }
}
__device__ __forceinline__ bool is_gemm(int kind) { return kind == PK_QKV || kind == PK_O || kind == PK_GU || kind == PK_DOWN || kind == PK_LM; }
// Output tiles per task: 2 for the paired tiles of QKV (rotary partners) and gate/up, and for the
// LM head (halves its activation re-reads); 1 for O and down, which have only h/16 tiles.
__device__ __forceinline__ int tiles_per_task(int kind) { return (kind == PK_O || kind == PK_DOWN) ? 1 : 2; }

struct GemmDesc {
    const u32x4 *A_hi, *A_lo;
    int KT;                 // k tiles
    int n_tasks;
    const u32x4 *W[3];      // QKV: wq, wk, wv; gate/up: gate, up; others: W[0]
    int NT;                 // n tiles of W[0] (O, down, LM head)
    const uint16_t *gamma_next;  // O, down: gains of the norm that consumes the updated stream
    const float *ssq_in;         // sums of squares of the stream this GEMM consumes (QKV, gate/up, LM head)
    float *ssq_out;              // O, down: sums of squares of the updated stream
    uint16_t *out_hi, *out_lo;   // O, down, gate/up: packed operands for the next GEMM
    int layer, kind;
};

// Operand buffers are versioned: every (layer, role) has its own copy, written in exactly one
// phase and read only after the barrier that follows it.  No address is ever read before its
// final write within a launch, so ordinary cached loads cannot see stale lines and the
// barrier needs no cache invalidation.
__device__ __forceinline__ uint16_t *abuf(CArgs &a, int role, int version) { return a.A[role] + (size_t)version * a.A_stride[role]; }

__device__ __forceinline__ GemmDesc make_desc(CArgs &a, int kind, int layer)
{
    GemmDesc g{};
    const auto &D = a.D;
    const int KTh = (D.h + 31) >> 5, KTq = (D.qd + 31) >> 5, KTf = (D.f + 31) >> 5;
    const size_t ssq_stride = (size_t)48 * (D.h >> 4);
    g.layer = layer;
    g.kind = kind;
    auto in = [&](int role, int version) {
        g.A_hi = (const u32x4 *)abuf(a, role, version);
        g.A_lo = (const u32x4 *)(abuf(a, role, version) + a.A_half[role]);
    };
    auto out = [&](int role, int version) {
        g.out_hi = abuf(a, role, version);
        g.out_lo = g.out_hi + a.A_half[role];
    };
    if (kind == PK_LM) {
        in(AK_QKV, D.L); g.KT = KTh; g.ssq_in = a.ssq + (size_t)(2 * D.L) * ssq_stride;
        g.NT = D.V >> 4; g.n_tasks = (g.NT + 1) / 2; g.W[0] = (const u32x4 *)a.lm_head;
    } else {
        const LayerPtrs *lw = a.layers + layer;
        if (kind == PK_QKV) {
            in(AK_QKV, layer); g.KT = KTh; g.ssq_in = a.ssq + (size_t)(2 * layer) * ssq_stride;
            g.W[0] = (const u32x4 *)lw->wq; g.W[1] = (const u32x4 *)lw->wk; g.W[2] = (const u32x4 *)lw->wv;
            g.n_tasks = (D.nq + 2 * D.nkv) * (D.d >> 5);
        } else if (kind == PK_O) {
            in(AK_ATT, layer); g.KT = KTq; out(AK_GU, layer); g.ssq_out = a.ssq + (size_t)(2 * layer + 1) * ssq_stride;
            g.W[0] = (const u32x4 *)lw->wo; g.NT = D.h >> 4; g.n_tasks = g.NT; g.gamma_next = lw->mlp_norm;
        } else if (kind == PK_GU) {
            in(AK_GU, layer); g.KT = KTh; out(AK_F, layer); g.ssq_in = a.ssq + (size_t)(2 * layer + 1) * ssq_stride;
            g.W[0] = (const u32x4 *)lw->wg; g.W[1] = (const u32x4 *)lw->wu; g.n_tasks = D.f >> 4;
        } else {  // PK_DOWN
            in(AK_F, layer); g.KT = KTf; out(AK_QKV, layer + 1); g.ssq_out = a.ssq + (size_t)(2 * layer + 2) * ssq_stride;
            g.W[0] = (const u32x4 *)lw->wd; g.NT = D.h >> 4; g.n_tasks = g.NT;
            g.gamma_next = layer + 1 < D.L ? a.layers[layer + 1].attn_norm : a.final_norm;
        }
    }
    return g;
}

template <int NG> struct TaskTiles {
    const u32x4 *wt[NG];   // per tile: this lane's record of k-tile 0
    int tile0;             // first output tile (tiles of O / down / LM-head tasks are consecutive)
    int qkind, head, pair; // QKV only: 0 = Q, 1 = K, 2 = V; head within its kind; tile pair within the head
};

template <int NG, typename DimsT>
__device__ __forceinline__ TaskTiles<NG> resolve_task(const DimsT &D, const GemmDesc &g, int task, int lane)
{
    TaskTiles<NG> t;
    t.qkind = t.head = t.pair = 0;
    const int KT = g.KT;
    if (NG == 2 && g.kind == PK_QKV) {
        const int TH = D.d >> 4, per_head = TH >> 1;
        int head = task / per_head;
        t.pair = task % per_head;
        const u32x4 *Wm = g.W[0];
        if (head >= D.nq + D.nkv) { t.qkind = 2; head -= D.nq + D.nkv; Wm = g.W[2]; }
        else if (head >= D.nq) { t.qkind = 1; head -= D.nq; Wm = g.W[1]; }
        t.head = head;
        t.tile0 = head * TH + t.pair;
        t.wt[0] = Wm + (size_t)t.tile0 * KT * 64 + lane;
        t.wt[NG - 1] = Wm + (size_t)(t.tile0 + per_head) * KT * 64 + lane;   // rotary partner tile
    } else if (NG == 2 && g.kind == PK_GU) {
        t.tile0 = task;
        t.wt[0] = g.W[0] + (size_t)task * KT * 64 + lane;
        t.wt[NG - 1] = g.W[1] + (size_t)task * KT * 64 + lane;
    } else {
        t.tile0 = task * NG;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int tc = t.tile0 + i < g.NT ? t.tile0 + i : g.NT - 1;  // a dead tile re-reads the last one
            t.wt[i] = g.W[0] + (size_t)tc * KT * 64 + lane;
        }
    }
    return t;
}

// The k-tiles a wave holds in flight: a ring of RING slots, each one k-tile of every tile of
// the task (weights) plus the hi/lo activation tiles of that k-tile.  A slot is refilled with
// the k-tile RING positions ahead right after it is consumed, so loads are issued continuously.
__host__ __device__ constexpr int ring_slots(int MT) { return MT == 1 ? 8 : 4; }
constexpr int WRING = 16;  // weight registers of the ring (RING * 2 tiles at most); they also carry
                           // the first k-tiles of the NEXT phase across the barrier

struct KRange {
    int kt0, kt1;   // this wave's k-tiles
    int nk_pad;     // k-tiles walked per task (same for every wave), a multiple of RING
};
template <int RING> __device__ __forceinline__ KRange wave_range(int KT)
{
    const int wave = threadIdx.x >> 6;
    KRange r;
    r.kt0 = (int)(((long)KT * wave) / WAVES);
    r.kt1 = (int)(((long)KT * (wave + 1)) / WAVES);
    const int widest = (KT + WAVES - 1) / WAVES;
    r.nk_pad = (widest + RING - 1) / RING * RING;
    return r;
}

// Weight loads of ring slot j at k-tile ktb + j for the tiles of tt (k-tiles past the wave's
// range re-read its last tile; their activations are zeroed at use).
template <int NG, int RING>
__device__ __forceinline__ void issue_w_slot(const TaskTiles<NG> &tt, int ktb, int j, const KRange &kr, u32x4 (&wr)[WRING])
{
    const int ktc = ktb + j < kr.kt1 ? ktb + j : kr.kt1 - 1;
#pragma unroll
    for (int i = 0; i < NG; ++i) wr[j * NG + i] = __builtin_nontemporal_load(tt.wt[i] + (size_t)ktc * 64);
}

// Before a barrier: put the weights of the first ring of the NEXT GEMM phase in flight.  They
// do not depend on anything the step computes, so HBM keeps streaming through the barrier.
template <int MT> __device__ __forceinline__ void prefetch_next_w(CArgs &a, int kind, int layer, u32x4 (&wr)[WRING])
{
    constexpr int RING = ring_slots(MT);
    if (!is_gemm(kind)) return;
    const GemmDesc g = make_desc(a, kind, layer);
    const KRange kr = wave_range<RING>(g.KT);
    const int lane = threadIdx.x & 63;
    if ((int)blockIdx.x >= g.n_tasks || kr.kt0 >= kr.kt1) return;
    if (tiles_per_task(kind) == 1) {
        const TaskTiles<1> tt = resolve_task<1>(a.D, g, blockIdx.x, lane);
#pragma unroll
        for (int j = 0; j < RING; ++j) issue_w_slot<1, RING>(tt, kr.kt0, j, kr, wr);
    } else {
        const TaskTiles<2> tt = resolve_task<2>(a.D, g, blockIdx.x, lane);
#pragma unroll
        for (int j = 0; j < RING; ++j) issue_w_slot<2, RING>(tt, kr.kt0, j, kr, wr);
    }
}

// Cross-wave reduction of the K split through LDS, then the phase's epilogue.
template <int MT, int NG>
__device__ __forceinline__ void gemm_epilogue(CArgs &a, const GemmDesc &g, const TaskTiles<NG> &tt,
                                              f32x4 (&acc)[NG][MT], float *red, const RowInfo &ri)
{
    const auto &D = a.D;
    const int M = a.io.B * (a.io.k + 1);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool paired = NG == 2 && g.kind != PK_LM;   // QKV, gate/up: both tiles of a task meet in one thread
    const int n_out = (paired ? 1 : NG) * MT * 256;
    constexpr int ITERS = (NG * MT * 256 + THREADS - 1) / THREADS;

    // The residual epilogue's inputs do not depend on the reduction: fetch them first.
    float xprev[ITERS], gnext[ITERS];
    if (NG == 1) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int o = threadIdx.x + it * THREADS;
            const int rem = o % (MT * 256);
            const int mt = rem >> 8, r = (rem >> 6) & 3, l = rem & 63;
            const int m = mt * 16 + 4 * (l >> 4) + r, nt = tt.tile0, n = nt * 16 + (l & 15);
            const bool live = o < n_out && m < M && nt < g.NT;
            xprev[it] = live ? a.X[(size_t)m * D.h + n] : 0.f;   // a tile of the stream always belongs to the same workgroup
            gnext[it] = live ? bf16_to_f32(g.gamma_next[n]) : 0.f;
        }
    }

#pragma unroll
    for (int i = 0; i < NG; ++i)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[((wave * NG + i) * MT + mt) * 256 + r * 64 + lane] = acc[i][mt][r];
    __syncthreads();

#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int o = threadIdx.x + it * THREADS;
        if (o >= n_out) break;   // whole waves leave together (256 is a multiple of 64)
        const int i0 = o / (MT * 256), rem = o % (MT * 256);
        const int mt = rem >> 8, r = (rem >> 6) & 3, l = rem & 63;
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            v0 += red[((w * NG + i0) * MT + mt) * 256 + r * 64 + l];
            if (NG == 2) v1 += red[((w * NG + 1) * MT + mt) * 256 + r * 64 + l];   // used by paired tasks only
        }
        const int m = mt * 16 + 4 * (l >> 4) + r, c = l & 15;
        const bool valid = m < M;
        if (NG == 1) {   // O, down: residual update, operands and sums of squares for the next norm
            const int nt = tt.tile0, n = nt * 16 + c;
            float xn = 0.f;
            if (valid && nt < g.NT) {
                xn = xprev[it] + v0;
                a.X[(size_t)m * D.h + n] = xn;
                uint16_t hi, lo;
                split_bf16(xn * gnext[it], hi, lo);
                const size_t idx = packed_index(m, n, (D.h + 31) >> 5);
                g.out_hi[idx] = hi;
                g.out_lo[idx] = lo;
            }
            float ss = xn * xn;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
            if (valid && nt < g.NT && c == 0) g.ssq_out[(size_t)m * (D.h >> 4) + nt] = ss;
        } else if (g.kind == PK_QKV) {
            if (valid) {
                const float rs = ri.rstd[m];
                v0 *= rs;
                v1 *= rs;
                const int b = m / (a.io.k + 1), j = m % (a.io.k + 1);
                const int pos = ri.pos[m];
                const int half = D.d >> 1, ch = tt.pair * 16 + c;  // channel of v0; v1 is ch + half
                const size_t slab = (size_t)g.layer * a.kv_layer_elems + (size_t)b * D.nkv * D.seq_pad * D.d;
                if (tt.qkind < 2) {
                    const float2 cs = *reinterpret_cast<const float2 *>(a.rope_cs + ((size_t)pos * half + ch) * 2);
                    const float y0 = v0 * cs.x - v1 * cs.y, y1 = v0 * cs.y + v1 * cs.x;
                    if (tt.qkind == 0) {
                        const int kvh = tt.head / D.g, hl = tt.head % D.g, rr = j * D.g + hl;
                        const size_t qs = ((size_t)b * D.nkv + kvh) * a.q_rows_pad * D.d;
                        uint16_t h0, l0, h1, l1;
                        split_bf16(y0, h0, l0);
                        split_bf16(y1, h1, l1);
                        const size_t i_0 = qs + packed_index(rr, ch, D.d >> 5), i_1 = qs + packed_index(rr, ch + half, D.d >> 5);
                        a.Qp[i_0] = h0; a.Qp_lo[i_0] = l0;
                        a.Qp[i_1] = h1; a.Qp_lo[i_1] = l1;
                    } else {
                        uint16_t *kr = a.Kc + slab + ((size_t)tt.head * D.seq_pad + pos) * D.d;
                        kr[ch] = f32_to_bf16(y0);
                        kr[ch + half] = f32_to_bf16(y1);
                    }
                } else {
                    uint16_t *vv = a.Vc + slab + (size_t)tt.head * D.seq_pad * D.d;
                    vv[vcache_index(pos, ch, D.d)] = f32_to_bf16(v0);
                    vv[vcache_index(pos, ch + half, D.d)] = f32_to_bf16(v1);
                }
            }
        } else if (g.kind == PK_GU) {
            if (valid) {
                const float rs = ri.rstd[m];
                const float gt = v0 * rs, up = v1 * rs;
                const float hval = gt / (1.f + __expf(-gt)) * up;
                uint16_t hi, lo;
                split_bf16(hval, hi, lo);
                const size_t idx = packed_index(m, tt.tile0 * 16 + c, (D.f + 31) >> 5);
                g.out_hi[idx] = hi;
                g.out_lo[idx] = lo;
            }
        } else {  // PK_LM: two independent tiles per task
            const int nt = tt.tile0 + i0, n = nt * 16 + c;
            const bool live = valid && nt < g.NT;
            const float logit = live ? v0 * ri.rstd[m] : -INFINITY;
            if (live && a.dbg_logits) a.dbg_logits[(size_t)m * D.V + n] = logit;
            float bv = logit;
            int bi = n;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off, 16);
                const int oi = __shfl_xor(bi, off, 16);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (live && c == 0) {
                a.part_val[(size_t)m * g.NT + nt] = bv;
                a.part_idx[(size_t)m * g.NT + nt] = bi;
            }
        }
    }
    __syncthreads();  // red is reused by the next task
}

// One GEMM phase.  A task is NG output tiles (16 columns each) over the full K; the waves of
// the workgroup split K and reduce through LDS in fixed order.  `prefetched`: the weights of
// the first ring were put in flight before the barrier that precedes the phase.  At its end
// the phase puts the first ring of phase (next_kind, next_layer) in flight.
template <int MT, int NG>
__device__ __forceinline__ void phase_gemm(CArgs &a, int kind, int layer, float *red, RowInfo &ri, u32x4 (&wr)[WRING],
                                           bool prefetched, int next_kind, int next_layer)
{
    constexpr int RING = ring_slots(MT);
    static_assert(RING * NG <= WRING, "ring does not fit the weight registers");
    const GemmDesc g = make_desc(a, kind, layer);
    const auto &D = a.D;
    const int M = a.io.B * (a.io.k + 1);
    const int lane = threadIdx.x & 63;
    const KRange kr = wave_range<RING>(g.KT);
    const bool has_k = kr.kt0 < kr.kt1;
    const int n_mine = (int)blockIdx.x < g.n_tasks ? (g.n_tasks - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    const int ipt = kr.nk_pad / RING;          // ring turns per task
    const int n_turns = n_mine * ipt;

    u32x4 xh[RING][MT], xl[RING][MT];
    auto issue_x_slot = [&](int ktb, int j) {
        const int ktc = ktb + j < kr.kt1 ? ktb + j : kr.kt1 - 1;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            xh[j][mt] = g.A_hi[((size_t)mt * g.KT + ktc) * 64 + lane];
            xl[j][mt] = g.A_lo[((size_t)mt * g.KT + ktc) * 64 + lane];
        }
    };

    TaskTiles<NG> tt = resolve_task<NG>(D, g, blockIdx.x, lane);
    if (n_mine > 0 && has_k) {
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            if (!prefetched) issue_w_slot<NG, RING>(tt, kr.kt0, j, kr, wr);
            issue_x_slot(kr.kt0, j);
        }
    }
    if (NG == 2) load_rstd<MT>(a, g.ssq_in, M, ri);
    __syncthreads();
    if (n_mine == 0) {
        prefetch_next_w<MT>(a, next_kind, next_layer, wr);
        return;
    }

    f32x4 acc[NG][MT];
    TaskTiles<NG> tn = tt;
    for (int turn = 0; turn < n_turns; ++turn) {
        const int sub = turn % ipt;
        if (sub == 0) {
#pragma unroll
            for (int i = 0; i < NG; ++i)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[i][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const int ktb = kr.kt0 + sub * RING;
        // where the slots are refilled from: the next turn of this task, or the first of the next task
        const bool more = turn + 1 < n_turns;
        const bool task_ends = sub + 1 == ipt;
        if (task_ends && more) tn = resolve_task<NG>(D, g, blockIdx.x + (turn + 1) / ipt * gridDim.x, lane);
        const int ktb_next = task_ends ? kr.kt0 : ktb + RING;
        if (has_k) {
#pragma unroll
            for (int j = 0; j < RING; ++j) {
                const bool live = ktb + j < kr.kt1;
                const u32x4 z = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const u32x4 h = live ? xh[j][mt] : z, l = live ? xl[j][mt] : z;
#pragma unroll
                    for (int i = 0; i < NG; ++i) {
                        acc[i][mt] = mfma(h, wr[j * NG + i], acc[i][mt]);
                        acc[i][mt] = mfma(l, wr[j * NG + i], acc[i][mt]);
                    }
                }
                if (more) {
                    issue_w_slot<NG, RING>(task_ends ? tn : tt, ktb_next, j, kr, wr);
                    issue_x_slot(ktb_next, j);
                }
            }
        }
        if (task_ends) {
            if (!more) prefetch_next_w<MT>(a, next_kind, next_layer, wr);
            gemm_epilogue<MT, NG>(a, g, tt, acc, red, ri);
            tt = tn;
        }
    }
}

// Attention partials: one wave per (sequence, kv head, chunk, query-row tile).
template <int HD> __device__ __noinline__ void phase_attention(CArgs &a, const RowInfo &ri, int layer)
{
    constexpr int KS = HD / 32, DT = HD / 16;
    const auto &D = a.D;
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int k = a.io.k;
    const int rt_total = (D.g * (k + 1) + 15) >> 4;
    const int n_tasks = a.io.B * D.nkv * D.max_splits * rt_total;
    const int wave_id = blockIdx.x * WAVES + (threadIdx.x >> 6), n_waves = gridDim.x * WAVES;
    const float scale = 1.4426950408889634f * rsqrtf((float)HD);

    for (int task = wave_id; task < n_tasks; task += n_waves) {
        const int rt = task % rt_total;
        const int split = (task / rt_total) % D.max_splits;
        const int kvh = (task / (rt_total * D.max_splits)) % D.nkv;
        const int b = task / (rt_total * D.max_splits * D.nkv);
        const int len = ri.pos[b * (k + 1)], total = len + k + 1;
        const int t_begin = split * D.chunk;
        if (t_begin >= total) continue;
        const int t_end = min(total, t_begin + D.chunk);
        const size_t slab = (size_t)layer * a.kv_layer_elems + ((size_t)b * D.nkv + kvh) * D.seq_pad * HD;
        const uint16_t *Kc = a.Kc + slab;
        const u32x4 *Vc = reinterpret_cast<const u32x4 *>(a.Vc + slab);
        const size_t qs = ((size_t)b * D.nkv + kvh) * a.q_rows_pad * HD;
        const u32x4 *Qh = reinterpret_cast<const u32x4 *>(a.Qp + qs), *Ql = reinterpret_cast<const u32x4 *>(a.Qp_lo + qs);
        u32x4 qh[KS], ql[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qh[ks] = ld_shared16(Qh + ((size_t)rt * KS + ks) * 64 + lane);
            ql[ks] = ld_shared16(Ql + ((size_t)rt * KS + ks) * 64 + lane);
        }
        f32x4 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m_run = NEG_BIG, l_run = 0.f;
        int j = (rt * 16 + c) / D.g;
        if (j > k) j = k;
        const int limit = len + j;

        for (int t0 = t_begin; t0 < t_end; t0 += 32) {
            u32x4 kreg[2][KS], vreg[DT];
            if (t0 + 32 > len) {   // the block holds rows appended in this launch by other workgroups
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        kreg[u][ks] = ld_shared16(reinterpret_cast<const u32x4 *>(Kc + (size_t)(t0 + 16 * u + c) * HD + ks * 32 + 8 * q));
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) vreg[dt] = ld_shared16(Vc + ((size_t)(t0 >> 5) * DT + dt) * 64 + lane);
            } else {
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        kreg[u][ks] = *reinterpret_cast<const u32x4 *>(Kc + (size_t)(t0 + 16 * u + c) * HD + ks * 32 + 8 * q);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) vreg[dt] = Vc[((size_t)(t0 >> 5) * DT + dt) * 64 + lane];
            }
            f32x4 s[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[u] = mfma(kreg[u][ks], qh[ks], s[u]);
                    s[u] = mfma(kreg[u][ks], ql[ks], s[u]);
                }
            }
            float v[8], mx = NEG_BIG;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = t0 + 16 * u + 4 * q + r;
                    float x = s[u][r] * scale;
                    if (t > limit) x = NEG_BIG;
                    v[u * 4 + r] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx), alpha = exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
            uint32_t pk[4], pkl[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float p0 = exp2f(v[e] - m_new), p1 = exp2f(v[e + 1] - m_new);
                uint16_t h0, l0, h1, l1;
                split_bf16(p0, h0, l0);
                split_bf16(p1, h1, l1);
                psum += p0 + p1;
                pk[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                pkl[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            l_run = l_run * alpha + psum;
            const u32x4 pb = u32x4{pk[0], pk[1], pk[2], pk[3]}, pl = u32x4{pkl[0], pkl[1], pkl[2], pkl[3]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[dt] *= alpha;
                o[dt] = mfma(vreg[dt], pb, o[dt]);
                o[dt] = mfma(vreg[dt], pl, o[dt]);
            }
        }
        float l = l_run;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const size_t slot = ((size_t)b * D.nkv + kvh) * D.max_splits + split;
        const size_t row = slot * a.q_rows_pad + (size_t)rt * 16 + c;
        float *po = a.part_o + row * HD;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4 *>(po + dt * 16 + 4 * q) = o[dt];
        if (q == 0) {
            a.part_ml[row * 2] = m_run;
            a.part_ml[row * 2 + 1] = l;
        }
    }
}

// Merge the chunks of every (sequence, kv head, query row): one wave per row.  Lanes first
// work across chunks (weights), then across channels (values, loaded eight chunks at a time).
__device__ __noinline__ void phase_combine(CArgs &a, const RowInfo &ri, int layer)
{
    uint16_t *out_hi = abuf(a, AK_ATT, layer), *out_lo = out_hi + a.A_half[AK_ATT];
    const auto &D = a.D;
    const int lane = threadIdx.x & 63, k = a.io.k;
    const int R = D.g * (k + 1);
    const int n_tasks = a.io.B * D.nkv * R;
    const int wave_id = blockIdx.x * WAVES + (threadIdx.x >> 6), n_waves = gridDim.x * WAVES;
    const int KTq = (D.qd + 31) >> 5;
    const int ch = lane * 2;  // head_dim 128: two channels per lane; head_dim 64: lanes 0..31
    for (int task = wave_id; task < n_tasks; task += n_waves) {
        const int r = task % R, kvh = (task / R) % D.nkv, b = task / (R * D.nkv);
        const int total = ri.pos[b * (k + 1)] + k + 1;
        const int n_splits = (total + D.chunk - 1) / D.chunk;
        const size_t slot0 = ((size_t)b * D.nkv + kvh) * D.max_splits;
        float m_star = NEG_BIG;
        for (int s = lane; s < n_splits; s += 64) m_star = fmaxf(m_star, ld_shared(a.part_ml + ((slot0 + s) * a.q_rows_pad + r) * 2));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m_star = fmaxf(m_star, __shfl_xor(m_star, off));
        float den = 0.f, num0 = 0.f, num1 = 0.f;
        for (int base = 0; base < n_splits; base += 64) {
            const int s_mine = base + lane;
            float w_lane = 0.f;
            if (s_mine < n_splits) {
                const float2 ml = ld_shared2(a.part_ml + ((slot0 + s_mine) * a.q_rows_pad + r) * 2);
                w_lane = exp2f(ml.x - m_star);
                den += w_lane * ml.y;
            }
            const int n_here = n_splits - base < 64 ? n_splits - base : 64;
            for (int s0 = 0; s0 < n_here; s0 += 8) {
                float2 pv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const size_t row = (slot0 + base + s0 + u) * a.q_rows_pad + r;
                    pv[u] = (s0 + u < n_here && ch < D.d) ? ld_shared2(a.part_o + row * D.d + ch) : float2{0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float w = __shfl(w_lane, s0 + u);   // lanes past n_here hold 0
                    num0 += w * pv[u].x;
                    num1 += w * pv[u].y;
                }
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
        if (ch < D.d) {
            const int j = r / D.g, hl = r % D.g, m = b * (k + 1) + j;
            const int col = (kvh * D.g + hl) * D.d + ch;
            uint16_t h0, l0, h1, l1;
            split_bf16(num0 / den, h0, l0);
            split_bf16(num1 / den, h1, l1);
            const size_t idx = packed_index(m, col, KTq);  // col is even: both channels share a lane record
            out_hi[idx] = h0; out_hi[idx + 1] = h1;
            out_lo[idx] = l0; out_lo[idx + 1] = l1;
        }
    }
}

// Row arg-max from the LM head's per-tile partials, then greedy prefix acceptance.
__device__ __noinline__ void phase_accept(CArgs &a)
{
    __shared__ float sv[WAVES];
    __shared__ int si[WAVES];
    __shared__ int that[32];
    const int sq = a.io.k + 1, NT = a.D.V >> 4;
    for (int b = blockIdx.x; b < a.io.B; b += gridDim.x) {
        for (int j = 0; j < sq; ++j) {
            const size_t row = (size_t)(b * sq + j) * NT;
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
            for (int t = threadIdx.x; t < NT; t += THREADS) {
                const float v = ld_shared(a.part_val + row + t);
                const int id = ld_shared(a.part_idx + row + t);
                if (v > bv || (v == bv && id < bi)) { bv = v; bi = id; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oi = __shfl_xor(bi, off);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
            __syncthreads();
            if (threadIdx.x == 0) {
                for (int w = 1; w < WAVES; ++w)
                    if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
                that[j] = bi;
                if (a.that_dbg) a.that_dbg[b * sq + j] = bi;
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            int n = 0;
            while (n < a.io.k && a.io.tokens[b * sq + n + 1] == that[n]) ++n;
            a.io.accepted_len[b] = n;
            a.io.next_token[b] = that[n];
        }
        __syncthreads();
    }
}

template <int MT> __global__ __launch_bounds__(THREADS) void verify_mega_kernel(MegaArgs args)
{
    extern __shared__ float red[];  // WAVES x 2 tiles x MT x 256 floats
    __shared__ RowInfo ri;
    (void)args;
    CArgs &a = *(CArgs *)__builtin_amdgcn_kernarg_segment_ptr();
    const auto &D = a.D;
    unsigned epoch = 0;
    const int n_phases = 3 + 6 * D.L;
    const int lo = a.phase_lo, hi = a.phase_hi < n_phases ? a.phase_hi : n_phases;
    const bool pers = lo == 0 && hi == n_phases;   // the whole step in this launch: prefetch across barriers
    const bool stamp = a.tstamps && blockIdx.x == 0 && threadIdx.x == 0;
    u32x4 wr[WRING];
#pragma unroll
    for (int i = 0; i < WRING; ++i) wr[i] = u32x4{0u, 0u, 0u, 0u};
    if (lo > 0) load_positions(a, ri);   // written by phase 0 of an earlier launch

    for (int ph = lo; ph < hi; ++ph) {
        int kind, layer, next_kind, next_layer;
        decode_phase(ph, D.L, kind, layer);
        decode_phase(ph + 1, D.L, next_kind, next_layer);
        if (!pers) next_kind = PK_NONE;
        if (stamp) a.tstamps[ph] = wall_clock64();
        switch (kind) {
        case PK_EMBED:
            phase_embed(a);
            prefetch_next_w<MT>(a, next_kind, next_layer, wr);
            break;
        case PK_QKV: case PK_GU: case PK_LM:
            if (kind == PK_LM && a.dbg_hidden) {
                const int M = a.io.B * (a.io.k + 1);
                for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < (size_t)M * D.h; i += (size_t)gridDim.x * THREADS)
                    a.dbg_hidden[i] = ld_shared(a.X + i);
            }
            phase_gemm<MT, 2>(a, kind, layer, red, ri, wr, pers, next_kind, next_layer);
            break;
        case PK_O: case PK_DOWN:
            phase_gemm<MT, 1>(a, kind, layer, red, ri, wr, pers, next_kind, next_layer);
            break;
        case PK_ATT:
            if (D.d == 128) phase_attention<128>(a, ri, layer);
            else phase_attention<64>(a, ri, layer);
            break;
        case PK_COMB:
            phase_combine(a, ri, layer);
            prefetch_next_w<MT>(a, next_kind, next_layer, wr);
            break;
        default:
            phase_accept(a);
            break;
        }
        if (stamp) a.tstamps[n_phases + 1 + ph] = wall_clock64();
        if (ph + 1 < hi) {
            if (!grid_barrier(a.bar, epoch, gridDim.x)) return;
            if (ph == 0) load_positions(a, ri);   // written by phase 0, constant afterwards
        }
    }
    if (stamp) a.tstamps[n_phases] = wall_clock64();
}

template <int MT> hipError_t launch_mt(const MegaArgs &a, int grid, bool cooperative, hipStream_t s)
{
    const size_t lds = (size_t)WAVES * 2 * MT * 256 * sizeof(float);
    auto kern = verify_mega_kernel<MT>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (cooperative) {
        MegaArgs copy = a;
        void *params[] = {&copy};
        return hipLaunchCooperativeKernel((const void *)kern, dim3(grid), dim3(THREADS), params, (unsigned)lds, s);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(THREADS), lds, s, a);
    return hipGetLastError();
}

}  // namespace

int mega_max_rows() { return 48; }

hipError_t mega_occupancy(int M, int *blocks_per_cu)
{
    const int mt = (M + 15) / 16;
    const size_t lds = (size_t)WAVES * 2 * mt * 256 * sizeof(float);
    const void *k = mt == 1 ? (const void *)verify_mega_kernel<1> : mt == 2 ? (const void *)verify_mega_kernel<2> : (const void *)verify_mega_kernel<3>;
    hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k, THREADS, lds);
}

hipError_t launch_mega(const MegaArgs &a, int grid, bool cooperative, hipStream_t s)
{
    const int M = a.io.B * (a.io.k + 1);
    const int mt = (M + 15) / 16;
    switch (mt) {
    case 1: return launch_mt<1>(a, grid, cooperative, s);
    case 2: return launch_mt<2>(a, grid, cooperative, s);
    case 3: return launch_mt<3>(a, grid, cooperative, s);
    default: return hipErrorInvalidValue;
    }
}
