// Fused per-operation kernels of the verify step: six launches per decoder layer.
//
//   QKV GEMM (+ RMSNorm scale, rotary embedding, Q operand packing, in-place KV append)
//   attention partials, chunk merge                       (attention.hip)
//   O GEMM      (+ residual add, next norm's gains, operand packing, sums of squares)
//   gate/up GEMM (+ RMSNorm scale, SwiGLU, operand packing)
//   down GEMM   (+ residual add, next norm's gains, operand packing, sums of squares)
// and the LM head GEMM (+ RMSNorm scale, per-tile arg-max).  These are the linear rows of
// the paper's Table 2 (App. B) with everything the table leaves out folded into their
// epilogues.  RMSNorm needs no pass of its own: the kernel that updates the residual stream
// x also writes x*gamma as packed bf16 hi/lo operands and per-16-column sums of squares, and
// the consuming GEMM scales its fp32 results by rsqrt(mean(x^2)+eps), which commutes with
// the matrix product.
//
// The GEMM itself is the weight streamer of gemm.hip: one workgroup per task of NG output
// tiles, its waves split K, weights go HBM -> registers -> MFMA with fully coalesced
// 16-byte-per-lane loads, the K split is reduced through LDS in fixed order.
#include "kernels.h"

namespace {

__device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int MT, int EPI> struct Shape {
    static constexpr int NG = EPI == FEPI_RESID ? 1 : 2;
    // Few output tiles (h/16) for O and down: more waves per workgroup keep enough loads in flight.
    static constexpr int WAVES = EPI == FEPI_RESID ? (MT <= 2 ? 16 : (MT <= 5 ? 8 : 4)) : (MT <= 2 ? 8 : (MT <= 5 ? 4 : 2));
    static constexpr int U = MT == 1 ? 8 : (MT == 2 ? 4 : (MT <= 5 ? 2 : 1));  // k-tiles loaded per batch
};

template <int MT, int EPI>
__global__ __launch_bounds__((Shape<MT, EPI>::WAVES * 64)) void fused_gemm_kernel(FusedGemmArgs a, int m_base)
{
    constexpr int NG = Shape<MT, EPI>::NG, WAVES = Shape<MT, EPI>::WAVES, U = Shape<MT, EPI>::U, THREADS = WAVES * 64;
    __shared__ float red[WAVES * NG * MT * 256];
    __shared__ float rstd[MT * 16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int task = blockIdx.x;
    const int KT = a.KT;
    const int kt0 = (int)(((long)KT * wave) / WAVES), kt1 = (int)(((long)KT * (wave + 1)) / WAVES);

    // ---- which tiles ----
    const u32x4 *wt[NG];
    int tile0 = 0, qkind = 0, head = 0, pair = 0;
    if (EPI == FEPI_QKV) {
        const int TH = a.d >> 4, per_head = TH >> 1;
        head = task / per_head;
        pair = task % per_head;
        const u32x4 *Wm = a.W0;
        if (head >= a.nq + a.nkv) { qkind = 2; head -= a.nq + a.nkv; Wm = a.W2; }
        else if (head >= a.nq) { qkind = 1; head -= a.nq; Wm = a.W1; }
        tile0 = head * TH + pair;
        wt[0] = Wm + (size_t)tile0 * KT * 64 + lane;
        wt[NG - 1] = Wm + (size_t)(tile0 + per_head) * KT * 64 + lane;   // rotary partner tile
    } else if (EPI == FEPI_SWIGLU) {
        tile0 = task;
        wt[0] = a.W0 + (size_t)task * KT * 64 + lane;
        wt[NG - 1] = a.W1 + (size_t)task * KT * 64 + lane;
    } else {
        tile0 = task * NG;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int tc = tile0 + i < a.NT ? tile0 + i : a.NT - 1;  // a dead tile re-reads the last one
            wt[i] = a.W0 + (size_t)tc * KT * 64 + lane;
        }
    }

    f32x4 acc[NG][MT];
#pragma unroll
    for (int i = 0; i < NG; ++i)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[i][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const size_t mt_base = (size_t)(m_base >> 4);
    const u32x4 *ah = a.A_hi + mt_base * KT * 64 + lane, *al = a.A_lo + mt_base * KT * 64 + lane;

    // rstd of this pass's rows is needed only by the epilogue.  With few rows per wave its
    // loads are issued here, ahead of the main loop, so they cost no extra round trip.
    constexpr int RROWS = (MT * 16 + WAVES - 1) / WAVES;
    constexpr bool EARLY = RROWS <= 2;
    float ssq_v[EARLY ? RROWS : 1][8];
    const int NSS = a.h >> 4;
    if (EPI != FEPI_RESID && EARLY) {
#pragma unroll
        for (int r = 0; r < RROWS; ++r) {
            const int ml = wave + r * WAVES, m = m_base + ml;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int t = lane + 64 * q;
                ssq_v[r][q] = (ml < MT * 16 && m < a.M && t < NSS) ? a.ssq_in[(size_t)m * NSS + t] : 0.f;
            }
        }
    }

    int kt = kt0;
    for (; kt + U <= kt1; kt += U) {
        u32x4 wv[NG][U], xh[MT][U], xl[MT][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < NG; ++i) wv[i][u] = __builtin_nontemporal_load(wt[i] + (size_t)(kt + u) * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                xh[mt][u] = ah[((size_t)mt * KT + kt + u) * 64];
                xl[mt][u] = al[((size_t)mt * KT + kt + u) * 64];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < NG; ++i) {
                    acc[i][mt] = mfma(xh[mt][u], wv[i][u], acc[i][mt]);
                    acc[i][mt] = mfma(xl[mt][u], wv[i][u], acc[i][mt]);
                }
    }
    for (; kt < kt1; ++kt) {
        u32x4 wv[NG];
#pragma unroll
        for (int i = 0; i < NG; ++i) wv[i] = __builtin_nontemporal_load(wt[i] + (size_t)kt * 64);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const u32x4 xh = ah[((size_t)mt * KT + kt) * 64], xl = al[((size_t)mt * KT + kt) * 64];
#pragma unroll
            for (int i = 0; i < NG; ++i) {
                acc[i][mt] = mfma(xh, wv[i], acc[i][mt]);
                acc[i][mt] = mfma(xl, wv[i], acc[i][mt]);
            }
        }
    }

    // ---- the residual epilogue's own inputs: fetch before the reduction ----
    constexpr int NOUT = EPI == FEPI_LM ? NG : 1;   // QKV, gate/up: the two tiles of a task meet in one thread
    constexpr int N_OUT = NOUT * MT * 256;
    constexpr int ITERS = (N_OUT + THREADS - 1) / THREADS;
    float xprev[ITERS], gnext[ITERS];
    if (EPI == FEPI_RESID) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int o = threadIdx.x + it * THREADS;
            const int rem = o % (MT * 256);
            const int mt = rem >> 8, r = (rem >> 6) & 3, l = rem & 63;
            const int m = m_base + mt * 16 + 4 * (l >> 4) + r, n = tile0 * 16 + (l & 15);
            const bool live = o < N_OUT && m < a.M;
            xprev[it] = live ? a.X[(size_t)m * a.h + n] : 0.f;
            gnext[it] = live ? bf16_to_f32(a.gamma_next[n]) : 0.f;
        }
    }

    // ---- cross-wave reduction of the K split; rstd ----
#pragma unroll
    for (int i = 0; i < NG; ++i)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[((wave * NG + i) * MT + mt) * 256 + r * 64 + lane] = acc[i][mt][r];
    if (EPI != FEPI_RESID) {
        if (EARLY && NSS <= 512) {
#pragma unroll
            for (int r = 0; r < RROWS; ++r) {
                float sum = 0.f;
#pragma unroll
                for (int q = 0; q < 8; ++q) sum += ssq_v[r][q];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0 && wave + r * WAVES < MT * 16) rstd[wave + r * WAVES] = rsqrtf(sum / (float)a.h + a.eps);
            }
        } else {
            for (int ml = wave; ml < MT * 16; ml += WAVES) {
                const int m = m_base + ml;
                float sum = 0.f;
                if (m < a.M)
                    for (int t = lane; t < NSS; t += 64) sum += a.ssq_in[(size_t)m * NSS + t];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0) rstd[ml] = rsqrtf(sum / (float)a.h + a.eps);
            }
        }
    }
    __syncthreads();

#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int o = threadIdx.x + it * THREADS;
        if (o >= N_OUT) break;   // whole waves leave together (256 is a multiple of 64)
        const int i0 = o / (MT * 256), rem = o % (MT * 256);
        const int mt = rem >> 8, r = (rem >> 6) & 3, l = rem & 63;
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            v0 += red[((w * NG + i0) * MT + mt) * 256 + r * 64 + l];
            if (NG == 2 && NOUT == 1) v1 += red[((w * NG + 1) * MT + mt) * 256 + r * 64 + l];
        }
        const int ml = mt * 16 + 4 * (l >> 4) + r, m = m_base + ml, c = l & 15;
        const bool valid = m < a.M;
        if (EPI == FEPI_RESID) {
            const int n = tile0 * 16 + c;
            float xn = 0.f;
            if (valid) {
                xn = xprev[it] + v0;
                a.X[(size_t)m * a.h + n] = xn;
                uint16_t hi, lo;
                split_bf16(xn * gnext[it], hi, lo);
                const size_t idx = packed_index(m, n, (a.h + 31) >> 5);
                a.out_hi[idx] = hi;
                a.out_lo[idx] = lo;
            }
            float ss = xn * xn;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
            if (valid && c == 0) a.ssq_out[(size_t)m * (a.h >> 4) + tile0] = ss;
        } else if (EPI == FEPI_QKV) {
            if (valid) {
                const float rs = rstd[ml];
                v0 *= rs;
                v1 *= rs;
                const int b = m / (a.k + 1), j = m % (a.k + 1);
                const int pos = a.pos_base[b] + j;
                const int half = a.d >> 1, ch = pair * 16 + c;  // channel of v0; v1 is ch + half
                const size_t slab = (size_t)b * a.nkv * a.seq_pad * a.d;
                if (qkind < 2) {
                    const float2 cs = *reinterpret_cast<const float2 *>(a.rope_cs + ((size_t)pos * half + ch) * 2);
                    const float y0 = v0 * cs.x - v1 * cs.y, y1 = v0 * cs.y + v1 * cs.x;
                    if (qkind == 0) {
                        const int g = a.nq / a.nkv, kvh = head / g, hl = head % g, rr = j * g + hl;
                        const size_t qs = ((size_t)b * a.nkv + kvh) * a.q_rows_pad * a.d;
                        uint16_t h0, l0, h1, l1;
                        split_bf16(y0, h0, l0);
                        split_bf16(y1, h1, l1);
                        const size_t i_0 = qs + packed_index(rr, ch, a.d >> 5), i_1 = qs + packed_index(rr, ch + half, a.d >> 5);
                        a.Qp[i_0] = h0; a.Qp_lo[i_0] = l0;
                        a.Qp[i_1] = h1; a.Qp_lo[i_1] = l1;
                    } else {
                        uint16_t *kr = a.Kc + slab + ((size_t)head * a.seq_pad + pos) * a.d;
                        kr[ch] = f32_to_bf16(y0);
                        kr[ch + half] = f32_to_bf16(y1);
                    }
                } else {
                    uint16_t *vv = a.Vc + slab + (size_t)head * a.seq_pad * a.d;
                    vv[vcache_index(pos, ch, a.d)] = f32_to_bf16(v0);
                    vv[vcache_index(pos, ch + half, a.d)] = f32_to_bf16(v1);
                }
            }
        } else if (EPI == FEPI_SWIGLU) {
            if (valid) {
                const float rs = rstd[ml];
                const float gt = v0 * rs, up = v1 * rs;
                const float hval = gt / (1.f + __expf(-gt)) * up;
                uint16_t hi, lo;
                split_bf16(hval, hi, lo);
                const size_t idx = packed_index(m, tile0 * 16 + c, a.KT_out);
                a.out_hi[idx] = hi;
                a.out_lo[idx] = lo;
            }
        } else {  // FEPI_LM: two independent tiles per task
            const int nt = tile0 + i0, n = nt * 16 + c;
            const bool live = valid && nt < a.NT;
            const float logit = live ? v0 * rstd[ml] : -INFINITY;
            if (live && a.logits) a.logits[(size_t)m * a.vocab + n] = logit;
            float bv = logit;
            int bi = n;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off, 16);
                const int oi = __shfl_xor(bi, off, 16);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (live && c == 0) {
                a.part_val[(size_t)m * a.NT + nt] = bv;
                a.part_idx[(size_t)m * a.NT + nt] = bi;
            }
        }
    }
}

template <int MT, int EPI> hipError_t launch_one(const FusedGemmArgs &a, int m_base, hipStream_t s)
{
    hipLaunchKernelGGL((fused_gemm_kernel<MT, EPI>), dim3(a.n_tasks), dim3(Shape<MT, EPI>::WAVES * 64), 0, s, a, m_base);
    return hipGetLastError();
}

template <int EPI> hipError_t launch_epi(const FusedGemmArgs &a, hipStream_t s)
{
    // Passes of at most 10 row tiles; the packed activation buffers hold whole passes.
    const int mt_total = (a.M + 15) / 16;
    for (int t0 = 0; t0 < mt_total; t0 += 10) {
        const int mt = mt_total - t0 < 10 ? mt_total - t0 : 10;
        hipError_t e;
        switch (mt) {
        case 1: e = launch_one<1, EPI>(a, t0 * 16, s); break;
        case 2: e = launch_one<2, EPI>(a, t0 * 16, s); break;
        case 3: e = launch_one<3, EPI>(a, t0 * 16, s); break;
        case 4: e = launch_one<4, EPI>(a, t0 * 16, s); break;
        case 5: e = launch_one<5, EPI>(a, t0 * 16, s); break;
        case 6: e = launch_one<6, EPI>(a, t0 * 16, s); break;
        case 7: case 8: e = launch_one<8, EPI>(a, t0 * 16, s); break;
        default: e = launch_one<10, EPI>(a, t0 * 16, s); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// grid = M rows, 512 threads.  Validates lens/tokens; x = E[token]; packed x*gamma; sums of squares.
__global__ __launch_bounds__(512) void fused_embed_kernel(Dims D, StepIO io, const uint16_t *embed, const uint16_t *gamma,
                                                          float *X, uint16_t *A_hi, uint16_t *A_lo, float *ssq,
                                                          int32_t *pos_base, int32_t *err_flag)
{
    const int m = blockIdx.x, b = m / (io.k + 1), j = m % (io.k + 1);
    int tok = io.tokens[m];
    if (tok < 0 || tok >= D.V) {
        if (threadIdx.x == 0) *err_flag = 1;
        tok = 0;
    }
    if (j == 0 && threadIdx.x == 0) {
        int len = io.lens[b];
        if (len < 0 || len + io.k + 1 > D.max_seq) {
            *err_flag = 1;
            len = 0;
        }
        pos_base[b] = len;
    }
    const uint16_t *row = embed + (size_t)tok * D.h;
    const int KT = (D.h + 31) >> 5, NSS = D.h >> 4;
    for (int i = threadIdx.x; i < D.h; i += blockDim.x) {
        const float x = bf16_to_f32(row[i]);
        X[(size_t)m * D.h + i] = x;
        uint16_t hi, lo;
        split_bf16(x * bf16_to_f32(gamma[i]), hi, lo);
        const size_t idx = packed_index(m, i, KT);
        A_hi[idx] = hi;
        A_lo[idx] = lo;
        float ss = x * x;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
        if ((i & 15) == 0) ssq[(size_t)m * NSS + (i >> 4)] = ss;
    }
}

}  // namespace

hipError_t launch_fused_gemm(const FusedGemmArgs &a, int epilogue, hipStream_t s)
{
    switch (epilogue) {
    case FEPI_QKV: return launch_epi<FEPI_QKV>(a, s);
    case FEPI_RESID: return launch_epi<FEPI_RESID>(a, s);
    case FEPI_SWIGLU: return launch_epi<FEPI_SWIGLU>(a, s);
    default: return launch_epi<FEPI_LM>(a, s);
    }
}

hipError_t launch_fused_embed(const Dims &D, const StepIO &io, const uint16_t *embed, const uint16_t *gamma, float *X,
                              uint16_t *A_hi, uint16_t *A_lo, float *ssq, int32_t *pos_base, int32_t *err_flag,
                              hipStream_t s)
{
    hipLaunchKernelGGL(fused_embed_kernel, dim3(io.B * (io.k + 1)), dim3(512), 0, s, D, io, embed, gamma, X, A_hi, A_lo, ssq,
                       pos_base, err_flag);
    return hipGetLastError();
}
