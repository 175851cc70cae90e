// Skinny bf16 GEMM  Y[M][N] = X[M][K] . W[N][K]^T  for M = B*(k+1) <= 160 rows per pass.
//
// These are the linear rows of the paper's Table 2 (App. B): Q/K_new/V_new = X W,
// Y = A_out W_o, H = SwiGLU(Y W_1), Z = H W_2, plus the LM head.  Their FLOPs:IO
// ratio is ~ b*s_q, far below the MI355X ridge (~312 flop/byte), so the kernel is a
// weight streamer: every weight byte is read from HBM exactly once, with one
// fully coalesced 16-byte-per-lane load per operand tile, straight into the
// registers that feed v_mfma_f32_16x16x32_bf16.  No LDS staging of weights: at
// small M a weight tile is consumed by exactly one wave, so LDS would only add a
// hop.  One workgroup owns one 16-column output tile; its waves split K and
// reduce through LDS in a fixed order (deterministic, no float atomics).
//
// Activations arrive pre-packed in operand-tile order as a bf16 "hi" part and
// (optionally) a bf16 "lo" residual, x ~= hi + lo; while HBM-bound the second
// MFMA per tile is free and makes the activation rounding error negligible.
#include "kernels.h"

namespace {

__device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int MT> struct Tune {
    static constexpr int WAVES = MT <= 2 ? 8 : (MT <= 5 ? 4 : 2);
    static constexpr int U = MT == 1 ? 8 : (MT == 2 ? 4 : (MT <= 5 ? 2 : 1));
};

template <int MT, bool SPLIT, int EPI>
__global__ __launch_bounds__(Tune<MT>::WAVES * 64) void gemm_skinny_kernel(GemmArgs a, int m_base)
{
    constexpr int WAVES = Tune<MT>::WAVES, U = Tune<MT>::U;
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    __shared__ float red[WAVES * NW * MT * 256];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nt = blockIdx.x;
    const int KT = a.KT;
    const int kt0 = (int)(((long)KT * wave) / WAVES), kt1 = (int)(((long)KT * (wave + 1)) / WAVES);

    f32x4 acc[NW][MT];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[w][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const u32x4 *wp[NW];
    wp[0] = a.W0 + (size_t)nt * KT * 64 + lane;
    if (NW == 2) wp[NW - 1] = a.W1 + (size_t)nt * KT * 64 + lane;
    const size_t mt_base = (size_t)(m_base >> 4);
    const u32x4 *ah = a.A_hi + mt_base * KT * 64 + lane;
    const u32x4 *al = SPLIT ? a.A_lo + mt_base * KT * 64 + lane : nullptr;

    int kt = kt0;
    for (; kt + U <= kt1; kt += U) {
        u32x4 wv[NW][U], xv[MT][U], xl[SPLIT ? MT : 1][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int w = 0; w < NW; ++w)
                wv[w][u] = __builtin_nontemporal_load(wp[w] + (size_t)(kt + u) * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                xv[mt][u] = ah[((size_t)mt * KT + kt + u) * 64];
                if (SPLIT) xl[mt][u] = al[((size_t)mt * KT + kt + u) * 64];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    acc[w][mt] = mfma(xv[mt][u], wv[w][u], acc[w][mt]);
                    if (SPLIT) acc[w][mt] = mfma(xl[mt][u], wv[w][u], acc[w][mt]);
                }
    }
    for (; kt < kt1; ++kt) {
        u32x4 wv[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w)
            wv[w] = __builtin_nontemporal_load(wp[w] + (size_t)kt * 64);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            u32x4 xv = ah[((size_t)mt * KT + kt) * 64];
#pragma unroll
            for (int w = 0; w < NW; ++w)
                acc[w][mt] = mfma(xv, wv[w], acc[w][mt]);
            if (SPLIT) {
                u32x4 xl = al[((size_t)mt * KT + kt) * 64];
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    acc[w][mt] = mfma(xl, wv[w], acc[w][mt]);
            }
        }
    }

    // Cross-wave reduction of the K split.  acc[w][mt][r] of lane l = 16*q + c is
    // output row mt*16 + 4*q + r, column nt*16 + c.
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                red[((wave * NW + w) * MT + mt) * 256 + r * 64 + lane] = acc[w][mt][r];
    __syncthreads();

    for (int o = threadIdx.x; o < MT * 256; o += WAVES * 64) {
        const int mt = o >> 8, r = (o >> 6) & 3, l = o & 63;
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int wv = 0; wv < WAVES; ++wv) {
            v0 += red[((wv * NW + 0) * MT + mt) * 256 + r * 64 + l];
            if (NW == 2) v1 += red[((wv * NW + (NW - 1)) * MT + mt) * 256 + r * 64 + l];
        }
        const int m = m_base + mt * 16 + 4 * (l >> 4) + r;
        const int n = nt * 16 + (l & 15);
        const bool valid = m < a.M;
        if (EPI == EPI_STORE) {
            if (valid) a.out_f32[(size_t)m * a.ld + n] = v0;
        } else if (EPI == EPI_RESID) {
            if (valid) a.out_f32[(size_t)m * a.ld + n] += v0;
        } else if (EPI == EPI_SWIGLU) {
            if (valid) {
                const float hval = v0 / (1.f + __expf(-v0)) * v1;
                uint16_t hi, lo;
                split_bf16(hval, hi, lo);
                const size_t idx = packed_index(m, n, a.KT_out);
                a.out_hi[idx] = hi;
                if (SPLIT) a.out_lo[idx] = lo;
            }
        } else {  // EPI_LMHEAD
            if (valid && a.logits) a.logits[(size_t)m * a.ld + n] = v0;
            float bv = v0;
            int bi = n;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {  // arg-max over the 16 columns; lowest id wins ties
                const float ov = __shfl_xor(bv, off, 16);
                const int oi = __shfl_xor(bi, off, 16);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (valid && (l & 15) == 0) {
                a.part_val[(size_t)m * a.NT + nt] = bv;
                a.part_idx[(size_t)m * a.NT + nt] = bi;
            }
        }
    }
}

template <int MT, bool SPLIT, int EPI> hipError_t launch_one(const GemmArgs &a, int m_base, hipStream_t s)
{
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, SPLIT, EPI>), dim3(a.NT), dim3(Tune<MT>::WAVES * 64), 0, s, a, m_base);
    return hipGetLastError();
}

template <bool SPLIT, int EPI> hipError_t launch_mt(const GemmArgs &a, int mt, int m_base, hipStream_t s)
{
    switch (mt) {
    case 1: return launch_one<1, SPLIT, EPI>(a, m_base, s);
    case 2: return launch_one<2, SPLIT, EPI>(a, m_base, s);
    case 3: return launch_one<3, SPLIT, EPI>(a, m_base, s);
    case 4: return launch_one<4, SPLIT, EPI>(a, m_base, s);
    case 5: return launch_one<5, SPLIT, EPI>(a, m_base, s);
    case 6: return launch_one<6, SPLIT, EPI>(a, m_base, s);
    case 7: case 8: return launch_one<8, SPLIT, EPI>(a, m_base, s);
    default: return launch_one<10, SPLIT, EPI>(a, m_base, s);
    }
}

template <int EPI> hipError_t launch_epi(const GemmArgs &a, bool split, hipStream_t s)
{
    // Passes of at most 10 row tiles.  The packed activation buffers always hold
    // whole tiles up to the pass boundary the template covers (they are sized for
    // the padded maximum), so computing a few dead rows is safe.
    const int mt_total = (a.M + 15) / 16;
    for (int t0 = 0; t0 < mt_total; t0 += 10) {
        const int mt = mt_total - t0 < 10 ? mt_total - t0 : 10;
        hipError_t e = split ? launch_mt<true, EPI>(a, mt, t0 * 16, s) : launch_mt<false, EPI>(a, mt, t0 * 16, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void pack_weight_kernel(const uint16_t *src, u32x4 *dst, int N, int K, int KT)
{
    const size_t rec = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte lane record
    const size_t total = (size_t)(N >> 4) * KT * 64;
    if (rec >= total) return;
    const int lane = (int)(rec & 63);
    const size_t tile = rec >> 6;
    const int kt = (int)(tile % KT);
    const int nt = (int)(tile / KT);
    const int n = nt * 16 + (lane & 15), k = kt * 32 + 8 * (lane >> 4);
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (k + 8 <= K) {
        v = *reinterpret_cast<const u32x4 *>(src + (size_t)n * K + k);
    } else if (k < K) {
        uint16_t tmp[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int e = 0; e < 8 && k + e < K; ++e) tmp[e] = src[(size_t)n * K + k + e];
        v = *reinterpret_cast<u32x4 *>(tmp);
    }
    dst[rec] = v;
}

}  // namespace

hipError_t launch_gemm(const GemmArgs &a, int epilogue, bool split, hipStream_t s)
{
    switch (epilogue) {
    case EPI_STORE: return launch_epi<EPI_STORE>(a, split, s);
    case EPI_RESID: return launch_epi<EPI_RESID>(a, split, s);
    case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(a, split, s);
    default: return launch_epi<EPI_LMHEAD>(a, split, s);
    }
}

hipError_t launch_pack_weight(const uint16_t *src, uint16_t *dst, int N, int K, hipStream_t s)
{
    const int KT = (K + 31) / 32;
    const size_t total = (size_t)(N / 16) * KT * 64;
    const int threads = 256;
    const unsigned blocks = (unsigned)((total + threads - 1) / threads);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(threads), 0, s, src, reinterpret_cast<u32x4 *>(dst), N, K, KT);
    return hipGetLastError();
}
