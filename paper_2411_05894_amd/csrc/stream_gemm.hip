// Weight-streaming GEMMs of the verify step and their fused epilogues.
//
// The linear rows of the paper's Table 2 (App. B) -- Q/K_new/V_new = X W, Y = A_out W_o,
// H = SwiGLU(Y W_1), Z = H W_2 -- and the LM head have FLOPs:IO ~ b*s_q, far below the
// MI355X ridge (~312 flop/byte), so each launch is a stream of the weight matrix through
// the matrix cores with everything else hidden behind it.
//
//   pgemm_kernel   M <= 16 rows.  Persistent: one workgroup of 16 waves per compute unit walks a
//                  list of 16-column output tiles.  Each wave owns a fixed k-slice and keeps the
//                  activations of that slice (bf16 hi and lo parts) in registers for the whole
//                  launch, so the inner loop touches memory only for weights.  Weight registers
//                  are refilled for the NEXT tile right after the MFMA that consumed them: a
//                  rolling prefetch with a constant number of bytes in flight per wave and no
//                  bubble at tile boundaries.  The k-split is reduced through LDS in fixed order.
//   epi_kernel     Sums split-K partial results (when K is split over workgroups) in fixed order
//                  and applies the epilogue.
//
// Epilogues (everything Table 2 leaves out is folded into them):
//   QKV     RMSNorm scale, rotary embedding, Q -> packed hi/lo operand, K/V -> cache (in place)
//   RESID   X += acc; packed X*gamma_next hi/lo; sums of squares per 16 columns
//   SWIGLU  RMSNorm scale, silu(gate)*up -> packed hi/lo operand
//   LM      RMSNorm scale, per-tile arg-max (logits are never materialised unless asked for)
// RMSNorm needs no pass of its own: the producer of the residual stream x writes x*gamma and
// partial sums of squares, the consuming GEMM scales its fp32 results by rsqrt(mean(x^2)+eps),
// which commutes with the matrix product.
#include "kernels.h"

namespace {

__device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// A "unit" is what one epilogue invocation needs: a rotary tile pair (QKV), a gate tile and its
// up tile (SWIGLU), or a single tile.
template <int EPI> struct Unit {
    static constexpr int TILES = (EPI == FEPI_QKV || EPI == FEPI_SWIGLU) ? 2 : 1;
};

// Tile index of (unit, part) in the concatenated output [Q | K | V] or [gate | up].
template <int EPI> __device__ __forceinline__ int unit_tile(const FusedGemmArgs &a, int unit, int part)
{
    if (EPI == FEPI_QKV) {
        const int TH = a.d >> 4, per_head = TH >> 1;
        return (unit / per_head) * TH + unit % per_head + part * per_head;
    }
    if (EPI == FEPI_SWIGLU) return unit + part * a.NT;
    return unit;
}

// Packed weights of concatenated tile gt (k-tile 0, lane record 0).
template <int EPI> __device__ __forceinline__ const u32x4 *tile_weights(const FusedGemmArgs &a, int gt)
{
    const size_t stride = (size_t)a.KT * 64;
    if (EPI == FEPI_QKV) {
        const int TH = a.d >> 4, nqT = a.nq * TH, nkT = a.nkv * TH;
        if (gt < nqT) return a.W0 + gt * stride;
        if (gt < nqT + nkT) return a.W1 + (gt - nqT) * stride;
        return a.W2 + (gt - nqT - nkT) * stride;
    }
    if (EPI == FEPI_SWIGLU) return gt < a.NT ? a.W0 + gt * stride : a.W1 + (gt - a.NT) * stride;
    return a.W0 + gt * stride;
}

// One output element pair of a unit: row m, column c of the 16-column tile(s).  v0/v1 are the
// fp32 results of the unit's first/second tile.  The 16 lanes c = 0..15 of a row are adjacent
// lanes of one wave (RESID and LM reduce over them).
template <int EPI>
__device__ __forceinline__ void epilogue(const FusedGemmArgs &a, int unit, int m, int c, bool valid, float v0, float v1, float rs)
{
    if (EPI == FEPI_RESID) {
        const int n = unit * 16 + c;
        float xn = 0.f;
        if (valid) {
            xn = a.X[(size_t)m * a.h + n] + v0;
            a.X[(size_t)m * a.h + n] = xn;
            uint16_t hi, lo;
            split_bf16(xn * bf16_to_f32(a.gamma_next[n]), hi, lo);
            const size_t idx = packed_index(m, n, (a.h + 31) >> 5);
            a.out_hi[idx] = hi;
            a.out_lo[idx] = lo;
        }
        float ss = xn * xn;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
        if (valid && c == 0) a.ssq_out[(size_t)m * (a.h >> 4) + unit] = ss;
    } else if (EPI == FEPI_QKV) {
        if (!valid) return;
        const int TH = a.d >> 4, per_head = TH >> 1;
        int head = unit / per_head;
        const int pair = unit % per_head;
        v0 *= rs;
        v1 *= rs;
        const int b = m / (a.k + 1), j = m % (a.k + 1);
        const int pos = a.pos_base[b] + j;
        const int half = a.d >> 1, ch = pair * 16 + c;  // channel of v0; v1 is ch + half
        const size_t slab = (size_t)b * a.nkv * a.seq_pad * a.d;
        if (head < a.nq + a.nkv) {
            const float2 cs = *reinterpret_cast<const float2 *>(a.rope_cs + ((size_t)pos * half + ch) * 2);
            const float y0 = v0 * cs.x - v1 * cs.y, y1 = v0 * cs.y + v1 * cs.x;
            if (head < a.nq) {
                const int g = a.nq / a.nkv, kvh = head / g, hl = head % g, rr = j * g + hl;
                const size_t qs = ((size_t)b * a.nkv + kvh) * a.q_rows_pad * a.d;
                uint16_t h0, l0, h1, l1;
                split_bf16(y0, h0, l0);
                split_bf16(y1, h1, l1);
                const size_t i_0 = qs + packed_index(rr, ch, a.d >> 5), i_1 = qs + packed_index(rr, ch + half, a.d >> 5);
                a.Qp[i_0] = h0; a.Qp_lo[i_0] = l0;
                a.Qp[i_1] = h1; a.Qp_lo[i_1] = l1;
            } else {
                head -= a.nq;
                uint16_t *kr = a.Kc + slab + ((size_t)head * a.seq_pad + pos) * a.d;
                kr[ch] = f32_to_bf16(y0);
                kr[ch + half] = f32_to_bf16(y1);
            }
        } else {
            head -= a.nq + a.nkv;
            uint16_t *vv = a.Vc + slab + (size_t)head * a.seq_pad * a.d;
            vv[vcache_index(pos, ch, a.d)] = f32_to_bf16(v0);
            vv[vcache_index(pos, ch + half, a.d)] = f32_to_bf16(v1);
        }
    } else if (EPI == FEPI_SWIGLU) {
        if (!valid) return;
        const float gt = v0 * rs, up = v1 * rs;
        const float hval = gt / (1.f + __expf(-gt)) * up;
        uint16_t hi, lo;
        split_bf16(hval, hi, lo);
        const size_t idx = packed_index(m, unit * 16 + c, a.KT_out);
        a.out_hi[idx] = hi;
        a.out_lo[idx] = lo;
    } else {  // FEPI_LM
        const int n = unit * 16 + c;
        const float logit = valid ? v0 * rs : -INFINITY;
        if (valid && a.logits) a.logits[(size_t)m * a.vocab + n] = logit;
        float bv = logit;
        int bi = n;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 16);
            const int oi = __shfl_xor(bi, off, 16);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (valid && c == 0) {
            a.part_val[(size_t)m * a.NT + unit] = bv;
            a.part_idx[(size_t)m * a.NT + unit] = bi;
        }
    }
}

// rsqrt(mean(x^2) + eps) of row m from the producer's per-16-column sums of squares; whole wave.
__device__ __forceinline__ float row_rstd(const FusedGemmArgs &a, int m, int lane)
{
    const int NSS = a.h >> 4;
    float sum = 0.f;
    if (m < a.M)
        for (int t = lane; t < NSS; t += 64) sum += a.ssq_in[(size_t)m * NSS + t];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    return rsqrtf(sum / (float)a.h + a.eps);
}

// ------------------------------------------------------------------ M <= 16 ----
constexpr int PW = 16;  // waves per workgroup

template <int KPW, bool PREFETCH>
__device__ __forceinline__ f32x4 stream_tile(const u32x4 (&ah)[KPW], const u32x4 (&al)[KPW], u32x4 (&w)[KPW], const u32x4 *wn,
                                             const int (&koff)[KPW])
{
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
        s0 = mfma(ah[i], w[i], s0);
        s1 = mfma(al[i], w[i], s1);
        if (PREFETCH) w[i] = __builtin_nontemporal_load(wn + koff[i]);
    }
    return s0 + s1;
}

// grid = n_groups * J workgroups of 1024 threads.  Workgroup (grp, j) computes units
// [grp*upw, (grp+1)*upw) over k-tiles [j*16*KPW, (j+1)*16*KPW); with J > 1 it stores fp32
// partial tiles for epi_kernel instead of applying the epilogue.
template <int EPI, int KPW>
__global__ __launch_bounds__(PW * 64) void pgemm_kernel(FusedGemmArgs a)
{
    constexpr int TPU = Unit<EPI>::TILES;
    __shared__ float red[2][PW][256];
    __shared__ float rstd_s[16];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int J = a.J, j = blockIdx.x % J, grp = blockIdx.x / J;
    const int KT = a.KT;
    const int kt0 = (j * PW + wave) * KPW;
    const int u_begin = grp * a.upw;
    const int u_end = u_begin + a.upw < a.n_units ? u_begin + a.upw : a.n_units;
    if (u_begin >= u_end) return;
    const int n_steps = (u_end - u_begin) * TPU;

    // k-tiles past the matrix (ragged K split) contribute zero activations and re-read the last tile.
    int koff[KPW];
#pragma unroll
    for (int i = 0; i < KPW; ++i) koff[i] = (kt0 + i < KT ? kt0 + i : KT - 1) * 64;

    u32x4 w[KPW], ah[KPW], al[KPW];
    const u32x4 *wp = tile_weights<EPI>(a, unit_tile<EPI>(a, u_begin, 0)) + lane;
#pragma unroll
    for (int i = 0; i < KPW; ++i) w[i] = __builtin_nontemporal_load(wp + koff[i]);
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
        const bool live = kt0 + i < KT;
        ah[i] = live ? a.A_hi[(size_t)koff[i] + lane] : u32x4{0, 0, 0, 0};
        al[i] = live ? a.A_lo[(size_t)koff[i] + lane] : u32x4{0, 0, 0, 0};
    }
    if (EPI != FEPI_RESID && J == 1) rstd_s[wave] = row_rstd(a, wave, lane);   // published by the first barrier

    float keep = 0.f;
    for (int s = 0; s < n_steps; ++s) {
        const int unit = u_begin + s / TPU, part = s % TPU;
        f32x4 acc;
        if (s + 1 < n_steps) {
            const u32x4 *wn = tile_weights<EPI>(a, unit_tile<EPI>(a, u_begin + (s + 1) / TPU, (s + 1) % TPU)) + lane;
            acc = stream_tile<KPW, true>(ah, al, w, wn, koff);
        } else {
            acc = stream_tile<KPW, false>(ah, al, w, nullptr, koff);
        }
        float *rb = &red[s & 1][0][0];
#pragma unroll
        for (int r = 0; r < 4; ++r) rb[wave * 256 + r * 64 + lane] = acc[r];
        __syncthreads();
        // Buffer s&1 is rewritten at step s+2, after the barrier of step s+1, which the four
        // reducing waves reach only after they have read it.
        if (wave < 4) {
            float v = 0.f;
#pragma unroll
            for (int ww = 0; ww < PW; ++ww) v += rb[ww * 256 + wave * 64 + lane];
            const int m = 4 * (lane >> 4) + wave, c = lane & 15;
            if (J > 1) {
                a.partials[((size_t)j * a.part_rows + m) * a.Ntot + unit_tile<EPI>(a, unit, part) * 16 + c] = v;
            } else if (TPU == 2 && part == 0) {
                keep = v;
            } else {
                const float rs = EPI == FEPI_RESID ? 1.f : rstd_s[m];
                if (TPU == 2) epilogue<EPI>(a, unit, m, c, m < a.M, keep, v, rs);
                else epilogue<EPI>(a, unit, m, c, m < a.M, v, 0.f, rs);
            }
        }
    }
}

// grid = (unit blocks, row tiles of 16), 256 threads.  Sums the J partial results of each unit
// in the order j = 0..J-1 and applies the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void epi_kernel(FusedGemmArgs a, int units_per_block)
{
    constexpr int TPU = Unit<EPI>::TILES;
    __shared__ float rstd_s[16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = blockIdx.y * 16;
    if (EPI != FEPI_RESID) {
        for (int r = wave; r < 16; r += 4) {
            const float rs = row_rstd(a, m0 + r, lane);
            if (lane == 0) rstd_s[r] = rs;
        }
        __syncthreads();
    }
    const int ml = 4 * (lane >> 4) + wave, m = m0 + ml, c = lane & 15;
    const bool valid = m < a.M;
    const float rs = EPI == FEPI_RESID ? 1.f : rstd_s[ml];
    const int u_begin = blockIdx.x * units_per_block;
    const int u_end = u_begin + units_per_block < a.n_units ? u_begin + units_per_block : a.n_units;
    const size_t jstride = (size_t)a.part_rows * a.Ntot;
    for (int unit = u_begin; unit < u_end; ++unit) {
        float v[TPU];
#pragma unroll
        for (int part = 0; part < TPU; ++part) {
            const float *p = a.partials + (size_t)m * a.Ntot + unit_tile<EPI>(a, unit, part) * 16 + c;
            float s = 0.f;
            if (valid)
                for (int j = 0; j < a.J; ++j) s += p[j * jstride];
            v[part] = s;
        }
        epilogue<EPI>(a, unit, m, c, valid, v[0], v[TPU - 1], rs);
    }
}

template <int EPI> hipError_t launch_small(FusedGemmArgs a, hipStream_t s)
{
    // k-tiles per wave: 7 when K is a multiple of 16*7*32 but not of 16*8*32 (the FFN widths of the
    // Llama shapes), else 8; a ragged K split is legal either way.
    const bool seven = a.KT % (PW * 7) == 0 && a.KT % (PW * 8) != 0;
    const int kpw = seven ? 7 : 8;
    a.J = (a.KT + PW * kpw - 1) / (PW * kpw);
    const int n_cu = a.n_cu > 0 ? a.n_cu : 256;
    int groups_target = n_cu / a.J;
    if (groups_target < 1) groups_target = 1;
    a.upw = (a.n_units + groups_target - 1) / groups_target;
    const int groups = (a.n_units + a.upw - 1) / a.upw;
    a.part_rows = 16;
    if (a.J > 1 && (size_t)a.J * a.part_rows * a.Ntot * sizeof(float) > a.partial_bytes) return hipErrorInvalidValue;
    if (seven) hipLaunchKernelGGL((pgemm_kernel<EPI, 7>), dim3(groups * a.J), dim3(PW * 64), 0, s, a);
    else hipLaunchKernelGGL((pgemm_kernel<EPI, 8>), dim3(groups * a.J), dim3(PW * 64), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.J == 1) return e;
    int upb = (a.n_units + 4 * n_cu - 1) / (4 * n_cu);
    if (upb < 1) upb = 1;
    hipLaunchKernelGGL((epi_kernel<EPI>), dim3((a.n_units + upb - 1) / upb, 1), dim3(256), 0, s, a, upb);
    return hipGetLastError();
}

}  // namespace

int stream_gemm_max_rows() { return 16; }

// Split-K scratch needed for M rows: the largest J * rows * Ntot over the model's GEMMs.
size_t stream_gemm_partial_bytes(const Dims &D, int M)
{
    (void)M;
    auto slices = [](int K) {
        const int KT = (K + 31) / 32;
        const bool seven = KT % (PW * 7) == 0 && KT % (PW * 8) != 0;
        const int ks = PW * (seven ? 7 : 8);
        return (size_t)((KT + ks - 1) / ks);
    };
    size_t best = 0;
    auto consider = [&](int K, size_t ntot) {
        const size_t j = slices(K);
        if (j > 1 && j * 16 * ntot > best) best = j * 16 * ntot;
    };
    consider(D.h, (size_t)D.qd + 2 * D.kd);
    consider(D.qd, D.h);
    consider(D.h, 2 * (size_t)D.f);
    consider(D.f, D.h);
    consider(D.h, D.V);
    return best * sizeof(float);
}

hipError_t launch_stream_gemm(const FusedGemmArgs &a, int epilogue, hipStream_t s)
{
    switch (epilogue) {
    case FEPI_QKV: return launch_small<FEPI_QKV>(a, s);
    case FEPI_RESID: return launch_small<FEPI_RESID>(a, s);
    case FEPI_SWIGLU: return launch_small<FEPI_SWIGLU>(a, s);
    default: return launch_small<FEPI_LM>(a, s);
    }
}
