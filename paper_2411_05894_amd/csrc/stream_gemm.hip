// Weight-streaming GEMMs of the verify step and their fused epilogues.
//
// The linear rows of the paper's Table 2 (App. B) -- Q/K_new/V_new = X W, Y = A_out W_o,
// H = SwiGLU(Y W_1), Z = H W_2 -- and the LM head have FLOPs:IO ~ b*s_q, far below the
// MI355X ridge (~312 flop/byte), so each launch is a stream of the weight matrix through
// the matrix cores with everything else hidden behind it.
//
//   pgemm_kernel   M <= 32 rows (one or two 16-row tiles).  Persistent: one workgroup of 16 waves per compute unit walks a
//                  list of 16-column output tiles.  Each wave owns a fixed k-slice and keeps the
//                  activations of that slice (bf16 hi and lo parts) in registers for the whole
//                  launch, so the inner loop touches memory only for weights.  Weight registers
//                  are refilled for the NEXT tile right after the MFMA that consumed them: a
//                  rolling prefetch with a constant number of bytes in flight per wave and no
//                  bubble at tile boundaries.  The k-split is reduced through LDS in fixed order.
//   qgemm16_kernel M > 48 rows (up to 160 per pass).  v_mfma_f32_16x16x32_bf16 tiles: each wave of a
//                  workgroup of eight (four for the small matrices) owns 32 output columns and streams
//                  their weights HBM -> registers (rolling prefetch, every weight byte read once), while
//                  the activation k-tiles of the workgroup's k-slice, which all its waves need, are staged
//                  through a register ring and a two-deep LDS ring.  Results go to split-K partials for
//                  epi_kernel.
//   qgemm_kernel   33..48 rows (and the rows a pass of 160 leaves over): the same launch on
//                  v_mfma_f32_32x32x16_bf16, the 16-row operand tiles of the packed layout read as the
//                  halves of 32-row MFMA operands, so one weight layout serves every kernel.
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

#include <hip/hip_ext.h>

#include "gemm_device.h"

namespace {

// ------------------------------------------------------------------ M <= 32 ----
constexpr int PW = 16;  // waves per workgroup

// Weight tile load.  One reader per byte (RH == 1): streaming, the line is not worth keeping.  Two
// workgroups of a die reading the same tiles (RH == 2): an ordinary load, so that the line is still in
// the die's L2 when the second request comes.
template <int RH> __device__ __forceinline__ u32x4 wload(const u32x4 *p)
{
    return RH == 1 ? __builtin_nontemporal_load(p) : *p;
}

template <int KPW, bool PREFETCH, int RH>
__device__ __forceinline__ f32x4 stream_tile(const u32x4 (&ah)[KPW], const u32x4 (&al)[KPW], u32x4 (&w)[KPW], const u32x4 *wn,
                                             const int (&koff)[KPW])
{
    f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
        s0 = mfma(ah[i], w[i], s0);
        s1 = mfma(al[i], w[i], s1);
        if (PREFETCH) w[i] = wload<RH>(wn + koff[i]);
    }
    return s0 + s1;
}

// grid = RH * n_groups * J workgroups of 1024 threads, each on one row tile of 16.  Workgroup
// (grp, j) computes its units over k-tiles [j*16*KPW, (j+1)*16*KPW); with J > 1 (SPLIT) it stores
// fp32 partial tiles, and the workgroup of a column group that arrives last sums them and applies the
// epilogue (epi_kernel does, in a second launch, when the launcher has no arrival counters for it).
// The unsplit instantiation carries none of that code (the QKV kernel is at the register limit).
//
// RH == 2 serves 17..32 rows without giving up the register-resident activations: the launch holds
// every workgroup twice, once for rows 0..15 and once for rows 16..31 (row tile rt), and the two copies
// sit 8 apart in the grid, i.e. on the same die, where they start together and ask for the same weight
// tiles: one of the two requests is served by the die's L2 (or merged with the other in flight), so
// HBM still sees each weight byte once (measured: 1.02 x the matrix bytes fetched per launch).
template <int EPI, int KPW, bool SPLIT, int RH>
__global__ __launch_bounds__(PW * 64) void pgemm_kernel(FusedGemmArgs a)
{
    constexpr int TPU = Unit<EPI>::TILES;
    __shared__ float red[2][PW][256];
    __shared__ float rstd_s[16];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // logical workgroup `bid` of `nblk`, and the row tile it serves
    int bid = blockIdx.x, nblk = gridDim.x, rt = 0;
    if (RH == 2) {
        nblk >>= 1;
        const int paired = nblk & ~7, b = blockIdx.x;           // whole sets of 8 logical workgroups, then the rest
        if (b < 2 * paired) {
            rt = (b >> 3) & 1;
            bid = ((b >> 4) << 3) | (b & 7);
        } else {
            const int rem = nblk - paired;
            rt = (b - 2 * paired) / rem;
            bid = paired + (b - 2 * paired) % rem;
        }
    }
    const int m_base = 16 * rt;
    const int J = SPLIT ? a.J : 1, j = SPLIT ? bid % J : 0, grp = SPLIT ? bid / J : bid;
    const int KT = a.KT;
    const int kt0 = (j * PW + wave) * KPW;
    // Units grp, grp + groups, grp + 2*groups, ... so that at any time the workgroups of a launch
    // read neighbouring tiles (measured 3 % faster on the layer matrices); the LM head, 30 times as
    // many tiles, measured 3 % faster with a contiguous run of upw units per workgroup.
    const int groups = nblk / J;
    constexpr bool RUNS = EPI == FEPI_LM;
    const int u_begin = RUNS ? grp * a.upw : grp, u_stride = RUNS ? 1 : groups;
    if (u_begin >= a.n_units) return;
    const int n_mine = RUNS ? (u_begin + a.upw < a.n_units ? a.upw : a.n_units - u_begin) : (a.n_units - grp + groups - 1) / groups;
    const int n_steps = n_mine * TPU;

    // k-tiles past the matrix (ragged K split) contribute zero activations and re-read the last tile.
    int koff[KPW];
#pragma unroll
    for (int i = 0; i < KPW; ++i) koff[i] = (kt0 + i < KT ? kt0 + i : KT - 1) * 64;

    u32x4 w[KPW], ah[KPW], al[KPW];
    const u32x4 *wp = tile_weights<EPI>(a, unit_tile<EPI>(a, u_begin, 0)) + lane;
#pragma unroll
    for (int i = 0; i < KPW; ++i) w[i] = wload<RH>(wp + koff[i]);
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
        const bool live = kt0 + i < KT;
        const size_t at = (size_t)rt * KT * 64 + koff[i] + lane;
        ah[i] = live ? a.A_hi[at] : u32x4{0, 0, 0, 0};
        al[i] = live ? a.A_lo[at] : u32x4{0, 0, 0, 0};
    }
    if (EPI != FEPI_RESID && EPI != FEPI_STORE && !SPLIT) rstd_s[wave] = row_rstd(a, m_base + wave, lane);   // published by the first barrier

    float keep = 0.f;
    for (int s = 0; s < n_steps; ++s) {
        const int unit = u_begin + (s / TPU) * u_stride, part = s % TPU;
        f32x4 acc;
        if (s + 1 < n_steps) {
            const u32x4 *wn = tile_weights<EPI>(a, unit_tile<EPI>(a, u_begin + ((s + 1) / TPU) * u_stride, (s + 1) % TPU)) + lane;
            acc = stream_tile<KPW, true, RH>(ah, al, w, wn, koff);
        } else {
            acc = stream_tile<KPW, false, RH>(ah, al, w, nullptr, koff);
        }
        float *rb = &red[s & 1][0][0];
#pragma unroll
        for (int r = 0; r < 4; ++r) rb[wave * 256 + r * 64 + lane] = acc[r];
        __syncthreads();
        // Buffer s&1 is rewritten at step s+2, after the barrier of step s+1, which the reducing waves
        // reach only after they have read it.
        if (wave < 4) {
            float v = 0.f;
#pragma unroll
            for (int ww = 0; ww < PW; ++ww) v += rb[ww * 256 + wave * 64 + lane];
            const int ml = 4 * (lane >> 4) + wave, m = m_base + ml, c = lane & 15;
            if (SPLIT) {
                // device-scope: read back by the last workgroup of the group, on whichever die it runs
                st<true>(a.partials + ((size_t)j * a.part_rows + m) * a.Ntot + unit_tile<EPI>(a, unit, part) * 16 + c, v);
            } else if (TPU == 2 && part == 0) {
                keep = v;
            } else {
                const float rs = (EPI == FEPI_RESID || EPI == FEPI_STORE) ? 1.f : rstd_s[ml];
                if (TPU == 2) epilogue<EPI>(a, unit, m, c, m < a.M, keep, v, rs);
                else epilogue<EPI>(a, unit, m, c, m < a.M, v, 0.f, rs);
            }
        }
    }

    // Split K with arrival counters: the workgroup of a (row tile, column group) that finishes last
    // sums the group's slices (in slice order, so the result does not depend on which one that is)
    // and applies the epilogue -- no second launch.  The slices were stored device-scope and each wave
    // waits for its stores before the workgroup is counted; they are read back device-scope.  The
    // counter is back at zero for the next launch on the stream.
    if (SPLIT && a.tail_count) {
        __shared__ int last_s;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            int *count = a.tail_count + rt * groups + grp;
            const int old = __hip_atomic_fetch_add(count, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last_s = old == J - 1;
            if (old == J - 1) __hip_atomic_store(count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!last_s) return;
        constexpr bool SCALED = EPI != FEPI_RESID && EPI != FEPI_STORE;
        if (SCALED) {
            rstd_s[wave] = row_rstd(a, m_base + wave, lane);
            __syncthreads();
        }
        if (EPI == FEPI_RESID) {
            // thread for thread what epi_kernel does (same order of every sum): a wave takes two units,
            // 8 columns per thread, lanes 16 apart share a unit's sum of squares
            const int r = lane & 15, kg = lane >> 4;
            for (int i = 2 * wave + (kg >> 1); i - (kg >> 1) < n_mine; i += 2 * PW) {
                const int unit = u_begin + i * u_stride, col = unit * 16 + (kg & 1) * 8;
                const int m = m_base + r;
                const bool live = i < n_mine && m < a.M;
                Vec8 v0{};
                if (live) v0 = sum_slices<true>(a, m, col);
                resid_block<false>(a, m, col, live, kg, v0);
            }
        } else {
            const size_t jstride = (size_t)a.part_rows * a.Ntot;
            for (int e = threadIdx.x; e < n_mine * 256; e += PW * 64) {   // 16 adjacent lanes: one row of a unit
                const int unit = u_begin + (e >> 8) * u_stride, ml = (e & 255) >> 4, m = m_base + ml, c = e & 15;
                float v[TPU];
#pragma unroll
                for (int part = 0; part < TPU; ++part) {
                    const float *pp = a.partials + (size_t)m * a.Ntot + unit_tile<EPI>(a, unit, part) * 16 + c;
                    float sum = ld<true>(pp);
                    for (int jj = 1; jj < J; ++jj) sum += ld<true>(pp + jj * jstride);
                    v[part] = sum;
                }
                epilogue<EPI>(a, unit, m, c, m < a.M, v[0], TPU == 2 ? v[TPU - 1] : 0.f, SCALED ? rstd_s[ml] : 1.f);
            }
        }
    }
}

// ---- epilogue from split-K partials ----
// The same four epilogues on 8 consecutive output columns per thread: thread (row r = lane%16,
// column group kg = lane/16) of a wave owns columns 8*kg..8*kg+7 of a 32-column block, which is
// exactly one 16-byte lane record of the packed operand layout, so a wave writes whole operand
// tiles (1 KiB, contiguous) and reads 128 contiguous bytes of each partial row.
// Column blocks of 32 per epilogue: plain output columns, except QKV, whose blocks run over the
// first-half channels of each head (the rotary partner columns come along).
template <int EPI> __device__ __host__ __forceinline__ int column_blocks(const FusedGemmArgs &a)
{
    if (EPI == FEPI_QKV) return (a.nq + 2 * a.nkv) * ((a.d / 2 + 31) / 32);
    if (EPI == FEPI_SWIGLU) return (a.Ntot / 2 + 31) / 32;
    return (a.Ntot + 31) / 32;
}

// grid = (column-block groups, row tiles of 16), 256 threads; each wave takes column blocks
// cb0 + wave, cb0 + wave + 4, ...  The partial sums of a block are fetched one block ahead (the
// first block's before the row scales are reduced), so the kernel's dependent memory round trips
// overlap.
template <int EPI>
__global__ __launch_bounds__(256) void epi_kernel(FusedGemmArgs a, int blocks_per_wg)
{
    __shared__ float rstd_s[16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = blockIdx.y * 16;
    constexpr bool SCALED = EPI != FEPI_RESID && EPI != FEPI_STORE;
    constexpr bool PAIRED = EPI == FEPI_QKV || EPI == FEPI_SWIGLU;
    const int r = lane & 15, kg = lane >> 4, m = m0 + r;
    const bool row_ok = m < a.M;
    const int n_cb = column_blocks<EPI>(a);
    const int cb_begin = blockIdx.x * blocks_per_wg;
    const int cb_end = cb_begin + blocks_per_wg < n_cb ? cb_begin + blocks_per_wg : n_cb;
    const int half = a.d >> 1, bph = (half + 31) / 32;   // QKV: column blocks per head

    // first output column of this thread in block cb (QKV: of the head's first half), or -1
    auto column = [&](int cb) -> int {
        if (!row_ok) return -1;
        if (EPI == FEPI_QKV) {
            const int ch = (cb % bph) * 32 + kg * 8;
            return ch < half ? (cb / bph) * a.d + ch : -1;
        }
        const int n0 = cb * 32 + kg * 8;
        return n0 < (EPI == FEPI_SWIGLU ? a.Ntot >> 1 : a.Ntot) ? n0 : -1;
    };
    auto fetch = [&](int cb, Vec8 &v0, Vec8 &v1) {
        const int col = cb < cb_end ? column(cb) : -1;
        if (col >= 0) {
            v0 = sum_slices(a, m, col);
            if (PAIRED) v1 = sum_slices(a, m, col + (EPI == FEPI_QKV ? half : a.Ntot >> 1));
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v0.v[e] = v1.v[e] = 0.f;
        }
    };

    // Row scales: four rows per wave.  Their loads go out first and the first block's partial
    // sums right behind them, so the two dependent round trips overlap.
    constexpr int SV = 8;                     // sums of squares per lane and row held in registers (h <= 8192)
    const int NSS = a.h >> 4;
    float sv[4][SV];
    if (SCALED) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int mm = m0 + wave + 4 * q;
#pragma unroll
            for (int i = 0; i < SV; ++i) {
                const int t = lane + 64 * i;
                sv[q][i] = (mm < a.M && t < NSS) ? a.ssq_in[(size_t)mm * NSS + t] : 0.f;
            }
        }
    }
    Vec8 v0, v1;
    fetch(cb_begin + wave, v0, v1);
    if (SCALED) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int mm = m0 + wave + 4 * q;
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < SV; ++i) sum += sv[q][i];
            if (mm < a.M)
                for (int t = lane + 64 * SV; t < NSS; t += 64) sum += a.ssq_in[(size_t)mm * NSS + t];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
            if (lane == 0) rstd_s[wave + 4 * q] = rsqrtf(sum / (float)a.h + a.eps);
        }
        __syncthreads();
    }
    const float rs = SCALED ? rstd_s[r] : 1.f;

    for (int cb = cb_begin + wave; cb < cb_end; cb += 4) {
        Vec8 n0v, n1v;
        fetch(cb + 4, n0v, n1v);
        const int col = column(cb);
        const bool live = col >= 0;
        if (EPI == FEPI_QKV) {
            if (live) {
                int head = cb / bph;
                const int ch = col - head * a.d;              // first-half channel of v0[0]
                const int b = m / (a.k + 1), j = m % (a.k + 1);
                const int base = a.pos_base[b];               // < 0: a rejected sequence, which must not touch the cache
                const int pos = base + j;                     // cache row of node j
#pragma unroll
                for (int e = 0; e < 8; ++e) { v0.v[e] *= rs; v1.v[e] *= rs; }
                if (head < a.nq + a.nkv) {
                    const float *cs = a.rope_cs + ((size_t)a.rope_pos[m] * half + ch) * 2;
                    const Vec8 cs0 = load8(cs), cs1 = load8(cs + 8);   // (cos, sin) of channels ch..ch+3, ch+4..ch+7
                    Vec8 y0, y1;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float co = e < 4 ? cs0.v[2 * e] : cs1.v[2 * (e - 4)], si = e < 4 ? cs0.v[2 * e + 1] : cs1.v[2 * (e - 4) + 1];
                        y0.v[e] = v0.v[e] * co - v1.v[e] * si;
                        y1.v[e] = v0.v[e] * si + v1.v[e] * co;
                    }
                    if (head < a.nq) {
                        const int g = a.nq / a.nkv, kvh = head / g, hl = head % g, rr = j * g + hl;
                        const size_t qs = ((size_t)b * a.nkv + kvh) * a.q_rows_pad * a.d;
                        u32x4 h0, l0, h1, l1;
                        split8(y0, h0, l0);
                        split8(y1, h1, l1);
                        const size_t i_0 = qs + packed_index(rr, ch, a.d >> 5), i_1 = qs + packed_index(rr, ch + half, a.d >> 5);
                        *reinterpret_cast<u32x4 *>(a.Qp + i_0) = h0; *reinterpret_cast<u32x4 *>(a.Qp_lo + i_0) = l0;
                        *reinterpret_cast<u32x4 *>(a.Qp + i_1) = h1; *reinterpret_cast<u32x4 *>(a.Qp_lo + i_1) = l1;
                    } else if (base >= 0) {
                        head -= a.nq;
                        uint16_t *kr = a.Kc + kcache_offset(a.kv, b, head, pos, 0);
                        *reinterpret_cast<u32x4 *>(kr + ch) = round8(y0);
                        *reinterpret_cast<u32x4 *>(kr + ch + half) = round8(y1);
                    }
                } else if (base >= 0) {
                    head -= a.nq + a.nkv;
                    uint16_t *vv = a.Vc + kv_block_offset(a.kv, kv_page(a.kv, b, pos >> 5), head);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        vv[vblock_index(pos & 31, ch + e, a.d)] = f32_to_bf16(v0.v[e]);
                        vv[vblock_index(pos & 31, ch + half + e, a.d)] = f32_to_bf16(v1.v[e]);
                    }
                }
            }
        } else if (EPI == FEPI_SWIGLU) {
            if (live) {
                Vec8 hv;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float gg = v0.v[e] * rs;
                    hv.v[e] = gg / (1.f + __expf(-gg)) * (v1.v[e] * rs);
                }
                u32x4 hi, lo;
                split8(hv, hi, lo);
                const size_t idx = packed_index(m, col, a.KT_out);
                *reinterpret_cast<u32x4 *>(a.out_hi + idx) = hi;
                *reinterpret_cast<u32x4 *>(a.out_lo + idx) = lo;
            }
        } else if (EPI == FEPI_STORE) {
            if (live) store8(a.out + (size_t)m * a.Ntot + col, v0);
        } else if (EPI == FEPI_RESID) {
            resid_block<false>(a, m, col, live, kg, v0);
        } else {  // FEPI_LM
            const int n0 = cb * 32 + kg * 8;
            float bv = -INFINITY;
            int bi = n0;
            if (live) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float logit = v0.v[e] * rs;
                    v0.v[e] = logit;
                    if (logit > bv) { bv = logit; bi = n0 + e; }   // ascending columns: the lowest index keeps a tie
                }
                if (a.logits) store8(a.logits + (size_t)m * a.vocab + n0, v0);
            }
            const float ov = __shfl_xor(bv, 16);
            const int oi = __shfl_xor(bi, 16);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            if (live && !(kg & 1)) {
                a.part_val[(size_t)m * a.NT + (n0 >> 4)] = bv;
                a.part_idx[(size_t)m * a.NT + (n0 >> 4)] = bi;
            }
        }
        v0 = n0v;
        v1 = n1v;
    }
}

template <int EPI> hipError_t launch_epi(const FusedGemmArgs &a, hipStream_t s)
{
    const int n_cu = a.n_cu > 0 ? a.n_cu : 256;
    const int row_tiles = (a.M + 15) / 16;
    const int n_cb = column_blocks<EPI>(a);
    // about 4 workgroups per compute unit, whole groups of four column blocks (one per wave)
    const int groups_x = (4 * n_cu + row_tiles - 1) / row_tiles;
    int bpw = (n_cb + groups_x - 1) / groups_x;
    bpw = (bpw + 3) / 4 * 4;
    hipLaunchKernelGGL((epi_kernel<EPI>), dim3((n_cb + bpw - 1) / bpw, row_tiles), dim3(256), 0, s, a, bpw);
    return hipGetLastError();
}

// ------------------------------------------------------------------- M > 32 ----
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mfma32(const u32x4 &a, const u32x4 &b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Packed weights of concatenated 16-column tile gt for any epilogue: the output is up to three
// matrices side by side, the first two of seg0 and seg1 tiles.
__device__ __forceinline__ const u32x4 *tile_weights_seg(const FusedGemmArgs &a, int gt)
{
    const size_t stride = (size_t)a.KT * 64;
    const u32x4 *base = a.W0;
    if (gt >= a.seg0) {
        gt -= a.seg0;
        base = a.W1;
        if (gt >= a.seg1) {
            gt -= a.seg1;
            base = a.W2;
        }
    }
    return base + gt * stride;
}

constexpr int QNG = 1;   // 32-column tiles per wave
constexpr int QDW = 4;   // weight k-tiles in flight per wave

// A 32 x 16 MFMA operand (rows l%32, k-slots 8*(l/32)..+7) assembled from two packed 16 x 32
// tiles T0 (rows 0..15) and T1 (rows 16..31): for k-half hh of the k-tile, lane l takes lane
// record (l%16) + 16*(l/32 + 2*hh) of tile T[(l/16)%2].  Both operands use the same rule, so the
// k-slots pair up.
__device__ __forceinline__ int half_record(int lane, int hh) { return (lane & 15) + 16 * ((lane >> 5) + 2 * hh); }

// grid = n_groups * J workgroups of QW waves; rows [m_base, m_base + 32*MT32) of the packed
// activations; writes partials[j][row][col].  One 32-column tile per wave, so two or more waves
// share a SIMD and cover each other's LDS and barrier waits; QW = 8 (256 columns per workgroup)
// for the large matrices, QW = 4 for the small ones, whose K then splits half as often (measured:
// 8 waves 15 % faster on gate/up and down at M = 160, 4 waves 10-15 % faster on QKV and O, and on
// every matrix at up to 64 rows).
template <int MT32, int QW>
__global__ __launch_bounds__(QW * 64) void qgemm_kernel(FusedGemmArgs a, int m_base, int NT16)
{
    constexpr int MT16 = 2 * MT32;
    constexpr int CHUNK = MT16 * 2 * 64;          // lane records of one activation k-tile (hi and lo)
    constexpr int APT = (CHUNK + QW * 64 - 1) / (QW * 64);   // records staged per thread
    constexpr bool AFULL = CHUNK % (QW * 64) == 0;
    __shared__ u32x4 ring[2][CHUNK];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int J = a.J, j = blockIdx.x % J, grp = blockIdx.x / J;
    const int KT = a.KT;
    const int kps = a.kps;
    const int kt_begin = j * kps, kt_end = kt_begin + kps < KT ? kt_begin + kps : KT;
    const int n_iter = kt_end - kt_begin;

    // this wave's weight tiles
    const u32x4 *wp[QNG];
    int n32[QNG];
#pragma unroll
    for (int g = 0; g < QNG; ++g) {
        n32[g] = (grp * QW + wave) * QNG + g;
        int t16 = 2 * n32[g] + ((lane >> 4) & 1);
        if (t16 >= NT16) t16 = NT16 - 1;          // columns past the matrix re-read the last tile, never stored
        wp[g] = tile_weights_seg(a, t16);
    }
    const int r0 = half_record(lane, 0), r1 = half_record(lane, 1);

    // activation staging: thread t moves records t, t+256, ... of each k-tile chunk
    const size_t mt_base = (size_t)(m_base >> 4);
    const u32x4 *asrc[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        int q = threadIdx.x + i * QW * 64;
        if (!AFULL && q >= CHUNK) q = CHUNK - 1;  // surplus threads re-read the last record, never stored
        const int tile = q >> 6, rec = q & 63;    // tile = mt16 * 2 + (0: hi, 1: lo)
        const u32x4 *base = (tile & 1) ? a.A_lo : a.A_hi;
        asrc[i] = base + ((mt_base + (tile >> 1)) * KT) * 64 + rec;
    }
    auto stage_load = [&](int kt, u32x4 (&v)[APT]) {
#pragma unroll
        for (int i = 0; i < APT; ++i) v[i] = asrc[i][(size_t)kt * 64];
    };
    auto stage_store = [&](int buf, const u32x4 (&v)[APT]) {
#pragma unroll
        for (int i = 0; i < APT; ++i)
            if (AFULL || threadIdx.x + i * QW * 64 < CHUNK) ring[buf][threadIdx.x + i * QW * 64] = v[i];
    };

    f32x16 acc[MT32][QNG];
#pragma unroll
    for (int i = 0; i < MT32; ++i)
#pragma unroll
        for (int g = 0; g < QNG; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.f;

    // All loads of a wave retire in issue order, so the activation loads (L2 hits) are issued
    // QDW k-tiles ahead, each right before the weight loads of the same k-tile, and parked in
    // registers: by the time chunk c moves to LDS (iteration c-1) everything issued before it has
    // been consumed already, and waiting for it never waits for a weight load still in flight.
    u32x4 w[QDW][QNG][2], apre[QDW][APT];
    auto issue = [&](int u, int it) {   // activation chunk and weights of iteration `it` into slot u
        const int kt = kt_begin + (it < n_iter ? it : n_iter - 1);
        stage_load(kt, apre[u]);
#pragma unroll
        for (int g = 0; g < QNG; ++g) {
            w[u][g][0] = __builtin_nontemporal_load(wp[g] + (size_t)kt * 64 + r0);
            w[u][g][1] = __builtin_nontemporal_load(wp[g] + (size_t)kt * 64 + r1);
        }
    };
#pragma unroll
    for (int u = 0; u < QDW; ++u) issue(u, u);
    stage_store(0, apre[0]);
    __syncthreads();

    // One k-tile: MFMAs on LDS slot it&1 with weight slot u, refill both register slots for
    // iteration it+QDW, move chunk it+1 to the other LDS slot.  The steady-state loop below runs it
    // with every branch resolved at compile time: a load that is only conditionally issued would
    // force the wait counters in front of every later use down to "nothing outstanding".
    auto ktile = [&](int u, int it, bool refill, bool next_chunk) {
        const u32x4 *buf = ring[it & 1];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int rec = hh ? r1 : r0;
#pragma unroll
            for (int i = 0; i < MT32; ++i) {
                // tile index in the chunk: (mt16 * 2 + hi/lo) with mt16 = 2i + (lane/16)%2
                const int t_hi = ((2 * i + ((lane >> 4) & 1)) * 2) * 64 + rec;
                const u32x4 xh = buf[t_hi], xl = buf[t_hi + 64];
#pragma unroll
                for (int g = 0; g < QNG; ++g) {
                    acc[i][g] = mfma32(xh, w[u][g][hh], acc[i][g]);
                    acc[i][g] = mfma32(xl, w[u][g][hh], acc[i][g]);
                }
            }
        }
        if (refill) issue(u, it + QDW);
        // LDS slot (it+1)&1 held chunk it-1, which every wave finished before the barrier that
        // ended iteration it-1.
        if (next_chunk) stage_store((it + 1) & 1, apre[(u + 1) % QDW]);
        __syncthreads();
    };
    int it0 = 0;
    for (; it0 + 2 * QDW <= n_iter; it0 += QDW) {   // every iteration of the group refills
#pragma unroll
        for (int u = 0; u < QDW; ++u) ktile(u, it0 + u, true, true);
    }
    for (; it0 < n_iter; it0 += QDW) {              // the last groups drain the pipeline
#pragma unroll
        for (int u = 0; u < QDW; ++u) {
            const int it = it0 + u;
            if (it < n_iter) ktile(u, it, it + QDW < n_iter, it + 1 < n_iter);
        }
    }

    // acc[i][g][v] of lane l: row 32i + 8*(v/4) + 4*(l/32) + v%4, column 32*n32[g] + l%32
#pragma unroll
    for (int g = 0; g < QNG; ++g) {
        const int col = n32[g] * 32 + (lane & 31);
        if (col >= a.Ntot) continue;
#pragma unroll
        for (int i = 0; i < MT32; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m_base + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.part_rows) a.partials[((size_t)j * a.part_rows + row) * a.Ntot + col] = acc[i][g][v];
            }
    }
}

// The same launch with v_mfma_f32_16x16x32_bf16 on MT16 row tiles of 16: the form used from 49 rows up.  An
// odd number of 16-row tiles spends no MFMA on a half-empty 32-row tile (144 rows: 36 instead of 40 units of MFMA
// time per k-tile and wave, 18 instead of 20 operand reads from LDS, nine instead of ten tiles staged), and both
// operands are the packed tiles as stored -- lane l holds (row or column l%16, k-slots 8*(l/16)..+7) of a 16 x 32
// tile -- so a wave's weight loads are two whole 1 KiB records per k-tile.  Staging, prefetch distance and the K
// split are those of qgemm_kernel.  Measured against it, whole steps in one session (ms): 8B shape 80 rows
// 6.20 -> 5.93, 112 rows 6.93 -> 6.72, 144 rows 8.02 -> 7.80, 64 / 96 / 128 / 160 rows 0-1.5 % ahead; 70B shape
// (16 layers) 80 rows 7.67 -> 7.03, 144 rows 10.79 -> 10.28, 64 / 160 rows 3 % ahead; at 36 rows the 32 x 32 form
// stays 4 % ahead on the 8B shape (same on the 70B shape at 48), so up to 48 rows keep it.
template <int MT16, int QW>
__global__ __launch_bounds__(QW * 64) void qgemm16_kernel(FusedGemmArgs a, int m_base, int NT16)
{
    constexpr int QDW = 4;
    constexpr int CHUNK = MT16 * 2 * 64;          // lane records of one activation k-tile (hi and lo)
    constexpr int APT = (CHUNK + QW * 64 - 1) / (QW * 64);
    constexpr bool AFULL = CHUNK % (QW * 64) == 0;
    __shared__ u32x4 ring[2][CHUNK];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int J = a.J, j = blockIdx.x % J, grp = blockIdx.x / J;
    const int KT = a.KT;
    const int kps = a.kps;
    const int kt_begin = j * kps, kt_end = kt_begin + kps < KT ? kt_begin + kps : KT;
    const int n_iter = kt_end - kt_begin;

    const int n32 = grp * QW + wave;
    const u32x4 *wp[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        int t16 = 2 * n32 + ct;
        if (t16 >= NT16) t16 = NT16 - 1;          // columns past the matrix re-read the last tile, never stored
        wp[ct] = tile_weights_seg(a, t16) + lane;
    }

    const size_t mt_base = (size_t)(m_base >> 4);
    const u32x4 *asrc[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        int q = threadIdx.x + i * QW * 64;
        if (!AFULL && q >= CHUNK) q = CHUNK - 1;  // surplus threads re-read the last record, never stored
        const int tile = q >> 6, rec = q & 63;    // tile = mt16 * 2 + (0: hi, 1: lo)
        const u32x4 *base = (tile & 1) ? a.A_lo : a.A_hi;
        asrc[i] = base + ((mt_base + (tile >> 1)) * KT) * 64 + rec;
    }
    auto stage_load = [&](int kt, u32x4 (&v)[APT]) {
#pragma unroll
        for (int i = 0; i < APT; ++i) v[i] = asrc[i][(size_t)kt * 64];
    };
    auto stage_store = [&](int buf, const u32x4 (&v)[APT]) {
#pragma unroll
        for (int i = 0; i < APT; ++i)
            if (AFULL || threadIdx.x + i * QW * 64 < CHUNK) ring[buf][threadIdx.x + i * QW * 64] = v[i];
    };

    f32x4 acc[MT16][2];
#pragma unroll
    for (int i = 0; i < MT16; ++i)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) acc[i][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 w[QDW][2], apre[QDW][APT];
    auto issue = [&](int u, int it) {   // activation chunk and weights of iteration `it` into slot u
        const int kt = kt_begin + (it < n_iter ? it : n_iter - 1);
        stage_load(kt, apre[u]);
        w[u][0] = __builtin_nontemporal_load(wp[0] + (size_t)kt * 64);
        w[u][1] = __builtin_nontemporal_load(wp[1] + (size_t)kt * 64);
    };
#pragma unroll
    for (int u = 0; u < QDW; ++u) issue(u, u);
    stage_store(0, apre[0]);
    __syncthreads();

    auto ktile = [&](int u, int it, bool refill, bool next_chunk) {
        const u32x4 *buf = ring[it & 1] + lane;
#pragma unroll
        for (int i = 0; i < MT16; ++i) {
            const u32x4 xh = buf[(2 * i) * 64], xl = buf[(2 * i + 1) * 64];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                acc[i][ct] = mfma(xh, w[u][ct], acc[i][ct]);
                acc[i][ct] = mfma(xl, w[u][ct], acc[i][ct]);
            }
        }
        if (refill) issue(u, it + QDW);
        if (next_chunk) stage_store((it + 1) & 1, apre[(u + 1) % QDW]);
        __syncthreads();
    };
    int it0 = 0;
    for (; it0 + 2 * QDW <= n_iter; it0 += QDW) {
#pragma unroll
        for (int u = 0; u < QDW; ++u) ktile(u, it0 + u, true, true);
    }
    for (; it0 < n_iter; it0 += QDW) {
#pragma unroll
        for (int u = 0; u < QDW; ++u) {
            const int it = it0 + u;
            if (it < n_iter) ktile(u, it, it + QDW < n_iter, it + 1 < n_iter);
        }
    }

    // acc[i][ct][v] of lane l: row 16i + 4*(l/16) + v, column 32*n32 + 16*ct + l%16
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        const int col = n32 * 32 + ct * 16 + (lane & 15);
        if (col >= a.Ntot) continue;
#pragma unroll
        for (int i = 0; i < MT16; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m_base + 16 * i + 4 * (lane >> 4) + v;
                if (row < a.part_rows) a.partials[((size_t)j * a.part_rows + row) * a.Ntot + col] = acc[i][ct][v];
            }
    }
}

struct QPlan {
    int groups, J, kps;   // column groups, K slices (none empty), k-tiles per slice
    int qw;               // waves (32-column tiles) per workgroup
};

// Column groups and the K split.  The split is the smallest J whose groups*J workgroups fill whole
// rounds of one workgroup per compute unit to at least 85 % (else the best-filling one), with at least
// 8 k-tiles per slice and at most 16 slices.  More slices than that would still find room on the device at
// up to 96 rows (two workgroups fit a compute unit there), but every slice is another fp32 copy of the
// output to write and read back: measured on the 70B shapes at 80 rows, filling 256 slots instead of 512
// took QKV from 52 to 43 us, down from 113 to 91 us, O from 46 to 41 us.
__host__ QPlan q_plan(int Ntot, int K, int M)
{
    const int NT32 = (Ntot / 16 + 1) / 2, KT = (K + 31) / 32;
    const int mt32 = M >= 160 ? 5 : (M + 31) / 32;
    const size_t bytes = (size_t)Ntot * (size_t)K * 2;
    QPlan p;
    // Four waves (128 columns per workgroup, K split half as often): the small matrices, and every matrix but
    // the very large ones at up to 64 rows (measured at 36 and 64 rows on the 8B shapes: gate/up 59 -> 48 and
    // 64 -> 51 us, down 34 -> 32 and 37 -> 33 us; from 65 rows on eight waves win on the large matrices, and
    // on the 940 MB gate/up matrix of the 70B shape they win at 48 rows already: 189 -> 153 us without a split).
    p.qw = (bytes < ((size_t)64 << 20) || (mt32 <= 2 && bytes < ((size_t)512 << 20))) ? 4 : 8;
    const int slots = 256;
    p.groups = (NT32 + p.qw * QNG - 1) / (p.qw * QNG);
    int jmax = KT / 8;
    if (jmax > 16) jmax = 16;
    if (jmax < 1) jmax = 1;
    int best = 1;
    double best_fill = 0.0;
    for (int J = 1; J <= jmax; ++J) {
        const long tasks = (long)p.groups * J;
        const long rounds = (tasks + slots - 1) / slots;
        const double fill = (double)tasks / (double)(rounds * slots);
        if (fill > best_fill + 1e-9) { best_fill = fill; best = J; }
        if (fill >= 0.85) { best = J; break; }
    }
    p.kps = (KT + best - 1) / best;
    p.J = (KT + p.kps - 1) / p.kps;
    return p;
}

template <int EPI> hipError_t launch_large(FusedGemmArgs &a, hipStream_t s, bool *needs_epilogue, hipEvent_t t0, hipEvent_t t1)
{
    *needs_epilogue = true;
    const int NT16 = a.Ntot / 16;
    const QPlan p = q_plan(a.Ntot, a.KT * 32, a.M);
    a.J = p.J;
    a.kps = p.kps;
    a.part_rows = round_up(a.M, 16);
    if (EPI == FEPI_QKV) { a.seg0 = a.nq * (a.d >> 4); a.seg1 = a.nkv * (a.d >> 4); }
    else if (EPI == FEPI_SWIGLU) { a.seg0 = a.NT; a.seg1 = a.NT; }
    else { a.seg0 = NT16; a.seg1 = 0; }
    if ((size_t)a.J * a.part_rows * a.Ntot * sizeof(float) > a.partial_bytes) return hipErrorInvalidValue;
    const dim3 grid(p.groups * a.J), block(p.qw * 64);
    for (int m_base = 0; m_base < a.M; m_base += 160) {
        const int mt32 = (a.M - m_base + 31) / 32;
        const int mt16 = (a.M - m_base + 15) / 16;
        hipEvent_t e0 = m_base == 0 ? t0 : nullptr, e1 = m_base + 160 >= a.M ? t1 : nullptr;   // first pass starts, last pass stops
        if (mt16 >= 4) {   // 49 rows and more: the 16 x 16 x 32 form (measured ahead at every tile count from 4 up)
#define SSSD_Q16LAUNCH(MT)                                                                                      \
    do {                                                                                                        \
        if (p.qw == 8) hipExtLaunchKernelGGL((qgemm16_kernel<MT, 8>), grid, block, 0, s, e0, e1, 0, a, m_base, NT16); \
        else hipExtLaunchKernelGGL((qgemm16_kernel<MT, 4>), grid, block, 0, s, e0, e1, 0, a, m_base, NT16);     \
    } while (0)
            switch (mt16) {
            case 4: SSSD_Q16LAUNCH(4); break;
            case 5: SSSD_Q16LAUNCH(5); break;
            case 6: SSSD_Q16LAUNCH(6); break;
            case 7: SSSD_Q16LAUNCH(7); break;
            case 8: SSSD_Q16LAUNCH(8); break;
            case 9: SSSD_Q16LAUNCH(9); break;
            default: SSSD_Q16LAUNCH(10); break;
            }
#undef SSSD_Q16LAUNCH
            hipError_t e16 = hipGetLastError();
            if (e16 != hipSuccess) return e16;
            continue;
        }
#define SSSD_QLAUNCH(MT)                                                                                        \
    do {                                                                                                        \
        if (p.qw == 8) hipExtLaunchKernelGGL((qgemm_kernel<MT, 8>), grid, block, 0, s, e0, e1, 0, a, m_base, NT16); \
        else hipExtLaunchKernelGGL((qgemm_kernel<MT, 4>), grid, block, 0, s, e0, e1, 0, a, m_base, NT16);       \
    } while (0)
        if (mt32 == 1) SSSD_QLAUNCH(1);   // the rows left over by a pass of 160
        else SSSD_QLAUNCH(2);             // 33..48 rows
#undef SSSD_QLAUNCH
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// k-tiles per wave: 7 when K is a multiple of 16*7*32 but not of 16*8*32 (the FFN widths of the
// Llama shapes), else 8.  A ragged K split is legal in every case.
__host__ int small_kpw(int KT) { return (KT % (PW * 7) == 0 && KT % (PW * 8) != 0) ? 7 : 8; }

struct SmallPlan {
    int rh, kpw, J, upw, groups;
};

__host__ SmallPlan small_plan(const FusedGemmArgs &a)
{
    SmallPlan p;
    p.rh = a.M > 16 ? 2 : 1;   // 17..32 rows: every workgroup twice, one per row tile
    p.kpw = small_kpw(a.KT);
    p.J = (a.KT + PW * p.kpw - 1) / (PW * p.kpw);
    const int n_cu = (a.n_cu > 0 ? a.n_cu : 256) / p.rh;
    int groups_target = n_cu / p.J;
    if (groups_target < 1) groups_target = 1;
    p.upw = (a.n_units + groups_target - 1) / groups_target;
    p.groups = (a.n_units + p.upw - 1) / p.upw;
    return p;
}

template <int EPI> hipError_t launch_small(FusedGemmArgs &a, hipStream_t s, bool *needs_epilogue, hipEvent_t t0, hipEvent_t t1)
{
    const SmallPlan sp = small_plan(a);
    const int kpw = sp.kpw, groups = sp.groups;
    a.J = sp.J;
    a.upw = sp.upw;
    a.groups = sp.groups;
    a.part_rows = 16 * sp.rh;
    if (a.J > 1 && (size_t)a.J * a.part_rows * a.Ntot * sizeof(float) > a.partial_bytes) return hipErrorInvalidValue;
    const dim3 grid(groups * a.J * sp.rh), block(PW * 64);
    if (groups * sp.rh > a.tail_slots) a.tail_count = nullptr;   // no counter for every group: epilogue launch
#define SSSD_PLAUNCH(KPW, RH)                                                                                   \
    do {                                                                                                        \
        if (a.J > 1) hipExtLaunchKernelGGL((pgemm_kernel<EPI, KPW, true, RH>), grid, block, 0, s, t0, t1, 0, a); \
        else hipExtLaunchKernelGGL((pgemm_kernel<EPI, KPW, false, RH>), grid, block, 0, s, t0, t1, 0, a);       \
    } while (0)
    if (sp.rh == 2 && kpw == 7) SSSD_PLAUNCH(7, 2);
    else if (sp.rh == 2) SSSD_PLAUNCH(8, 2);
    else if (kpw == 7) SSSD_PLAUNCH(7, 1);
    else SSSD_PLAUNCH(8, 1);
#undef SSSD_PLAUNCH
    *needs_epilogue = a.J > 1 && !a.tail_count;
    return hipGetLastError();
}

}  // namespace

int stream_gemm_max_rows() { return 32; }

const char *stream_gemm_kernel_name(int M)
{
    if (M <= stream_gemm_max_rows()) return "pgemm_kernel";
    return (M < 160 ? M : 160) > 48 ? "qgemm16_kernel" : "qgemm_kernel";
}

// Split-K scratch needed for M rows: the largest J * rows * Ntot over the model's GEMMs.
size_t stream_gemm_partial_bytes(const Dims &D, int M)
{
    size_t best = 0;
    const size_t rows_small = M > 16 ? 32 : 16;
    auto consider = [&](int K, size_t ntot) {
        const int KT = (K + 31) / 32, ks = PW * small_kpw(KT);
        const size_t need = (size_t)((KT + ks - 1) / ks) * rows_small * ntot;
        if (need > rows_small * ntot && need > best) best = need;   // only a split K needs scratch
    };
    consider(D.h, (size_t)D.qd + 2 * D.kd);
    consider(D.qd, D.h);
    consider(D.h, 2 * (size_t)D.f);
    consider(D.f, D.h);
    consider(D.h, D.V);
    // larger steps: the K split depends on the row count's class (32-row tiles), so take the worst
    // case over every step size up to M
    for (int mc = 32; M > stream_gemm_max_rows(); mc += 32) {
        const int rows_c = mc < M ? mc : M;
        const size_t rows = (size_t)round_up(rows_c, 16);
        auto large = [&](int K, size_t ntot) {
            const size_t need = (size_t)q_plan((int)ntot, K, rows_c).J * rows * ntot;
            if (need > best) best = need;
        };
        large(D.h, (size_t)D.qd + 2 * D.kd);
        large(D.qd, D.h);
        large(D.h, 2 * (size_t)D.f);
        large(D.f, D.h);
        large(D.h, D.V);
        if (mc >= M) break;
    }
    return best * sizeof(float);
}

size_t stream_gemm_scratch_bytes(int M, int N, int K)
{
    const int KT = (K + 31) / 32;
    if (M > stream_gemm_max_rows()) return (size_t)q_plan(N, K, M).J * round_up(M, 16) * N * sizeof(float);
    const int ks = PW * small_kpw(KT);
    const size_t j = (size_t)((KT + ks - 1) / ks);
    return j > 1 ? j * (M <= 16 ? 16 : 32) * N * sizeof(float) : 0;
}

hipError_t launch_stream_gemm(FusedGemmArgs &a, int epilogue, hipStream_t s, bool *needs_epilogue, hipEvent_t t0,
                              hipEvent_t t1)
{
    if (a.M > stream_gemm_max_rows()) {
        switch (epilogue) {
        case FEPI_QKV: return launch_large<FEPI_QKV>(a, s, needs_epilogue, t0, t1);
        case FEPI_RESID: return launch_large<FEPI_RESID>(a, s, needs_epilogue, t0, t1);
        case FEPI_SWIGLU: return launch_large<FEPI_SWIGLU>(a, s, needs_epilogue, t0, t1);
        case FEPI_STORE: return launch_large<FEPI_STORE>(a, s, needs_epilogue, t0, t1);
        default: return launch_large<FEPI_LM>(a, s, needs_epilogue, t0, t1);
        }
    }
    switch (epilogue) {
    case FEPI_QKV: return launch_small<FEPI_QKV>(a, s, needs_epilogue, t0, t1);
    case FEPI_RESID: return launch_small<FEPI_RESID>(a, s, needs_epilogue, t0, t1);
    case FEPI_SWIGLU: return launch_small<FEPI_SWIGLU>(a, s, needs_epilogue, t0, t1);
    case FEPI_STORE: return launch_small<FEPI_STORE>(a, s, needs_epilogue, t0, t1);
    default: return launch_small<FEPI_LM>(a, s, needs_epilogue, t0, t1);
    }
}

hipError_t launch_stream_epilogue(const FusedGemmArgs &a, int epilogue, hipStream_t s)
{
    switch (epilogue) {
    case FEPI_QKV: return launch_epi<FEPI_QKV>(a, s);
    case FEPI_RESID: return launch_epi<FEPI_RESID>(a, s);
    case FEPI_SWIGLU: return launch_epi<FEPI_SWIGLU>(a, s);
    case FEPI_STORE: return launch_epi<FEPI_STORE>(a, s);
    default: return launch_epi<FEPI_LM>(a, s);
    }
}
