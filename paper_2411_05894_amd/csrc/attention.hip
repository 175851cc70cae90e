// Causal grouped-query attention of the k+1 new rows against the per-sequence KV cache.
//
// Table 2 (App. B), attention row: A_out = softmax(Q K^T / sqrt(d) + M) V with
// K, V of shape (b, n_kv, s_kv + s_q, d).  Its FLOPs:IO ratio is ~ g*s_q, so the
// operation is bound by streaming the cache; the mask M of a linear draft chain
// is "row j sees positions 0 .. lens[b]+j" and is applied arithmetically (no mask
// tensor is read).
//
// One wavefront owns one (sequence, kv head, position chunk): all g*(k+1) query
// rows that share the kv head ride in the MFMA column dimension, so every cached
// byte is read once per step.  Per block of 32 positions:
//   S^T = K . Q^T        (A operand = 16 cached K rows straight from memory)
//   online softmax in registers; the row statistics need only two cross-lane xors
//   O^T += V^T . P^T     (A operand = V in its block-transposed cache order,
//                         B operand = the lane's own probabilities)
// The transposed forms are chosen so that the lane that owns a query row's
// statistics also owns that row's accumulator columns: no shuffles to rescale.
// Chunks are merged by a second kernel in fixed order (deterministic).
#include "kernels.h"

namespace {

__device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr float NEG_BIG = -1.0e30f;

template <int HD, int RT>
__global__ __launch_bounds__(64) void attn_partial_kernel(Dims D, AttnArgs a, int q_rows_pad, int rt_base)
{
    constexpr int KS = HD / 32, DT = HD / 16;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int q = lane >> 4, c = lane & 15;
    const int len = a.pos_base[b];
    const int total = len + a.k + 1;
    const int t_begin = split * D.chunk;
    if (t_begin >= total) return;
    const int t_end = min(total, t_begin + D.chunk);

    const size_t slab = ((size_t)b * D.nkv + kvh) * D.seq_pad * HD;
    const uint16_t *Kc = a.Kc + slab;
    const u32x4 *Vc = reinterpret_cast<const u32x4 *>(a.Vc + slab);
    const u32x4 *Qs = reinterpret_cast<const u32x4 *>(a.Qp + ((size_t)b * D.nkv + kvh) * q_rows_pad * HD);
    const u32x4 *Ql = reinterpret_cast<const u32x4 *>(a.Qp_lo + ((size_t)b * D.nkv + kvh) * q_rows_pad * HD);

    // q ~= hi + lo (two bf16), so the scores carry fp32-level accuracy although K is bf16.
    u32x4 qreg[RT][KS], qlo[RT][KS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qreg[rt][ks] = Qs[((size_t)(rt_base + rt) * KS + ks) * 64 + lane];
            qlo[rt][ks] = Ql[((size_t)(rt_base + rt) * KS + ks) * 64 + lane];
        }

    f32x4 o[RT][DT];
    float m_run[RT], l_run[RT];
    int limit[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = NEG_BIG;
        l_run[rt] = 0.f;
        int j = ((rt_base + rt) * 16 + c) / D.g;   // query row -> draft index
        if (j > a.k) j = a.k;
        limit[rt] = len + j;                        // last visible position
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[rt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale = 1.4426950408889634f * rsqrtf((float)HD);  // log2(e)/sqrt(d)

    for (int t0 = t_begin; t0 < t_end; t0 += 32) {
        u32x4 kreg[2][KS];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kreg[u][ks] = *reinterpret_cast<const u32x4 *>(Kc + (size_t)(t0 + 16 * u + c) * HD + ks * 32 + 8 * q);
        u32x4 vreg[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vreg[dt] = Vc[((size_t)(t0 >> 5) * DT + dt) * 64 + lane];

        u32x4 pb[RT], pl[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            f32x4 s[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[u] = mfma(kreg[u][ks], qreg[rt][ks], s[u]);
                    s[u] = mfma(kreg[u][ks], qlo[rt][ks], s[u]);
                }
            }
            // s[u][r] is the score of position t0 + 16u + 4q + r for query row rt*16 + c.
            float v[8];
            float mx = NEG_BIG;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = t0 + 16 * u + 4 * q + r;
                    float x = s[u][r] * scale;
                    if (t > limit[rt]) x = NEG_BIG;
                    v[u * 4 + r] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[rt], mx);
            const float alpha = exp2f(m_run[rt] - m_new);
            m_run[rt] = m_new;
            float psum = 0.f;
            uint32_t pk[4], pkl[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float p0 = exp2f(v[e] - m_new), p1 = exp2f(v[e + 1] - m_new);
                uint16_t h0, l0, h1, l1;   // p ~= hi + lo: the probabilities keep ~16 mantissa bits
                split_bf16(p0, h0, l0);
                split_bf16(p1, h1, l1);
                psum += p0 + p1;
                pk[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                pkl[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            l_run[rt] = l_run[rt] * alpha + psum;
            pb[rt] = u32x4{pk[0], pk[1], pk[2], pk[3]};
            pl[rt] = u32x4{pkl[0], pkl[1], pkl[2], pkl[3]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[rt][dt] *= alpha;
            }
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                o[rt][dt] = mfma(vreg[dt], pb[rt], o[rt][dt]);
                o[rt][dt] = mfma(vreg[dt], pl[rt], o[rt][dt]);
            }
    }

    // o[rt][dt][r] of lane (q, c): channel dt*16 + 4q + r of query row rt*16 + c.
    const size_t slot = ((size_t)b * D.nkv + kvh) * D.max_splits + split;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float l = l_run[rt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const size_t row = slot * q_rows_pad + (size_t)(rt_base + rt) * 16 + c;
        float *po = a.part_o + row * HD;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4 *>(po + dt * 16 + 4 * q) = o[rt][dt];
        if (q == 0) {
            a.part_ml[row * 2] = m_run[rt];
            a.part_ml[row * 2 + 1] = l;
        }
    }
}

// One wave per (sequence, kv head, query row); 4 waves per block.  Lanes first work across
// chunks (weights), then across channels (values, eight chunks' loads in flight at a time).
__global__ __launch_bounds__(256) void attn_combine_kernel(Dims D, AttnArgs a, int q_rows_pad)
{
    const int lane = threadIdx.x & 63, k = a.k;
    const int R = D.g * (k + 1);
    const int n_tasks = a.B * D.nkv * R;
    const int task = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (task >= n_tasks) return;
    const int KTq = (D.qd + 31) >> 5;
    const int ch = lane * 2;  // head_dim 128: two channels per lane; head_dim 64: lanes 0..31
    const int r = task % R, kvh = (task / R) % D.nkv, b = task / (R * D.nkv);
    const int total = a.pos_base[b] + k + 1;
    const int n_splits = (total + D.chunk - 1) / D.chunk;
    const size_t slot0 = ((size_t)b * D.nkv + kvh) * D.max_splits;
    float m_star = NEG_BIG;
    for (int s = lane; s < n_splits; s += 64) m_star = fmaxf(m_star, a.part_ml[((slot0 + s) * q_rows_pad + r) * 2]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m_star = fmaxf(m_star, __shfl_xor(m_star, off));
    float den = 0.f, num0 = 0.f, num1 = 0.f;
    for (int base = 0; base < n_splits; base += 64) {
        const int s_mine = base + lane;
        float w_lane = 0.f;
        if (s_mine < n_splits) {
            const float2 ml = *reinterpret_cast<const float2 *>(a.part_ml + ((slot0 + s_mine) * q_rows_pad + r) * 2);
            w_lane = exp2f(ml.x - m_star);
            den += w_lane * ml.y;
        }
        const int n_here = n_splits - base < 64 ? n_splits - base : 64;
        for (int s0 = 0; s0 < n_here; s0 += 8) {
            float2 pv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const size_t row = (slot0 + base + s0 + u) * q_rows_pad + r;
                pv[u] = (s0 + u < n_here && ch < D.d) ? *reinterpret_cast<const float2 *>(a.part_o + row * D.d + ch) : float2{0.f, 0.f};
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
        a.out_hi[idx] = h0; a.out_hi[idx + 1] = h1;
        a.out_lo[idx] = l0; a.out_lo[idx + 1] = l1;
    }
}

template <int HD> hipError_t launch_partial(const Dims &D, const AttnArgs &a, int q_rows_pad, hipStream_t s)
{
    const int rows = D.g * (a.k + 1);
    const int rt_total = (rows + 15) / 16;
    const dim3 grid(D.max_splits, D.nkv, a.B);
    // Up to 3 query-row tiles per wave; more rows take further passes over the cache.
    for (int rt0 = 0; rt0 < rt_total; rt0 += 3) {
        const int rt = rt_total - rt0 < 3 ? rt_total - rt0 : 3;
        switch (rt) {
        case 1: hipLaunchKernelGGL((attn_partial_kernel<HD, 1>), grid, dim3(64), 0, s, D, a, q_rows_pad, rt0); break;
        case 2: hipLaunchKernelGGL((attn_partial_kernel<HD, 2>), grid, dim3(64), 0, s, D, a, q_rows_pad, rt0); break;
        default: hipLaunchKernelGGL((attn_partial_kernel<HD, 3>), grid, dim3(64), 0, s, D, a, q_rows_pad, rt0); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_attention(const Dims &D, const AttnArgs &a, hipStream_t s)
{
    const int q_rows_pad = round_up(D.g * (D.max_k + 1), 16);
    hipError_t e = D.d == 128 ? launch_partial<128>(D, a, q_rows_pad, s) : launch_partial<64>(D, a, q_rows_pad, s);
    if (e != hipSuccess) return e;
    const int n_tasks = a.B * D.nkv * D.g * (a.k + 1);
    hipLaunchKernelGGL(attn_combine_kernel, dim3((n_tasks + 3) / 4), dim3(256), 0, s, D, a, q_rows_pad);
    return hipGetLastError();
}
