// Device helpers of the weight-streaming GEMM kernels (stream_gemm.hip): MFMA wrapper, tile addressing
// of the concatenated outputs, device-scope accesses, the fused epilogues and the split-K slice sums.
#pragma once
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

// Device-scope accesses (COH) for data that a workgroup of the SAME launch on another die wrote or
// will read: stores go through to memory, loads do not take a line this die cached earlier.  Plain
// accesses are enough across launches.
template <bool COH, typename T> __device__ __forceinline__ void st(T *p, T v)
{
    if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}

template <bool COH, typename T> __device__ __forceinline__ T ld(const T *p)
{
    if (COH) return __hip_atomic_load(const_cast<T *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

// One output element pair of a unit: row m, column c of the 16-column tile(s).  v0/v1 are the
// fp32 results of the unit's first/second tile.  The 16 lanes c = 0..15 of a row are adjacent
// lanes of one wave (RESID and LM reduce over them).
template <int EPI, bool COH = false>
__device__ __forceinline__ void epilogue(const FusedGemmArgs &a, int unit, int m, int c, bool valid, float v0, float v1, float rs)
{
    if (EPI == FEPI_STORE) {
        if (valid) a.out[(size_t)m * a.Ntot + unit * 16 + c] = v0;
    } else if (EPI == FEPI_RESID) {
        const int n = unit * 16 + c;
        float xn = 0.f;
        if (valid) {
            xn = ld<COH>(a.X + (size_t)m * a.h + n) + v0;
            st<COH>(a.X + (size_t)m * a.h + n, xn);
            uint16_t hi, lo;
            split_bf16(xn * bf16_to_f32(a.gamma_next[n]), hi, lo);
            const size_t idx = packed_index(m, n, (a.h + 31) >> 5);
            st<COH>(a.out_hi + idx, hi);
            st<COH>(a.out_lo + idx, lo);
        }
        float ss = xn * xn;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 16);
        if (valid && c == 0) st<COH>(a.ssq_out + (size_t)m * (a.h >> 4) + unit, ss);
    } else if (EPI == FEPI_QKV) {
        if (!valid) return;
        const int TH = a.d >> 4, per_head = TH >> 1;
        int head = unit / per_head;
        const int pair = unit % per_head;
        v0 *= rs;
        v1 *= rs;
        const int b = m / (a.k + 1), j = m % (a.k + 1);
        const int base = a.pos_base[b];                 // < 0: a rejected sequence, which must not touch the cache
        const int pos = base + j;                       // cache row of node j
        const int half = a.d >> 1, ch = pair * 16 + c;  // channel of v0; v1 is ch + half
        if (head < a.nq + a.nkv) {
            const float2 cs = *reinterpret_cast<const float2 *>(a.rope_cs + ((size_t)a.rope_pos[m] * half + ch) * 2);
            const float y0 = v0 * cs.x - v1 * cs.y, y1 = v0 * cs.y + v1 * cs.x;
            if (head < a.nq) {
                const int g = a.nq / a.nkv, kvh = head / g, hl = head % g, rr = j * g + hl;
                const size_t qs = ((size_t)b * a.nkv + kvh) * a.q_rows_pad * a.d;
                uint16_t h0, l0, h1, l1;
                split_bf16(y0, h0, l0);
                split_bf16(y1, h1, l1);
                const size_t i_0 = qs + packed_index(rr, ch, a.d >> 5), i_1 = qs + packed_index(rr, ch + half, a.d >> 5);
                st<COH>(a.Qp + i_0, h0); st<COH>(a.Qp_lo + i_0, l0);
                st<COH>(a.Qp + i_1, h1); st<COH>(a.Qp_lo + i_1, l1);
            } else if (base >= 0) {
                head -= a.nq;
                uint16_t *kr = a.Kc + kcache_offset(a.kv, b, head, pos, 0);
                st<COH>(kr + ch, f32_to_bf16(y0));
                st<COH>(kr + ch + half, f32_to_bf16(y1));
            }
        } else if (base >= 0) {
            head -= a.nq + a.nkv;
            uint16_t *vv = a.Vc + kv_block_offset(a.kv, kv_page(a.kv, b, pos >> 5), head);
            st<COH>(vv + vblock_index(pos & 31, ch, a.d), f32_to_bf16(v0));
            st<COH>(vv + vblock_index(pos & 31, ch + half, a.d), f32_to_bf16(v1));
        }
    } else if (EPI == FEPI_SWIGLU) {
        if (!valid) return;
        const float gt = v0 * rs, up = v1 * rs;
        const float hval = gt / (1.f + __expf(-gt)) * up;
        uint16_t hi, lo;
        split_bf16(hval, hi, lo);
        const size_t idx = packed_index(m, unit * 16 + c, a.KT_out);
        st<COH>(a.out_hi + idx, hi);
        st<COH>(a.out_lo + idx, lo);
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
template <bool COH = false> __device__ __forceinline__ float row_rstd(const FusedGemmArgs &a, int m, int lane)
{
    const int NSS = a.h >> 4;
    float sum = 0.f;
    if (m < a.M)
        for (int t = lane; t < NSS; t += 64) sum += ld<COH>(a.ssq_in + (size_t)m * NSS + t);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    return rsqrtf(sum / (float)a.h + a.eps);
}

// ---- eight columns per thread ----
struct Vec8 {
    float v[8];
};

template <bool COH = false> __device__ __forceinline__ Vec8 load8(const float *p)
{
    if (COH) {   // device-scope: four 8-byte loads
        Vec8 r;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned long long u = ld<true>(reinterpret_cast<const unsigned long long *>(p) + q);
            r.v[2 * q] = __uint_as_float((uint32_t)u);
            r.v[2 * q + 1] = __uint_as_float((uint32_t)(u >> 32));
        }
        return r;
    }
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
    return Vec8{{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]}};
}

template <bool COH = false> __device__ __forceinline__ void store8(float *p, const Vec8 &x)
{
    if (COH) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            st<true>(reinterpret_cast<unsigned long long *>(p) + q,
                     (unsigned long long)__float_as_uint(x.v[2 * q]) | ((unsigned long long)__float_as_uint(x.v[2 * q + 1]) << 32));
        return;
    }
    *reinterpret_cast<f32x4 *>(p) = f32x4{x.v[0], x.v[1], x.v[2], x.v[3]};
    *reinterpret_cast<f32x4 *>(p + 4) = f32x4{x.v[4], x.v[5], x.v[6], x.v[7]};
}

template <bool COH = false> __device__ __forceinline__ void st_record(uint16_t *p, const u32x4 &r)
{
    if (COH) {
        st<true>(reinterpret_cast<unsigned long long *>(p), (unsigned long long)r[0] | ((unsigned long long)r[1] << 32));
        st<true>(reinterpret_cast<unsigned long long *>(p) + 1, (unsigned long long)r[2] | ((unsigned long long)r[3] << 32));
        return;
    }
    *reinterpret_cast<u32x4 *>(p) = r;
}

// x[0..7] -> one lane record of bf16 hi parts and one of lo parts
__device__ __forceinline__ void split8(const Vec8 &x, u32x4 &hi, u32x4 &lo)
{
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        uint16_t h0, l0, h1, l1;
        split_bf16(x.v[e], h0, l0);
        split_bf16(x.v[e + 1], h1, l1);
        h[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        l[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
    }
    hi = u32x4{h[0], h[1], h[2], h[3]};
    lo = u32x4{l[0], l[1], l[2], l[3]};
}

__device__ __forceinline__ u32x4 round8(const Vec8 &x)
{
    uint32_t h[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) h[e >> 1] = (uint32_t)f32_to_bf16(x.v[e]) | ((uint32_t)f32_to_bf16(x.v[e + 1]) << 16);
    return u32x4{h[0], h[1], h[2], h[3]};
}

// Sum of the J slices of 8 columns starting at (row m, column col), slices in order.
template <bool COH = false> __device__ __forceinline__ Vec8 sum_slices(const FusedGemmArgs &a, int m, int col)
{
    const float *p = a.partials + (size_t)m * a.Ntot + col;
    const size_t jstride = (size_t)a.part_rows * a.Ntot;
    Vec8 s = load8<COH>(p);
    for (int j = 1; j < a.J; ++j) {
        const Vec8 t = load8<COH>(p + j * jstride);
#pragma unroll
        for (int e = 0; e < 8; ++e) s.v[e] += t.v[e];
    }
    return s;
}

// Residual epilogue on 8 columns (col..col+7 of row m) per thread, v0 = the projection's result there;
// kg: which 8-column group of its 32-column block the thread holds (lanes kg and kg^1, 16 lanes
// apart, share a 16-column sum of squares).  Whole waves call this.
template <bool COH> __device__ __forceinline__ void resid_block(const FusedGemmArgs &a, int m, int col, bool live, int kg, const Vec8 &v0)
{
    float ss = 0.f;
    if (live) {
        const Vec8 x = load8<COH>(a.X + (size_t)m * a.h + col);
        Vec8 xn, xg;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            xn.v[e] = x.v[e] + v0.v[e];
            xg.v[e] = xn.v[e] * bf16_to_f32(a.gamma_next[col + e]);   // caller's array: no alignment assumed
            ss += xn.v[e] * xn.v[e];
        }
        store8<COH>(a.X + (size_t)m * a.h + col, xn);
        u32x4 hi, lo;
        split8(xg, hi, lo);
        const size_t idx = packed_index(m, col, (a.h + 31) >> 5);
        st_record<COH>(a.out_hi + idx, hi);
        st_record<COH>(a.out_lo + idx, lo);
    }
    ss += __shfl_xor(ss, 16);   // the other 8 columns of the 16-column group
    if (live && !(kg & 1)) st<COH>(a.ssq_out + (size_t)m * (a.h >> 4) + (col >> 4), ss);
}

}  // namespace
