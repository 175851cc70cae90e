// Shared device helpers and layout definitions of the SSSD verify library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // one 16-byte lane record

#define SSSD_WAVE 64

// ---- bf16 helpers (round to nearest even, finite inputs) ----
__device__ __forceinline__ uint32_t f32_bits(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float bits_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = f32_bits(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }
// x ~= hi + lo with both parts bf16: the pair carries ~16 mantissa bits.
__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - bf16_to_f32(hi));
}

// Two values at once through the hardware conversion (v_cvt_pk_bf16_f32, round to nearest even):
// the bf16 pair (x0 low half, x1 high half), and the hi + lo split of both.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float x0, float x1)
{
    const f32x2_t v = {x0, x1};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ void split_bf16x2(float x0, float x1, uint32_t &hi, uint32_t &lo)
{
    hi = pack_bf16x2(x0, x1);
    lo = pack_bf16x2(x0 - bits_f32(hi << 16), x1 - bits_f32(hi & 0xFFFF0000u));
}

// ---- MFMA operand tile order -------------------------------------------------
// v_mfma_f32_16x16x32_bf16 reads, per lane l, 8 bf16 of a 16 x 32 operand tile:
// row/column l % 16, k-slots 8*(l/16) .. 8*(l/16)+7.  A "packed" matrix stores
// each such tile as 64 consecutive 16-byte lane records (1 KiB), tiles ordered
// [row_tile][k_tile], so that a wave fetches a whole tile with one fully
// coalesced 16-byte-per-lane load.  Element (r, k) of a packed matrix with KT
// k-tiles lives at bf16 index:
__host__ __device__ __forceinline__ size_t packed_index(int r, int k, int KT)
{
    return ((((size_t)(r >> 4) * KT + (k >> 5)) * 64 + (size_t)(((k & 31) >> 3) * 16 + (r & 15))) << 3) + (k & 7);
}

// ---- KV cache: pages of 32 positions ---------------------------------------------
// The cache of one layer is a pool of pages; a page holds 32 consecutive positions of ONE sequence for
// all kv heads: K as [kv head][32 rows][head_dim] (row-major), V as [kv head][head_dim/16 operand
// tiles of 1 KiB].  Block i of sequence b (positions 32i .. 32i+31) lives in page table[b][i], or in
// page b * blocks_per_seq + i when no table is set (every sequence then owns a contiguous run of
// pages).  A (sequence, kv head, block) is 32*head_dim contiguous bf16 in both caches: the unit the
// attention kernel streams.
//
// Within a V block, lane l = 16*q + c of tile dt holds channel dt*16 + c at the 8 positions
// {4q..4q+3} u {16+4q..16+4q+3} of the block: exactly the positions whose scores that lane owns
// after the two 16-position score MFMAs, so probabilities feed the second MFMA without any
// cross-lane movement.  bf16 index of (row r of the block, channel ch) within the block:
__host__ __device__ __forceinline__ size_t vblock_index(int r, int ch, int head_dim)
{
    (void)head_dim;
    const int q = (r & 15) >> 2, e = (r & 3) + ((r >> 4) << 2);
    return ((((size_t)(ch >> 4)) * 64 + (size_t)(q * 16 + (ch & 15))) << 3) + e;
}

struct KvGeom {
    const int32_t *table;   // device [max_batch][blocks_per_seq], or nullptr: contiguous runs
    int blocks_per_seq, n_pages, nkv, d;
};
// Page of block blk of sequence b, forced into the pool.  The embedding kernel reports a bad table
// entry and marks its sequence so that no kernel WRITES through it; readers come here and must only
// not fault.
__device__ __forceinline__ int kv_page(const KvGeom &g, int b, int blk)
{
    int page = g.table ? g.table[(size_t)b * g.blocks_per_seq + blk] : b * g.blocks_per_seq + blk;
    if (page < 0) page = 0;
    if (page >= g.n_pages) page = g.n_pages - 1;
    return page;
}
// True when every block of positions [t_first, t_last] of sequence b maps to a page inside the pool:
// what a kernel that WRITES through the table checks first (it skips the sequence otherwise).
__device__ __forceinline__ bool kv_pages_ok(const KvGeom &g, int b, int t_first, int t_last)
{
    if (!g.table) return true;
    for (int blk = t_first >> 5; blk <= (t_last >> 5); ++blk) {
        const int page = g.table[(size_t)b * g.blocks_per_seq + blk];
        if (page < 0 || page >= g.n_pages) return false;
    }
    return true;
}
// bf16 offset of the (page, kv head) block inside a layer's K or V pool
__device__ __forceinline__ size_t kv_block_offset(const KvGeom &g, int page, int kvh)
{
    return ((size_t)page * g.nkv + kvh) * 32 * g.d;
}
// bf16 offsets of element (position t, channel ch) of (sequence b, kv head kvh)
__device__ __forceinline__ size_t kcache_offset(const KvGeom &g, int b, int kvh, int t, int ch)
{
    return kv_block_offset(g, kv_page(g, b, t >> 5), kvh) + (size_t)(t & 31) * g.d + ch;
}
__device__ __forceinline__ size_t vcache_offset(const KvGeom &g, int b, int kvh, int t, int ch)
{
    return kv_block_offset(g, kv_page(g, b, t >> 5), kvh) + vblock_index(t & 31, ch, g.d);
}

// Model dimensions and buffer map handed to every kernel launcher.
struct Dims {
    int L, h, nq, nkv, d, f, V;
    int qd, kd, g;       // nq*d, nkv*d, nq/nkv
    int max_batch, max_k, max_seq, seq_pad;  // seq_pad = max_seq rounded up to 32
    int blocks_per_seq, n_pages;             // KV pages of 32 positions: per sequence, in the pool
    float eps, rope_base;
};

__host__ __device__ __forceinline__ int round_up(int x, int m) { return (x + m - 1) / m * m; }
