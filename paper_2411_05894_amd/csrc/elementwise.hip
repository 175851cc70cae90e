// Small bandwidth-trivial kernels around the GEMMs: token/length validation with the
// embedding gather (which also writes the first layer's packed operands and sums of
// squares), arg-max merge + greedy prefix acceptance, rollback, cache import/export,
// weight reordering at init, and the packing helpers of the kernel-level entry points.
// None of them is in the paper's Table 2 (it lists the matrix operations only); they move
// O(M*h) bytes against O(params) for the GEMMs.
#include "kernels.h"

namespace {

// grid = M rows, block = 1024.  Row arg-max from the LM head's per-tile partials; the lowest
// token id wins a tie.  The loads go out eight at a time (the kernel is one memory round trip long
// per batch, not per element).
__global__ __launch_bounds__(1024) void row_argmax_kernel(const float *part_val, const int *part_idx, int NT, int32_t *that)
{
    __shared__ float sv[16];
    __shared__ int si[16];
    const size_t row = (size_t)blockIdx.x * NT;
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    constexpr int U = 8;
    for (int t0 = threadIdx.x; t0 < NT; t0 += U * 1024) {
        float v[U];
        int id[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * 1024;
            v[u] = t < NT ? part_val[row + t] : -INFINITY;
            id[u] = t < NT ? part_idx[row + t] : 0x7FFFFFFF;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (v[u] > bv || (v[u] == bv && id[u] < bi)) { bv = v[u]; bi = id[u]; }
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
        for (int w = 1; w < 16; ++w)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        that[blockIdx.x] = bi;
    }
}

// One thread per sequence: the longest draft prefix the arg-max chain reproduces, and the bonus token.
__global__ void accept_kernel(StepIO io, const int32_t *that)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= io.B) return;
    const int sq = io.k + 1;
    int n = 0;
    while (n < io.k && io.tokens[b * sq + n + 1] == that[b * sq + n]) ++n;
    io.accepted_len[b] = n;
    io.next_token[b] = that[b * sq + n];
}

// Greedy acceptance on draft trees (the candidate tree the paper verifies, Sec. 3.1): from the
// root, step to the child whose token is the arg-max after the current node (the lowest node index
// if several children carry it) until none does.  One thread per sequence.
__global__ void accept_tree_kernel(StepIO io, const int32_t *that)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= io.B) return;
    const int sq = io.k + 1;
    const int32_t *tok = io.tokens + b * sq, *par = io.parents + b * sq, *th = that + b * sq;
    int32_t *path = io.path + b * sq;
    int cur = 0, n = 0;
    path[0] = 0;
    for (;;) {
        int next = -1;
        for (int c = cur + 1; c <= io.k; ++c)
            if (par[c] == cur && tok[c] == th[cur]) { next = c; break; }
        if (next < 0) break;
        cur = next;
        path[++n] = cur;
    }
    for (int i = n + 1; i <= io.k; ++i) path[i] = -1;
    io.accepted_len[b] = n;
    io.next_token[b] = th[cur];
}

// grid = (nkv, B, L), block = d threads.  Thread i moves channel i of the accepted rows, one row
// after the other in path order: destinations lens + 1 .. lens + n never run ahead of the sources
// still to be read (path[i] >= i, increasing), and each thread touches its own channel only.
__global__ void kv_compact_kernel(Dims D, KvGeom kv, uint16_t *Kc, uint16_t *Vc, size_t kv_layer_elems, int k, const int32_t *lens,
                                  const int32_t *accepted_len, const int32_t *path)
{
    const int kvh = blockIdx.x, b = blockIdx.y, l = blockIdx.z, i = threadIdx.x;
    const int len = lens[b], n = accepted_len[b];
    if (len < 0 || n < 0 || n > k || len + k + 1 > D.max_seq) return;   // flagged by kv_commit_kernel
    if (!kv_pages_ok(kv, b, len, len + k)) return;                       // likewise: nothing moves through a bad page
    uint16_t *kc = Kc + (size_t)l * kv_layer_elems, *vc = Vc + (size_t)l * kv_layer_elems;
    int prev = 0;
    for (int s = 1; s <= n; ++s) {
        const int node = path[b * (k + 1) + s];
        if (node <= prev || node > k) return;        // not an increasing path: leave the rest alone (flagged)
        prev = node;
        if (node == s) continue;
        kc[kcache_offset(kv, b, kvh, len + s, i)] = kc[kcache_offset(kv, b, kvh, len + node, i)];
        vc[vcache_offset(kv, b, kvh, len + s, i)] = vc[vcache_offset(kv, b, kvh, len + node, i)];
    }
}

// After kv_compact_kernel: lens[b] += accepted_len[b] + 1; malformed input raises the error flag
// and leaves lens[b] alone.
__global__ void kv_commit_kernel(Dims D, KvGeom kv, int B, int k, int32_t *lens, const int32_t *accepted_len, const int32_t *path,
                                 int32_t *err_flag)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int len = lens[b], n = accepted_len[b];
    bool ok = len >= 0 && n >= 0 && n <= k && len + k + 1 <= D.max_seq;
    ok = ok && kv_pages_ok(kv, b, len, len + k);
    int prev = 0;
    for (int s = 1; ok && s <= n; ++s) {
        const int node = path[b * (k + 1) + s];
        ok = node > prev && node <= k;
        prev = node;
    }
    if (ok) lens[b] = len + n + 1;
    else *err_flag = 1;
}

__global__ void rollback_kernel(int B, int32_t *lens, const int32_t *accepted_len, const int32_t *new_lens)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    if (accepted_len) lens[b] += accepted_len[b] + 1;
    else lens[b] = new_lens[b];
}

// grid = (n_rows, nkv), block = d.  ext layout [nkv][n_rows][d]; Kc/Vc: the layer's pools.
// A row whose block the table sends outside the pool is skipped (nothing written on either side) and
// raises the sticky flag.
__global__ void kv_copy_kernel(Dims D, KvGeom kv, uint16_t *Kc, uint16_t *Vc, int b, int t0, int n_rows, uint16_t *k_ext,
                               uint16_t *v_ext, bool import, int32_t *err_flag)
{
    (void)D;
    const int t = blockIdx.x, kvh = blockIdx.y, i = threadIdx.x;
    if (!kv_pages_ok(kv, b, t0 + t, t0 + t)) {
        if (i == 0 && kvh == 0) *err_flag = 1;
        return;
    }
    uint16_t *kc = Kc + kcache_offset(kv, b, kvh, t0 + t, i);
    uint16_t *vc = Vc + vcache_offset(kv, b, kvh, t0 + t, i);
    const size_t e = ((size_t)kvh * n_rows + t) * kv.d + i;
    if (import) {
        *kc = k_ext[e];
        *vc = v_ext[e];
    } else {
        k_ext[e] = *kc;
        v_ext[e] = *vc;
    }
}


// grid = M rows.  Plain fp32 -> packed bf16 hi/lo (no normalisation).
__global__ __launch_bounds__(256) void pack_act_kernel(const float *X, int K, int KT, uint16_t *A_hi, uint16_t *A_lo)
{
    const int m = blockIdx.x;
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        uint16_t hi, lo;
        split_bf16(X[(size_t)m * K + i], hi, lo);
        const size_t idx = packed_index(m, i, KT);
        A_hi[idx] = hi;
        A_lo[idx] = lo;
    }
}

// grid = M rows.  packed hi + lo -> fp32 [M][K].
__global__ __launch_bounds__(256) void unpack_act_kernel(const uint16_t *A_hi, const uint16_t *A_lo, int K, int KT, float *X)
{
    const int m = blockIdx.x;
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        const size_t idx = packed_index(m, i, KT);
        X[(size_t)m * K + i] = bf16_to_f32(A_hi[idx]) + bf16_to_f32(A_lo[idx]);
    }
}

// grid = (M, nq), block = d.  Already-rotated fp32 queries -> packed Q operand buffer.
__global__ void q_pack_kernel(Dims D, const float *q, int k, uint16_t *Qp, uint16_t *Qp_lo, int q_rows_pad)
{
    const int m = blockIdx.x, head = blockIdx.y, i = threadIdx.x;
    const int b = m / (k + 1), j = m % (k + 1);
    const int kvh = head / D.g, hl = head % D.g, r = j * D.g + hl;
    const size_t idx = ((size_t)b * D.nkv + kvh) * q_rows_pad * D.d + packed_index(r, i, D.d >> 5);
    uint16_t hi, lo;
    split_bf16(q[((size_t)m * D.nq + head) * D.d + i], hi, lo);
    Qp[idx] = hi;
    Qp_lo[idx] = lo;
}

// Validated lens and the row geometry of linear chains (kernel-level attention entry point).
__global__ void lens_kernel(Dims D, int B, int k, const int32_t *lens, int32_t *pos_base, int32_t *rope_pos, uint32_t *anc,
                            int32_t *err_flag)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int len = lens[b];
    if (len < 0 || len + k + 1 > D.max_seq) {
        *err_flag = 1;
        len = 0;
    }
    pos_base[b] = len;
    for (int j = 0; j <= k; ++j) {
        rope_pos[b * (k + 1) + j] = len + j;
        anc[b * (k + 1) + j] = 0xFFFFFFFFu >> (31 - j);
    }
}

// Reorder a row-major bf16 matrix [N][K] into operand tiles (one 16-byte lane record per thread).
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


// grid = M rows, 512 threads.  Validates lens/tokens/parents; row geometry (depth and visible new
// rows of the node, from the draft tree or the chain); x = E[token]; packed x*gamma; sums of squares.
__global__ __launch_bounds__(512) void fused_embed_kernel(Dims D, StepIO io, KvGeom kv, const uint16_t *embed, const uint16_t *gamma,
                                                          float *X, uint16_t *A_hi, uint16_t *A_lo, float *ssq,
                                                          int32_t *pos_base, int32_t *rope_pos, uint32_t *anc,
                                                          int32_t *err_flag)
{
    const int m = blockIdx.x, b = m / (io.k + 1), j = m % (io.k + 1);
    int tok = io.tokens[m];
    if (tok < 0 || tok >= D.V) {
        if (threadIdx.x == 0) *err_flag = 1;
        tok = 0;
    }
    if (threadIdx.x == 0) {
        int len = io.lens[b];
        bool reject = false;   // the sequence must not write the cache: its rows would land on live data
        if (len < 0 || len + io.k + 1 > D.max_seq) {
            reject = true;
            len = 0;
        }
        if (j == 0) {
            if (kv.table && !reject) {   // every page the step reads or writes must lie in the pool
                const int last_blk = (len + io.k) >> 5;
                for (int blk = 0; blk <= last_blk; ++blk) {
                    const int page = kv.table[(size_t)b * kv.blocks_per_seq + blk];
                    if (page < 0 || page >= kv.n_pages) reject = true;
                }
            }
            // pos_base < 0 marks the rejected sequence for the K/V writers; readers take it as length 0
            pos_base[b] = reject ? -1 : len;
        }
        if (reject) *err_flag = 1;
        int depth = j;
        uint32_t vis = 0xFFFFFFFFu >> (31 - j);
        if (io.parents) {
            // walk to the root; a parent outside [0, node) is treated as node-1 and flagged
            depth = 0;
            vis = 1u << j;
            for (int i = j; i > 0;) {
                int p = io.parents[b * (io.k + 1) + i];
                if (p < 0 || p >= i) {
                    *err_flag = 1;
                    p = i - 1;
                }
                i = p;
                vis |= 1u << i;
                ++depth;
            }
        }
        rope_pos[m] = len + depth;
        anc[m] = vis;
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

// Plain read-only stream over a buffer: workgroup b reads the 16 KiB pieces b, b + grid, b + 2 grid, ...,
// each as four 16-byte loads per lane, all in flight together.  What it reaches is the read bandwidth a
// kernel on this device can get from HBM with no arithmetic in the way: the yardstick the weight
// streamers are held against.  (Measured on 2 GiB: 7.0-7.3 TB/s for 512 to 4096 workgroups of this shape;
// the same bytes fetched thread by thread at a grid-wide stride, four loads 8 MB apart per lane, reach
// 6.0 TB/s; 256 workgroups of 1024 threads with eight loads per lane, the launch shape of the weight
// streamers, 6.6-6.8 TB/s.)  The XOR of everything read goes to sink[workgroup] so that the loads are live.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *src, size_t n16, uint32_t *sink)
{
    constexpr size_t PIECE = 1024;   // records of a 16 KiB piece
    const size_t n_pieces = n16 / PIECE;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (size_t c = blockIdx.x; c < n_pieces; c += gridDim.x) {
        const u32x4 *p = src + c * PIECE + threadIdx.x;
        const u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 256);
        const u32x4 cc = __builtin_nontemporal_load(p + 512), d = __builtin_nontemporal_load(p + 768);
        acc ^= a ^ b ^ cc ^ d;
    }
    for (size_t i = n_pieces * PIECE + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        acc ^= __builtin_nontemporal_load(src + i);
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

}  // namespace

hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int n_cu, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    const int grid = n_cu * 2 < STREAM_READ_SINK_WORDS ? n_cu * 2 : STREAM_READ_SINK_WORDS;
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, s, (const u32x4 *)src, n16, sink);
    return hipGetLastError();
}

hipError_t launch_accept(const Dims &D, const StepIO &io, const float *part_val, const int *part_idx, int NT,
                         int32_t *that, hipStream_t s)
{
    (void)D;
    if (part_val) {
        hipLaunchKernelGGL(row_argmax_kernel, dim3(io.B * (io.k + 1)), dim3(1024), 0, s, part_val, part_idx, NT, that);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (io.parents) hipLaunchKernelGGL(accept_tree_kernel, dim3((io.B + 63) / 64), dim3(64), 0, s, io, that);
    else hipLaunchKernelGGL(accept_kernel, dim3((io.B + 63) / 64), dim3(64), 0, s, io, that);
    return hipGetLastError();
}

hipError_t launch_rollback(int B, int32_t *lens, const int32_t *accepted_len, const int32_t *new_lens, hipStream_t s)
{
    hipLaunchKernelGGL(rollback_kernel, dim3((B + 63) / 64), dim3(64), 0, s, B, lens, accepted_len, new_lens);
    return hipGetLastError();
}

hipError_t launch_kv_compact(const Dims &D, const KvGeom &kv, uint16_t *Kc, uint16_t *Vc, size_t kv_layer_elems, int B, int k,
                             int32_t *lens, const int32_t *accepted_len, const int32_t *path, int32_t *err_flag, hipStream_t s)
{
    hipLaunchKernelGGL(kv_compact_kernel, dim3(D.nkv, B, D.L), dim3(D.d), 0, s, D, kv, Kc, Vc, kv_layer_elems, k, lens,
                       accepted_len, path);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kv_commit_kernel, dim3((B + 63) / 64), dim3(64), 0, s, D, kv, B, k, lens, accepted_len, path, err_flag);
    return hipGetLastError();
}

hipError_t launch_kv_copy(const Dims &D, const KvGeom &kv, uint16_t *Kc_layer, uint16_t *Vc_layer, int b, int t0, int n_rows,
                          uint16_t *k_ext, uint16_t *v_ext, bool import, int32_t *err_flag, hipStream_t s)
{
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(kv_copy_kernel, dim3(n_rows, D.nkv), dim3(D.d), 0, s, D, kv, Kc_layer, Vc_layer, b, t0, n_rows, k_ext,
                       v_ext, import, err_flag);
    return hipGetLastError();
}

hipError_t launch_pack_act(const float *X, int M, int K, uint16_t *A_hi, uint16_t *A_lo, hipStream_t s)
{
    hipLaunchKernelGGL(pack_act_kernel, dim3(M), dim3(256), 0, s, X, K, (K + 31) / 32, A_hi, A_lo);
    return hipGetLastError();
}

hipError_t launch_unpack_act(const uint16_t *A_hi, const uint16_t *A_lo, int M, int K, float *X, hipStream_t s)
{
    hipLaunchKernelGGL(unpack_act_kernel, dim3(M), dim3(256), 0, s, A_hi, A_lo, K, (K + 31) / 32, X);
    return hipGetLastError();
}

hipError_t launch_q_pack(const Dims &D, const float *q, int B, int k, uint16_t *Qp, uint16_t *Qp_lo, hipStream_t s)
{
    const int q_rows_pad = round_up(D.g * (D.max_k + 1), 16);
    hipLaunchKernelGGL(q_pack_kernel, dim3(B * (k + 1), D.nq), dim3(D.d), 0, s, D, q, k, Qp, Qp_lo, q_rows_pad);
    return hipGetLastError();
}

hipError_t launch_lens(const Dims &D, int B, int k, const int32_t *lens, int32_t *pos_base, int32_t *rope_pos, uint32_t *anc,
                       int32_t *err_flag, hipStream_t s)
{
    hipLaunchKernelGGL(lens_kernel, dim3((B + 63) / 64), dim3(64), 0, s, D, B, k, lens, pos_base, rope_pos, anc, err_flag);
    return hipGetLastError();
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

hipError_t launch_fused_embed(const Dims &D, const StepIO &io, const KvGeom &kv, const uint16_t *embed, const uint16_t *gamma,
                              float *X, uint16_t *A_hi, uint16_t *A_lo, float *ssq, int32_t *pos_base, int32_t *rope_pos,
                              uint32_t *anc, int32_t *err_flag, hipStream_t s)
{
    hipLaunchKernelGGL(fused_embed_kernel, dim3(io.B * (io.k + 1)), dim3(512), 0, s, D, io, kv, embed, gamma, X, A_hi, A_lo, ssq,
                       pos_base, rope_pos, anc, err_flag);
    return hipGetLastError();
}
