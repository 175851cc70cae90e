// Causal grouped-query attention of the k+1 new rows against the per-sequence KV cache.
//
// Table 2 (App. B), attention row: A_out = softmax(Q K^T / sqrt(d) + M) V with
// K, V of shape (b, n_kv, s_kv + s_q, d).  Its FLOPs:IO ratio is ~ g*s_q, so the
// operation is bound by streaming the cache.  The mask M is never read as a tensor:
// every query row sees the old cache (rows below lens[b]) and, of the k+1 new rows, the
// ones named by a 32-bit word per query node -- itself and its ancestors in the draft
// tree (Sec. 3.1); for a linear chain that is "row j sees new rows 0..j".
//
// One workgroup owns one (sequence, kv head, position chunk).  All g*(k+1) query rows
// that share the kv head are processed against the chunk, one 16-row tile per wave,
// so every cached byte is read from HBM once per step: the waves stage each block of
// 32 positions through LDS together (double buffered, the next block's loads in flight
// during the current block's arithmetic) and every wave reads its operands from there.
// Per block and wave:
//   S^T = K . Q^T        (A operand = 16 cached K rows; LDS rows are padded by 32 bytes, the
//                         pitch at which this 16-rows-by-4-records read of a wave measured free
//                         of bank conflicts -- 16 bytes of padding cost 1.5x the cycles)
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
constexpr int MAX_WAVES = 6;   // query-row tiles per launch

// grid = (splits, kv heads, sequences); block = NW waves; wave w owns query-row tile rt_base + w.
// The kernel is bound by bytes in flight, i.e. by resident workgroups: with three or more waves the
// register allocator is held to three waves per SIMD (four workgroups per compute unit).
template <int HD, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW >= 3 ? 3 : NW, 3))) void attn_partial_kernel(Dims D, AttnArgs a, int q_rows_pad, int rt_base)
{
    constexpr int KS = HD / 32, DT = HD / 16;
    constexpr int CPR = HD / 8;          // 16-byte records per cached K row
    constexpr int KROW = CPR + 2;        // LDS row pitch in records (two records of padding)
    constexpr int NREC = 32 * CPR;       // records of a 32-position block, K and V alike
    constexpr int T = NW * 64;
    constexpr int SPT = (NREC + T - 1) / T;   // records staged per thread and operand
    __shared__ u32x4 Ks[2][32 * KROW];
    __shared__ u32x4 Vs[2][NREC];

    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int q = lane >> 4, c = lane & 15;
    const int len = max(a.pos_base[b], 0);   // a rejected sequence (< 0) is read as empty
    const int total = len + a.k + 1;
    const int t_begin = split * a.chunk;
    if (t_begin >= total) return;
    const int t_end = min(total, t_begin + a.chunk);

    // Pages of the chunk's blocks: lane l keeps the page of block first_blk + 64*group + l, so the
    // page of any block of the current group of 64 is one cross-lane read away.
    const u32x4 *Kpool = reinterpret_cast<const u32x4 *>(a.Kc), *Vpool = reinterpret_cast<const u32x4 *>(a.Vc);
    const int first_blk = t_begin >> 5;
    int pg_group = 0;
    auto load_pages = [&](int group) {
        const int blk = min(first_blk + 64 * group + lane, a.kv.blocks_per_seq - 1);
        return kv_page(a.kv, b, blk);
    };
    int pg = load_pages(0);
    // 16-byte record offset of block (t0 / 32) of this (sequence, kv head) in either pool
    auto block_records = [&](int t0) -> size_t {
        const int rel = (t0 >> 5) - first_blk;
        if ((rel >> 6) != pg_group) {   // wave-uniform, once per 64 blocks
            pg_group = rel >> 6;
            pg = load_pages(pg_group);
        }
        const int page = __shfl(pg, rel & 63);
        return (((size_t)page * D.nkv + kvh) * 32 * HD) >> 3;
    };
    const int rt = rt_base + wave;
    const u32x4 *Qs = reinterpret_cast<const u32x4 *>(a.Qp + ((size_t)b * D.nkv + kvh) * q_rows_pad * HD) + (size_t)rt * KS * 64 + lane;
    const u32x4 *Ql = reinterpret_cast<const u32x4 *>(a.Qp_lo + ((size_t)b * D.nkv + kvh) * q_rows_pad * HD) + (size_t)rt * KS * 64 + lane;

    // staging: record i of a block; K rows are contiguous in the cache, so is a whole V block.
    // Two register stages: while block i is processed out of LDS, block i+1 sits in one stage
    // (loaded during the previous iteration, moved to LDS at the end of this one) and block i+2 is
    // being fetched into the other, so two blocks (32 KiB with d = 128) are in flight per workgroup.
    // Every load is issued unconditionally -- past the chunk's end all lanes re-read one record of the
    // last block (a single cache line of traffic), which is never stored -- because a load under a
    // branch would make every later wait a full drain.
    struct Stage {
        u32x4 k[SPT], v[SPT];
    };
    const int t_last = t_begin + ((t_end - t_begin - 1) & ~31);   // first position of the chunk's last block
    auto stage_load = [&](Stage &st, int t0) {
        const bool past = t0 > t_last;   // nothing left to fetch: every lane reads one and the same record
        if (past) t0 = t_last;
        const size_t base = block_records(t0);
#pragma unroll
        for (int i = 0; i < SPT; ++i) {
            int rec = threadIdx.x + i * T;
            if (NREC % T != 0 && rec >= NREC) rec = NREC - 1;
            if (past) rec = 0;
            st.k[i] = __builtin_nontemporal_load(Kpool + base + rec);
            st.v[i] = __builtin_nontemporal_load(Vpool + base + rec);
        }
    };
    auto stage_store = [&](int buf, const Stage &st) {
#pragma unroll
        for (int i = 0; i < SPT; ++i) {
            const int rec = threadIdx.x + i * T;
            if (NREC % T == 0 || rec < NREC) {
                Ks[buf][(rec / CPR) * KROW + rec % CPR] = st.k[i];
                Vs[buf][rec] = st.v[i];
            }
        }
    };
    Stage sa, sb;
    stage_load(sa, t_begin);

    // q ~= hi + lo (two bf16), so the scores carry fp32-level accuracy although K is bf16.
    u32x4 qreg[KS], qlo[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qreg[ks] = Qs[ks * 64];
        qlo[ks] = Ql[ks * 64];
    }
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = NEG_BIG, l_run = 0.f;
    int j = (rt * 16 + c) / D.g;   // query row -> node of the chain or tree
    if (j > a.k) j = a.k;
    const uint32_t vis = a.anc[b * (a.k + 1) + j];   // visible new rows: bit i = cache row len + i
    const float scale = 1.4426950408889634f * rsqrtf((float)HD);  // log2(e)/sqrt(d)

    stage_store(0, sa);
    stage_load(sa, t_begin + 32);
    __syncthreads();

    // one block of 32 positions out of LDS buffer `buf`
    auto block = [&](int buf, int t0) {
        f32x4 s[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const u32x4 kk = Ks[buf][(16 * u + c) * KROW + ks * 4 + q];
                s[u] = mfma(kk, qreg[ks], s[u]);
                s[u] = mfma(kk, qlo[ks], s[u]);
            }
        }
        // s[u][r] is the score of position t0 + 16u + 4q + r for query row rt*16 + c.
        float v[8];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[u * 4 + r] = s[u][r] * scale;
        if (t0 + 32 > len) {   // the block holds new rows: apply the node's visibility word
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int rel = t0 + 16 * u + 4 * q + r - len;   // < 0: old cache, always visible
                    if (rel >= 0 && (rel > 31 || !((vis >> rel) & 1u))) v[u * 4 + r] = NEG_BIG;
                }
        }
        float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // The exponent's reference m_run follows the running maximum lazily: it moves (and the
        // accumulators are rescaled) only when some row's maximum has outgrown it by more than 2^8,
        // so most blocks skip the rescale.  Any reference gives the same softmax; probabilities stay
        // below 2^8 and the partial (o, l, m_run) handed to the merge is consistent with it.
        if (__any(mx > m_run + 8.f)) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
        }
        float psum = 0.f;
        uint32_t pk[4], pkl[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(v[e] - m_run), p1 = __builtin_amdgcn_exp2f(v[e + 1] - m_run);
            split_bf16x2(p0, p1, pk[e >> 1], pkl[e >> 1]);   // p ~= hi + lo: the probabilities keep ~16 mantissa bits
            psum += p0 + p1;
        }
        l_run += psum;
        const u32x4 pb = u32x4{pk[0], pk[1], pk[2], pk[3]}, pl = u32x4{pkl[0], pkl[1], pkl[2], pkl[3]};
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const u32x4 vv = Vs[buf][dt * 64 + lane];
            o[dt] = mfma(vv, pb, o[dt]);
            o[dt] = mfma(vv, pl, o[dt]);
        }
    };

    // Entering an iteration at t0: LDS buffer 0 holds block t0, stage sa block t0+32.  The LDS buffer
    // written at the end of a half-iteration was read in the previous one, which every wave left
    // through a barrier before anyone got here.
    for (int t0 = t_begin; t0 < t_end; t0 += 64) {
        stage_load(sb, t0 + 64);
        block(0, t0);
        if (t0 + 32 >= t_end) break;
        stage_store(1, sa);
        __syncthreads();
        stage_load(sa, t0 + 96);
        block(1, t0 + 32);
        if (t0 + 64 >= t_end) break;
        stage_store(0, sb);
        __syncthreads();
    }

    // o[dt][r] of lane (q, c): channel dt*16 + 4q + r of query row rt*16 + c.
    const size_t slot = ((size_t)b * D.nkv + kvh) * a.n_splits + split;
    float l = l_run;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const size_t row = slot * q_rows_pad + (size_t)rt * 16 + c;
    float *po = a.part_o + row * HD;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4 *>(po + dt * 16 + 4 * q) = o[dt];
    if (q == 0) {
        a.part_ml[row * 2] = m_run;
        a.part_ml[row * 2 + 1] = l;
    }
}

// One wave per (sequence, kv head, query row); 4 waves per block.  The wave reads the row's
// partial outputs of up to 4*BATCH chunks in one round of independent loads: lanes 16s..16s+15
// take chunk s, s+4, ... with 8 channels each, and the four lane groups are summed at the end
// in fixed order.
template <int HD>
__global__ __launch_bounds__(256) void attn_combine_kernel(Dims D, AttnArgs a, int q_rows_pad)
{
    constexpr int BATCH = 9;
    constexpr int LPR = HD / 8;   // lanes that cover a row of HD channels, 8 each
    const int lane = threadIdx.x & 63, k = a.k;
    const int R = D.g * (k + 1);
    const int n_tasks = a.B * D.nkv * R;
    const int task = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (task >= n_tasks) return;
    const int KTq = (D.qd + 31) >> 5;
    const int sg = lane >> 4, cl = lane & 15;
    const int r = task % R, kvh = (task / R) % D.nkv, b = task / (R * D.nkv);
    const int total = max(a.pos_base[b], 0) + k + 1;
    const int n_splits = (total + a.chunk - 1) / a.chunk;   // at most 64 (launch_attention)
    const size_t slot0 = ((size_t)b * D.nkv + kvh) * a.n_splits;

    float2 ml = float2{NEG_BIG, 0.f};
    if (lane < n_splits) ml = *reinterpret_cast<const float2 *>(a.part_ml + ((slot0 + lane) * q_rows_pad + r) * 2);
    float num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float m_star = 0.f, w_lane = 0.f;
    for (int base = 0; base < n_splits; base += 4 * BATCH) {
        f32x4 pv[BATCH][2];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int s = base + 4 * u + sg;
            const bool live = s < n_splits && cl < LPR;
            const f32x4 *p = reinterpret_cast<const f32x4 *>(a.part_o + ((slot0 + (live ? s : 0)) * q_rows_pad + r) * HD + (cl < LPR ? cl : 0) * 8);
            pv[u][0] = live ? p[0] : f32x4{0.f, 0.f, 0.f, 0.f};
            pv[u][1] = live ? p[1] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if (base == 0) {
            m_star = ml.x;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) m_star = fmaxf(m_star, __shfl_xor(m_star, off));
            w_lane = lane < n_splits ? exp2f(ml.x - m_star) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int s = base + 4 * u + sg;
            const float w = __shfl(w_lane, s < 64 ? s : 0);   // chunks past n_splits carry weight 0
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                num[e] += w * pv[u][0][e];
                num[4 + e] += w * pv[u][1][e];
            }
        }
    }
    float den = w_lane * ml.y;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        num[e] += __shfl_xor(num[e], 16);
        num[e] += __shfl_xor(num[e], 32);
    }
    if (sg == 0 && cl < LPR) {
        const int j = r / D.g, hl = r % D.g, m = b * (k + 1) + j;
        const int col = (kvh * D.g + hl) * HD + cl * 8;
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            uint16_t h0, l0, h1, l1;
            split_bf16(num[e] / den, h0, l0);
            split_bf16(num[e + 1] / den, h1, l1);
            hi[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            lo[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        const size_t idx = packed_index(m, col, KTq);   // col % 8 == 0: one whole lane record
        *reinterpret_cast<u32x4 *>(a.out_hi + idx) = u32x4{hi[0], hi[1], hi[2], hi[3]};
        *reinterpret_cast<u32x4 *>(a.out_lo + idx) = u32x4{lo[0], lo[1], lo[2], lo[3]};
    }
}

template <int HD, int NW> void launch_nw(const Dims &D, const AttnArgs &a, int q_rows_pad, int rt0, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((attn_partial_kernel<HD, NW>), grid, dim3(NW * 64), 0, s, D, a, q_rows_pad, rt0);
}

template <int HD> hipError_t launch_partial(const Dims &D, const AttnArgs &a, int q_rows_pad, hipStream_t s)
{
    const int rows = D.g * (a.k + 1);
    const int rt_total = (rows + 15) / 16;
    const dim3 grid(a.n_splits, D.nkv, a.B);
    // One wave per query-row tile; more than MAX_WAVES tiles take further passes over the cache.
    for (int rt0 = 0; rt0 < rt_total; rt0 += MAX_WAVES) {
        const int nw = rt_total - rt0 < MAX_WAVES ? rt_total - rt0 : MAX_WAVES;
        switch (nw) {
        case 1: launch_nw<HD, 1>(D, a, q_rows_pad, rt0, grid, s); break;
        case 2: launch_nw<HD, 2>(D, a, q_rows_pad, rt0, grid, s); break;
        case 3: launch_nw<HD, 3>(D, a, q_rows_pad, rt0, grid, s); break;
        case 4: launch_nw<HD, 4>(D, a, q_rows_pad, rt0, grid, s); break;
        case 5: launch_nw<HD, 5>(D, a, q_rows_pad, rt0, grid, s); break;
        default: launch_nw<HD, 6>(D, a, q_rows_pad, rt0, grid, s); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

// Positions per workgroup for a step of B sequences with `rows` query rows per kv head.  The device
// holds four workgroups per compute unit with up to three waves (row tiles) each, three with four
// waves, two with five or six, i.e. 1024 / 768 / 512 at once, and a launch is kept to one such round
// at most (a round and a half measured 8 % slower than one or two).  Within that, fewer and longer
// chunks are faster -- every chunk is a partial result of g*(k+1) rows to write and merge, and HBM
// serves 512 concurrent streams better than 1024 -- as long as ragged batches still even out:
//   target = max(512, 3 chunks per (sequence, kv head)), capped at the round.
// Measured, 8B shape, ms per step at 512 / 768 / 1024 workgroups: B = 4, context 32768, k = 8 (three
// waves) 7.47 / 7.71 / 8.23; k = 4 (two) 6.79 / 6.95 / 6.98; k = 12 (four) 7.84 / 7.95 / 8.41; B = 16,
// context 4096, k = 8: 9.12 / 9.22 / 9.42; 32 ragged sequences of 1024..4096 at k = 4: 9.89 / 9.54 /
// 9.59 (two chunks per sequence leave the compute units unevenly loaded).  70B shape at k = 8, five
// waves: 13 chunks of 160 positions per sequence -> 4 of 544: attention 7.3 -> 5.3 ms per step.  With five or
// six waves and long caches, 256 workgroups beat 512 (70B shape, 16 layers, B = 8, context 8192, k = 8:
// 8.21 against 8.55 ms; 8B shape, B = 4, context 16384, k = 23: 8.09 against 8.45; context 32768, k = 16:
// 9.82 against 10.09), while at B = 16, context 2048 (chunks of 1030 positions) 512 stay 1 % ahead.
// In whole 32-position blocks, at most 64 chunks per sequence (128 measured 4 % slower per step at
// B = 1, context 32768) and at least 128 positions per chunk (shorter chunks only add partial
// results for the merge: at B = 1, context 2048 the merge takes 6.8 us with 64-position chunks, 5.6 us
// with 128, the partial kernel the same).
int attention_chunk(const Dims &D, int B, int rows)
{
    const int waves = (rows + 15) / 16 < MAX_WAVES ? (rows + 15) / 16 : MAX_WAVES;
    const long round = waves <= 3 ? 1024 : (waves == 4 ? 768 : 512);
    const long positions = (long)D.seq_pad * B * D.nkv;
    long target = 3L * B * D.nkv;
    // five or six waves: one workgroup per compute unit when that still leaves it 2048 positions or more
    const long least = (waves >= 5 && positions >= 256L * 2048) ? 256 : 512;
    if (target < least) target = least;
    if (target > round) target = round;
    long chunk = (positions + target - 1) / target;
    const long floor64 = (D.seq_pad + 63) / 64;
    if (chunk < floor64) chunk = floor64;
    chunk = (chunk + 31) / 32 * 32;
    if (chunk < 128) chunk = 128;
    return (int)chunk;
}

// Chunks per sequence at the narrowest step (the most chunks any step of B sequences uses): what the
// partial-result buffers are sized for.
int attention_splits(const Dims &D, int B)
{
    const int chunk = attention_chunk(D, B, 1);
    return (D.seq_pad + chunk - 1) / chunk;
}

hipError_t launch_attention(const Dims &D, const AttnArgs &a_in, hipStream_t s)
{
    AttnArgs a = a_in;
    a.chunk = attention_chunk(D, a.B, D.g * (a.k + 1));
    a.n_splits = (D.seq_pad + a.chunk - 1) / a.chunk;
    const int q_rows_pad = round_up(D.g * (D.max_k + 1), 16);
    hipError_t e = D.d == 128 ? launch_partial<128>(D, a, q_rows_pad, s) : launch_partial<64>(D, a, q_rows_pad, s);
    if (e != hipSuccess) return e;
    const int n_tasks = a.B * D.nkv * D.g * (a.k + 1);
    if (D.d == 128) hipLaunchKernelGGL(attn_combine_kernel<128>, dim3((n_tasks + 3) / 4), dim3(256), 0, s, D, a, q_rows_pad);
    else hipLaunchKernelGGL(attn_combine_kernel<64>, dim3((n_tasks + 3) / 4), dim3(256), 0, s, D, a, q_rows_pad);
    return hipGetLastError();
}
