// Target-only speculative sampling: one token per tree node drawn from the target model's own
// distribution (temperature, top-k, top-p), so that acceptance needs no draft probabilities.
//
// Beyond greedy decoding the paper runs SSSD with a reduced form of speculative sampling that keeps
// the target distribution exact and needs no probabilities from the draft side (Sec. 4.4, at
// temperature 0.6 / top-p 0.95; Fig. 5 uses temperature 0.7, top-p 0.8, top-k 20).
// n-gram drafts carry no probabilities: the draft distribution of a proposed token is a point mass,
// for which the acceptance test of speculative sampling (accept with probability min(1, p/q), else
// resample from the normalised residual) is the same as drawing ONE token t from the target
// distribution p of the node and accepting the child that carries t, if any; otherwise t itself is
// emitted and the walk stops.  Every emitted token is an exact sample of p given its prefix.
//
// Distribution of a row (logits z, temperature T > 0, top_k, top_p):
//   order O: by logit descending, token id ascending among equal logits
//   S_k = the first top_k tokens of O (all tokens if top_k is 0 or >= vocab)
//   w_i = exp((z_i - max z) / T);  Z_k = sum of w over S_k
//   S   = the shortest prefix of O (at least one token) whose w-sum reaches top_p * Z_k
//   the sample: r = u * Z_S, the first token of S in ascending TOKEN ID order whose running
//   w-sum exceeds r (u is the caller's uniform number in [0, 1) for this row).
//
// One workgroup of 1024 threads per row.  Both selections are radix selects over the 32-bit logit
// pattern (four 8-bit digits, most significant first): top-k on counts, top-p on masses.  Masses
// are 1.31 fixed-point integers accumulated in 64 bits with integer LDS atomics, so every sum is exact and
// independent of the order of accumulation: the kernel is deterministic, and a tie at a threshold
// is resolved by token id exactly as the definition says.  The row stays in L2 across the passes.
#include "kernels.h"

namespace {

constexpr int ST = 1024;   // threads per row
constexpr int MAX_BATCH = 64;   // batches of 512 ids per wave: vocabularies up to 16 * 64 * 512 tokens

// Order-preserving map of a finite float to uint32: larger float -> larger key.
__device__ __forceinline__ uint32_t order_key(float z)
{
    const uint32_t u = f32_bits(z);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct RowCtx {
    const float *z;
    int V;
    float mx, scale;   // w = exp2((z - mx) * scale)
};

// Weight of a token as a 1.31 fixed-point integer: w * 2^31 is exact in fp32 (a power-of-two scale)
// and fits 32 bits because w <= 1.
__device__ __forceinline__ uint64_t fix_mass(const RowCtx &r, float z)
{
    const float w = __builtin_amdgcn_exp2f((z - r.mx) * r.scale);   // in [0, 1]
    return (uint64_t)(uint32_t)(w * 2147483648.0f);
}

// Wave 0 scans 256 bins from the top: the bin g with above + (sum of higher bins) < target <= that + bins[g]
// (bin 0 if the target is never reached).  Every lane returns g and the sum of the bins above g;
// lane l owns bins 4l .. 4l+3.
template <typename T> __device__ int pick_bin(const T *bins, T target, T above, T &higher, int lane)
{
    T v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = bins[4 * lane + e];
    const T mine = v[0] + v[1] + v[2] + v[3];
    T suffix = mine;   // sum over lanes >= lane
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const T o = __shfl_down(suffix, off);
        if (lane + off < 64) suffix += o;
    }
    T hi = suffix - mine;   // sum of the bins of higher lanes
    int g = -1;
    T hg = 0;
#pragma unroll
    for (int e = 3; e >= 0; --e) {
        if (g < 0 && above + hi + v[e] >= target) { g = 4 * lane + e; hg = hi; }
        hi += v[e];
    }
    // the highest bin that qualifies wins
    const unsigned long long found = __ballot(g >= 0);
    const int src = found ? 63 - __clzll(found) : 0;
    int gs = __shfl(g, src);
    T hs = __shfl(hg, src);
    if (!found) { gs = 0; hs = __shfl(suffix, 0) - __shfl(v[0], 0); }
    higher = hs;
    return gs;
}

// Histogram accumulation through a private run per thread: consecutive elements that fall into the
// same bin (the leading digits of a row's logits mostly do) are summed in registers and reach LDS as
// one atomic add when the bin changes, so a hot bin is not hit by an atomic per element.
struct BinRun {
    uint32_t bin, count;
    uint64_t mass;
    bool open;
};
__device__ __forceinline__ void run_flush(BinRun &r, uint32_t *chist, uint64_t *mhist)
{
    if (!r.open) return;
    if (chist) atomicAdd(&chist[r.bin], r.count);
    if (mhist) atomicAdd((unsigned long long *)&mhist[r.bin], (unsigned long long)r.mass);
    r.open = false;
}
__device__ __forceinline__ void run_add(BinRun &r, uint32_t bin, uint64_t mass, uint32_t *chist, uint64_t *mhist)
{
    if (r.open && r.bin == bin) {
        r.count += 1;
        r.mass += mass;
        return;
    }
    run_flush(r, chist, mhist);
    r.bin = bin;
    r.count = 1;
    r.mass = mass;
    r.open = true;
}

// body(i, z, valid) for i = begin + first, begin + first + stride, ... below end, in ascending order.
// The loads go out eight at a time: a pass is bound by load latency, not by bandwidth (the row is in L2).
// Every thread makes the same number of calls (valid = false past the end), so body may use wave-wide
// operations.
constexpr int SU = 8;
template <typename F>
__device__ __forceinline__ void for_row(const float *z, int begin, int end, int first, int stride, F body)
{
    for (int base = begin; base < end; base += stride * SU) {
        float zz[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int i = base + u * stride + first;
            zz[u] = i < end ? z[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int i = base + u * stride + first;
            body(i, zz[u], i < end);
        }
    }
}

// The whole row, any order: 16-byte loads (four tokens per thread and load) when the row allows it.
template <typename F> __device__ __forceinline__ void for_whole_row(const float *z, int V, bool vec4, int tid, F body)
{
    if (!vec4) {
        for_row(z, 0, V, tid, ST, body);
        return;
    }
    const f32x4 *z4 = reinterpret_cast<const f32x4 *>(z);
    const int V4 = V >> 2;
    for (int base = 0; base < V4; base += ST * SU) {
        f32x4 zz[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int i = base + u * ST + tid;
            zz[u] = i < V4 ? z4[i] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int i = base + u * ST + tid;
#pragma unroll
            for (int e = 0; e < 4; ++e) body(4 * i + e, zz[u][e], i < V4);
        }
    }
}

// ---- several workgroups per row ----
// One compute unit pulls a 513 KB row out of L2 in 10-15 us, and the exact selections need seven to
// twelve passes: with few rows (a step of B = 1 has k+1 of them) the kernel's time is that of one row on
// one compute unit.  So a row is given to a CLUSTER of C workgroups, each on its own contiguous range of
// token ids; what a pass finds (maximum, histogram bins, tie counts, member mass) is merged through a
// small scratch block in global memory and a barrier among the C workgroups, after which every workgroup
// takes the same decision from the same merged numbers.  All merged quantities are integers (or a
// maximum), so the result does not depend on C: the cluster of one is the plain kernel.
//
// The barrier is a counter per cluster that only grows: barrier number n of a launch waits for n*C
// arrivals.  Shared words are written with device-scope atomics (or device-scope stores, waited for,
// before the workgroup is counted in) and read with device-scope loads, as in the split-K hand-over of
// the GEMM kernels.  Waiting is bounded: a cluster whose workgroups are not all resident (the launch
// assumes the device to itself: grid <= compute units) gives up after SPIN_LIMIT polls, raises *err and
// leaves its rows unsampled (-1) instead of hanging.
constexpr int MAX_CLUSTER = 16;
constexpr int HIST_PASSES = 8;            // four count passes (top-k) and four mass passes (top-p)
constexpr unsigned SPIN_LIMIT = 1u << 20;
struct SampleScratch {                    // one per cluster; the two counters are zero when a launch starts
    uint32_t arrivals;
    uint32_t departures;                  // the last workgroup to leave puts both counters back to zero
    uint32_t pad[14];
    float gmax[MAX_CLUSTER];
    uint32_t gties[MAX_CLUSTER];
    uint64_t gsub[MAX_CLUSTER];
    uint32_t chist[HIST_PASSES][256];
    uint64_t mhist[HIST_PASSES][256];
};

struct Cluster {
    SampleScratch *s;
    int C, c;
    uint32_t passed;   // barriers passed so far in this launch (same in every workgroup of the cluster)
    bool failed;
};

// All threads of all workgroups of the cluster.  Returns false when the wait ran out.
__device__ __forceinline__ bool cluster_sync(Cluster &cl, int32_t *err)
{
    if (cl.C == 1) return true;
    __shared__ int ok_s;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    cl.passed += 1;
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(&cl.s->arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t want = cl.passed * (uint32_t)cl.C;
        unsigned spins = 0;
        while (__hip_atomic_load(&cl.s->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want && spins < SPIN_LIMIT) {
            __builtin_amdgcn_s_sleep(2);
            ++spins;
        }
        ok_s = spins < SPIN_LIMIT;
        if (!ok_s && err) atomicOr(err, 2);
    }
    __syncthreads();
    const bool ok = ok_s != 0;
    __syncthreads();
    if (!ok) cl.failed = true;
    return ok;
}

// Local 256-bin histograms -> the cluster's bins of this pass -> back into LDS (every workgroup then holds
// the merged bins).  Whole workgroup; tid < 256 owns bin tid.
__device__ __forceinline__ bool merge_bins(Cluster &cl, int pass, uint32_t *chist, uint64_t *mhist, bool counts, bool masses, int tid,
                                           int32_t *err)
{
    if (cl.C == 1) return true;
    if (tid < 256) {
        if (counts && chist[tid]) __hip_atomic_fetch_add(&cl.s->chist[pass][tid], chist[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (masses && mhist[tid])
            __hip_atomic_fetch_add((unsigned long long *)&cl.s->mhist[pass][tid], (unsigned long long)mhist[tid], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!cluster_sync(cl, err)) return false;
    if (tid < 256) {
        if (counts) chist[tid] = __hip_atomic_load(&cl.s->chist[pass][tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (masses)
            mhist[tid] = __hip_atomic_load((unsigned long long *)&cl.s->mhist[pass][tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return true;
}

// grid = clusters * C workgroups of 1024 threads; cluster g takes rows g, g + clusters, ...
__global__ __launch_bounds__(ST) void sample_rows_kernel(const float *logits, int rows, int V, float inv_temperature, int top_k, float top_p,
                                                         const float *uniforms, int32_t *sampled, int C, SampleScratch *scratch,
                                                         int32_t *err)
{
    __shared__ uint32_t chist[256];
    __shared__ uint64_t mhist[256];
    __shared__ float red_f[16];
    __shared__ uint32_t red_c[16];
    __shared__ uint32_t sh_prefix, sh_need, sh_count_b;
    __shared__ uint64_t sh_above, sh_total, sh_target;
    __shared__ int sh_wave, sh_batch, sh_token;
    __shared__ uint64_t sub[16][MAX_BATCH];   // mass of S per (wave, batch of 512 ids)

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_clusters = gridDim.x / C;
    Cluster cl{C > 1 ? scratch + blockIdx.x / C : nullptr, C, (int)(blockIdx.x % C), 0u, false};
    // this workgroup's token ids: [seg_lo, seg_hi), whole groups of four so that 16-byte loads stay aligned
    const int seg_len = ((V + C - 1) / C + 3) & ~3;
    const int seg_lo = min(V, cl.c * seg_len), seg_hi = min(V, seg_lo + seg_len), Vs = seg_hi - seg_lo;

  for (int row = blockIdx.x / C; row < rows; row += n_clusters) {
    RowCtx r;
    r.z = logits + (size_t)row * V;
    r.V = V;
    const float *zs = r.z + seg_lo;   // the segment
    auto give_up = [&]() { if (cl.c == 0 && tid == 0) sampled[row] = -1; };
    if (cl.failed) {                  // an earlier wait ran out: nothing more is sampled by this cluster
        give_up();
        continue;
    }
    // the cluster's bins of the previous row are dead (everyone left that row through a barrier that
    // came after its last read of them): clear them for this row
    if (C > 1) {
        uint32_t *w = &cl.s->chist[0][0];
        constexpr int WORDS = HIST_PASSES * 256 * 3;
        for (int i = cl.c * ST + tid; i < WORDS; i += C * ST) __hip_atomic_store(w + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- max ----
    float mx = -INFINITY;
    const bool vec4 = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(r.z) & 15) == 0;
    for_whole_row(zs, Vs, vec4, tid, [&](int, float z, bool ok) { if (ok) mx = fmaxf(mx, z); });
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) red_f[wave] = mx;
    __syncthreads();
    mx = red_f[0];
    for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red_f[w]);
    __syncthreads();
    if (C > 1) {
        if (tid == 0) __hip_atomic_store(&cl.s->gmax[cl.c], mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!cluster_sync(cl, err)) { give_up(); continue; }
        for (int w = 0; w < C; ++w) mx = fmaxf(mx, __hip_atomic_load(&cl.s->gmax[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    r.mx = mx;
    r.scale = 1.4426950408889634f * inv_temperature;

    // ---- top-k: key_a = key of the top_k-th token of O, n_a = how many tokens with exactly that key are kept ----
    uint32_t key_a = 0, n_a = 0, total_a = 0;   // total_a: tokens of the row with key == key_a
    const bool use_k = top_k > 0 && top_k < V;
    bool lost = false;
    if (use_k) {
        uint32_t prefix = 0, need = (uint32_t)top_k;
        for (int d = 3; d >= 0 && !lost; --d) {
            if (tid < 256) chist[tid] = 0;
            __syncthreads();
            BinRun run{0, 0, 0, false};
            for_whole_row(zs, Vs, vec4, tid, [&](int, float z, bool ok) {
                const uint32_t key = order_key(z);
                if (ok && (d == 3 || (key >> (8 * (d + 1))) == prefix)) run_add(run, (key >> (8 * d)) & 255u, 0, chist, nullptr);
            });
            run_flush(run, chist, nullptr);
            __syncthreads();
            if (!merge_bins(cl, 3 - d, chist, nullptr, true, false, tid, err)) { lost = true; break; }
            if (wave == 0) {
                uint32_t higher;
                const int g = pick_bin<uint32_t>(chist, need, 0u, higher, lane);
                if (lane == 0) {
                    sh_prefix = (prefix << 8) | (uint32_t)g;
                    sh_need = need - higher;
                    sh_count_b = chist[g];   // after the last digit: every token of the row with exactly this key
                }
            }
            __syncthreads();
            prefix = sh_prefix;
            need = sh_need;
            __syncthreads();
        }
        key_a = prefix;   // the key of the k-th token
        n_a = need;       // 1 <= n_a <= total_a
        total_a = sh_count_b;
        __syncthreads();
    }
    if (lost) { give_up(); continue; }

    // the n_a kept tokens at the top-k threshold all carry the same logit, hence the same mass
    uint64_t mass_a = 0;
    if (use_k) {
        const uint32_t u = (key_a & 0x80000000u) ? (key_a & 0x7FFFFFFFu) : ~key_a;   // invert order_key
        mass_a = fix_mass(r, bits_f32(u));
    }

    // ---- top-p: key_b = key of the last token of S, n_b = how many tokens with exactly that key are in S.
    // The first pass's bins add up to Z_k, from which the target mass follows. ----
    uint32_t key_b = key_a, n_b = n_a;
    uint32_t count_b = n_a;   // kept tokens with key == key_b
    uint32_t total_b = total_a;   // tokens of the row with key == key_b
    {
        const bool nucleus = top_p < 1.f;
        uint64_t target = 0, above = 0;
        uint32_t prefix = 0;
        for (int d = 3; nucleus && d >= 0 && !lost; --d) {
            if (tid < 256) { mhist[tid] = 0; chist[tid] = 0; }
            __syncthreads();
            BinRun run{0, 0, 0, false};
            uint32_t *cbins = d == 0 ? chist : nullptr;   // counts matter only for the exact key (the ties at key_b)
            for_whole_row(zs, Vs, vec4, tid, [&](int, float z, bool ok) {
                const uint32_t key = order_key(z);
                if (ok && (!use_k || key > key_a) && (d == 3 || (key >> (8 * (d + 1))) == prefix))
                    run_add(run, (key >> (8 * d)) & 255u, fix_mass(r, z), cbins, mhist);
            });
            run_flush(run, cbins, mhist);
            // the kept tokens at the top-k threshold are added once per row, by the cluster's first workgroup
            if (tid == 0 && cl.c == 0 && use_k && (d == 3 || (key_a >> (8 * (d + 1))) == prefix)) {
                const uint32_t g = (key_a >> (8 * d)) & 255u;
                atomicAdd((unsigned long long *)&mhist[g], (unsigned long long)n_a * mass_a);
                atomicAdd(&chist[g], n_a);
            }
            __syncthreads();
            if (!merge_bins(cl, 4 + (3 - d), chist, mhist, d == 0, true, tid, err)) { lost = true; break; }
            if (wave == 0) {
                if (d == 3) {   // Z_k = the sum of all bins; the nucleus target follows from it
                    uint64_t tot = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) tot += mhist[4 * lane + e];
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) tot += __shfl_xor(tot, off);
                    target = (uint64_t)((double)top_p * (double)tot);
                    if (target < 1) target = 1;
                    if (target > tot) target = tot;
                    if (lane == 0) { sh_total = tot; sh_target = target; }
                }
                if (nucleus) {
                    uint64_t higher;
                    const int g = pick_bin<uint64_t>(mhist, target, above, higher, lane);
                    if (lane == 0) {
                        sh_prefix = (prefix << 8) | (uint32_t)g;
                        sh_above = above + higher;
                        sh_count_b = chist[g];
                    }
                }
            }
            __syncthreads();
            target = sh_target;
            if (nucleus) {
                prefix = sh_prefix;
                above = sh_above;
            }
            __syncthreads();
        }
        if (nucleus && !lost) {
            key_b = prefix;
            count_b = sh_count_b;   // after the last digit: kept tokens with exactly this key
            const uint32_t ub = (key_b & 0x80000000u) ? (key_b & 0x7FFFFFFFu) : ~key_b;
            const uint64_t mass_b = fix_mass(r, bits_f32(ub));
            uint64_t nb = mass_b ? (target - above + mass_b - 1) / mass_b : 1;
            if (nb < 1) nb = 1;
            if (nb > count_b) nb = count_b;
            n_b = (uint32_t)nb;
            total_b = (use_k && key_b == key_a) ? total_a : count_b;
        }
    }
    if (lost) { give_up(); continue; }
    const bool all_kept = !use_k && !(top_p < 1.f);   // S is the whole vocabulary

    // ---- sample in token-id order.  Wave w of this workgroup owns ids [lo, hi) of the segment; lanes stride by 64. ----
    const int per = (Vs + 15) / 16;
    const int lo = seg_lo + min(Vs, wave * per), hi = min(seg_hi, lo + per);
    // (1) ties at key_b below each wave, so that "the n_b lowest ids" is decidable per element
    uint32_t ties = 0;
    const bool partial_ties = !all_kept && n_b < total_b;   // else every tie is a member: no ranks needed
    if (partial_ties)
        for_row(r.z, lo, hi, lane, 64, [&](int, float z, bool ok) {
            ties += (uint32_t)__popcll(__ballot(ok && order_key(z) == key_b));
        });
    if (lane == 0) red_c[wave] = ties;
    __syncthreads();
    uint32_t tie_base = 0;
    for (int w = 0; w < wave; ++w) tie_base += red_c[w];
    if (C > 1 && partial_ties) {   // ties in the workgroups before this one
        uint32_t mine = 0;
        for (int w = 0; w < 16; ++w) mine += red_c[w];
        if (tid == 0) __hip_atomic_store(&cl.s->gties[cl.c], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!cluster_sync(cl, err)) { give_up(); continue; }
        for (int w = 0; w < cl.c; ++w) tie_base += __hip_atomic_load(&cl.s->gties[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // (2) mass of S inside each wave
    auto member_mass = [&](float z, bool in_range, uint32_t &tie_seen) -> uint64_t {   // wave-uniform call; updates the running tie count
        const uint32_t key = order_key(z);
        const bool tie = in_range && !all_kept && key == key_b;
        uint32_t rank = 0;
        if (partial_ties) {
            const uint64_t bal = __ballot(tie);
            rank = tie_seen + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
            tie_seen += (uint32_t)__popcll(bal);
        }
        const bool member = in_range && (all_kept || key > key_b || (tie && rank < n_b));
        return member ? fix_mass(r, z) : 0ull;
    };
    // One entry per batch of 8 x 64 consecutive ids of every wave: the target is then located in one
    // batch instead of a walk through the wave's whole range.
    if (lane < MAX_BATCH) sub[wave][lane] = 0;   // ranges past the vocabulary leave their entries at zero
    {
        uint32_t seen = tie_base;
        uint64_t bsum = 0;
        int calls = 0, calls_total = 0;
        for_row(r.z, lo, hi, lane, 64, [&](int, float z, bool ok) {
            bsum += member_mass(z, ok, seen);
            if (++calls == SU) {
                uint64_t t = bsum;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off);
                const int batch = (calls_total++);
                if (lane == 0) sub[wave][batch] = t;
                calls = 0;
                bsum = 0;
            }
        });
    }
    __syncthreads();
    // (3) the (workgroup, wave, batch) whose id range holds the target, then the element inside it
    const int n_batch = (per + 64 * SU - 1) / (64 * SU);
    uint64_t wg_before = 0, row_total = 0;   // member mass in the workgroups before this one / in the whole row
    if (C > 1) {
        uint64_t mine = 0;
        if (tid == 0)
            for (int w = 0; w < 16; ++w)
                for (int bt = 0; bt < n_batch; ++bt) mine += sub[w][bt];
        if (tid == 0) __hip_atomic_store((unsigned long long *)&cl.s->gsub[cl.c], (unsigned long long)mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!cluster_sync(cl, err)) { give_up(); continue; }
        for (int w = 0; w < C; ++w) {
            const uint64_t m = __hip_atomic_load((unsigned long long *)&cl.s->gsub[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (w < cl.c) wg_before += m;
            row_total += m;
        }
    }
    if (tid == 0) {
        uint64_t tot = 0;
        for (int w = 0; w < 16; ++w)
            for (int bt = 0; bt < n_batch; ++bt) tot += sub[w][bt];
        const uint64_t mine = tot;
        if (C > 1) tot = row_total;
        // the draw uses this recomputed total, so that it always lands inside S
        const double u = (double)uniforms[row];
        uint64_t target = (uint64_t)(u * (double)tot);
        if (target >= tot) target = tot ? tot - 1 : 0;
        // the workgroup whose ids hold the target walks on; with no mass at all the last one answers
        const bool here = C == 1 || (tot ? (target >= wg_before && target < wg_before + mine) : cl.c == C - 1);
        target -= here ? wg_before : 0;
        uint64_t acc = 0;
        int w = 0, bt = 0;
        bool done = false;
        for (w = 0; w < 16 && !done; ++w)
            for (bt = 0; bt < n_batch; ++bt) {
                if (acc + sub[w][bt] > target) { done = true; break; }
                acc += sub[w][bt];
            }
        if (done) --w; else { w = 15; bt = n_batch > 0 ? n_batch - 1 : 0; }   // an empty range walks nothing and falls through to the arg-max
        sh_wave = here ? w : -1;
        sh_batch = bt;
        sh_above = target - acc;   // offset of the target inside that batch
        sh_token = -1;
    }
    __syncthreads();
    if (wave == sh_wave) {
        const uint64_t target = sh_above;
        const int b_lo = lo + sh_batch * 64 * SU, b_hi = min(hi, b_lo + 64 * SU);
        // ties before this batch inside the wave's range (only needed when ties are taken partially)
        uint32_t seen = tie_base;
        if (partial_ties)
            for_row(r.z, lo, b_lo, lane, 64, [&](int, float z, bool ok) {
                seen += (uint32_t)__popcll(__ballot(ok && order_key(z) == key_b));
            });
        uint64_t carry = 0;
        int found = -1;
        int last_member = -1;
        for_row(r.z, b_lo, b_hi, lane, 64, [&](int i, float z, bool ok) {
            if (found >= 0) return;                     // wave-uniform
            const int base = i - lane;
            const uint64_t m = member_mass(z, ok, seen);
            uint64_t inc = m;   // inclusive scan over lanes
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint64_t o = __shfl_up(inc, off);
                if (lane >= off) inc += o;
            }
            const bool hit = m > 0 && carry + inc > target;
            const uint64_t hb = __ballot(hit);
            const uint64_t mb = __ballot(m > 0);
            if (mb) last_member = base + 63 - __clzll(mb);
            if (hb) found = base + __ffsll((long long)hb) - 1;
            carry += __shfl(inc, 63);
        });
        if (lane == 0) sh_token = found >= 0 ? found : last_member;
    }
    __syncthreads();
    if (tid == 0 && sh_wave >= 0) {
        int t = sh_token;
        if (t < 0) {   // no mass at all in the chosen range (cannot happen with finite logits): the arg-max
            t = 0;
            for (int i = 1; i < V; ++i)
                if (r.z[i] > r.z[t]) t = i;
        }
        sampled[row] = t;
    }
    __syncthreads();   // the shared words above are rewritten by the next row
  }
    // Leave the counters at zero for the next launch on this scratch (a cluster that gave up leaves them as
    // they are: the launcher's caller learns of it through *err and clears the scratch).
    if (C > 1 && !cl.failed && tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(&cl.s->departures, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == (uint32_t)C - 1) {
            __hip_atomic_store(&cl.s->arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&cl.s->departures, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Clears the clusters' scratch blocks (a kernel, not a memset: the launch may be captured in a graph).
__global__ void sample_scratch_clear_kernel(uint32_t *words, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0u;
}

}  // namespace

// Workgroups per row for a launch of `rows` rows on a device of n_cu compute units: the largest power of two
// (at most 16) that keeps the whole grid resident at one workgroup per compute unit; 1 without scratch.
static int sample_cluster_size(int rows, int n_cu)
{
    int c = 1;
    while (c * 2 <= MAX_CLUSTER && (long)rows * (c * 2) <= n_cu) c *= 2;
    return c;
}

size_t sample_scratch_bytes(int rows, int n_cu)
{
    const int c = sample_cluster_size(rows, n_cu);
    return c > 1 ? (size_t)rows * sizeof(SampleScratch) : 0;
}

hipError_t launch_sample_rows(const float *logits, int rows, int V, float temperature, int top_k, float top_p,
                              const float *uniforms, int32_t *sampled, void *scratch, size_t scratch_bytes, bool scratch_clean, int n_cu,
                              int32_t *err, hipStream_t s)
{
    if ((long)V > 16L * MAX_BATCH * 64 * SU) return hipErrorInvalidValue;
    int C = scratch ? sample_cluster_size(rows, n_cu > 0 ? n_cu : 256) : 1;
    if (C > 1 && scratch_bytes < (size_t)rows * sizeof(SampleScratch)) C = 1;
    if (C > 1 && (long)(V / C) > (long)MAX_BATCH * 16 * 64 * SU) return hipErrorInvalidValue;
    if (C > 1 && !scratch_clean) {
        const size_t words = (size_t)rows * sizeof(SampleScratch) / 4;
        hipLaunchKernelGGL(sample_scratch_clear_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, (uint32_t *)scratch, words);
    }
    hipLaunchKernelGGL(sample_rows_kernel, dim3(rows * C), dim3(ST), 0, s, logits, rows, V, 1.f / temperature, top_k, top_p, uniforms,
                       sampled, C, (SampleScratch *)scratch, err);
    return hipGetLastError();
}
