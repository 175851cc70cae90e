// Target-only speculative sampling: one token per tree node drawn from the target model's own
// distribution (temperature, top-k, top-p), so that acceptance needs no draft probabilities.
//
// The paper evaluates SSSD beyond greedy decoding with "a simplified speculative sampling procedure
// ... which preserves the target distribution without requiring draft probability estimates"
// (Sec. 4.4, with temperature 0.6 / top-p 0.95; Fig. 5 uses temperature 0.7, top-p 0.8, top-k 20).
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
// are 32.32 fixed-point integers accumulated with integer LDS atomics, so every sum is exact and
// independent of the order of accumulation: the kernel is deterministic, and a tie at a threshold
// is resolved by token id exactly as the definition says.  The row stays in L2 across the passes.
#include "kernels.h"

namespace {

constexpr int ST = 1024;   // threads per row

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

__device__ __forceinline__ uint64_t fix_mass(const RowCtx &r, float z)
{
    const float w = __builtin_amdgcn_exp2f((z - r.mx) * r.scale);   // in (0, 1]
    return (uint64_t)((double)w * 4294967296.0);
}

// Scan 256 bins from the top: the first bin g with above + (mass of higher bins) + bin[g] >= target.
// Returns g and adds the mass of the higher bins to `above`.  One thread.
template <typename T> __device__ int pick_bin(const T *bins, T target, T &above)
{
    T acc = 0;
    for (int g = 255; g >= 0; --g) {
        if (above + acc + bins[g] >= target) {
            above += acc;
            return g;
        }
        acc += bins[g];
    }
    above += acc - bins[0];
    return 0;
}

// grid = rows, block = 1024.
__global__ __launch_bounds__(ST) void sample_rows_kernel(const float *logits, int V, float inv_temperature, int top_k, float top_p,
                                                         const float *uniforms, int32_t *sampled)
{
    __shared__ uint32_t chist[256];
    __shared__ uint64_t mhist[256];
    __shared__ float red_f[16];
    __shared__ uint64_t red_u[16];
    __shared__ uint32_t red_c[16];
    __shared__ uint32_t sh_prefix, sh_need, sh_count_b;
    __shared__ uint64_t sh_above, sh_total;
    __shared__ int sh_wave, sh_token;

    const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    RowCtx r;
    r.z = logits + (size_t)row * V;
    r.V = V;

    // ---- max ----
    float mx = -INFINITY;
    for (int i = tid; i < V; i += ST) mx = fmaxf(mx, r.z[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) red_f[wave] = mx;
    __syncthreads();
    mx = red_f[0];
    for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red_f[w]);
    r.mx = mx;
    r.scale = 1.4426950408889634f * inv_temperature;
    __syncthreads();

    // ---- top-k: key_a = key of the top_k-th token of O, n_a = how many tokens with exactly that key are kept ----
    uint32_t key_a = 0, n_a = 0;
    const bool use_k = top_k > 0 && top_k < V;
    if (use_k) {
        uint32_t prefix = 0, need = (uint32_t)top_k;
        for (int d = 3; d >= 0; --d) {
            if (tid < 256) chist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < V; i += ST) {
                const uint32_t key = order_key(r.z[i]);
                if (d == 3 || (key >> (8 * (d + 1))) == prefix) atomicAdd(&chist[(key >> (8 * d)) & 255u], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t above = 0;
                const int g = pick_bin<uint32_t>(chist, need, above);
                sh_prefix = (prefix << 8) | (uint32_t)g;
                sh_need = need - above;
            }
            __syncthreads();
            prefix = sh_prefix;
            need = sh_need;
            __syncthreads();
        }
        key_a = prefix;   // the key of the k-th token
        n_a = need;       // 1 <= n_a <= number of tokens with that key
    }

    // ---- Z_k ----
    uint64_t part = 0;
    for (int i = tid; i < V; i += ST) {
        const float z = r.z[i];
        if (!use_k || order_key(z) > key_a) part += fix_mass(r, z);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
    if (lane == 0) red_u[wave] = part;
    __syncthreads();
    uint64_t Zk = 0;
    for (int w = 0; w < 16; ++w) Zk += red_u[w];
    // the n_a kept tokens at the top-k threshold all carry the same logit, hence the same mass
    uint64_t mass_a = 0;
    if (use_k) {
        // recover the logit of key_a: invert order_key
        const uint32_t u = (key_a & 0x80000000u) ? (key_a & 0x7FFFFFFFu) : ~key_a;
        mass_a = fix_mass(r, bits_f32(u));
        Zk += (uint64_t)n_a * mass_a;
    }
    __syncthreads();

    // ---- top-p: key_b = key of the last token of S, n_b = how many tokens with exactly that key are in S ----
    uint32_t key_b = key_a, n_b = n_a;
    uint64_t above_b = use_k ? Zk - (uint64_t)n_a * mass_a : 0;   // mass of the tokens of S with key > key_b
    if (top_p < 1.f) {
        uint64_t target = (uint64_t)((double)top_p * (double)Zk);
        if (target < 1) target = 1;
        if (target > Zk) target = Zk;
        uint32_t prefix = 0;
        uint64_t above = 0;
        for (int d = 3; d >= 0; --d) {
            if (tid < 256) { mhist[tid] = 0; chist[tid] = 0; }
            __syncthreads();
            for (int i = tid; i < V; i += ST) {
                const float z = r.z[i];
                const uint32_t key = order_key(z);
                if ((!use_k || key > key_a) && (d == 3 || (key >> (8 * (d + 1))) == prefix)) {
                    const uint32_t g = (key >> (8 * d)) & 255u;
                    atomicAdd((unsigned long long *)&mhist[g], (unsigned long long)fix_mass(r, z));
                    atomicAdd(&chist[g], 1u);
                }
            }
            if (tid == 0 && use_k && (d == 3 || (key_a >> (8 * (d + 1))) == prefix)) {
                const uint32_t g = (key_a >> (8 * d)) & 255u;
                atomicAdd((unsigned long long *)&mhist[g], (unsigned long long)n_a * mass_a);
                atomicAdd(&chist[g], n_a);
            }
            __syncthreads();
            if (tid == 0) {
                uint64_t ab = above;
                const int g = pick_bin<uint64_t>(mhist, target, ab);
                sh_prefix = (prefix << 8) | (uint32_t)g;
                sh_above = ab;
                sh_count_b = chist[g];
            }
            __syncthreads();
            prefix = sh_prefix;
            above = sh_above;
            __syncthreads();
        }
        key_b = prefix;
        above_b = above;
        const uint32_t avail = sh_count_b;   // kept tokens with key == key_b (after the last digit: exact key)
        const uint32_t ub = (key_b & 0x80000000u) ? (key_b & 0x7FFFFFFFu) : ~key_b;
        const uint64_t mass_b = fix_mass(r, bits_f32(ub));
        uint64_t nb = mass_b ? (target - above + mass_b - 1) / mass_b : 1;
        if (nb < 1) nb = 1;
        if (nb > avail) nb = avail;
        n_b = (uint32_t)nb;
        // total of S below
        sh_total = above_b + (uint64_t)n_b * mass_b;
    } else {
        sh_total = Zk;
    }
    __syncthreads();
    const uint64_t ZS = sh_total;
    const bool all_kept = !use_k && !(top_p < 1.f);   // S is the whole vocabulary

    // ---- sample in token-id order.  Wave w owns ids [w*per, (w+1)*per); lanes stride by 64. ----
    const int per = (V + 15) / 16;
    const int lo = wave * per, hi = min(V, lo + per);
    // (1) ties at key_b below each wave, so that "the n_b lowest ids" is decidable per element
    uint32_t ties = 0;
    if (!all_kept)
        for (int base = lo; base < hi; base += 64) {
            const int i = base + lane;
            const bool tie = i < hi && order_key(r.z[i]) == key_b;
            ties += (uint32_t)__popcll(__ballot(tie));
        }
    if (lane == 0) red_c[wave] = ties;
    __syncthreads();
    uint32_t tie_base = 0;
    for (int w = 0; w < wave; ++w) tie_base += red_c[w];
    // (2) mass of S inside each wave
    auto member_mass = [&](int i, uint32_t &tie_seen) -> uint64_t {   // wave-uniform call; updates the running tie count
        const float z = i < hi ? r.z[i] : 0.f;
        const uint32_t key = order_key(z);
        const bool in_range = i < hi;
        const bool tie = in_range && !all_kept && key == key_b;
        const uint64_t bal = __ballot(tie);
        const uint32_t rank = tie_seen + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
        tie_seen += (uint32_t)__popcll(bal);
        const bool member = in_range && (all_kept || key > key_b || (tie && rank < n_b));
        return member ? fix_mass(r, z) : 0ull;
    };
    uint64_t wsum = 0;
    {
        uint32_t seen = tie_base;
        for (int base = lo; base < hi; base += 64) wsum += member_mass(base + lane, seen);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wsum += __shfl_xor(wsum, off);
    if (lane == 0) red_u[wave] = wsum;
    __syncthreads();
    // (3) the wave whose id range holds the target, then the element inside it
    if (tid == 0) {
        uint64_t tot = 0;
        for (int w = 0; w < 16; ++w) tot += red_u[w];
        // tot equals ZS by construction; the draw uses the recomputed total so that it always lands inside
        const double u = (double)uniforms[row];
        uint64_t target = (uint64_t)(u * (double)tot);
        if (target >= tot) target = tot ? tot - 1 : 0;
        uint64_t acc = 0;
        int w = 0;
        for (; w < 15; ++w) {
            if (acc + red_u[w] > target) break;
            acc += red_u[w];
        }
        sh_wave = w;
        sh_above = target - acc;   // offset of the target inside wave w's mass
        sh_token = -1;
        (void)ZS;
    }
    __syncthreads();
    if (wave == sh_wave) {
        const uint64_t target = sh_above;
        uint64_t carry = 0;
        uint32_t seen = tie_base;
        int found = -1;
        int last_member = -1;
        for (int base = lo; base < hi && found < 0; base += 64) {
            const int i = base + lane;
            const uint64_t m = member_mass(i, seen);
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
        }
        if (lane == 0) sh_token = found >= 0 ? found : last_member;
    }
    __syncthreads();
    if (tid == 0) {
        int t = sh_token;
        if (t < 0) {   // no mass at all in the chosen range (cannot happen with finite logits): the arg-max
            t = 0;
            for (int i = 1; i < V; ++i)
                if (r.z[i] > r.z[t]) t = i;
        }
        sampled[row] = t;
    }
}

}  // namespace

hipError_t launch_sample_rows(const float *logits, int rows, int V, float temperature, int top_k, float top_p,
                              const float *uniforms, int32_t *sampled, hipStream_t s)
{
    hipLaunchKernelGGL(sample_rows_kernel, dim3(rows), dim3(ST), 0, s, logits, V, 1.f / temperature, top_k, top_p, uniforms,
                       sampled);
    return hipGetLastError();
}
