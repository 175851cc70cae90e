// Native driver of the C ABI (no Python, no PyTorch): builds a model of a given shape with
// pseudo-random bf16 weights, runs verify steps, prints the step time.  It exists for
// profiler runs that need a plain executable (hardware-counter collection), and it includes
// a plain copy kernel of known traffic (--copy-gib) to calibrate byte counters against.
//
//   step_driver --shape 8b --batch 1 --ctx 2048 --k 8 --steps 5 [--copy-gib 1] [--layers n]
#include "../../include/sssd_verify.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            std::fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            return 1;                                                                          \
        }                                                                                      \
    } while (0)
#define SK(x)                                                                                  \
    do {                                                                                       \
        int r_ = (x);                                                                          \
        if (r_ != SSSD_OK) {                                                                   \
            std::fprintf(stderr, "sssd error %s at %s:%d\n", sssd_strerror(r_), __FILE__, __LINE__); \
            return 1;                                                                          \
        }                                                                                      \
    } while (0)

// bf16 values of magnitude ~0.02 from a counter hash (benchmark filler, not the test generator).
__global__ void fill_bf16(uint16_t *p, size_t n, uint32_t seed, float scale)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t x = (uint32_t)i * 2654435761u + seed;
        x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
        const float u = ((x & 0xFFFF) + ((x >> 16) & 0xFFFF)) * (1.0f / 65536.0f) - 1.0f;   // triangular on (-1, 1)
        const float v = u * scale;
        uint32_t b = __builtin_bit_cast(uint32_t, v);
        b += 0x7FFFu + ((b >> 16) & 1u);
        p[i] = (uint16_t)(b >> 16);
    }
}
__global__ void fill_ones_bf16(uint16_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0x3F80;
}
__global__ void fill_i32(int32_t *p, int n, int value, uint32_t seed, int modulo)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t x = (uint32_t)i * 2654435761u + seed;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    p[i] = modulo > 0 ? (int32_t)(x % (uint32_t)modulo) : value;
}
// Plain copy: reads n*16 bytes, writes n*16 bytes.
__global__ void calibration_copy_kernel(const uint4 *src, uint4 *dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int main(int argc, char **argv)
{
    std::string shape = "8b";
    int B = 1, ctx = 2048, k = 8, steps = 5, warmup = 2, layers = 0;
    double copy_gib = 0.0;
    for (int i = 1; i + 1 < argc; i += 2) {
        const std::string f = argv[i];
        const char *v = argv[i + 1];
        if (f == "--shape") shape = v;
        else if (f == "--batch") B = std::atoi(v);
        else if (f == "--ctx") ctx = std::atoi(v);
        else if (f == "--k") k = std::atoi(v);
        else if (f == "--steps") steps = std::atoi(v);
        else if (f == "--warmup") warmup = std::atoi(v);
        else if (f == "--copy-gib") copy_gib = std::atof(v);
        else if (f == "--layers") layers = std::atoi(v);   // override the layer count of the shape (shorter runs)
        else { std::fprintf(stderr, "unknown flag %s\n", f.c_str()); return 2; }
    }
    sssd_model_config cfg{};
    if (shape == "8b") { cfg.n_layers = 32; cfg.hidden = 4096; cfg.n_q_heads = 32; cfg.n_kv_heads = 8; cfg.head_dim = 128; cfg.ffn = 14336; cfg.vocab = 128256; cfg.rope_base = 500000.f; }
    else if (shape == "70b") { cfg.n_layers = 80; cfg.hidden = 8192; cfg.n_q_heads = 64; cfg.n_kv_heads = 8; cfg.head_dim = 128; cfg.ffn = 28672; cfg.vocab = 128256; cfg.rope_base = 500000.f; }
    else if (shape == "tiny") { cfg.n_layers = 2; cfg.hidden = 256; cfg.n_q_heads = 4; cfg.n_kv_heads = 2; cfg.head_dim = 64; cfg.ffn = 688; cfg.vocab = 1024; cfg.rope_base = 10000.f; }
    else { std::fprintf(stderr, "unknown shape\n"); return 2; }
    if (layers > 0) cfg.n_layers = layers;
    cfg.rms_eps = 1e-5f; cfg.max_batch = B; cfg.max_k = k; cfg.max_seq = ctx + k + 1;
    const bool in_place = shape == "70b";

    if (copy_gib > 0) {
        const size_t n = (size_t)(copy_gib * (1 << 30)) / 16;
        uint4 *src, *dst;
        CK(hipMalloc(&src, n * 16)); CK(hipMalloc(&dst, n * 16));
        CK(hipMemset(src, 1, n * 16));
        for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(calibration_copy_kernel, dim3(4096), dim3(256), 0, 0, src, dst, n);
        CK(hipDeviceSynchronize());
        CK(hipFree(src)); CK(hipFree(dst));
    }

    const size_t qd = (size_t)cfg.n_q_heads * cfg.head_dim, kd = (size_t)cfg.n_kv_heads * cfg.head_dim, h = cfg.hidden, f = cfg.ffn, V = cfg.vocab;
    auto make = [&](size_t n, uint32_t seed, bool ones) -> uint16_t * {
        uint16_t *p = nullptr;
        if (hipMalloc(&p, n * 2) != hipSuccess) return nullptr;
        if (ones) hipLaunchKernelGGL(fill_ones_bf16, dim3(256), dim3(256), 0, 0, p, n);
        else hipLaunchKernelGGL(fill_bf16, dim3(4096), dim3(256), 0, 0, p, n, seed, 0.049f);   // std ~0.02
        return p;
    };
    std::vector<const void *> wq(cfg.n_layers), wk(cfg.n_layers), wv(cfg.n_layers), wo(cfg.n_layers), wg(cfg.n_layers),
        wu(cfg.n_layers), wd(cfg.n_layers), an(cfg.n_layers), mn(cfg.n_layers);
    uint32_t seed = 1;
    for (int l = 0; l < cfg.n_layers; ++l) {
        wq[l] = make(qd * h, seed++, false); wk[l] = make(kd * h, seed++, false); wv[l] = make(kd * h, seed++, false);
        wo[l] = make(h * qd, seed++, false); wg[l] = make(f * h, seed++, false); wu[l] = make(f * h, seed++, false);
        wd[l] = make(h * f, seed++, false); an[l] = make(h, 0, true); mn[l] = make(h, 0, true);
        if (!wq[l] || !wk[l] || !wv[l] || !wo[l] || !wg[l] || !wu[l] || !wd[l] || !an[l] || !mn[l]) { std::fprintf(stderr, "out of device memory\n"); return 1; }
    }
    sssd_weights w{};
    w.embed = make(V * h, seed++, false); w.lm_head = make(V * h, seed++, false); w.final_norm = make(h, 0, true);
    w.wq = wq.data(); w.wk = wk.data(); w.wv = wv.data(); w.wo = wo.data(); w.w_gate = wg.data(); w.w_up = wu.data();
    w.w_down = wd.data(); w.attn_norm = an.data(); w.mlp_norm = mn.data();
    CK(hipDeviceSynchronize());

    size_t kv_b, ws_b, pk_b;
    SK(sssd_verify_sizes(&cfg, &kv_b, &ws_b, &pk_b));
    void *kv, *ws, *pk = nullptr;
    CK(hipMalloc(&kv, kv_b)); CK(hipMalloc(&ws, ws_b));
    if (!in_place) CK(hipMalloc(&pk, pk_b));
    sssd_ctx *vc = nullptr;
    SK(sssd_verify_init(&cfg, &w, kv, kv_b, ws, ws_b, pk, in_place ? 0 : pk_b, in_place ? SSSD_PACK_IN_PLACE : 0, &vc));
    // cache contents: finite pseudo-random rows everywhere (import is not needed for timing)
    hipLaunchKernelGGL(fill_bf16, dim3(4096), dim3(256), 0, 0, (uint16_t *)kv, kv_b / 2, 12345u, 2.4f);
    int32_t *tok, *lens, *acc, *nxt;
    CK(hipMalloc(&tok, (size_t)B * (k + 1) * 4)); CK(hipMalloc(&lens, B * 4)); CK(hipMalloc(&acc, B * 4)); CK(hipMalloc(&nxt, B * 4));
    hipLaunchKernelGGL(fill_i32, dim3((B * (k + 1) + 63) / 64), dim3(64), 0, 0, tok, B * (k + 1), 0, 77u, (int)V);
    hipLaunchKernelGGL(fill_i32, dim3((B + 63) / 64), dim3(64), 0, 0, lens, B, ctx, 0u, 0);
    CK(hipDeviceSynchronize());

    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int i = 0; i < warmup; ++i) SK(sssd_verify_step(vc, B, k, tok, lens, acc, nxt, nullptr));
    CK(hipEventRecord(e0, nullptr));
    for (int i = 0; i < steps; ++i) SK(sssd_verify_step(vc, B, k, tok, lens, acc, nxt, nullptr));
    CK(hipEventRecord(e1, nullptr));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    SK(sssd_verify_sync(vc, nullptr));
    std::printf("{\"shape\": \"%s\", \"B\": %d, \"ctx\": %d, \"k\": %d, \"steps\": %d, \"ms_per_step\": %.4f}\n",
                shape.c_str(), B, ctx, k, steps, ms / steps);
    SK(sssd_verify_destroy(vc));
    return 0;
}
