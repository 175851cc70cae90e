/*
 * sssd_ops.h -- kernel-level entry points of libsssd_verify, for parity tests and
 * micro-benchmarks of single operations of the verify step (the rows of the
 * paper's Table 2, App. B).  Same conventions as sssd_verify.h: device pointers
 * are caller-owned, calls enqueue on `stream` and return 0 or a negative SSSD_E*.
 */
#ifndef SSSD_OPS_H
#define SSSD_OPS_H

#include "sssd_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of the tile-ordered form of a bf16 matrix [N][K] (K padded to 32; N % 16 == 0),
 * and of one half (hi or lo) of the tile-ordered activations of M rows x K. */
size_t sssd_op_packed_weight_bytes(int32_t N, int32_t K);
size_t sssd_op_packed_act_bytes(int32_t M, int32_t K);

/* w: device bf16 [N][K] row-major -> packed: device, sssd_op_packed_weight_bytes(N, K). */
int sssd_op_pack_weight(const void *w, void *packed, int32_t N, int32_t K, void *stream);

/* x: device fp32 [M][K] -> a_hi, a_lo: device, sssd_op_packed_act_bytes(M, K) each, which
 * the caller zero-filled once (padding must read as zero); x ~= hi + lo, both bf16. */
int sssd_op_pack_activation(const float *x, int32_t M, int32_t K, void *a_hi, void *a_lo, void *stream);

/* Table 2 linear rows: out[M][N] (device fp32, row-major) = X[M][K] . W[N][K]^T with fp32
 * accumulation, X = a_hi + a_lo.  scratch: device, at least sssd_op_gemm_scratch_bytes(M, N, K)
 * bytes (split-K partial sums; may be NULL when that is 0); SSSD_ECAPACITY if it is smaller. */
size_t sssd_op_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K);
int sssd_op_gemm(const void *a_hi, const void *a_lo, const void *w_packed, int32_t M, int32_t N, int32_t K,
                 float *out, void *scratch, size_t scratch_bytes, void *stream);

/*
 * sssd_op_gemm for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The split-K partial sums live in
 * a device array that is part of the library image (SSSD_OP_GEMM_STATIC_SCRATCH_BYTES, one copy per
 * GPU, held until the process ends), so the call allocates and frees nothing, on the device or
 * through any allocating runtime routine; its first call on a device only looks the array's address
 * up.  Same arguments, result (bit for bit) and errors as sssd_op_gemm, except:
 *  - SSSD_ECAPACITY when sssd_op_gemm_scratch_bytes(M, N, K) exceeds the array: the shape needs
 *    sssd_op_gemm with a caller-provided scratch;
 *  - all calls on one GPU share the one array: calls that overlap in time on the same GPU (different
 *    streams, different threads) race on it and must be ordered by the caller.  Nothing in it has to
 *    be cleared between calls: a launch only reads the partial sums it wrote itself.
 */
#define SSSD_OP_GEMM_STATIC_SCRATCH_BYTES (32u << 20)
size_t sssd_op_gemm_static_scratch_limit(void);
int sssd_op_gemm_static(const void *a_hi, const void *a_lo, const void *w_packed, int32_t M, int32_t N, int32_t K,
                        float *out, void *stream);

/* Largest M = B*(k+1) that the small-step GEMM kernel (pgemm_kernel) serves; steps above it run the
 * large-M kernels (qgemm_kernel up to 48 rows, qgemm16_kernel above).  For benchmarks. */
int32_t sssd_op_gemm_small_step_rows(void);

/* Name of the weight-streaming kernel that a GEMM of M rows launches (static string; for M > 160, of its
 * first pass of 160 rows): "pgemm_kernel", "qgemm_kernel" or "qgemm16_kernel". */
const char *sssd_op_gemm_kernel_name(int32_t M);

/* Measurement aid: one read-only pass over `bytes` (>= 16, src 16-byte aligned) of device memory by a
 * kernel that does nothing else, i.e. the read bandwidth a kernel can reach on this device, against
 * which the weight-streaming GEMMs (Table 2 linear rows: FLOPs:IO ~ b*s_q, so HBM-bound) are rated.
 * sink: device uint32 [4096], receives per-workgroup XORs of the data (keeps the loads live). */
int sssd_op_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

/* Table 2 attention row on a context's cache: q device fp32 [B][k+1][n_q_heads][head_dim]
 * (already rotated), lens device int32 [B] (the k+1 new K/V rows of `layer` must already be
 * in the cache at lens[b]..lens[b]+k, e.g. via sssd_kv_import); row j attends to cache rows
 * 0..lens[b]+j.  out device fp32 [B][k+1][n_q_heads*head_dim].  Uses the context's scratch. */
int sssd_op_attention(sssd_ctx *ctx, int32_t layer, int32_t B, int32_t k, const float *q, const int32_t *lens,
                      float *out, void *stream);

/* The row sampler of sssd_verify_step_tree_sampled on its own: logits device fp32 [rows][vocab],
 * uniforms device fp32 [rows], sampled device int32 [rows] out; `sampling` is host memory. */
int sssd_op_sample(const float *logits, int32_t rows, int32_t vocab, const sssd_sampling_params *sampling,
                   const float *uniforms, int32_t *sampled, void *stream);


/* The same sampler with a row spread over several workgroups when there are few rows (at most half as
 * many as the device has compute units): a step of B = 1 samples k+1 rows, and one compute unit needs
 * 10-15 us per pass over a 128k-token row.  The workgroups of a row merge what they find (maximum,
 * integer histogram bins, tie counts, member mass) through `scratch` and take the same decisions from the
 * same numbers, so the tokens are exactly those of sssd_op_sample.
 *   scratch  device, at least sssd_op_sample_scratch_bytes(rows) bytes (0: no scratch needed, may be
 *            NULL; the call then is sssd_op_sample), any contents; SSSD_ECAPACITY if it is smaller
 * The workgroups of a row wait for each other inside the kernel, which takes the device to itself (the
 * grid never exceeds the compute units); the wait is bounded: a row whose workgroups could not all meet
 * comes back as -1 instead of hanging the device.  sssd_verify_step_tree_sampled uses this form with
 * scratch from the context's workspace and reports such a failure as SSSD_EHIP from sssd_verify_sync. */
size_t sssd_op_sample_scratch_bytes(int32_t rows);
int sssd_op_sample_wide(const float *logits, int32_t rows, int32_t vocab, const sssd_sampling_params *sampling,
                        const float *uniforms, int32_t *sampled, void *scratch, size_t scratch_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SSSD_OPS_H */
