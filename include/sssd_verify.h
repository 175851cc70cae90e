/*
 * sssd_verify.h -- C ABI of the SSSD verification step on one MI355X (gfx950).
 *
 * The paper (SSSD, arXiv 2411.05894) drafts candidate tokens on the host and
 * has the target model check them in one forward pass over the newest accepted
 * token followed by the drafts (Sec. 2; Sec. 3.2, first paragraph).  This
 * library is that device-side step for k drafts per sequence, given as a
 * linear chain (sssd_verify_step) or as a draft tree (sssd_verify_step_tree):
 * one pass of a Llama-style decoder over b sequences x s_q = k+1
 * tokens (the operations of Table 2, App. B, with p = 1), K/V of all k+1 rows
 * appended in place to a per-sequence cache, then greedy acceptance.
 *
 * Conventions
 *  - "device" pointers are HIP device memory owned by the CALLER; the library
 *    never allocates or frees device memory.  "host" pointers are ordinary
 *    process memory.
 *  - All weights are bf16 (2 bytes, Table 2 caption), matrices row-major
 *    [out][in] (the transpose of the paper's X.W orientation, same product).
 *  - Every function returns 0 (SSSD_OK) or a negative SSSD_E* code; nothing
 *    is printed and nothing aborts.  sssd_strerror() names a code.
 *  - Calls that take a `stream` only enqueue work on that hipStream_t (passed
 *    as void*; NULL = the default stream) and return without waiting.
 */
#ifndef SSSD_VERIFY_H
#define SSSD_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSSD_OK 0
#define SSSD_EINVAL (-1)    /* null pointer, bad handle, unsupported shape            */
#define SSSD_ECAPACITY (-2) /* B > max_batch, k > max_k, buffer too small             */
#define SSSD_ENOSPACE (-3)  /* some lens[b] + k + 1 > max_seq, or a token id, parent or
                               page out of range (found on the device, reported by
                               sssd_verify_sync)                                       */
#define SSSD_EHIP (-4)      /* a HIP runtime call failed                              */

typedef struct sssd_ctx sssd_ctx; /* opaque, host memory owned by the library */

/* Model and capacity.  Notation of Table 2: hidden = h, n_q_heads = n_q,
 * n_kv_heads = n_kv, head_dim = d, ffn = h_mlp.  Supported: head_dim 64 or 128;
 * n_q_heads a multiple of n_kv_heads; hidden, n_q*d, n_kv*d, ffn, vocab multiples of 16;
 * max_k <= 31.  No biases, untied embedding / LM head, RMSNorm with eps inside the
 * square root, rotary embedding pairing element i with i + d/2 at angle
 * pos * rope_base^(-2i/d), softmax scale 1/sqrt(d), SwiGLU = silu(gate) * up. */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rms_eps, rope_base;
    int32_t max_batch; /* largest B of any step                                   */
    int32_t max_k;     /* largest number of drafts per sequence                   */
    int32_t max_seq;   /* KV rows kept per sequence (context + k+1 must fit)      */
} sssd_model_config;

/* Device pointers to the bf16 weights.  wq..mlp_norm are HOST arrays of
 * n_layers device pointers.  Shapes: embed, lm_head [vocab][hidden];
 * wq [n_q*d][hidden]; wk, wv [n_kv*d][hidden]; wo [hidden][n_q*d];
 * w_gate, w_up [ffn][hidden]; w_down [hidden][ffn]; norms [hidden]. */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *w_gate, *const *w_up, *const *w_down;
    const void *const *attn_norm, *const *mlp_norm;
} sssd_weights;

/* Flags of sssd_verify_init. */
#define SSSD_PACK_IN_PLACE 1u /* reorder each weight matrix inside the caller's own buffer
                                 (needs hidden, n_q*d and ffn to be multiples of 32);
                                 the caller's matrices are then in the library's private
                                 tile order until the process frees them                  */

/* Bytes the caller must provide for a configuration (host computation only): the KV cache of Table 2's
 * caption (2 bytes per element, b x n_kv x s_kv x d per layer for K and for V), the workspace of one pass of
 * App. B's operations over b x s_q rows, and the reordered copy of the 2-byte weights.
 * packed_weight_bytes is what `packed` must hold when SSSD_PACK_IN_PLACE is not
 * used (0 bytes are needed with it).  Any out pointer may be NULL. */
int sssd_verify_sizes(const sssd_model_config *cfg, size_t *kv_bytes, size_t *ws_bytes,
                      size_t *packed_weight_bytes);

/* Host computation only, no device needed: SSSD_OK when every launch of a step of B sequences x k
 * drafts fits the buffers sssd_verify_sizes asks for under cfg (row buffers, the split-K scratch each of
 * the five GEMM launchers plans at B*(k+1) rows, the attention partial slots), SSSD_ECAPACITY when B or
 * k exceed the configuration -- or when the sizing and a launcher's plan ever disagree, which is what
 * the host-side self-test sweeps for.  Follows the same statement of the step as sssd_verify_step
 * (Sec. 3.2: b sequences x s_q = k+1 positions per pass). */
int sssd_verify_plan_check(const sssd_model_config *cfg, int32_t B, int32_t k);

/*
 * Create a context for the decoder of App. B / Table 2 (the operations of one layer, p = 1) with the weights
 * given.  Synchronous (it waits for its own device work):
 *  - zero-fills kv_cache (device, >= kv_bytes) -- the cache layout is private,
 *    use sssd_kv_import / sssd_kv_export to move rows in and out;
 *  - reorders every weight matrix into the tile order the GEMM kernels stream,
 *    either into `packed` (device, >= packed_weight_bytes; the caller may free
 *    the original matrices afterwards, but not embed and the three norm
 *    vectors, which are used where they are) or in place (SSSD_PACK_IN_PLACE,
 *    packed may be NULL);
 *  - lays out `workspace` (device, >= ws_bytes, 256-byte aligned).
 * All buffers must outlive the context.  *out is written only on success.
 */
int sssd_verify_init(const sssd_model_config *cfg, const sssd_weights *weights, void *kv_cache,
                     size_t kv_bytes, void *workspace, size_t ws_bytes, void *packed,
                     size_t packed_bytes, uint32_t flags, sssd_ctx **out);

/*
 * One verification step, enqueued on `stream`.
 *   tokens       device int32 [B][k+1]; tokens[b][0] is the last accepted token
 *                (not yet in the cache), tokens[b][1..k] the drafts
 *   lens         device int32 [B]; valid cache rows of sequence b BEFORE the step
 *   accepted_len device int32 [B] out; number of drafts accepted, in 0..k: the
 *                longest prefix with tokens[b][i+1] == argmax(logits[b][i])
 *   next_token   device int32 [B] out; argmax(logits[b][accepted_len[b]]), the
 *                bonus token, so accepted drafts + next_token is exactly what greedy
 *                decoding emits.  Ties in argmax go to the lowest token id.
 * Sequence b is cache slot b (0 <= b < B <= max_batch).  The step writes K/V
 * rows lens[b] .. lens[b]+k of every layer and does NOT change lens; rows of
 * rejected drafts stay behind as dead data and are overwritten by the next
 * step (sssd_kv_rollback computes the new lens).
 * If some lens[b] is negative or lens[b] + k + 1 > max_seq, that sequence is
 * rejected: it writes NOTHING to the cache (every live row of every sequence
 * keeps its bits), it is computed as an empty context so that all accesses
 * stay in bounds, and its outputs are meaningless.  A token id outside
 * [0, vocab) is computed as token 0; the rows it writes (lens[b] ..
 * lens[b]+k) are dead rows in any case.  Either condition sets a sticky
 * device flag that makes the next sssd_verify_sync return SSSD_ENOSPACE.
 * Steps on the same context must be ordered (same stream, or synchronised).
 */
int sssd_verify_step(sssd_ctx *ctx, int32_t B, int32_t k, const int32_t *tokens,
                     const int32_t *lens, int32_t *accepted_len, int32_t *next_token,
                     void *stream);

/*
 * Commit or roll back, enqueued on `stream`: after verification only the accepted drafts and the token that
 * follows them extend a sequence (Sec. 2; Sec. 3.2), so the cache keeps accepted_len + 1 of the k + 1 rows a
 * step appended.  lens is device int32 [B], in-out.
 *   accepted_len != NULL: lens[b] += accepted_len[b] + 1  (root + accepted drafts stay)
 *   else new_lens != NULL: lens[b]  = new_lens[b]          (arbitrary rollback / chunked prefill)
 * No cache data moves: rows at or beyond lens[b] are simply dead.
 */
int sssd_kv_rollback(sssd_ctx *ctx, int32_t B, int32_t *lens, const int32_t *accepted_len,
                     const int32_t *new_lens, void *stream);

/*
 * One verification step over draft TREES, enqueued on `stream`.  The paper merges its
 * candidates into a draft tree and verifies all nodes in one pass under an attention mask
 * built from the tree (Sec. 3.1; the mask M of Table 2's attention row, App. B); a linear
 * chain (sssd_verify_step) is the tree in which node i's parent is node i-1.
 *   tokens        device int32 [B][k+1]; node 0 is the root = the last accepted token,
 *                 nodes 1..k the drafts
 *   parents       device int32 [B][k+1]; parents[b][i] in [0, i) for i >= 1 (entry 0 unused):
 *                 nodes are numbered so that a parent precedes its children
 *   accepted_len  device int32 [B] out; number of drafts on the accepted path, in 0..depth
 *   next_token    device int32 [B] out; arg-max after the last accepted node (bonus token)
 *   accepted_path device int32 [B][k+1] out; accepted_path[b][0] = 0, then the nodes
 *                 walked: from the current node step to the child whose token equals the
 *                 arg-max after the current node (the lowest node index if several children
 *                 carry that token) until none does; entries past accepted_len[b] are -1.
 *                 Accepted tokens + next_token is exactly what greedy decoding emits.
 * Node i attends to the old cache, its ancestors and itself; its rotary position is
 * lens[b] + depth(i); its K/V go to cache row lens[b] + i of every layer.  lens is not
 * changed: sssd_kv_commit_tree moves the accepted rows into place and advances lens.
 * Errors as for sssd_verify_step; a parent outside [0, i) is treated as i-1 and raises the
 * same sticky flag.
 */
int sssd_verify_step_tree(sssd_ctx *ctx, int32_t B, int32_t k, const int32_t *tokens,
                          const int32_t *parents, const int32_t *lens, int32_t *accepted_len,
                          int32_t *next_token, int32_t *accepted_path, void *stream);

/*
 * The tree step with SAMPLING instead of greedy acceptance, enqueued on `stream`.  The paper runs
 * SSSD beyond greedy decoding with a simplified speculative sampling that preserves the target
 * distribution without draft probabilities (Sec. 4.4: temperature 0.6, top-p 0.95; Fig. 5:
 * temperature 0.7, top-p 0.8, top-k 20).  An n-gram draft is a point mass, for which the
 * accept/resample rule of speculative sampling equals: draw ONE token t from the target
 * distribution of the current node; step to the child that carries t if there is one (the lowest
 * node index among equal tokens), else emit t and stop.  Per row the distribution is
 *   order O : logit descending, token id ascending among equal logits
 *   S_k     : the first top_k tokens of O (all if top_k == 0 or top_k >= vocab)
 *   w_i     : exp((logit_i - max logit) / temperature)
 *   S       : the shortest prefix of O, at least one token, whose w-sum reaches top_p * sum(w over S_k)
 *   sample  : r = u * sum(w over S); the first token of S in ascending token id whose running
 *             w-sum exceeds r.
 *   sampling       host; temperature > 0, top_k >= 0, 0 < top_p <= 1
 *   uniforms       device float [B][k+1]; u in [0, 1) for node i of sequence b (the caller's
 *                  random numbers: the library draws none)
 *   logits_scratch device float, at least B*(k+1)*vocab elements (the step's logits; also the
 *                  row order of sssd_debug_outputs)
 *   accepted_len / next_token / accepted_path as in sssd_verify_step_tree, with the sampled
 *   token in place of the arg-max.  Everything else (cache rows, positions, lens, errors) is
 *   identical to sssd_verify_step_tree; sssd_kv_commit_tree commits the step.
 */
typedef struct {
    float temperature;
    int32_t top_k; /* 0 = off */
    float top_p;   /* 1 = off */
} sssd_sampling_params;
int sssd_verify_step_tree_sampled(sssd_ctx *ctx, int32_t B, int32_t k, const int32_t *tokens,
                                  const int32_t *parents, const int32_t *lens,
                                  const sssd_sampling_params *sampling, const float *uniforms,
                                  float *logits_scratch, int32_t *accepted_len, int32_t *next_token,
                                  int32_t *accepted_path, void *stream);

/*
 * Commit a tree step, enqueued on `stream`: in every layer the K/V rows of the accepted nodes
 * accepted_path[b][1..n] (n = accepted_len[b]) move from cache rows lens[b] + node to rows
 * lens[b] + 1 .. lens[b] + n, so that the cache again holds one row per position; then
 * lens[b] += n + 1 (device int32 [B], in-out).  accepted_len / accepted_path are the outputs
 * of the tree step (device).  A path that is not strictly increasing within 1..k, or an
 * n outside 0..k, leaves that sequence untouched and raises the sticky flag
 * (sssd_verify_sync returns SSSD_ENOSPACE).
 */
int sssd_kv_commit_tree(sssd_ctx *ctx, int32_t B, int32_t k, int32_t *lens,
                        const int32_t *accepted_len, const int32_t *accepted_path, void *stream);

/*
 * Paged cache and continuous batching.  The cache of a layer is a pool of n_pages pages of
 * rows_per_page = 32 positions (all kv heads of one sequence); kv_bytes of sssd_verify_sizes covers
 * max_batch * blocks_per_seq pages, blocks_per_seq = ceil(max_seq / 32).  Without a block table
 * sequence b owns pages b*blocks_per_seq .. (b+1)*blocks_per_seq - 1 (one contiguous run each: the
 * behaviour described everywhere else in this header).  With a table, block i of sequence b
 * (positions 32i .. 32i+31) lives in page block_table[b*blocks_per_seq + i] of every layer, so
 * sequences of unequal length share the pool, and "sequence b" is whatever row b of the table says
 * in THIS step: a serving loop that admits and retires sequences between steps (the batched
 * serving the paper targets, Sec. 2 "Batching") only rewrites rows of the table and lens.
 *   block_table  device int32 [max_batch][blocks_per_seq], or NULL to return to contiguous runs.
 *                It is read on the device when each later call executes (steps, commit,
 *                import/export, sssd_op_attention), so it may be updated in stream order between
 *                calls; entries for blocks a step does not touch are ignored.  An entry outside
 *                [0, n_pages) that a step would use rejects that sequence as a bad lens does (it
 *                writes nothing to the cache; its reads are forced into the pool) and raises the
 *                sticky flag.  Two sequences of one step must not share a page they write.
 */
int sssd_kv_geometry(const sssd_model_config *cfg, int32_t *rows_per_page, int32_t *blocks_per_seq,
                     int32_t *n_pages);
int sssd_kv_set_block_table(sssd_ctx *ctx, const int32_t *block_table);

/* Wait for `stream`, then return SSSD_ENOSPACE if any step since the last call raised
 * the device flag (a sequence that does not fit its cache rows, a token id, parent or page out of
 * range) and clear it, SSSD_EHIP if the runtime reported an error or the row sampler of a sampled step
 * could not synchronise its workgroups (another kernel held part of the device; the step's outputs
 * are then meaningless), else SSSD_OK. */
int sssd_verify_sync(sssd_ctx *ctx, void *stream);

/* Parity aid.  logits != NULL: every following step also stores its fp32
 * logits to `logits`, device float [B*(k+1)][vocab] (row b*(k+1)+j).
 * hidden != NULL: and the residual stream after the last layer, device float
 * [B*(k+1)][hidden].  NULL switches a store off again. */
int sssd_debug_outputs(sssd_ctx *ctx, float *logits, float *hidden);
/* The logits half of sssd_debug_outputs alone (the hidden-state store keeps its setting). */
int sssd_debug_logits(sssd_ctx *ctx, float *logits);
/* that != NULL: every following step also stores the token the step itself chose per row, device
 * int32 [B*(k+1)] (row b*(k+1)+j): the arg-max the LM-head epilogue and the merge kernel compute
 * without materialising logits (lowest id among equal logits), or the drawn token in the sampled
 * step.  This is the vector the acceptance walk consumes, so a test can hold it against an
 * independent arg-max row by row.  NULL switches the store off. */
int sssd_debug_argmax(sssd_ctx *ctx, int32_t *that);

/*
 * Copy cache rows in (e.g. a prefilled prompt) or out, enqueued on `stream`.
 * src/dst are device bf16 [n_kv_heads][n_rows][head_dim] for cache slot b of
 * `layer`, covering rows t0 .. t0+n_rows-1 (t0 + n_rows <= max_seq).  With a block
 * table, a row whose block is mapped outside the pool is skipped (neither side is
 * written) and raises the sticky flag of sssd_verify_sync.
 */
int sssd_kv_import(sssd_ctx *ctx, int32_t layer, int32_t b, int32_t t0, int32_t n_rows,
                   const void *k_src, const void *v_src, void *stream);
int sssd_kv_export(sssd_ctx *ctx, int32_t layer, int32_t b, int32_t t0, int32_t n_rows,
                   void *k_dst, void *v_dst, void *stream);

/*
 * Timing aid for benchmarks.  With profiling on, sssd_verify_step brackets its
 * launches of each kernel class with HIP events on the step's stream (no other
 * change to the work).  sssd_profile_read waits for the stream and returns, per
 * class c < SSSD_PROF_CLASSES, the summed milliseconds ms[c] and launch counts
 * n[c] since profiling was switched on (host arrays), then resets them.
 */
#define SSSD_PROF_CLASSES 8
enum {
    SSSD_PROF_GEMM = 0,  /* all weight GEMMs                   */
    SSSD_PROF_ATTN = 1,  /* attention + its split combine      */
    SSSD_PROF_ELEM = 2,  /* embed, split-K epilogue launches   */
    SSSD_PROF_ACCEPT = 3  /* arg-max merge + prefix acceptance  */
};
int sssd_profile_enable(sssd_ctx *ctx, int32_t on);
int sssd_profile_read(sssd_ctx *ctx, void *stream, double *ms, int64_t *n);

int sssd_verify_destroy(sssd_ctx *ctx);
const char *sssd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SSSD_VERIFY_H */
