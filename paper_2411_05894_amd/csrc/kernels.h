// Private launcher interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include "common.h"

// ---------------------------------------------------------- elementwise ----
// Reorder a row-major bf16 matrix [N][K] into packed tiles (K padded to 32 with zeros).
hipError_t launch_pack_weight(const uint16_t *src, uint16_t *dst, int N, int K, hipStream_t s);

struct StepIO {
    const int32_t *tokens, *lens;
    int32_t *accepted_len, *next_token;
    int B, k;
    const int32_t *parents;   // draft trees [B][k+1] (node 0 = root, parents[b][i] < i), or nullptr: linear chains
    int32_t *path;            // tree steps: accepted root-to-node path [B][k+1] out (entries past accepted_len = -1)
};

// Per-row geometry of a step, written by the embedding kernel and read by the QKV epilogue and
// the attention kernel: node j of sequence b is row m = b*(k+1)+j; its K/V go to cache row
// pos_base[b] + j, its rotary position is rope_pos[m] = pos_base[b] + depth(j), and it attends to
// the old cache plus the new rows whose bit is set in anc[m] (itself and its ancestors).  A
// linear chain is the tree with parent(j) = j-1: depth j, bits 0..j.

// ------------------------------------------------------------ fused GEMMs ----
enum FusedEpilogue {
    FEPI_QKV = 0,    // RMSNorm scale, rotary embedding, Q operand packing, KV append; units = rotary tile pairs
    FEPI_RESID = 1,  // X += acc; packed X*gamma_next; sums of squares per 16 columns; units = single tiles
    FEPI_SWIGLU = 2, // RMSNorm scale, silu(gate)*up, operand packing; units = (gate tile, up tile)
    FEPI_LM = 3,     // RMSNorm scale, per-tile arg-max, optional logits; units = single tiles
    FEPI_STORE = 4   // out[m][n] = acc (kernel-level entry point only)
};

struct FusedGemmArgs {
    const u32x4 *A_hi, *A_lo;     // packed activations x*gamma (or attention output / SwiGLU output)
    const u32x4 *W0, *W1, *W2;    // QKV: wq, wk, wv; SWIGLU: gate, up; else W0
    int KT, NT, M;                // k tiles, n tiles of W0, valid rows
    int h, d, nq, nkv, seq_pad, k, q_rows_pad, vocab;
    float eps;
    const float *ssq_in;          // [M][h/16] sums of squares of the consumed stream (not RESID)
    float *X, *ssq_out;           // RESID: residual stream [M][h], sums of squares of the updated stream
    const uint16_t *gamma_next;   // RESID: gains of the norm that consumes the updated stream
    uint16_t *out_hi, *out_lo;    // RESID (K = h) / SWIGLU (KT_out k-tiles): packed operands of the next GEMM
    int KT_out;
    const float *rope_cs;         // QKV
    const int32_t *pos_base;      // QKV: cache row of (b, j) is pos_base[b] + j
    const int32_t *rope_pos;      // QKV: rotary position of row m
    uint16_t *Qp, *Qp_lo, *Kc, *Vc;  // Kc, Vc: this layer's cache pools
    KvGeom kv;                    // QKV: page geometry of the cache
    float *logits, *part_val;     // LM
    int *part_idx;
    // weight streamer (stream_gemm.hip)
    int n_units;                  // epilogue units: rotary tile pairs (QKV), gate/up tile pairs (SWIGLU), tiles (RESID, LM)
    int Ntot;                     // columns of the concatenated output: (nq+2nkv)*d, 2*ffn, h, vocab
    int n_cu;                     // compute units of the device
    float *out;                   // STORE: [M][Ntot] fp32
    float *partials;              // split-K scratch [J][part_rows][Ntot] fp32
    size_t partial_bytes;
    int *tail_count;              // M <= 32 with a split K: tail_slots arrival counters, zero between launches; with them
    int tail_slots;               // the last workgroup of a column group sums the slices itself (null: epilogue launch)
    int seg0, seg1;               // tiles of W0 and of W1 in the concatenated output (M > 16 kernel)
    int upw, J, part_rows, kps;   // filled in by the launcher: units per workgroup, K slices, rows per slice, k-tiles per slice
    int groups;                   // ... and column groups (M <= 32: the grid is groups * J workgroups)
};
// M <= stream_gemm_max_rows(): persistent weight streamer; NT must be the tile count of W0.
int stream_gemm_max_rows();
const char *stream_gemm_kernel_name(int M);   // the kernel that serves (the first pass of) a GEMM of M rows
size_t stream_gemm_partial_bytes(const Dims &D, int M);
size_t stream_gemm_scratch_bytes(int M, int N, int K);   // one GEMM (kernel-level entry point)
// Launches the weight-streaming kernel and records its plan (J, part_rows, ...) in `a`; when
// *needs_epilogue comes back true the results are split-K partials and launch_stream_epilogue
// must follow with the same `a`.  With t0/t1 non-null the dispatch stamps them at the kernel's own
// start and end (what a profiler reports as the kernel's duration).
hipError_t launch_stream_gemm(FusedGemmArgs &a, int epilogue, hipStream_t s, bool *needs_epilogue, hipEvent_t t0,
                              hipEvent_t t1);
hipError_t launch_stream_epilogue(const FusedGemmArgs &a, int epilogue, hipStream_t s);
hipError_t launch_fused_embed(const Dims &D, const StepIO &io, const KvGeom &kv, const uint16_t *embed, const uint16_t *gamma,
                              float *X, uint16_t *A_hi, uint16_t *A_lo, float *ssq, int32_t *pos_base, int32_t *rope_pos,
                              uint32_t *anc, int32_t *err_flag, hipStream_t s);

// Merge per-tile arg-max partials, then greedy acceptance (longest matching prefix of a chain, or
// the walk from the root of a draft tree when io.parents is set).
// With part_val == nullptr `that` already holds the target's choice per row (sampled tokens) and only the walk runs.
hipError_t launch_accept(const Dims &D, const StepIO &io, const float *part_val, const int *part_idx, int NT,
                         int32_t *that, hipStream_t s);
// One token per row drawn from softmax(logits / temperature) restricted by top_k (0: off) and top_p
// (1: off), with the caller's uniform number per row; sampling.hip states the exact definition.
// With scratch (sample_scratch_bytes(rows, n_cu) bytes) and few rows, a row is spread over a cluster of
// workgroups; *err gets bit 1 set if a cluster could not synchronise (its rows are then -1).  scratch_clean:
// the scratch is all zero or was last used by a launch that completed without such an error (a launch leaves
// its counters at zero); otherwise it is cleared first.
size_t sample_scratch_bytes(int rows, int n_cu);
hipError_t launch_sample_rows(const float *logits, int rows, int V, float temperature, int top_k, float top_p,
                              const float *uniforms, int32_t *sampled, void *scratch, size_t scratch_bytes, bool scratch_clean, int n_cu,
                              int32_t *err, hipStream_t s);
hipError_t launch_rollback(int B, int32_t *lens, const int32_t *accepted_len, const int32_t *new_lens,
                           hipStream_t s);
// Tree commit: in every layer move the K/V rows of the accepted nodes path[b][1..n] from cache rows
// lens[b] + path[b][i] to lens[b] + i, then lens[b] += n + 1.  Kc/Vc: whole cache (all layers).
hipError_t launch_kv_compact(const Dims &D, const KvGeom &kv, uint16_t *Kc, uint16_t *Vc, size_t kv_layer_elems, int B, int k,
                             int32_t *lens, const int32_t *accepted_len, const int32_t *path, int32_t *err_flag,
                             hipStream_t s);
hipError_t launch_kv_copy(const Dims &D, const KvGeom &kv, uint16_t *Kc_layer, uint16_t *Vc_layer, int b, int t0, int n_rows,
                          uint16_t *k_ext, uint16_t *v_ext, bool import, int32_t *err_flag, hipStream_t s);

// Kernel-level entry points only (parity tests, micro-benchmarks).
hipError_t launch_pack_act(const float *X, int M, int K, uint16_t *A_hi, uint16_t *A_lo, hipStream_t s);
hipError_t launch_unpack_act(const uint16_t *A_hi, const uint16_t *A_lo, int M, int K, float *X, hipStream_t s);
// Read-only stream over `bytes` of device memory (the achievable-bandwidth yardstick); sink holds
// STREAM_READ_SINK_WORDS words.
constexpr int STREAM_READ_SINK_WORDS = 4096;
hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int n_cu, hipStream_t s);
hipError_t launch_q_pack(const Dims &D, const float *q, int B, int k, uint16_t *Qp, uint16_t *Qp_lo, hipStream_t s);
hipError_t launch_lens(const Dims &D, int B, int k, const int32_t *lens, int32_t *pos_base, int32_t *rope_pos,
                       uint32_t *anc, int32_t *err_flag, hipStream_t s);

// ------------------------------------------------------------ attention ----
struct AttnArgs {
    const uint16_t *Qp;        // packed Q (bf16 hi part), one slab of q_rows_pad x d per (b, kv head)
    const uint16_t *Qp_lo;     // bf16 lo part: q ~= hi + lo
    const uint16_t *Kc, *Vc;   // this layer's cache pools
    KvGeom kv;                 // page geometry
    const int32_t *pos_base;   // validated lens
    const uint32_t *anc;       // [B*(k+1)] visible new rows of each query row (bit i = row pos_base + i)
    float *part_o;             // [b][kv head][n_splits][q_rows_pad][d]
    float *part_ml;            // [b][kv head][n_splits][q_rows_pad][2]  (running max in log2 units, sum)
    uint16_t *out_hi, *out_lo; // packed activations for the O projection (K = nq*d)
    int B, k;
    int chunk, n_splits;       // filled in by launch_attention: positions per workgroup, partial slots per (b, kv head)
};
// Positions per workgroup for a step of B sequences with `rows` query rows per kv head, and the most
// chunks per sequence any such step uses (sizes the partial buffers).
int attention_chunk(const Dims &D, int B, int rows);
int attention_splits(const Dims &D, int B);
hipError_t launch_attention(const Dims &D, const AttnArgs &a, hipStream_t s);
