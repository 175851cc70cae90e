/*
 * sssd_draft.h -- C ABI of the host-side drafter of SSSD (arXiv 2411.05894).
 *
 * The paper keeps drafting on the host (Sec. 3.1): the last tokens of a sequence
 * (the draft prefix) are matched against two n-gram sources -- a trie over the
 * prompt and the sequence's own output (Sec. 3.1.1, App. A Alg. 1) and a datastore
 * of suffix arrays over earlier text (Sec. 3.1.2 / 3.1.3, App. A Alg. 2) -- and the
 * continuations found are merged through a priority queue into one draft tree
 * (Sec. 3.1.4, App. A Alg. 3), which sssd_verify_step_tree then verifies.  The
 * speculation length follows the roofline rule s_q = I_knee / b (Sec. 3.2).
 *
 * Everything here is HOST code and every pointer is HOST memory owned by the
 * caller; the drafter owns its tries and suffix arrays.  Functions return 0
 * (SSSD_OK) or a negative SSSD_E* code of sssd_verify.h.  A drafter is not
 * thread-safe; different drafters are independent.
 */
#ifndef SSSD_DRAFT_H
#define SSSD_DRAFT_H

#include "sssd_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sssd_drafter sssd_drafter; /* opaque */

/* Constants of App. A, with the values the paper prints as defaults. */
typedef struct {
    int32_t prefix_len;     /* P, tokens of the tail matched against both sources (4, Sec. 3.1.1)  */
    int32_t branch_len;     /* max depth of a continuation below the root (Alg. 2, Alg. 3)         */
    int32_t max_tree_nodes; /* the datastore tree stops being extended at this size (50, Alg. 2)   */
    int32_t max_samples;    /* continuations sampled per datastore query, at regular intervals
                               over the sorted matches (100, Alg. 2 / Sec. 3.1.3), shared equally
                               by the sub-indices                                                  */
    int32_t max_sub_indices;/* suffix arrays kept; adding one more drops the oldest (cap 8)        */
    double input_discount;  /* scale of probabilities that come from the input (0.6, Alg. 3)       */
    double datastore_match; /* match length attributed to the datastore tree (4, Alg. 3)           */
    double child_disc_base; /* child discount = base + per_match * match length (0.6, 0.1, Alg. 3) */
    double child_disc_per_match;
} sssd_draft_params;

void sssd_draft_default_params(sssd_draft_params *p);

/* n_sequences independent inputs (one trie each) sharing one datastore. */
int sssd_draft_create(const sssd_draft_params *p, int32_t n_sequences, sssd_drafter **out);
int sssd_draft_destroy(sssd_drafter *d);

/* Input of sequence `seq` (prompt, then every accepted token): forget it / append n tokens.
 * After appending token i every n-gram of up to prefix_len + branch_len tokens that ends at i
 * has its trie count incremented, so a node's count is the number of occurrences of its n-gram. */
int sssd_draft_input_reset(sssd_drafter *d, int32_t seq);
int sssd_draft_input_append(sssd_drafter *d, int32_t seq, const int32_t *tokens, int32_t n);

/* Add one sub-index: a suffix array over tokens[0..n) (copied).  Suffixes are ordered
 * lexicographically by their first prefix_len + branch_len tokens, then by position. */
int sssd_draft_datastore_add(sssd_drafter *d, const int32_t *tokens, int64_t n);

/*
 * Draft tree for the current tail of sequence `seq` (Alg. 3): at most dec_len nodes INCLUDING
 * the root, so dec_len is the speculation length s_q of Sec. 3.2.  tokens[0] is the last input
 * token (the root), parents[0] = 0; node i >= 1 has parents[i] < i: the layout
 * sssd_verify_step_tree takes.  tokens and parents hold dec_len entries; *n_nodes gets the
 * number written (>= 1).  An empty input is SSSD_EINVAL.
 */
int sssd_draft_propose(sssd_drafter *d, int32_t seq, int32_t dec_len, int32_t *tokens, int32_t *parents,
                       int32_t *n_nodes);

/* s_q = I_knee / b rounded to the nearest integer, I_knee = peak_flops / peak_bytes_per_s, clamped
 * to [1, cap] (Sec. 3.2: the budget is capped, e.g. 32 at b = 1; App. B's example: 173.7 / 8 -> 22). */
int32_t sssd_draft_speculation_length(double peak_flops, double peak_bytes_per_s, int32_t b, int32_t cap);

/* ---- introspection for tests (the same numbers the algorithms use) ---- */
/* Count stored for the n-gram gram[0..n) in the trie of `seq` (0 if absent or n > depth). */
int64_t sssd_draft_input_count(const sssd_drafter *d, int32_t seq, const int32_t *gram, int32_t n);
/* The matches Alg. 1 looks for: suffixes of the sequence (at most prefix_len tokens long) that are
 * n-grams of its trie, as the library tracks them while appending; match_len[i] = length of the
 * i-th, longest first; returns how many (<= prefix_len), or a negative code. */
int32_t sssd_draft_match_input(const sssd_drafter *d, int32_t seq, int32_t *match_len);
/* Suffix-array range of `prefix` in sub-index `sub` (0 = oldest): positions in the token array
 * of the matching suffixes in suffix-array order, at most max_out of them; *total = their number. */
int sssd_draft_datastore_lookup(const sssd_drafter *d, int32_t sub, const int32_t *prefix, int32_t n,
                                int64_t *positions, int64_t max_out, int64_t *total);
/* Alg. 2 on the tail of `seq`: the datastore tree flattened in insertion order.
 * tokens/parents/counts must hold 1 + 2 * prefix_len * max_samples * branch_len entries (a round
 * samples up to twice max_samples continuations before the size test); node 0 is the root,
 * whose count is the number of continuations inserted. */
int sssd_draft_datastore_tree(const sssd_drafter *d, int32_t seq, int32_t *tokens, int32_t *parents,
                              int64_t *counts, int32_t *n_nodes);

#ifdef __cplusplus
}
#endif
#endif /* SSSD_DRAFT_H */
