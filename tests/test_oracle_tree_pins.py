"""Pins of the oracle's TREE verification (the paper verifies a draft tree with an explicit
attention mask: Sec. 3.1 and the caption / attention row of Table 2, App. B).  What the paper and
the mathematics fix: the masked softmax definition; a chain is a tree; a node depends only on its
root path, so every root-to-node path must equal plain sequential decoding of that path (Sec. 2:
exact output preserved); greedy acceptance on a tree is the longest root path the target's own
arg-max chain follows."""
import random

import numpy as np
import pytest
import torch

import oracle
from sssd_synth import MODEL_SHAPES, normal_bf16, uniform_int


def random_tree(rng: random.Random, k: int):
    """parents[0] = -1, parents[i] uniform in 0..i-1."""
    return [-1] + [rng.randrange(0, i) for i in range(1, k + 1)]


def ancestors(parents, j):
    out = []
    while True:
        out.append(j)
        if j == 0:
            return out[::-1]
        j = parents[j]


# ------------------------------------------------------------ tree helpers ----
def test_tree_mask_and_depths_closed_forms():
    k = 6
    chain = [-1] + list(range(k))
    assert oracle.tree_depths(chain) == list(range(k + 1))
    assert np.array_equal(oracle.tree_mask(chain), np.tril(np.ones((k + 1, k + 1), dtype=np.uint8)))
    star = [-1] + [0] * k
    assert oracle.tree_depths(star) == [0] + [1] * k
    m = np.eye(k + 1, dtype=np.uint8)
    m[:, 0] = 1
    assert np.array_equal(oracle.tree_mask(star), m)
    rng = random.Random(5)
    for _ in range(20):
        par = random_tree(rng, 9)
        mask, depth = oracle.tree_mask(par), oracle.tree_depths(par)
        for j in range(10):
            anc = ancestors(par, j)
            assert depth[j] == len(anc) - 1
            assert sorted(np.nonzero(mask[j])[0].tolist()) == anc


def test_masked_attention_row_vs_dense_brute_force():
    """softmax(q K^T / sqrt(d) + M) V with M in {0, -inf} written out in fp64 (Table 2, attention row)."""
    d, n = 16, 23
    q = normal_bf16(41, 1, (d,), 1.0).float() * 1.3
    K = normal_bf16(41, 2, (n, d), 1.0)
    V = normal_bf16(41, 3, (n, d), 1.0)
    rng = random.Random(3)
    for trial in range(6):
        mask = torch.tensor([1 if (rng.random() < 0.6 or t == 0) else 0 for t in range(n)], dtype=torch.uint8)
        add = torch.where(mask.bool(), 0.0, float("-inf")).double()
        s = (K.double() @ q.double()) / d ** 0.5
        s = s.float().double()              # the oracle rounds each score to fp32 once
        p = torch.softmax(s + add, dim=0)
        ref = (p[:, None] * V.double()).sum(0)
        got = oracle.attention_row_masked(q, K, V, mask)
        assert (got.double() - ref).abs().max().item() < 1e-6
    # all visible == the unmasked routine, bit for bit; one visible row returns that V row
    full = torch.ones(n, dtype=torch.uint8)
    assert torch.equal(oracle.attention_row_masked(q, K, V, full), oracle.attention_row(q, K, V, n))
    one = torch.zeros(n, dtype=torch.uint8)
    one[7] = 1
    assert torch.equal(oracle.attention_row_masked(q, K, V, one), V[7].float())


# ----------------------------------------------------------------- accept ----
def brute_force_accept(tokens, parents, that):
    """Enumerate every root path; valid iff each step's token is the parent's arg-max choice."""
    k = len(tokens) - 1
    best = [0]
    for j in range(1, k + 1):
        path = ancestors(parents, j)
        ok = all(tokens[path[i + 1]] == that[path[i]] for i in range(len(path) - 1))
        # with duplicate sibling tokens the lowest node index wins at every step
        ok = ok and all(not any(parents[c] == path[i] and tokens[c] == that[path[i]] for c in range(1, path[i + 1]))
                        for i in range(len(path) - 1))
        if ok and len(path) > len(best):
            best = path
    return len(best) - 1, that[best[-1]], best


def test_accept_tree_vs_enumeration_and_chain_special_case():
    rng = random.Random(11)
    for trial in range(300):
        k = rng.randrange(0, 9)
        par = random_tree(rng, k)
        tokens = [rng.randrange(0, 4) for _ in range(k + 1)]
        that = [rng.randrange(0, 4) for _ in range(k + 1)]
        assert oracle.accept_tree(tokens, par, that) == brute_force_accept(tokens, par, that)
    for trial in range(100):
        k = rng.randrange(0, 7)
        tokens = [rng.randrange(0, 3) for _ in range(k + 1)]
        that = [rng.randrange(0, 3) for _ in range(k + 1)]
        a, n = oracle.accept(tokens, that)
        a2, n2, path = oracle.accept_tree(tokens, [-1] + list(range(k)), that)
        assert (a, n) == (a2, n2) and path == list(range(a + 1))


# ------------------------------------------------------------ whole model ----
def prefilled(shape, seed, n_ctx, max_batch=1, max_seq=96):
    m = oracle.build_model(shape, seed=seed, max_batch=max_batch, max_seq=max_seq)
    prompt = uniform_int(seed, 77, (n_ctx,), 0, shape.vocab - 1)
    for b in range(max_batch):
        for t in range(n_ctx):
            m.decode_token(b, int(prompt[t]), t)
    return m


def test_chain_as_tree_is_bit_identical_to_the_chain_pass(tiny_shape):
    k, n_ctx = 5, 9
    a, b = prefilled(tiny_shape, 1, n_ctx), prefilled(tiny_shape, 1, n_ctx)
    tokens = uniform_int(2, 78, (1, k + 1), 0, tiny_shape.vocab - 1)
    lens = torch.tensor([n_ctx], dtype=torch.int32)
    ref = a.verify_step(tokens, lens)
    got = b.verify_step_tree(tokens, torch.tensor([[-1] + list(range(k))]), lens, compact=False)
    assert torch.equal(ref["logits"], got["logits"])
    assert torch.equal(a.K, b.K) and torch.equal(a.V, b.V)
    assert int(ref["accepted_len"][0]) == int(got["accepted_len"][0])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_every_root_path_equals_sequential_decode(tiny_shape, seed):
    """A node's logits depend on its root path only and equal decoding that path token by token
    (the model sees the same tokens at the same positions): bit for bit, for every node."""
    k, n_ctx = 7, 6
    rng = random.Random(seed)
    par = random_tree(rng, k)
    tokens = uniform_int(seed, 79, (1, k + 1), 0, tiny_shape.vocab - 1)
    tree = prefilled(tiny_shape, seed, n_ctx)
    out = tree.verify_step_tree(tokens, torch.tensor([par]), torch.tensor([n_ctx], dtype=torch.int32), compact=False)
    for j in range(k + 1):
        seq = prefilled(tiny_shape, seed, n_ctx)
        path = ancestors(par, j)
        for depth, node in enumerate(path):
            logits = seq.decode_token(0, int(tokens[0, node]), n_ctx + depth)
        assert torch.equal(logits, out["logits"][0, j]), f"node {j} (path {path})"


@pytest.mark.parametrize("kind", ["truth_plus_noise", "random"])
def test_tree_speculative_loop_equals_greedy_loop(tiny_shape, kind):
    """Drafting trees of any quality and verifying them emits exactly the greedy stream, and the
    compacted cache equals the cache of plain decoding (Sec. 2: exact output preserved)."""
    n_ctx, n_new, k = 5, 14, 6
    prompt = uniform_int(4, 77, (n_ctx,), 0, tiny_shape.vocab - 1)
    # greedy reference: rows 0..n_ctx-2 prefilled, then decode from the last prompt token on
    stream = []
    ref = prefilled(tiny_shape, 4, n_ctx - 1, max_seq=64)
    tok = int(prompt[n_ctx - 1])
    pos = n_ctx - 1
    for _ in range(n_new + k + 2):
        logits = ref.decode_token(0, tok, pos)
        tok = oracle.argmax(logits)
        stream.append(tok)
        pos += 1
    spec = prefilled(tiny_shape, 4, n_ctx - 1, max_seq=64)
    rng = random.Random(9)
    emitted, last, ln = [], int(prompt[n_ctx - 1]), n_ctx - 1
    while len(emitted) < n_new:
        par = random_tree(rng, k)
        toks = [last] + [rng.randrange(0, tiny_shape.vocab) for _ in range(k)]
        if kind == "truth_plus_noise":
            # plant the true continuation along one root path, noise elsewhere
            leaf = rng.randrange(1, k + 1)
            path = ancestors(par, leaf)
            for depth, node in enumerate(path[1:]):
                toks[node] = stream[len(emitted) + depth]
        out = spec.verify_step_tree(torch.tensor([toks]), torch.tensor([par]), torch.tensor([ln], dtype=torch.int32))
        acc, path = int(out["accepted_len"][0]), out["path"][0]
        emitted += [toks[n] for n in path[1:]] + [int(out["next_token"][0])]
        ln += acc + 1
        last = emitted[-1]
    assert emitted[:n_new] == stream[:n_new]
    # cache rows 0..ln-1 of the speculative run == plain decoding of the same tokens
    full = prefilled(tiny_shape, 4, n_ctx - 1, max_seq=64)
    seq_tokens = [int(prompt[n_ctx - 1])] + emitted[:-1]
    for i, t in enumerate(seq_tokens[: ln - (n_ctx - 1)]):
        full.decode_token(0, t, n_ctx - 1 + i)
    assert torch.equal(full.K[:, 0, :, :ln], spec.K[:, 0, :, :ln])
    assert torch.equal(full.V[:, 0, :, :ln], spec.V[:, 0, :, :ln])
