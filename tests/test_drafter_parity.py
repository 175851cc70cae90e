"""The C++ host drafter (include/sssd_draft.h) against its Python oracle, node by node, on seeded
repetitive token streams (App. A, Alg. 1-3; Sec. 3.2).  Host code only: no GPU needed."""
import random

import pytest

from oracle import drafter as od
from paper_2411_05894_amd import binding as sv
from paper_2411_05894_amd import drafter as dr
from sssd_synth import repetitive_stream, uniform_int


def make_pair(**kw):
    """A C++ drafter and an oracle drafter with the same parameters."""
    cp = dr.default_params()
    op = od.Params()
    for k, v in kw.items():
        setattr(cp, k, v)
        setattr(op, k, v)
    return dr.Drafter(cp), od.Drafter(op)


def canonical(tokens, parents, counts):
    """path below the root -> count, from a flattened tree."""
    out = {}
    paths = {0: ()}
    for i in range(1, len(tokens)):
        paths[i] = paths[parents[i]] + (tokens[i],)
        out[paths[i]] = counts[i]
    return out


def test_default_params_are_the_papers_constants():
    p = dr.default_params()
    o = od.Params()
    for name in ("prefix_len", "branch_len", "max_tree_nodes", "max_samples", "max_sub_indices", "input_discount",
                 "datastore_match", "child_disc_base", "child_disc_per_match"):
        assert getattr(p, name) == getattr(o, name)
    assert (p.prefix_len, p.max_tree_nodes, p.max_samples, p.max_sub_indices) == (4, 50, 100, 8)
    assert (p.input_discount, p.datastore_match, p.child_disc_base, p.child_disc_per_match) == (0.6, 4.0, 0.6, 0.1)


def test_trie_counts_and_matches():
    x = repetitive_stream(81, 1, 500, vocab=12)
    c, o = make_pair()
    rng = random.Random(3)
    for lo, hi in ((0, 1), (1, 3), (3, 200), (200, 500)):
        c.sssd_draft_input_append(0, x[lo:hi])
        o.input.append(x[lo:hi])
        assert c.sssd_draft_match_input(0) == [m for _, m in o.input.match_input(4)]
        for _ in range(200):
            n = rng.randrange(1, 10)
            s = rng.randrange(0, max(1, hi - n))
            g = x[s: s + n]
            node = o.input.find(g)
            assert c.sssd_draft_input_count(0, g) == (node.count if node else 0)
    assert c.sssd_draft_input_count(0, [99, 98]) == 0
    c.sssd_draft_input_reset(0)
    assert c.sssd_draft_input_count(0, x[:1]) == 0


def test_suffix_array_lookup():
    text = repetitive_stream(82, 1, 5000, vocab=9)
    c, o = make_pair()
    c.sssd_draft_datastore_add(text)
    o.datastore_add(text)
    rng = random.Random(4)
    for _ in range(200):
        n = rng.randrange(1, 7)
        s = rng.randrange(0, len(text) - n)
        pre = text[s: s + n]
        pos, total = c.sssd_draft_datastore_lookup(0, pre)
        assert total == len(pos) and pos == o.subs[0].positions(pre)
    pos, total = c.sssd_draft_datastore_lookup(0, [8, 8, 8, 8, 8, 8, 8, 8])
    assert pos == o.subs[0].positions([8] * 8)
    # the tail of the text as a key: suffixes that end inside the key do not match
    pos, total = c.sssd_draft_datastore_lookup(0, text[-2:] + [0])
    assert pos == o.subs[0].positions(text[-2:] + [0])


@pytest.mark.parametrize("n_sub", [1, 3])
def test_datastore_tree(n_sub):
    c, o = make_pair()
    for i in range(n_sub):
        text = repetitive_stream(83, 1 + (i % 2), 4000, vocab=15, noise=0.02 * i)
        c.sssd_draft_datastore_add(text)
        o.datastore_add(text)
    x = repetitive_stream(83, 1, 300, vocab=15)
    for cut in (1, 2, 3, 7, 50, 299):
        c.sssd_draft_input_reset(0)
        c.sssd_draft_input_append(0, x[:cut])
        tok, par, cnt = c.sssd_draft_datastore_tree(0)
        tree = od.get_cands(o.subs, x[:cut], o.p)
        assert tok[0] == tree.token and cnt[0] == tree.count
        assert canonical(tok, par, cnt) == od.paths(tree)


@pytest.mark.parametrize("kw", [{}, {"prefix_len": 2, "branch_len": 6}, {"max_samples": 7, "max_tree_nodes": 8},
                                {"input_discount": 1.0, "datastore_match": 1.0}])
def test_draft_trees_are_identical(kw):
    c, o = make_pair(**kw)
    corpus_a = repetitive_stream(84, 1, 6000, vocab=40)
    corpus_b = repetitive_stream(84, 2, 2500, vocab=40)
    x = repetitive_stream(84, 1, 260, vocab=40, noise=0.1)
    step = 0
    for lo, hi in ((0, 1), (1, 2), (2, 5), (5, 60), (60, 61), (61, 180), (180, 260)):
        c.sssd_draft_input_append(0, x[lo:hi])
        o.input.append(x[lo:hi])
        if hi == 5:
            c.sssd_draft_datastore_add(corpus_a); o.datastore_add(corpus_a)
        if hi == 61:
            c.sssd_draft_datastore_add(corpus_b); o.datastore_add(corpus_b)
        for dec_len in (1, 2, 9, 17, 32):
            assert c.sssd_draft_propose(0, dec_len) == o.propose(dec_len), (kw, hi, dec_len)
            step += 1
    assert step == 35


def test_oldest_sub_index_is_dropped():
    c, o = make_pair(max_sub_indices=2)
    texts = [repetitive_stream(85, i + 1, 800, vocab=10) for i in range(3)]
    for t in texts:
        c.sssd_draft_datastore_add(t)
        o.datastore_add(t)
    assert len(o.subs) == 2
    pre = texts[2][10:12]
    assert c.sssd_draft_datastore_lookup(0, pre)[0] == o.subs[0].positions(pre)       # sub 0 is now the second text
    assert c.sssd_draft_datastore_lookup(1, pre)[0] == o.subs[1].positions(pre)
    with pytest.raises(sv.SssdError):
        c.sssd_draft_datastore_lookup(2, pre)


def test_sequences_are_independent_and_errors():
    c = dr.Drafter(n_sequences=2)
    c.sssd_draft_input_append(0, [1, 2, 3, 1, 2])
    c.sssd_draft_input_append(1, [7, 7, 7, 7])
    assert c.sssd_draft_propose(0, 4) == ([2, 3, 1, 2], [0, 0, 1, 2])
    assert c.sssd_draft_propose(1, 3) == ([7, 7, 7], [0, 0, 1])
    with pytest.raises(sv.SssdError):
        c.sssd_draft_propose(2, 4)                          # no such sequence
    c.sssd_draft_input_reset(1)
    with pytest.raises(sv.SssdError):
        c.sssd_draft_propose(1, 4)                          # empty input
    with pytest.raises(sv.SssdError):
        c.sssd_draft_propose(0, 0)
    bad = dr.default_params()
    bad.prefix_len = 0
    with pytest.raises(sv.SssdError):
        dr.Drafter(bad)


def test_speculation_length_matches_the_oracle_rule():
    for tf, tb in ((165e12, 0.95e12), (2.5e15, 8e12), (1e12, 1e12)):
        for b in (1, 2, 7, 8, 32, 500):
            for cap in (1, 16, 32, 64):
                assert dr.sssd_draft_speculation_length(tf, tb, b, cap) == od.speculation_length(tf, tb, b, cap)
    assert dr.sssd_draft_speculation_length(165e12, 0.95e12, 8, 64) == 22     # the paper's example
    assert dr.sssd_draft_speculation_length(2.5e15, 8e12, 1, 32) == 32        # MI355X ridge 312, capped
