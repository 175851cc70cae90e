"""Pins of the drafter ORACLE (oracle/drafter.py) against what the paper and the mathematics fix:
n-gram counts by brute force, suffix-array lookups by linear scan of the text, a fusion example
worked by hand, structural invariants, and the source of every drafted path (App. A, Sec. 3.1-3.2)."""
import os
import random

import pytest

from oracle import drafter as od
from sssd_synth import repetitive_stream, uniform_int

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def occurrences(x, g):
    n = len(g)
    return sum(1 for s in range(len(x) - n + 1) if list(x[s: s + n]) == list(g))


def test_trie_counts_are_ngram_occurrence_counts():
    x = uniform_int(71, 1, (300,), 0, 5).tolist()
    t = od.InputTrie(6)
    t.append(x[:100])
    t.append(x[100:])                      # incremental updates give the same trie
    rng = random.Random(1)
    for _ in range(300):
        n = rng.randrange(1, 7)
        s = rng.randrange(0, len(x) - n)
        g = x[s: s + n]
        assert t.find(g).count == occurrences(x, g)
    assert t.find([0, 1, 2, 3, 4, 5, 0]) is None          # deeper than the trie
    # a node's count is the sum of its children's counts plus the occurrences that end the input
    for g in ([x[-1]], x[-2:], x[-3:]):
        node = t.find(g)
        assert node.count == sum(c.count for c in node.children.values()) + 1


def test_match_input_returns_every_suffix_of_the_tail():
    x = [7, 8, 9, 7, 8]
    t = od.InputTrie(8)
    t.append(x)
    res = t.match_input(4)
    assert [m for _, m in res] == [4, 3, 2, 1]
    assert [n.count for n, _ in res] == [1, 1, 2, 2]      # (8 9 7 8), (9 7 8), (7 8), (8)
    short = od.InputTrie(8)
    short.append([5, 6])
    assert [m for _, m in short.match_input(4)] == [2, 1]


def test_suffix_array_order_and_lookup_vs_linear_scan():
    text = uniform_int(72, 1, (400,), 0, 3).tolist()
    sub = od.SubIndex(text, 8)
    assert sorted(sub.sa) == list(range(len(text)))
    for a, b in zip(sub.sa, sub.sa[1:]):
        ka, kb = text[a: a + 8], text[b: b + 8]
        assert ka < kb or (ka == kb and a < b)            # list comparison: a proper prefix sorts first
    rng = random.Random(2)
    for _ in range(100):
        n = rng.randrange(1, 5)
        s = rng.randrange(0, len(text) - n)
        pre = text[s: s + n]
        want = sorted(i for i in range(len(text) - n + 1) if text[i: i + n] == pre)
        assert sorted(sub.positions(pre)) == want
        conts = sub.search(pre, 3)
        assert conts == [text[i + n: i + n + 3] for i in sub.positions(pre)]
        # suffix-array order makes the continuations non-decreasing
        assert all(a <= b for a, b in zip(conts, conts[1:]))
    assert sub.positions([9, 9]) == []


def test_get_cands_counts_and_interval_sampling():
    p = od.Params(prefix_len=3, branch_len=2, max_tree_nodes=10 ** 6)
    text = uniform_int(73, 1, (150,), 0, 2).tolist()
    tail = text[40:43]
    sub = od.SubIndex(text, 5)
    tree = od.get_cands([sub], tail, p)
    # few matches: every continuation is inserted, for prefix lengths 3 and 2
    want = {}
    for n in (3, 2):
        pre = tail[-n:]
        for i in range(len(text) - n + 1):
            if text[i: i + n] == pre:
                cont = text[i + n: i + n + 2]
                for d in range(1, len(cont) + 1):
                    want[tuple(cont[:d])] = want.get(tuple(cont[:d]), 0) + 1
    assert od.paths(tree) == want
    assert tree.token == tail[-1]
    # many matches: every step-th one, step = floor(matches / quota)
    text = [1, 2] * 250 + [3]
    sub = od.SubIndex(text, 6)
    p = od.Params(prefix_len=2, branch_len=2, max_samples=100)
    tree = od.get_cands([sub], [1, 2], p)
    matches = occurrences(text, [1, 2])
    assert matches == 250
    assert tree.count == len(range(0, matches, matches // 100))
    # two sub-indices share the sample budget
    tree2 = od.get_cands([sub, sub], [1, 2], p)
    assert tree2.count == 2 * len(range(0, matches, matches // 50))
    # the size test stops further rounds
    p_small = od.Params(prefix_len=4, branch_len=2, max_tree_nodes=2)
    t3 = od.get_cands([od.SubIndex([5, 6, 7, 8, 9, 1, 7, 8, 9, 2], 6)], [5, 6, 7, 8], p_small)
    assert od.paths(t3) == {(9,): 1, (9, 1): 1}            # only the length-4 round ran


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def test_fusion_example_worked_by_hand():
    g = read_golden("draft_fusion_example.txt")
    d = od.Drafter(od.Params(prefix_len=g["prefix_len"][0], branch_len=g["branch_len"][0]))
    d.input.append(g["input"])
    tokens, parents = d.propose(g["dec_len"][0])
    assert tokens == g["tokens"] and parents == g["parents"]
    assert d.propose(2) == ([2, 3], [0, 0])                 # dec_len counts the root
    assert d.propose(1) == ([2], [0])


def test_datastore_candidates_outrank_equal_input_candidates():
    """Alg. 3 scales input probabilities by 0.6 and leaves the datastore's alone."""
    d = od.Drafter(od.Params(prefix_len=2, branch_len=1))
    d.input.append([4, 5, 6, 4, 5])                         # input says 6 follows "4 5" (prob 1/2 * 0.6)
    d.datastore_add([4, 5, 7, 0, 4, 5, 7])                  # datastore says 7 (prob 1)
    tokens, parents = d.propose(3)
    assert tokens == [5, 7, 6] and parents == [0, 0, 0]


def path_of(tokens, parents, i):
    out = []
    while i != 0:
        out.append(tokens[i])
        i = parents[i]
    return out[::-1]


def test_draft_tree_invariants_and_sources():
    x = repetitive_stream(74, 1, 400, vocab=30)
    corpus = repetitive_stream(74, 2, 3000, vocab=30)        # shares no templates with x: seeded separately
    own = repetitive_stream(74, 1, 1500, vocab=30)           # same templates as x
    p = od.Params()
    d = od.Drafter(p)
    d.datastore_add(corpus)
    d.datastore_add(own)
    sizes = []
    for cut in (5, 40, 123, 250, 400):
        d.input = od.InputTrie(p.prefix_len + p.branch_len)
        d.input.append(x[:cut])
        for dec_len in (1, 4, 16, 32):
            tokens, parents = d.propose(dec_len)
            assert 1 <= len(tokens) <= dec_len and tokens[0] == x[cut - 1] and parents[0] == 0
            for i in range(1, len(tokens)):
                assert 0 <= parents[i] < i
            for i in range(len(tokens)):
                kids = [tokens[c] for c in range(1, len(tokens)) if parents[c] == i]
                assert len(kids) == len(set(kids))
            for i in range(1, len(tokens)):
                path = path_of(tokens, parents, i)
                assert len(path) <= p.branch_len
                # the path follows some suffix of the tail somewhere in the input or the datastore
                ok = False
                for m in range(1, p.prefix_len + 1):
                    gram = x[cut - m: cut] + path
                    if m <= cut and (occurrences(x[:cut], gram) or occurrences(corpus, gram) or occurrences(own, gram)):
                        ok = True
                assert ok, (cut, dec_len, path)
            sizes.append(len(tokens))
    assert max(sizes) == 32                                  # the repetitive stream really fills the budget


def test_periodic_input_drafts_its_own_continuation():
    period = [11, 12, 13, 14, 15, 16, 17]
    d = od.Drafter(od.Params())
    d.input.append(period * 4 + period[:3])
    tokens, parents = d.propose(5)
    assert tokens == [13, 14, 15, 16, 17] and parents == [0, 0, 1, 2, 3]


def test_speculation_length_rule():
    # the paper's example (App. B / Sec. 3.2): 165 TFLOP/s, 0.95 TB/s, b = 8 -> 22
    g = [l.split() for l in open(os.path.join(GOLDEN, "knee_example.txt")) if not l.startswith("#") and l.strip()][0]
    tf, tb, b, s_q = float(g[1]), float(g[2]), int(g[3]), int(g[5])
    assert od.speculation_length(tf * 1e12, tb * 1e12, b, 64) == s_q
    assert od.speculation_length(tf * 1e12, tb * 1e12, 1, 32) == 32      # capped
    assert od.speculation_length(tf * 1e12, tb * 1e12, 1000, 32) == 1    # never below the root itself
