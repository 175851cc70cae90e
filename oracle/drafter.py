"""Oracle of the SSSD host drafter -- TEST INFRASTRUCTURE ONLY.

Plain Python written from the paper's App. A: the input trie and its retrieval (Alg. 1), the
suffix-array datastore query with interval sampling (Alg. 2), and the priority-queue merge into
one draft tree (Alg. 3), each in the order and notation of the pseudocode, on dictionaries and
lists, with brute-force scans where the product uses binary search.  It shares no code with the
C++ drafter and is compared with it node by node in tests/test_drafter_parity.py.

The pseudocode is "logically equivalent, not exact" (App. A, first paragraph); the readings
taken where it leaves a choice:
  * node.prob = count(node) / count(parent(node)); the factors along a path telescope to
    count(v) / count(u), the definition given in the "Input tree" subsection;
  * children are visited in ascending token id; the queue returns the largest probability and,
    among equal probabilities, the element pushed first;
  * Alg. 2 shortens the ORIGINAL prefix by one token per round (lengths P, P-1, ..., 2) while the
    tree has fewer than `max_tree_nodes` nodes (the printed listing re-slices the already shortened
    prefix, which would skip lengths); every sub-index is sampled with step
    max(1, floor(|conts| / (max_samples // sub_indices)));
  * no draft node lies deeper than branch_len below the root (branch_len bounds the depth of a draft);
  * dec_len counts the root: it is the speculation length s_q of Sec. 3.2.

Pins (tests/test_oracle_drafter_pins.py): trie counts == brute-force n-gram occurrence counts;
suffix-array order == sorted suffixes and lookups == a linear scan; a fusion example worked by hand
(tests/golden/draft_fusion_example.txt); structural invariants of the draft tree; every root path of
a draft is a continuation that really follows a sub-prefix of the tail in one of the sources; the
knee example the paper prints.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple


@dataclass
class Params:
    prefix_len: int = 4            # P (Sec. 3.1.1)
    branch_len: int = 4            # max depth of a continuation
    max_tree_nodes: int = 50       # Alg. 2: |tree| < 50
    max_samples: int = 100         # Alg. 2: floor(|conts| / 100)
    max_sub_indices: int = 8       # Sec. 3.1.3
    input_discount: float = 0.6    # Alg. 3
    datastore_match: float = 4.0   # Alg. 3: <datastore_tree, 4>
    child_disc_base: float = 0.6   # Alg. 3: 0.6 + 0.1 * match
    child_disc_per_match: float = 0.1


@dataclass
class Node:
    token: int
    count: int = 0
    children: Dict[int, "Node"] = field(default_factory=dict)


def tree_insert(root: Node, cont: Sequence[int]) -> None:
    """Alg. 2's Insert (App. A, "Datastore"): missing nodes are added with count 1, the counts of
    the nodes already on the path are incremented; the root counts the inserted continuations."""
    root.count += 1
    node = root
    for t in cont:
        if t not in node.children:
            node.children[t] = Node(t, 0)
        node = node.children[t]
        node.count += 1


def tree_size(root: Node) -> int:
    return 1 + sum(tree_size(c) for c in root.children.values())


def paths(root: Node, prefix: Tuple[int, ...] = ()) -> Dict[Tuple[int, ...], int]:
    """Canonical form of a counted tree: path of tokens below the root -> count."""
    out: Dict[Tuple[int, ...], int] = {}
    for t, c in root.children.items():
        out[prefix + (t,)] = c.count
        out.update(paths(c, prefix + (t,)))
    return out


# ------------------------------------------------------------------ input ----
class InputTrie:
    """Trie over the prompt and the self-output (App. A, "Input tree"): inserting a sequence
    increments the count of every node on its path; every window of `depth` tokens of the input is
    inserted, so a node stores how often its n-gram occurred."""

    def __init__(self, depth: int):
        self.depth = depth
        self.root = Node(-1, 0)
        self.tokens: List[int] = []

    def append(self, toks: Sequence[int]) -> None:
        for t in toks:
            self.tokens.append(int(t))
            i = len(self.tokens) - 1
            # the n-grams that END at token i, one per start position
            for s in range(max(0, i - self.depth + 1), i + 1):
                node = self.root
                for u in self.tokens[s: i + 1]:
                    if u not in node.children:
                        node.children[u] = Node(u, 0)
                    node = node.children[u]
                node.count += 1
            self.root.count += 1

    def find(self, gram: Sequence[int]) -> Optional[Node]:
        node = self.root
        for t in gram:
            if t not in node.children:
                return None
            node = node.children[t]
        return node

    def match_input(self, P: int) -> List[Tuple[Node, int]]:
        """Alg. 1 (MatchInput) on the tail of the input."""
        prefix = self.tokens[-P:] if P <= len(self.tokens) else list(self.tokens)
        results = []
        it = 0
        while it < len(prefix):
            p = prefix[it:]
            node = self.root
            i = 0
            while i < len(p) and p[i] in node.children:
                node = node.children[p[i]]
                i += 1
            if i == len(p):
                results.append((node, len(p)))
            it += 1
        return results


# -------------------------------------------------------------- datastore ----
class SubIndex:
    """One suffix array (App. A, "Datastore"): the suffixes of the text in lexicographic order of
    their first `depth` tokens, ties by position."""

    def __init__(self, text: Sequence[int], depth: int):
        self.text = [int(t) for t in text]
        self.sa = sorted(range(len(self.text)), key=lambda i: (tuple(self.text[i: i + depth]), i))

    def search(self, prefix: Sequence[int], branch_len: int) -> List[List[int]]:
        """The continuations (up to branch_len tokens) of every occurrence of `prefix`, in
        suffix-array order.  A linear scan stands in for the two binary searches."""
        n = len(prefix)
        pre = list(prefix)
        return [self.text[i + n: i + n + branch_len] for i in self.sa if self.text[i: i + n] == pre]

    def positions(self, prefix: Sequence[int]) -> List[int]:
        n = len(prefix)
        pre = list(prefix)
        return [i for i in self.sa if self.text[i: i + n] == pre]


def get_cands(subs: Sequence[SubIndex], tail: Sequence[int], p: Params) -> Node:
    """Alg. 2 (GetCands) with the readings of the module docstring."""
    prefix = list(tail[-p.prefix_len:]) if len(tail) >= p.prefix_len else list(tail)
    tree = Node(prefix[-1], 0)
    if not subs:
        return tree
    quota = max(1, p.max_samples // len(subs))
    it = 0
    while it < len(prefix) - 1 and tree_size(tree) < p.max_tree_nodes:
        sub_prefix = prefix[it:]
        for sub in subs:
            conts = sub.search(sub_prefix, p.branch_len)
            step = max(1, len(conts) // quota)
            i = 0
            while i < len(conts):
                tree_insert(tree, conts[i])
                i += step
        it += 1
    return tree


# ------------------------------------------------------------------ fusion ----
def fuse(input_trees: Sequence[Tuple[Node, int]], datastore_tree: Optional[Node], root_token: int, dec_len: int,
         p: Params) -> Tuple[List[int], List[int]]:
    """Alg. 3: returns the draft tree as (tokens, parents), node 0 the root, parents first."""
    tokens, parents = [root_token], [0]
    kids: List[Dict[int, int]] = [{}]
    pq: List[Tuple[float, int, Node, float, int, int]] = []
    pushed = 0
    all_trees: List[Tuple[Optional[Node], float, bool]] = [(datastore_tree, p.datastore_match, True)]
    all_trees += [(node, float(match), False) for node, match in input_trees]
    for tree, match, is_ds in all_trees:
        if tree is None or not tree.children:
            continue
        node = tree
        for tok in sorted(node.children):
            child = node.children[tok]
            discount = 1.0 if is_ds else p.input_discount
            child_disc = p.child_disc_base + p.child_disc_per_match * match
            prob = (child.count / node.count) * 1.0 * discount
            heapq.heappush(pq, (-prob, pushed, child, child_disc, 0, 1))
            pushed += 1
    while pq and len(tokens) < dec_len:
        neg, _, node, child_disc, parent, depth = heapq.heappop(pq)
        prob = -neg
        # InsertTok: add the token under the parent unless it is there already
        if node.token in kids[parent]:
            new = kids[parent][node.token]
        else:
            new = len(tokens)
            tokens.append(node.token); parents.append(parent); kids.append({})
            kids[parent][node.token] = new
        if depth + 1 <= p.branch_len:
            for tok in sorted(node.children):
                child = node.children[tok]
                q = (child.count / node.count) * prob * child_disc
                heapq.heappush(pq, (-q, pushed, child, child_disc, new, depth + 1))
                pushed += 1
    return tokens, parents


class Drafter:
    """The three algorithms wired together for one sequence and a shared datastore."""

    def __init__(self, p: Optional[Params] = None):
        self.p = p or Params()
        self.input = InputTrie(self.p.prefix_len + self.p.branch_len)
        self.subs: List[SubIndex] = []

    def datastore_add(self, text: Sequence[int]) -> None:
        self.subs.append(SubIndex(text, self.p.prefix_len + self.p.branch_len))
        while len(self.subs) > self.p.max_sub_indices:
            self.subs.pop(0)

    def propose(self, dec_len: int) -> Tuple[List[int], List[int]]:
        tail = self.input.tokens
        ds = get_cands(self.subs, tail, self.p)
        matches = self.input.match_input(self.p.prefix_len)
        return fuse(matches, ds, tail[-1], dec_len, self.p)


def speculation_length(peak_flops: float, peak_bw: float, b: int, cap: int) -> int:
    """Sec. 3.2: s_q = I_knee / b to the nearest integer, clamped to [1, cap]."""
    return max(1, min(cap, int(peak_flops / peak_bw / b + 0.5)))
