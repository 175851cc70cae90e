"""GPU parity of TREE verification (the paper verifies a draft tree under an explicit attention
mask: Sec. 3.1, Table 2 attention row) against the CPU oracle, through the C ABI."""
import random

import pytest
import torch

import oracle
from harness import LOGIT_TOL, Pair, compare_step, compare_tree_step, step_tree
from paper_2411_05894_amd import binding as sv
from sssd_synth import MODEL_SHAPES, uniform_int

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def seeded_tree(seed: int, tid: int, k: int):
    """parents[0] = 0 (unused), parents[i] uniform in 0..i-1, from the shared counter hash."""
    raw = uniform_int(seed, tid, (k + 1,), 0, 1 << 20).tolist()
    return [0] + [raw[i] % i for i in range(1, k + 1)]


def plant_greedy_path(p: Pair, tokens: torch.Tensor, parents: torch.Tensor, lens: torch.Tensor, depth: int):
    """Rewrite draft tokens so that, per sequence, a root path of up to `depth` nodes carries the
    oracle's own greedy continuation (a node's logits depend only on its root path, so the path
    is planted one level per oracle pass).  The oracle's cache rows written here are dead rows."""
    B, sq = tokens.shape
    cur = [0] * B
    for _ in range(depth):
        ref = p.oracle.verify_step_tree(tokens, parents, lens, compact=False)
        moved = False
        for b in range(B):
            kids = [c for c in range(1, sq) if int(parents[b, c]) == cur[b]]
            if kids:
                tokens[b, kids[-1]] = int(ref["that"][b, cur[b]])   # the highest-numbered child: path != node order
                cur[b] = kids[-1]
                moved = True
        if not moved:
            break
    return tokens


def test_tree_step_random_trees_vs_oracle():
    s = MODEL_SHAPES["tiny"]
    B, k = 4, 9
    p = Pair(s, seed=21, max_batch=B, max_k=k, max_seq=160, unit_gains=False)
    ctxs = [0, 17, 40, 100]
    for b in range(B):
        p.prefill_random_kv(23, b, ctxs[b], oracle_slot=b)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    parents = torch.tensor([seeded_tree(24, b, k) for b in range(B)], dtype=torch.int32)
    tokens = uniform_int(25, 1, (B, k + 1), 0, s.vocab - 1)
    tokens = plant_greedy_path(p, tokens, parents, lens, depth=4)
    ref = p.oracle.verify_step_tree(tokens, parents, lens, compact=False)
    gpu = step_tree(p, tokens, parents, lens)
    e, ex, r = compare_tree_step(gpu, ref, tokens, parents)
    accepted = [int(a) for a in ref["accepted_len"]]
    say(f"tree step: worst logit err {e:.2e}, exempt rows {ex}/{r}, accepted {accepted}, trees {parents.tolist()}")
    assert sum(accepted) >= B                      # the planted paths are really accepted
    assert ex < r // 2


def test_largest_tree_and_degenerate_trees():
    """k = 31 (32 nodes: every bit of the visibility word), a star (all drafts children of the root),
    an empty context, and k = 0 (the root alone)."""
    s = MODEL_SHAPES["tiny"]
    B, k = 3, 31
    p = Pair(s, seed=23, max_batch=B, max_k=k, max_seq=128)
    ctxs = [0, 1, 64]
    for b in range(B):
        p.prefill_random_kv(28, b, ctxs[b], oracle_slot=b)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    parents = torch.tensor([seeded_tree(29, 0, k), [0] * (k + 1), [0] + list(range(k))], dtype=torch.int32)
    tokens = uniform_int(30, 1, (B, k + 1), 0, s.vocab - 1)
    tokens = plant_greedy_path(p, tokens, parents, lens, depth=3)
    ref = p.oracle.verify_step_tree(tokens, parents, lens, compact=False)
    gpu = step_tree(p, tokens, parents, lens)
    e, ex, r = compare_tree_step(gpu, ref, tokens, parents)
    say(f"k=31 trees: worst logit err {e:.2e}, exempt rows {ex}/{r}, accepted {ref['accepted_len'].tolist()}")
    # k = 0: the tree is the root
    t0 = tokens[:, :1].contiguous()
    p0 = parents[:, :1].contiguous()
    ref0 = p.oracle.verify_step_tree(t0, p0, lens, compact=False)
    gpu0 = step_tree(p, t0, p0, lens)
    compare_tree_step(gpu0, ref0, t0, p0)
    assert gpu0["accepted_len"].tolist() == [0, 0, 0] and gpu0["path"].tolist() == [[0], [0], [0]]


def test_chain_given_as_tree_is_the_chain_step():
    """parent(i) = i-1: the same kernels on the same geometry, so logits are bit-identical."""
    s = MODEL_SHAPES["tiny"]
    B, k = 3, 6
    p = Pair(s, seed=22, max_batch=B, max_k=k, max_seq=96)
    ctxs = [5, 33, 64]
    for b in range(B):
        p.prefill_random_kv(26, b, ctxs[b])
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(27, 1, (B, k + 1), 0, s.vocab - 1)
    parents = torch.tensor([[0] + list(range(k))] * B, dtype=torch.int32)
    a = p.step(tokens, lens)
    la = a["logits"].clone()
    t = step_tree(p, tokens, parents, lens)
    assert torch.equal(la, t["logits"])
    assert torch.equal(a["accepted_len"], t["accepted_len"]) and torch.equal(a["next_token"], t["next_token"])
    for b in range(B):
        n = int(t["accepted_len"][b])
        assert t["path"][b].tolist() == list(range(n + 1)) + [-1] * (k - n)


def test_tree_speculative_loop_emits_the_greedy_stream():
    """Chained tree steps with commit (cache compaction): the emitted tokens are the oracle's greedy
    stream, lens advance by accepted + 1, and the compacted cache rows equal the oracle's."""
    s = MODEL_SHAPES["tiny"]
    k, prompt_len, steps = 7, 48, 24
    max_seq = prompt_len + steps * (k + 1) + 8
    p = Pair(s, seed=31, max_batch=1, max_k=k, max_seq=max_seq)
    ref_model = oracle.build_model(s, 31, 1, max_seq)        # plain greedy decoding, its own cache
    prompt = uniform_int(32, 5, (prompt_len,), 0, s.vocab - 1)
    lens = 0
    while lens < prompt_len - 1:                              # prefill through the chain step, both sides
        n = min(k + 1, prompt_len - 1 - lens)
        chunk = prompt[lens: lens + n].view(1, n)
        p.step(chunk, torch.tensor([lens]))
        p.oracle.verify_step(chunk, torch.tensor([lens]))
        ref_model.verify_step(chunk, torch.tensor([lens]))
        lens += n
    # the greedy stream the loop must reproduce
    n_greedy = steps * (k + 1)
    greedy, t = [], int(prompt[-1])
    for i in range(n_greedy):
        t = oracle.argmax(ref_model.decode_token(0, t, prompt_len - 1 + i))
        greedy.append(t)
    rng = random.Random(7)
    dlens = torch.tensor([lens], dtype=torch.int32, device=DEV)
    last, emitted, worst, exempt, rows, acc_hist = int(prompt[-1]), [], 0.0, 0, 0, []
    for step in range(steps):
        # a draft tree: the true continuation for `good` levels (in shuffled node order), wrong siblings elsewhere
        good = rng.randrange(0, 5)
        parents, toks, spine = [0], [last] + [-1] * k, 0
        for i in range(1, k + 1):
            if rng.random() < 0.6:
                parents.append(spine)           # node i extends the spine
                spine = i
            else:
                parents.append(rng.randrange(0, i))
        # fill tokens: nodes on the spine get the true continuation while depth <= good, others random ids
        depth = oracle.tree_depths(parents)
        on = set()
        node = spine
        while node != 0:
            on.add(node)
            node = parents[node]
        base = len(emitted)
        for i in range(1, k + 1):
            if i in on and depth[i] <= good and base + depth[i] - 1 < len(greedy):
                toks[i] = greedy[base + depth[i] - 1]
            else:
                toks[i] = rng.randrange(0, s.vocab)
        tokens = torch.tensor([toks], dtype=torch.int32)
        par = torch.tensor([parents], dtype=torch.int32)
        cur_len = torch.tensor([lens], dtype=torch.int32)
        ref = p.oracle.verify_step_tree(tokens, par, cur_len, compact=True)
        gpu = step_tree(p, tokens, par, cur_len)
        e, ex, r = compare_tree_step(gpu, ref, tokens, par)
        worst, exempt, rows = max(worst, e), exempt + ex, rows + r
        n = int(ref["accepted_len"][0])
        path = ref["path"][0]
        if gpu["path"][0].tolist()[: int(gpu["accepted_len"][0]) + 1] == path:
            p.ctx.sssd_kv_commit_tree(dlens, gpu["dev"]["accepted_len"], gpu["dev"]["path"])
        else:                                   # an undecided row forked the walk: follow the oracle
            acc_d = torch.tensor([n], dtype=torch.int32, device=DEV)
            path_d = torch.tensor([path + [-1] * (k - n)], dtype=torch.int32, device=DEV)
            p.ctx.sssd_kv_commit_tree(dlens, acc_d, path_d)
        assert p.ctx.sssd_verify_sync() == 0
        emitted += [toks[i] for i in path[1:]] + [int(ref["next_token"][0])]
        acc_hist.append(n)
        lens += n + 1
        assert int(dlens.item()) == lens
        last = int(ref["next_token"][0])
        # the compacted rows of this step, all layers: library vs oracle (bf16 rows of values that differ
        # in the last fp32 bits may round differently: compare as numbers)
        if n > 0:
            for l in range(s.n_layers):
                Kb = torch.empty(s.n_kv_heads, n + 1, s.head_dim, dtype=torch.bfloat16, device=DEV)
                Vb = torch.empty_like(Kb)
                p.ctx.sssd_kv_export(l, 0, lens - n - 1, Kb, Vb)
                Ko = p.oracle.K[l, 0, :, lens - n - 1: lens].float()
                Vo = p.oracle.V[l, 0, :, lens - n - 1: lens].float()
                assert (Kb.cpu().float() - Ko).abs().max().item() <= 2e-2 * max(1.0, Ko.abs().max().item())
                assert (Vb.cpu().float() - Vo).abs().max().item() <= 2e-2 * max(1.0, Vo.abs().max().item())
    assert emitted == greedy[: len(emitted)]
    say(f"tree loop: {len(emitted)} tokens in {steps} steps (accepted {sum(acc_hist)}), worst logit err {worst:.2e}, "
        f"exempt rows {exempt}/{rows}")
    assert sum(acc_hist) >= steps // 2


def test_tree_error_reporting():
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=1, max_batch=2, max_k=4, max_seq=64)
    t = torch.zeros(2, 5, dtype=torch.int32, device=DEV)
    out = torch.zeros(2, dtype=torch.int32, device=DEV)
    path = torch.zeros(2, 5, dtype=torch.int32, device=DEV)
    lens = torch.tensor([10, 20], dtype=torch.int32, device=DEV)
    par = torch.tensor([[0, 0, 1, 1, 3], [0, 0, 0, 3, 2]], dtype=torch.int32, device=DEV)   # parents[1][3] = 3: not < 3
    p.ctx.sssd_verify_step_tree(t, par, lens, out, out.clone(), path)
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    assert p.ctx.sssd_verify_sync() == 0
    # commit with a path that does not increase: flagged, lens untouched
    acc = torch.tensor([2, 1], dtype=torch.int32, device=DEV)
    bad = torch.tensor([[0, 3, 2, -1, -1], [0, 4, -1, -1, -1]], dtype=torch.int32, device=DEV)
    l2 = lens.clone()
    p.ctx.sssd_kv_commit_tree(l2, acc, bad)
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    assert l2.cpu().tolist() == [10, 22]
    with pytest.raises(sv.SssdError) as ei:
        p.ctx.sssd_verify_step_tree(torch.zeros(2, 6, dtype=torch.int32, device=DEV),
                                    torch.zeros(2, 6, dtype=torch.int32, device=DEV), lens, out, out,
                                    torch.zeros(2, 6, dtype=torch.int32, device=DEV))
    assert ei.value.code == sv.SSSD_ECAPACITY
