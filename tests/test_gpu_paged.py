"""Paged KV cache and continuous batching: a per-step block table maps (sequence row, block of 32
positions) to a page of the pool.  The arithmetic does not depend on where pages live, so a step
through a shuffled table must be bit-identical to the same step on contiguous runs; and a sequence
must keep its state when it moves to another row between steps (the batched serving the paper
targets admits and retires sequences between steps)."""
import pytest
import torch

import oracle
from harness import Pair, compare_step, compare_tree_step, step_tree
from paper_2411_05894_amd import binding as sv
from sssd_synth import MODEL_SHAPES, uniform_int

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def shuffled_table(seed, max_batch, bps, n_pages):
    """Every (row, block) gets its own page: a seeded permutation of the pool."""
    keys = uniform_int(seed, 1, (n_pages,), 0, (1 << 30)).tolist()
    perm = sorted(range(n_pages), key=lambda i: (keys[i], i))
    return torch.tensor(perm[: max_batch * bps], dtype=torch.int32).view(max_batch, bps)


def test_shuffled_pages_are_bit_identical_to_contiguous_runs():
    s = MODEL_SHAPES["tiny"]
    B, k = 3, 7
    ctxs = [5, 40, 97]
    plain = Pair(s, seed=61, max_batch=B, max_k=k, max_seq=160, unit_gains=False)
    paged = Pair(s, seed=61, max_batch=B, max_k=k, max_seq=160, unit_gains=False)
    rows, bps, n_pages = sv.sssd_kv_geometry(paged.cfg)
    assert (rows, bps, n_pages) == (32, 5, 15)
    table = shuffled_table(62, B, bps, n_pages).to(DEV)
    paged.ctx.sssd_kv_set_block_table(table)
    for p in (plain, paged):
        for b in range(B):
            p.prefill_random_kv(63, b, ctxs[b], oracle_slot=b if p is plain else None)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    # a chain step
    tokens = uniform_int(64, 1, (B, k + 1), 0, s.vocab - 1)
    a, b_ = plain.step(tokens, lens), paged.step(tokens, lens)
    assert torch.equal(a["logits"], b_["logits"]) and torch.equal(a["accepted_len"], b_["accepted_len"])
    e, ex, r = compare_step(a, plain.oracle.verify_step(tokens, lens), tokens)
    # a tree step with commit, then a second step on the committed cache
    raw = uniform_int(65, 1, (B, k + 1), 0, 1 << 20).tolist()
    parents = torch.tensor([[0] + [raw[b][i] % i for i in range(1, k + 1)] for b in range(B)], dtype=torch.int32)
    ref = plain.oracle.verify_step_tree(tokens, parents, lens, compact=False)
    for b in range(B):                                   # plant one accepted child per sequence
        kid = max(c for c in range(1, k + 1) if int(parents[b, c]) == 0)
        tokens[b, kid] = int(ref["that"][b, 0])
    ta, tb = step_tree(plain, tokens, parents, lens), step_tree(paged, tokens, parents, lens)
    assert torch.equal(ta["logits"], tb["logits"]) and torch.equal(ta["path"], tb["path"])
    assert int(ta["accepted_len"].sum()) >= B
    la, lb = lens.to(DEV), lens.to(DEV)
    plain.ctx.sssd_kv_commit_tree(la, ta["dev"]["accepted_len"], ta["dev"]["path"])
    paged.ctx.sssd_kv_commit_tree(lb, tb["dev"]["accepted_len"], tb["dev"]["path"])
    assert torch.equal(la.cpu(), lb.cpu())
    nxt = ta["next_token"].view(B, 1).contiguous()
    a2, b2 = plain.step(nxt, la.cpu()), paged.step(nxt, lb.cpu())
    assert torch.equal(a2["logits"], b2["logits"])
    # the exported rows agree as well (export goes through the table)
    for b in range(B):
        n = int(la[b])
        Ka = torch.empty(s.n_kv_heads, n, s.head_dim, dtype=torch.bfloat16, device=DEV)
        Va, Kb, Vb = torch.empty_like(Ka), torch.empty_like(Ka), torch.empty_like(Ka)
        plain.ctx.sssd_kv_export(1, b, 0, Ka, Va)
        paged.ctx.sssd_kv_export(1, b, 0, Kb, Vb)
        assert torch.equal(Ka.view(torch.int16), Kb.view(torch.int16)) and torch.equal(Va.view(torch.int16), Vb.view(torch.int16))
    say(f"paged == contiguous bit for bit (chain, tree, commit, follow-up step); chain logit err vs oracle {e:.2e}")


def test_continuous_batching_rows_change_between_steps():
    """Four sequences A, B, C, D with their own pages.  Step 1 runs A, B, C in rows 0, 1, 2; then B is
    retired, D admitted, and step 2 runs C, D, A in rows 0, 1, 2.  The oracle keeps every sequence in a
    fixed slot; each library row must match the oracle's sequence of the same name."""
    s = MODEL_SHAPES["tiny"]
    k = 3
    p = Pair(s, seed=66, max_batch=4, max_k=k, max_seq=128)
    rows, bps, n_pages = sv.sssd_kv_geometry(p.cfg)
    owner = shuffled_table(67, 4, bps, n_pages)           # owner[x] = pages of sequence x (A..D = 0..3)
    ctxs = [33, 10, 64, 0]
    # prefill every sequence through row 0 of the table
    for x in range(4):
        table = torch.zeros(4, bps, dtype=torch.int32)
        table[0] = owner[x]
        p.ctx.sssd_kv_set_block_table(table.to(DEV))
        for l in range(s.n_layers):
            if ctxs[x]:
                from sssd_synth import make_kv_prefill
                K, V = make_kv_prefill(68 * 1000 + x, l, (s.n_kv_heads, ctxs[x], s.head_dim), device=DEV)
                p.ctx.sssd_kv_import(l, 0, 0, K, V)
                p.oracle.K[l, x, :, : ctxs[x]] = K.cpu()
                p.oracle.V[l, x, :, : ctxs[x]] = V.cpu()
        torch.cuda.synchronize()
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tok = uniform_int(69, 1, (4, k + 1), 0, s.vocab - 1)

    def run(order, tokens_all, lens_all):
        """order: sequence in each library row."""
        table = torch.zeros(4, bps, dtype=torch.int32)
        for row, x in enumerate(order):
            table[row] = owner[x]
        p.ctx.sssd_kv_set_block_table(table.to(DEV))
        t = tokens_all[order].contiguous()
        ln = lens_all[order].contiguous()
        gpu = p.step(t, ln)
        ref = p.oracle.verify_step(tokens_all, lens_all)          # all four, fixed slots
        sub = {key: ref[key][order] for key in ("logits", "that", "accepted_len", "next_token")}
        e, ex, r = compare_step(gpu, sub, t)
        return gpu, ref, e

    g1, r1, e1 = run([0, 1, 2], tok, lens)
    lens2 = lens + r1["accepted_len"] + 1                          # A, B, C advanced (D too in the oracle: harmless, reset below)
    lens2[3] = 0
    tok2 = uniform_int(70, 1, (4, k + 1), 0, s.vocab - 1)
    tok2[:, 0] = r1["next_token"]
    tok2[3] = uniform_int(71, 1, (k + 1,), 0, s.vocab - 1)         # D starts fresh
    g2, r2, e2 = run([2, 3, 0], tok2, lens2)
    say(f"continuous batching: logit err step 1 {e1:.2e}, step 2 (rows permuted, one retired, one admitted) {e2:.2e}")


def test_block_table_errors():
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=1, max_batch=2, max_k=2, max_seq=64)
    rows, bps, n_pages = sv.sssd_kv_geometry(p.cfg)
    table = torch.arange(2 * bps, dtype=torch.int32).view(2, bps)
    table[1, 0] = n_pages                                           # outside the pool
    p.ctx.sssd_kv_set_block_table(table.to(DEV))
    t = torch.zeros(2, 3, dtype=torch.int32, device=DEV)
    out = torch.zeros(2, dtype=torch.int32, device=DEV)
    p.ctx.sssd_verify_step(t, torch.tensor([0, 0], dtype=torch.int32, device=DEV), out, out.clone())
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    table[1, 0] = 3
    table[1, 1] = -7                                                # not touched by a step at lens 0, k 2
    p.ctx.sssd_kv_set_block_table(table.to(DEV))
    p.ctx.sssd_verify_step(t, torch.tensor([0, 0], dtype=torch.int32, device=DEV), out, out.clone())
    assert p.ctx.sssd_verify_sync() == 0
    # import / export / tree commit through a bad entry: the row is skipped on both sides and the flag is raised
    s_ = p.shape
    table[1, 1] = n_pages + 3
    p.ctx.sssd_kv_set_block_table(table.to(DEV))
    before = p.ctx.kv_cache.clone()
    K = torch.ones(s_.n_kv_heads, 40, s_.head_dim, dtype=torch.bfloat16, device=DEV)
    p.ctx.sssd_kv_import(0, 1, 0, K, K)                             # rows 0..31 go to page 3, rows 32..39 nowhere
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    out_k = torch.full_like(K, 7.0)
    p.ctx.sssd_kv_export(0, 1, 0, out_k, torch.full_like(K, 7.0))
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    assert torch.equal(out_k[:, :32], K[:, :32]) and bool((out_k[:, 32:] == 7.0).all())
    pages = lambda t: t.view(2, s_.n_layers, n_pages, -1)            # [K | V][layer][page][bytes]
    touched = (pages(p.ctx.kv_cache) != pages(before)).any(-1)
    assert bool(touched[:, 0, 3].all()) and int(touched.sum()) == 2   # page 3 of layer 0, in K and in V, and nothing else
    lens_d = torch.tensor([0, 30], dtype=torch.int32, device=DEV)
    acc_d = torch.tensor([0, 1], dtype=torch.int32, device=DEV)
    path_d = torch.tensor([[0, -1, -1], [0, 2, -1]], dtype=torch.int32, device=DEV)
    snap = p.ctx.kv_cache.clone()
    p.ctx.sssd_kv_commit_tree(lens_d, acc_d, path_d)                # sequence 1 would move row 32 -> 31 through the bad page
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    assert lens_d.tolist() == [1, 30] and torch.equal(p.ctx.kv_cache, snap)
    p.ctx.sssd_kv_set_block_table(None)
    p.ctx.sssd_verify_step(t, torch.tensor([0, 0], dtype=torch.int32, device=DEV), out, out.clone())
    assert p.ctx.sssd_verify_sync() == 0
