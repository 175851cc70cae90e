"""The optional chained launch (O, gate/up, down and the next QKV / the LM head in one launch with
grid-wide barriers): same arithmetic in the same order, so every output must be bit-identical to
the separate launches, and it must meet the oracle like they do."""
import pytest
import torch

from harness import Pair, compare_step, compare_tree_step, step_tree
from paper_2411_05894_amd import binding as sv
from sssd_synth import MODEL_SHAPES, uniform_int

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def test_tiny_chain_matches_separate_launches_and_oracle():
    """Tiny shape (no GEMM splits K): chained steps of several sizes, a tree step, and a step too
    large for the chained launch (17 rows: it must fall back without a trace)."""
    s = MODEL_SHAPES["tiny"]
    B, k = 2, 7
    a = Pair(s, seed=71, max_batch=B, max_k=k + 1, max_seq=200, unit_gains=False)
    b = Pair(s, seed=71, max_batch=B, max_k=k + 1, max_seq=200, unit_gains=False)
    b.ctx.sssd_set_gemm_chain(True)
    ctxs = [33, 90]
    for p in (a, b):
        for i in range(B):
            p.prefill_random_kv(72, i, ctxs[i], oracle_slot=i if p is a else None)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    for step, kk in enumerate([7, 0, 3, 7, 8]):            # 8: M = 18 rows, not chained
        tokens = uniform_int(73, step, (B, kk + 1), 0, s.vocab - 1)
        ra, rb = a.step(tokens, lens), b.step(tokens, lens)
        assert torch.equal(ra["logits"], rb["logits"]) and torch.equal(ra["hidden"], rb["hidden"])
        assert torch.equal(ra["accepted_len"], rb["accepted_len"]) and torch.equal(ra["next_token"], rb["next_token"])
        if step == 0:
            e, ex, r = compare_step(rb, a.oracle.verify_step(tokens, lens), tokens)
            say(f"chain tiny: logit err vs oracle {e:.2e}, exempt {ex}/{r}")
    raw = uniform_int(74, 1, (B, k + 1), 0, 1 << 20).tolist()
    parents = torch.tensor([[0] + [raw[i][j] % j for j in range(1, k + 1)] for i in range(B)], dtype=torch.int32)
    tokens = uniform_int(74, 2, (B, k + 1), 0, s.vocab - 1)
    ta, tb = step_tree(a, tokens, parents, lens), step_tree(b, tokens, parents, lens)
    assert torch.equal(ta["logits"], tb["logits"]) and torch.equal(ta["path"], tb["path"])
    e, ex, r = compare_tree_step(tb, a.oracle.verify_step_tree(tokens, parents, lens, compact=False), tokens, parents)
    say(f"chain tiny tree: logit err vs oracle {e:.2e}, exempt {ex}/{r}")


def test_barrier_give_up_is_reported_and_the_context_recovers():
    """The error path, forced from the host: with a limit of one poll per barrier wait every workgroup
    of the chained launches leaves through the give-up branch (the kernels end normally).  The sync call must say so once; the context then runs separate launches, and the
    chain again when asked to, both bit-identical to a context that never failed."""
    s = MODEL_SHAPES["tiny"]
    B, k = 2, 5
    a = Pair(s, seed=81, max_batch=B, max_k=k, max_seq=120, unit_gains=False)
    b = Pair(s, seed=81, max_batch=B, max_k=k, max_seq=120, unit_gains=False)
    ctxs = [17, 64]
    for p in (a, b):
        for i in range(B):
            p.prefill_random_kv(82, i, ctxs[i])
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(83, 1, (B, k + 1), 0, s.vocab - 1)
    ref = a.step(tokens, lens)
    b.ctx.sssd_set_gemm_chain(True)
    b.ctx.sssd_debug_chain_wait(1)
    dev = b.dev
    t, ln = tokens.to(dev, torch.int32), lens.to(dev, torch.int32)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    b.ctx.sssd_verify_step(t, ln, acc, nxt)
    rc = b.ctx.sssd_verify_sync()
    assert rc == -4, rc                                   # SSSD_EHIP
    assert b.ctx.sssd_verify_sync() == 0                  # reported once
    got = b.step(tokens, lens)                            # separate launches now
    assert torch.equal(ref["logits"], got["logits"]) and torch.equal(ref["next_token"], got["next_token"])
    b.ctx.sssd_set_gemm_chain(True)                       # counters and epoch were started over
    for _ in range(2):
        got = b.step(tokens, lens)
        assert torch.equal(ref["logits"], got["logits"]) and torch.equal(ref["accepted_len"], got["accepted_len"])
    say("chain give-up: reported as SSSD_EHIP once, separate launches and the re-enabled chain bit-identical")


def test_chain_writes_the_paged_cache_like_the_separate_launches():
    """The chained launch's last phase is the next layer's QKV projection, whose epilogue appends K/V
    through the block table: with a shuffled table the step and the cache rows it leaves behind (read
    back through the table) must equal those of separate launches on the same table."""
    s = MODEL_SHAPES["tiny"]
    B, k = 3, 4
    a = Pair(s, seed=91, max_batch=B, max_k=k, max_seq=130, unit_gains=False)
    b = Pair(s, seed=91, max_batch=B, max_k=k, max_seq=130, unit_gains=False)
    rows, bps, n_pages = sv.sssd_kv_geometry(a.cfg)
    keys = uniform_int(92, 1, (n_pages,), 0, 1 << 30).tolist()
    perm = sorted(range(n_pages), key=lambda i: (keys[i], i))
    table = torch.tensor(perm[: B * bps], dtype=torch.int32).view(B, bps).to(a.dev)
    ctxs = [3, 40, 95]
    for p in (a, b):
        p.ctx.sssd_kv_set_block_table(table)
        for i in range(B):
            p.prefill_random_kv(93, i, ctxs[i])
    b.ctx.sssd_set_gemm_chain(True)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(94, 1, (B, k + 1), 0, s.vocab - 1)
    ra, rb = a.step(tokens, lens), b.step(tokens, lens)
    assert torch.equal(ra["logits"], rb["logits"])
    for l in range(s.n_layers):
        for i in range(B):
            n = ctxs[i] + k + 1
            Ka = torch.empty(s.n_kv_heads, n, s.head_dim, dtype=torch.bfloat16, device=a.dev)
            Va, Kb, Vb = torch.empty_like(Ka), torch.empty_like(Ka), torch.empty_like(Ka)
            a.ctx.sssd_kv_export(l, i, 0, Ka, Va)
            b.ctx.sssd_kv_export(l, i, 0, Kb, Vb)
            assert torch.equal(Ka.view(torch.int16), Kb.view(torch.int16)), (l, i)
            assert torch.equal(Va.view(torch.int16), Vb.view(torch.int16)), (l, i)
    say("chain + paged cache: logits and appended K/V rows identical to separate launches")
