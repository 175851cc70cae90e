"""The whole SSSD loop on one GPU: the C++ host drafter proposes draft trees from the input trie
and the datastore (App. A, Alg. 1-3), the speculation length follows the roofline rule (Sec. 3.2),
the library verifies the trees and commits the accepted path, and the accepted tokens feed the
drafter again.  Every step is checked against the CPU oracle run on the same tree, and the emitted
stream against the oracle's plain greedy decoding (Sec. 2: the output is exactly preserved)."""
import pytest
import torch

import oracle
from harness import Pair, compare_tree_step, step_tree
from paper_2411_05894_amd import drafter as dr
from sssd_synth import MODEL_SHAPES, repetitive_stream

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def test_drafter_verify_commit_loop_emits_the_greedy_stream():
    s = MODEL_SHAPES["tiny"]
    B, prompt_len, steps = 2, 48, 28
    s_q = dr.sssd_draft_speculation_length(2.5e15, 8e12, B, 12)      # MI355X ridge 312 / b, capped at 12 here
    assert s_q == 12
    k = s_q - 1
    max_seq = prompt_len + steps * s_q + 8
    p = Pair(s, seed=41, max_batch=B, max_k=k, max_seq=max_seq)
    greedy_model = oracle.build_model(s, 41, B, max_seq)             # plain greedy decoding, its own cache
    prompts = [repetitive_stream(42, 1 + b, prompt_len, vocab=s.vocab, n_templates=4, noise=0.0) for b in range(B)]

    # prefill rows 0..prompt_len-2 through chain steps (library, oracle, and the greedy model)
    lens = 0
    while lens < prompt_len - 1:
        n = min(k + 1, prompt_len - 1 - lens)
        chunk = torch.tensor([pr[lens: lens + n] for pr in prompts], dtype=torch.int32)
        ln = torch.full((B,), lens, dtype=torch.int32)
        p.step(chunk, ln)
        p.oracle.verify_step(chunk, ln)
        greedy_model.verify_step(chunk, ln)
        lens += n
    n_greedy = steps * s_q
    greedy = []
    for b in range(B):
        out, t = [], prompts[b][-1]
        for i in range(n_greedy):
            t = oracle.argmax(greedy_model.decode_token(b, t, prompt_len - 1 + i))
            out.append(t)
        greedy.append(out)

    drafter = dr.Drafter(n_sequences=B)
    drafter.sssd_draft_datastore_add(repetitive_stream(42, 1, 4000, vocab=s.vocab, n_templates=4, noise=0.0))
    for b in range(B):
        drafter.sssd_draft_input_append(b, prompts[b])
    dlens = torch.full((B,), lens, dtype=torch.int32, device=DEV)
    cur = [lens] * B
    emitted = [[] for _ in range(B)]
    accepted, drafted, worst, exempt, rows = 0, 0, 0.0, 0, 0
    for step in range(steps):
        toks, pars = [], []
        for b in range(B):
            t, par = drafter.sssd_draft_propose(b, s_q)
            drafted += len(t) - 1
            t += [0] * (s_q - len(t))             # pad with children of the root; a padded node is accepted
            par += [0] * (s_q - len(par))         # only if its token IS the greedy token, so padding is harmless
            toks.append(t)
            pars.append(par)
        tokens = torch.tensor(toks, dtype=torch.int32)
        parents = torch.tensor(pars, dtype=torch.int32)
        ln = torch.tensor(cur, dtype=torch.int32)
        ref = p.oracle.verify_step_tree(tokens, parents, ln, compact=True)
        gpu = step_tree(p, tokens, parents, ln)
        e, ex, r = compare_tree_step(gpu, ref, tokens, parents)
        worst, exempt, rows = max(worst, e), exempt + ex, rows + r
        same = all(gpu["path"][b].tolist()[: int(gpu["accepted_len"][b]) + 1] == ref["path"][b] for b in range(B))
        if same:
            p.ctx.sssd_kv_commit_tree(dlens, gpu["dev"]["accepted_len"], gpu["dev"]["path"])
        else:                                     # an undecided row forked the walk: follow the oracle
            acc_d = ref["accepted_len"].to(DEV)
            path_d = torch.tensor([ref["path"][b] + [-1] * (s_q - len(ref["path"][b])) for b in range(B)],
                                  dtype=torch.int32, device=DEV)
            p.ctx.sssd_kv_commit_tree(dlens, acc_d, path_d)
        assert p.ctx.sssd_verify_sync() == 0
        for b in range(B):
            n = int(ref["accepted_len"][b])
            new = [toks[b][i] for i in ref["path"][b][1:]] + [int(ref["next_token"][b])]
            emitted[b] += new
            drafter.sssd_draft_input_append(b, new)
            cur[b] += n + 1
            accepted += n
        assert dlens.cpu().tolist() == cur
    for b in range(B):
        assert emitted[b] == greedy[b][: len(emitted[b])], f"sequence {b} left the greedy stream"
    tokens_out = sum(len(e) for e in emitted)
    say(f"e2e loop: {tokens_out} tokens in {steps} steps x {B} sequences ({tokens_out / (steps * B):.2f} per step), "
        f"{accepted}/{drafted} drafts accepted, worst logit err {worst:.2e}, exempt rows {exempt}/{rows}")
    assert accepted > 0
