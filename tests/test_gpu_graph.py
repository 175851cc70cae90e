"""The verify step under HIP graph capture: a serving loop may record the step once and replay it.  Nothing in
the step allocates, synchronises or records memsets, so the capture must succeed, and every replay -- with eager
steps and synchronisations between the replays -- must give the eager step's outputs bit for bit."""
import os
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu

from sssd_synth import MODEL_SHAPES, uniform_int

sys.path.insert(0, os.path.dirname(__file__))
from harness import Pair  # noqa: E402

DEV = "cuda:0"


@pytest.mark.parametrize("B,k", [(1, 8), (2, 12), (6, 7)])
def test_replayed_step_equals_the_eager_step(B, k):
    """M = 9 (small-step kernels), 26 (row halves), 48 (large-M kernels with their epilogue launches)."""
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=9, max_batch=B, max_k=k, max_seq=160)
    ctxs = [int(c) for c in uniform_int(31, B * 100 + k, (B,), 0, 100)]
    for b in range(B):
        p.prefill_random_kv(32, b, ctxs[b])
    tokens = uniform_int(33, B * 100 + k, (B, k + 1), 0, s.vocab - 1).to(DEV)
    lens = torch.tensor(ctxs, dtype=torch.int32, device=DEV)
    acc = torch.empty(B, dtype=torch.int32, device=DEV)
    nxt = torch.empty(B, dtype=torch.int32, device=DEV)
    M = B * (k + 1)

    def eager():
        p.ctx.sssd_verify_step(tokens, lens, acc, nxt)
        assert p.ctx.sssd_verify_sync() == 0
        return p.logits[:M].clone(), acc.clone(), nxt.clone()

    want = eager()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        p.ctx.sssd_verify_step(tokens, lens, acc, nxt)          # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            p.ctx.sssd_verify_step(tokens, lens, acc, nxt)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        p.logits[:M].zero_()
        acc.fill_(-5)
        nxt.fill_(-5)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(p.logits[:M], want[0]) and torch.equal(acc, want[1]) and torch.equal(nxt, want[2]), rep
        # the program's own eager work between replays: another step with other tokens, then the first one again
        other = (tokens + 1 + rep) % s.vocab
        p.ctx.sssd_verify_step(other.to(torch.int32), lens, acc, nxt)
        assert p.ctx.sssd_verify_sync() == 0
        again = eager()
        assert all(torch.equal(a, b) for a, b in zip(again, want))
    p.ctx.sssd_verify_destroy()
