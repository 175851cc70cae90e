"""Parity at the full sizes of the benchmark configurations (Llama-3-8B and 70B shapes),
in the launch configuration bench.py times.  The oracle cannot run whole batches of
these in seconds, so it recomputes SAMPLED sequences completely (every layer, every
logit of their k+1 rows); sequences are independent, so a sampled sequence of the
batched GPU step must match the oracle run on that sequence alone."""
import os
import sys
import time

import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_05894_amd import binding as sv
from sssd_synth import (MODEL_SHAPES, TensorId, global_weight_specs, layer_weight_specs, make_kv_prefill,
                        make_weight, uniform_int)

sys.path.insert(0, os.path.dirname(__file__))
from harness import LOGIT_TOL, Pair, compare_step  # noqa: E402

DEV = "cuda:0"
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg):
    """Progress lines for long tests: printed, and appended to a file the harness can watch."""
    print(msg, flush=True)
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


@pytest.fixture(scope="module")
def pair_8b():
    """8B-shaped weights (seed 3) once per module: capacity B=32, k<=16, 4128 rows per sequence."""
    progress("8b: generating weights")
    p = Pair(MODEL_SHAPES["8b"], seed=3, max_batch=32, max_k=16, max_seq=4096 + 17, oracle_batch=2)
    progress("8b: ready")
    yield p
    p.ctx.sssd_verify_destroy()


@pytest.mark.timeout(300)
def test_cfg2_8b_b1_ctx2048_k_sweep(pair_8b):
    """Config 2: B=1, KV context 2048 (random N(0,1) prefill), uniform-random drafts.  The oracle
    runs k=16 once; rows 0..k of that pass are the reference for every smaller k (row j never
    depends on later rows)."""
    p, s = pair_8b, pair_8b.shape
    p.prefill_random_kv(4, 0, 2048, oracle_slot=0)
    tokens = uniform_int(4, TensorId.TOKENS, (1, 17), 0, s.vocab - 1)
    lens = torch.tensor([2048], dtype=torch.int32)
    t = time.time()
    ref = p.oracle.verify_step(tokens, lens)
    progress(f"cfg2: oracle k=16 took {time.time() - t:.1f}s")
    for k in (16, 8, 3, 0):
        tk = tokens[:, : k + 1].contiguous()
        sub = {"logits": ref["logits"][:, : k + 1], "that": ref["that"][:, : k + 1]}
        a, n = oracle.accept(tk[0].tolist(), sub["that"][0].tolist())
        sub["accepted_len"], sub["next_token"] = torch.tensor([a]), torch.tensor([n])
        gpu = p.step(tk, lens)
        err, ex, rows = compare_step(gpu, sub, tk)
        progress(f"cfg2 k={k}: max logit err {err:.2e}, exempt rows {ex}/{rows}")


@pytest.mark.timeout(300)
def test_cfg3_8b_b32_ragged_k4(pair_8b):
    """Config 3: B=32, context lengths uniform in [1024, 4096], k=4.  Sequences 5 and 31 are
    recomputed by the oracle."""
    p, s = pair_8b, pair_8b.shape
    B, k = 32, 4
    lens = uniform_int(5, TensorId.LENS, (B,), 1024, 4096)
    sample = [5, 31]
    for b in range(B):
        p.prefill_random_kv(5, b, int(lens[b]), oracle_slot=sample.index(b) if b in sample else None)
    progress(f"cfg3: prefilled, lens[sample]={[int(lens[b]) for b in sample]}")
    tokens = uniform_int(5, TensorId.TOKENS, (B, k + 1), 0, s.vocab - 1)
    gpu = p.step(tokens, lens)
    t = time.time()
    ref = p.oracle.verify_step(tokens[sample].contiguous(), lens[sample].contiguous())
    progress(f"cfg3: oracle on 2 sequences took {time.time() - t:.1f}s")
    err, ex, rows = compare_step(gpu, ref, tokens, seqs=sample)
    progress(f"cfg3: max logit err {err:.2e}, exempt rows {ex}/{rows}")


@pytest.mark.timeout(300)
def test_cfg4_8b_b4_ctx32768_k8():
    """Config 4: B=4, KV context 32768, k=8 (attention-dominated).  Sequence 2 is recomputed."""
    s = MODEL_SHAPES["8b"]
    B, k, ctx = 4, 8, 32768
    progress("cfg4: generating weights")
    p = Pair(s, seed=3, max_batch=B, max_k=k, max_seq=ctx + k + 1, oracle_batch=1)
    for b in range(B):
        p.prefill_random_kv(6, b, ctx, oracle_slot=0 if b == 2 else None)
    progress("cfg4: prefilled")
    tokens = uniform_int(6, TensorId.TOKENS, (B, k + 1), 0, s.vocab - 1)
    lens = torch.full((B,), ctx, dtype=torch.int32)
    gpu = p.step(tokens, lens)
    t = time.time()
    ref = p.oracle.verify_step(tokens[2:3].contiguous(), lens[2:3].contiguous())
    progress(f"cfg4: oracle on 1 sequence took {time.time() - t:.1f}s")
    err, ex, rows = compare_step(gpu, ref, tokens, seqs=[2])
    progress(f"cfg4: max logit err {err:.2e}, exempt rows {ex}/{rows}")
    p.ctx.sssd_verify_destroy()
