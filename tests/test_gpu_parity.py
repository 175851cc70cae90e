"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle."""
import math
import os
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_05894_amd import binding as sv
from sssd_synth import MODEL_SHAPES, normal_bf16, uniform_bf16, uniform_int

sys.path.insert(0, os.path.dirname(__file__))
from harness import LOGIT_TOL, MARGIN, Pair, compare_step  # noqa: E402

DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------ generator ----
def test_generator_same_bits_on_cpu_and_gpu():
    for tid, shape, std in [(1, (333, 77), 0.02), (2, (5, 4096), 1.0)]:
        a = normal_bf16(9, tid, shape, std, device="cpu")
        b = normal_bf16(9, tid, shape, std, device=DEV).cpu()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(uniform_int(3, 4, (1000,), 5, 77), uniform_int(3, 4, (1000,), 5, 77, device=DEV).cpu())
    assert torch.equal(uniform_bf16(3, 5, (1000,), 0.5, 1.5).view(torch.int16),
                       uniform_bf16(3, 5, (1000,), 0.5, 1.5, device=DEV).cpu().view(torch.int16))


# ----------------------------------------------------------------- GEMM ----
GEMM_SHAPES = [  # (N, K): every distinct K of the three models, N a slice of the real matrix
    (512, 256), (256, 688), (688, 256), (1024, 256),        # tiny: QKV, down, gate, LM head
    (96, 4096), (48, 14336), (48, 8192), (32, 28672),       # 8B / 70B rows
]


@pytest.mark.parametrize("N,K", GEMM_SHAPES)
def test_gemm_vs_oracle(N, K):
    w = normal_bf16(21, N * 3 + K, (N, K), 0.02, device=DEV)
    wp = sv.sssd_op_pack_weight(w)
    wc = w.cpu()
    # 49 rows and more run the 16-row-tile form of the large-M kernel: every tile count from 4 to 10 (and a
    # second pass over left-over rows) is in the list, beside both row classes of the 32-row form (33..48).
    for M in (1, 5, 17, 32, 33, 36, 48, 49, 64, 80, 96, 100, 128, 144, 160, 163):
        say(f"gemm N={N} K={K} M={M}")
        x = normal_bf16(22, M * 7 + K, (M, K), 1.0, device=DEV).float() * 1.25
        x += 2.0 ** -10 * normal_bf16(23, M + K, (M, K), 1.0, device=DEV).float()     # not bf16-representable
        hi, lo = sv.sssd_op_pack_activation(x)
        ref = oracle.linear(x.cpu(), wc)
        scale = ref.abs().max().item()
        y2 = sv.sssd_op_gemm(hi, lo, wp, M, N, K).cpu()
        assert (y2 - ref).abs().max().item() <= 3e-5 * scale + 1e-6, "hi+lo activations"


@pytest.mark.parametrize("N,K", [(32768, 256), (24592, 352)])
def test_wide_gemm_vs_oracle(N, K):
    """Wide matrices (more column groups than compute units) through the large-M kernel: an even and an odd
    number of k-tiles, a last column group that is only partly inside the matrix."""
    w = normal_bf16(24, N * 3 + K, (N, K), 0.02, device=DEV)
    wp = sv.sssd_op_pack_weight(w)
    wc = w.cpu()
    for M in (33, 64, 100, 144, 160, 163):
        say(f"wide gemm N={N} K={K} M={M}")
        x = normal_bf16(25, M * 7 + K, (M, K), 1.0, device=DEV).float() * 1.25
        x += 2.0 ** -10 * normal_bf16(26, M + K, (M, K), 1.0, device=DEV).float()
        hi, lo = sv.sssd_op_pack_activation(x)
        ref = oracle.linear(x.cpu(), wc)
        y = sv.sssd_op_gemm(hi, lo, wp, M, N, K).cpu()
        assert (y - ref).abs().max().item() <= 3e-5 * ref.abs().max().item() + 1e-6


def test_stream_read_yardstick_reads_every_record():
    """The read-only bandwidth yardstick of bench.py: the XOR of the per-workgroup words it leaves behind must
    equal the XOR of every 32-bit word of the buffer's whole 16-byte records (a skipped or doubled record would
    show), for sizes that do and do not fill the grid's last round."""
    import numpy as np
    for n_words in (4, 4 * 1000 + 3, 4 * (1 << 20) + 8, 4 * 2048 * 256 * 4):
        buf = uniform_int(91, n_words, (n_words,), 0, (1 << 31) - 1, device=DEV).to(torch.int32)
        sink = torch.zeros(4096, dtype=torch.int32, device=DEV)
        sv.sssd_op_stream_read(buf, sink)
        torch.cuda.synchronize()
        got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
        want = int(np.bitwise_xor.reduce(buf.cpu().numpy().view(np.uint32)[: n_words // 4 * 4]))
        assert got == want, n_words


# ------------------------------------------------------------ attention ----
@pytest.mark.parametrize("shape_name,B,k,ctxs", [
    ("tiny", 2, 4, [0, 37]), ("tiny", 1, 0, [130]), ("tiny", 3, 7, [31, 32, 95]),
    ("8b", 2, 8, [2048, 1000]), ("8b", 1, 16, [300]),
    ("8b", 1, 31, [70]),          # the largest k: 128 query rows per kv head = 8 row tiles, two passes over the cache
    ("70b", 1, 5, [33]),          # g = 8
])
def test_attention_vs_oracle(shape_name, B, k, ctxs):
    s = MODEL_SHAPES[shape_name]
    s1 = type(s)(**{**s.__dict__, "n_layers": 1, "vocab": 1024})
    max_seq = max(ctxs) + k + 1
    layers = [{n: torch.zeros(shp, dtype=torch.bfloat16, device=DEV) for n, _, shp in
               __import__("sssd_synth").layer_weight_specs(s1)}]
    g = {n: torch.zeros(shp, dtype=torch.bfloat16, device=DEV) for n, _, shp in
         __import__("sssd_synth").global_weight_specs(s1)}
    ctx = sv.VerifyContext(sv.make_config(s1, B, k, max_seq), layers, g)
    sq, d, g_ = k + 1, s.head_dim, s.n_q_heads // s.n_kv_heads
    q = (normal_bf16(31, 1, (B, sq, s.n_q_heads, d), 1.0, device=DEV).float() * 1.28).contiguous()
    Ks, Vs = [], []
    for b in range(B):
        n = ctxs[b] + sq
        K = normal_bf16(32, 2 * b, (s.n_kv_heads, n, d), 1.0, device=DEV)
        V = normal_bf16(32, 2 * b + 1, (s.n_kv_heads, n, d), 1.0, device=DEV)
        ctx.sssd_kv_import(0, b, 0, K, V)
        Ks.append(K.cpu()); Vs.append(V.cpu())
    lens = torch.tensor(ctxs, dtype=torch.int32, device=DEV)
    out = torch.empty(B, sq, s.n_q_heads * d, dtype=torch.float32, device=DEV)
    say(f"attention {shape_name} B={B} k={k} ctx={ctxs}")
    ctx.sssd_op_attention(0, q, lens, out)
    assert ctx.sssd_verify_sync() == 0
    out = out.cpu().view(B, sq, s.n_q_heads, d)
    qc = q.cpu()
    worst = 0.0
    for b in range(B):
        for j in range(sq):
            for hq in range(s.n_q_heads):
                ref = oracle.attention_row(qc[b, j, hq], Ks[b][hq // g_], Vs[b][hq // g_], ctxs[b] + j + 1)
                worst = max(worst, (ref - out[b, j, hq]).abs().max().item())
    say("  worst abs err", worst)
    # q and the probabilities enter the MFMAs as bf16 hi+lo pairs (~2^-17 relative); outputs are O(1)
    assert worst <= 1e-4
    # round trip of the cache through its private layout
    Kb = torch.empty_like(Ks[0], device=DEV); Vb = torch.empty_like(Vs[0], device=DEV)
    ctx.sssd_kv_export(0, 0, 0, Kb, Vb)
    assert torch.equal(Kb.cpu().view(torch.int16), Ks[0].view(torch.int16))
    assert torch.equal(Vb.cpu().view(torch.int16), Vs[0].view(torch.int16))


# ----------------------------------------------------- cfg 1: tiny chain ----
def test_tiny_chained_verify_steps():
    """Tiny model, B=1, 128-token prompt, k=4 drafts from the oracle's greedy continuation with
    one token replaced at a seeded position in 0..4 (4 = no replacement), 64 chained steps."""
    s = MODEL_SHAPES["tiny"]
    k, prompt_len, steps = 4, 128, 64
    p = Pair(s, seed=1, max_batch=1, max_k=k, max_seq=prompt_len + steps * (k + 1) + 8)
    prompt = uniform_int(2, 5, (prompt_len,), 0, s.vocab - 1)
    # prefill rows 0..126 through the verify step itself, in chunks of k+1, on both sides
    lens = 0
    while lens < prompt_len - 1:
        n = min(k + 1, prompt_len - 1 - lens)
        chunk = prompt[lens: lens + n].view(1, n)
        p.step(chunk, torch.tensor([lens]))
        p.oracle.verify_step(chunk, torch.tensor([lens]))
        lens += n
    last = int(prompt[-1])
    pos_seed = uniform_int(2, 6, (steps,), 0, k).tolist()
    tok_seed = uniform_int(2, 7, (steps,), 0, s.vocab - 1).tolist()
    worst, exempt, rows, acc_hist = 0.0, 0, 0, []
    for step in range(steps):
        # oracle's own greedy continuation after `last` (writes only dead rows >= lens)
        drafts, t = [], last
        for j in range(k):
            t = oracle.argmax(p.oracle.decode_token(0, t, lens + j))
            drafts.append(t)
        if pos_seed[step] < k:
            drafts[pos_seed[step]] = tok_seed[step]
        tokens = torch.tensor([[last] + drafts], dtype=torch.int32)
        ref = p.oracle.verify_step(tokens, torch.tensor([lens]))
        gpu = p.step(tokens, torch.tensor([lens]))
        e, ex, r = compare_step(gpu, ref, tokens)
        worst, exempt, rows = max(worst, e), exempt + ex, rows + r
        acc = int(ref["accepted_len"][0])
        acc_hist.append(acc)
        lens += acc + 1                       # follow the oracle's decision (exempt rows cannot fork the chain)
        last = int(ref["next_token"][0])
    say(f"tiny chain: worst logit err {worst:.2e}, exempt rows {exempt}/{rows}, accepted {sum(acc_hist)}")
    assert sum(acc_hist) > steps              # the chain really accepts drafts
    assert exempt < rows // 2


def test_tiny_batched_ragged_and_rollback():
    s = MODEL_SHAPES["tiny"]
    B, k = 5, 7
    p = Pair(s, seed=3, max_batch=B, max_k=k, max_seq=200, unit_gains=False)
    ctxs = [0, 1, 31, 64, 150]
    for b in range(B):
        p.prefill_random_kv(11, b, ctxs[b], oracle_slot=b)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(12, 1, (B, k + 1), 0, s.vocab - 1)
    ref = p.oracle.verify_step(tokens, lens, return_hidden=True)
    gpu = p.step(tokens, lens)
    e, ex, r = compare_step(gpu, ref, tokens)
    herr = (gpu["hidden"] - ref["hidden"]).abs().max().item() / ref["hidden"].abs().max().item()
    say(f"tiny ragged batch: worst logit err {e:.2e}, hidden rel err {herr:.2e}, exempt {ex}/{r}")
    assert herr < 5e-3
    # k = 0 step on a sub-batch after committing
    dl = lens.to(DEV)
    p.ctx.sssd_kv_rollback(dl, accepted_len=gpu["accepted_len"].to(DEV))
    assert torch.equal(dl.cpu(), lens + gpu["accepted_len"] + 1)
    new = torch.tensor([3, 0, 9, 1, 2], dtype=torch.int32, device=DEV)
    p.ctx.sssd_kv_rollback(dl, new_lens=new)
    assert torch.equal(dl.cpu(), new.cpu())
    lens2 = lens + ref["accepted_len"] + 1
    tok2 = ref["next_token"].view(B, 1)[:3].contiguous()
    ref2 = p.oracle.verify_step(tok2, lens2[:3])
    gpu2 = p.step(tok2, lens2[:3])
    compare_step(gpu2, ref2, tok2)


@pytest.mark.parametrize("B,k", [(6, 7), (5, 15), (8, 12), (7, 15), (4, 31)])
def test_tiny_steps_across_the_row_tilings(B, k):
    """Whole steps with M = B*(k+1) = 48, 80, 104, 112, 128 rows: past the small-step GEMM kernel
    (M <= 32), through every row-tile count of the large-M kernel up to the largest step a tiny
    context of max_k = 31 allows, ragged contexts included."""
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=5, max_batch=B, max_k=k, max_seq=260, unit_gains=False)
    ctxs = [int(c) for c in uniform_int(14, B * 100 + k, (B,), 0, 200)]
    ctxs[0] = 0
    for b in range(B):
        p.prefill_random_kv(15, b, ctxs[b], oracle_slot=b)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(16, B * 100 + k, (B, k + 1), 0, s.vocab - 1)
    ref = p.oracle.verify_step(tokens, lens, return_hidden=True)
    gpu = p.step(tokens, lens)
    e, ex, r = compare_step(gpu, ref, tokens)
    herr = (gpu["hidden"] - ref["hidden"]).abs().max().item() / ref["hidden"].abs().max().item()
    say(f"tiny M={B * (k + 1)} (B={B}, k={k}): worst logit err {e:.2e}, hidden rel err {herr:.2e}, exempt {ex}/{r}")
    assert herr < 5e-3
    assert ex < r // 2
    p.ctx.sssd_verify_destroy()


@pytest.mark.parametrize("B,k", [(4, 8), (8, 7), (10, 9), (16, 9), (11, 15)])
def test_wide_ffn_and_vocabulary_take_the_unsplit_large_m_path(B, k):
    """A one-layer model whose gate/up matrices (ffn 14336) and LM head (vocabulary 32768) are wide enough that the
    large-M kernel does not split K (one slice of partial sums, more column groups than compute units), beside
    narrow QKV / O / down matrices that split it many ways.  M = 36, 64, 100, 160, 176 (two row passes)."""
    s0 = MODEL_SHAPES["tiny"]
    s = type(s0)(**{**s0.__dict__, "n_layers": 1, "ffn": 14336, "vocab": 32768})
    p = Pair(s, seed=7, max_batch=B, max_k=k, max_seq=96, unit_gains=False)
    ctxs = [int(c) for c in uniform_int(19, B * 100 + k, (B,), 0, 60)]
    for b in range(B):
        p.prefill_random_kv(20, b, ctxs[b], oracle_slot=b)
    lens = torch.tensor(ctxs, dtype=torch.int32)
    tokens = uniform_int(21, B * 100 + k, (B, k + 1), 0, s.vocab - 1)
    ref = p.oracle.verify_step(tokens, lens, return_hidden=True)
    gpu = p.step(tokens, lens)
    e, ex, r = compare_step(gpu, ref, tokens)
    herr = (gpu["hidden"] - ref["hidden"]).abs().max().item() / ref["hidden"].abs().max().item()
    say(f"wide model M={B * (k + 1)}: worst logit err {e:.2e}, hidden rel err {herr:.2e}, exempt {ex}/{r}")
    assert herr < 5e-3
    p.ctx.sssd_verify_destroy()


def test_error_reporting():
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=1, max_batch=2, max_k=4, max_seq=64)
    t = torch.zeros(2, 5, dtype=torch.int32, device=DEV)
    out = torch.zeros(2, dtype=torch.int32, device=DEV)
    lens = torch.tensor([10, 60], dtype=torch.int32, device=DEV)            # 60 + 5 > 64
    p.ctx.sssd_verify_step(t, lens, out, out.clone())
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    assert p.ctx.sssd_verify_sync() == 0                                    # flag is cleared
    t[1, 2] = s.vocab                                                       # token id out of range
    p.ctx.sssd_verify_step(t, torch.tensor([0, 0], dtype=torch.int32, device=DEV), out, out.clone())
    assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE
    with pytest.raises(sv.SssdError) as ei:
        p.ctx.sssd_verify_step(torch.zeros(3, 5, dtype=torch.int32, device=DEV), lens, out, out)
    assert ei.value.code == sv.SSSD_ECAPACITY
    with pytest.raises(sv.SssdError) as ei:
        p.ctx.sssd_verify_step(torch.zeros(2, 6, dtype=torch.int32, device=DEV), lens, out, out)
    assert ei.value.code == sv.SSSD_ECAPACITY


def _export_all(p, b, n_rows):
    s = p.shape
    out = []
    for l in range(s.n_layers):
        K = torch.empty(s.n_kv_heads, n_rows, s.head_dim, dtype=torch.bfloat16, device=DEV)
        V = torch.empty_like(K)
        p.ctx.sssd_kv_export(l, b, 0, K, V)
        out += [K.cpu().view(torch.int16), V.cpu().view(torch.int16)]
    return out


def test_rejected_sequence_leaves_the_cache_untouched():
    """A sequence whose lens does not fit (or whose block table names a page outside the pool) must not
    write a single cache row, of its own or of a neighbour: after the flagged step every row of the
    rejected sequence and every LIVE row of the accepted one hold the bits they held before, and the
    accepted sequence still gets the oracle's logits."""
    s = MODEL_SHAPES["tiny"]
    k, max_seq = 4, 64
    p = Pair(s, seed=1, max_batch=2, max_k=k, max_seq=max_seq)
    p.prefill_random_kv(17, 0, 40, oracle_slot=0)
    p.prefill_random_kv(17, 1, max_seq)
    tokens = uniform_int(18, 1, (2, k + 1), 0, s.vocab - 1)
    ref = p.oracle.verify_step(tokens[:1].contiguous(), torch.tensor([40]))
    rows, bps, n_pages = sv.sssd_kv_geometry(p.cfg)
    bad_table = torch.arange(2 * bps, dtype=torch.int32).view(2, bps)
    bad_table[1, 1] = n_pages + 5                                       # block 1 of sequence 1: outside the pool
    cases = [("lens too large", torch.tensor([40, 61], dtype=torch.int32), None),
             ("negative lens", torch.tensor([40, -3], dtype=torch.int32), None),
             ("page outside the pool", torch.tensor([40, 30], dtype=torch.int32), bad_table)]
    for name, lens, table in cases:
        before0, before1 = _export_all(p, 0, 40), _export_all(p, 1, 32 if table is not None else max_seq)
        if table is not None:
            p.ctx.sssd_kv_set_block_table(table.to(DEV))
        t = tokens.to(DEV)
        acc = torch.empty(2, dtype=torch.int32, device=DEV)
        nxt = torch.empty(2, dtype=torch.int32, device=DEV)
        p.ctx.sssd_verify_step(t, lens.to(DEV), acc, nxt)
        assert p.ctx.sssd_verify_sync() == sv.SSSD_ENOSPACE, name
        # block 0 of sequence 1 is a good page in every case; with the bad table only it can be exported
        after0, after1 = _export_all(p, 0, 40), _export_all(p, 1, 32 if table is not None else max_seq)
        p.ctx.sssd_kv_set_block_table(None)
        assert all(torch.equal(a, b) for a, b in zip(before0, after0)), name
        assert all(torch.equal(a, b) for a, b in zip(before1, after1)), name
        if table is not None:   # the rest of sequence 1, through the plain layout the table mirrored
            assert all(torch.equal(a, b) for a, b in zip(full1, _export_all(p, 1, max_seq))), name
        full1 = _export_all(p, 1, max_seq)
        err = (p.logits[: k + 1].cpu() - ref["logits"][0]).abs().max().item()
        assert err <= LOGIT_TOL, (name, err)
        say(f"rejected sequence ({name}): cache bits unchanged, neighbour's logits within {err:.2e}")


def test_step_is_deterministic():
    s = MODEL_SHAPES["tiny"]
    p = Pair(s, seed=1, max_batch=2, max_k=4, max_seq=64)
    tokens = uniform_int(13, 1, (2, 5), 0, s.vocab - 1)
    a = p.step(tokens, torch.tensor([0, 0]))["logits"].clone()
    b = p.step(tokens, torch.tensor([0, 0]))["logits"]
    assert torch.equal(a, b)
