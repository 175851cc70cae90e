"""Pins of the CPU oracle against things other than itself: fp64 library
routines, closed forms, dense brute force, and the equalities the paper fixes
(verify pass == sequential decoding; speculative output == greedy output)."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from sssd_synth import MODEL_SHAPES, ModelShape, normal_bf16, uniform_bf16, uniform_int


def bf16(x):
    return x.to(torch.bfloat16)


# ---------------------------------------------------------------- bf16 ----
def test_bf16_roundtrip_matches_torch():
    x = torch.randn(20000, generator=torch.Generator().manual_seed(0)) * 3
    x = torch.cat([x, torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, 3.3895e38])])
    ref = x.to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([oracle.lib().orc_f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert (ref == got).all()
    back = np.array([oracle.lib().orc_bf16_to_f32(int(b)) for b in ref[:1000]], dtype=np.float32)
    assert (back == x[:1000].to(torch.bfloat16).float().numpy()).all()


# ---------------------------------------------------------------- GEMM ----
SHAPES_NK = [(512, 256), (256, 256), (688, 256), (256, 688), (1024, 256),     # tiny
             (96, 4096), (64, 14336), (48, 8192), (32, 28672)]                 # rows of 8B/70B matrices


@pytest.mark.parametrize("N,K", SHAPES_NK)
@pytest.mark.parametrize("M", [1, 5])
def test_linear_vs_fp64_matmul(N, K, M):
    w = normal_bf16(11, N * 7 + K, (N, K), 0.02)
    x = normal_bf16(12, N + K * 3 + M, (M, K), 1.0).float() * 1.37
    y = oracle.linear(x, w)
    ref = x.double() @ w.double().T
    assert y.shape == (M, N)
    assert torch.allclose(y.double(), ref, rtol=1e-6, atol=1e-7)


def test_linear_is_not_transposed():
    # W = [[1,2],[3,4],[5,6]] (N=3, K=2), x = [1, 10] -> y = [21, 43, 65]
    w = bf16(torch.tensor([[1., 2.], [3., 4.], [5., 6.]]))
    y = oracle.linear(torch.tensor([[1., 10.]]), w)
    assert y.tolist() == [[21., 43., 65.]]


# ------------------------------------------------------------- RMSNorm ----
def test_rmsnorm_closed_form_constant_vector():
    n, c, eps = 256, 3.0, 1e-5
    gamma = uniform_bf16(3, 1, (n,), 0.5, 1.5)
    out = oracle.rmsnorm(torch.full((n,), c), gamma, eps)
    expect = gamma.double() * c / math.sqrt(c * c + eps)
    assert torch.allclose(out.double(), expect, rtol=1e-6)


def test_rmsnorm_vs_library_and_scale_invariance():
    n, eps = 688, 1e-5
    x = normal_bf16(4, 2, (3, n), 1.0).float()
    gamma = uniform_bf16(3, 2, (n,), 0.5, 1.5)
    out = oracle.rmsnorm(x, gamma, eps)
    ref = F.rms_norm(x.double(), (n,), gamma.double(), eps)
    assert torch.allclose(out.double(), ref, rtol=1e-6, atol=1e-7)
    out2 = oracle.rmsnorm(x * 64.0, gamma, eps)       # eps negligible against mean(x^2) ~ 1
    assert torch.allclose(out2, out, rtol=2e-5, atol=1e-6)


# ---------------------------------------------------------------- RoPE ----
@pytest.mark.parametrize("d,base", [(64, 10000.0), (128, 500000.0)])
def test_rope_identities(d, base):
    q = normal_bf16(5, d, (d,), 1.0).float()
    k = normal_bf16(6, d, (d,), 1.0).float()
    assert torch.equal(oracle.rope(q, 0, base), q)                       # position 0 is the identity
    for p in (1, 17, 4095, 40000):
        r = oracle.rope(q, p, base)
        assert abs(r.double().norm() - q.double().norm()) < 1e-5         # rotation preserves the norm
    # <R(p) q, R(p') k> depends only on p - p'
    for (p, pp), (s, ss) in [((5, 2), (1003, 1000)), ((40000, 39990), (10, 0)), ((7, 7), (0, 0))]:
        a = oracle.rope(q, p, base).double() @ oracle.rope(k, pp, base).double()
        b = oracle.rope(q, s, base).double() @ oracle.rope(k, ss, base).double()
        assert abs(a - b) < 2e-4 * max(1.0, abs(a))


@pytest.mark.parametrize("d,base", [(64, 10000.0), (128, 500000.0)])
def test_rope_is_complex_rotation_of_half_split_pairs(d, base):
    # Textbook statement: z_i = v_i + 1j*v_{i+d/2} is multiplied by exp(1j*p*base^(-2i/d)).
    v = normal_bf16(7, d, (d,), 1.0).double()
    p = 1234
    z = torch.complex(v[: d // 2], v[d // 2:])
    theta = p * torch.pow(torch.tensor(base, dtype=torch.float64), -2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    zr = z * torch.polar(torch.ones_like(theta), theta)
    ref = torch.cat([zr.real, zr.imag])
    assert torch.allclose(oracle.rope(v.float(), p, base).double(), ref, atol=2e-6)
    # unit vector e_1 at position p -> cos at slot 1, sin at slot 1 + d/2, zero elsewhere
    e = torch.zeros(d); e[1] = 1.0
    r = oracle.rope(e, 3, base).double()
    th = 3 * base ** (-2.0 / d)
    assert abs(r[1] - math.cos(th)) < 1e-6 and abs(r[1 + d // 2] - math.sin(th)) < 1e-6
    r[1] = 0; r[1 + d // 2] = 0
    assert r.abs().max() == 0


# ----------------------------------------------------------- attention ----
def dense_masked_attention(Q, K, V, lens_b, d):
    """softmax(Q K^T / sqrt(d) + M) V with the mask built explicitly (Table 2
    attention row); Q [sq, d], K/V [s_kv + sq, d], fp64."""
    sq = Q.shape[0]
    total = lens_b + sq
    mask = np.full((sq, total), -np.inf)
    for j in range(sq):
        mask[j, : lens_b + j + 1] = 0.0
    S = Q @ K[:total].T / math.sqrt(d) + mask
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    P /= P.sum(axis=1, keepdims=True)
    return P @ V[:total]


def test_attention_row_vs_dense_brute_force():
    d = 8
    for seed, (ctx, k) in enumerate([(0, 0), (1, 3), (16, 3), (5, 2), (13, 0)]):
        sq = k + 1
        Kc = normal_bf16(20 + seed, 1, (ctx + sq, d), 1.0)
        Vc = normal_bf16(20 + seed, 2, (ctx + sq, d), 1.0)
        Q = normal_bf16(20 + seed, 3, (sq, d), 1.0).float() * 2.0
        ref = dense_masked_attention(Q.double().numpy(), Kc.double().numpy(), Vc.double().numpy(), ctx, d)
        for j in range(sq):
            out = oracle.attention_row(Q[j], Kc, Vc, ctx + j + 1)
            assert np.allclose(out.double().numpy(), ref[j], rtol=1e-5, atol=1e-6)


def test_attention_row_vs_library_sdpa():
    d, n = 64, 77
    Kc = normal_bf16(31, 1, (n, d), 1.0)
    Vc = normal_bf16(31, 2, (n, d), 1.0)
    q = normal_bf16(31, 3, (d,), 1.0).float()
    ref = F.scaled_dot_product_attention(q.double().view(1, 1, 1, d), Kc.double().view(1, 1, n, d),
                                         Vc.double().view(1, 1, n, d)).view(d)
    out = oracle.attention_row(q, Kc, Vc, n)
    assert torch.allclose(out.double(), ref, rtol=1e-5, atol=1e-6)


def test_attention_closed_forms():
    d, n = 16, 9
    V = normal_bf16(32, 2, (n, d), 1.0)
    q = normal_bf16(32, 3, (d,), 1.0).float()
    same_k = normal_bf16(32, 4, (1, d), 1.0).expand(n, d).contiguous()
    out = oracle.attention_row(q, same_k, V, n)                      # equal keys -> mean of V
    assert torch.allclose(out.double(), V.double().mean(0), atol=1e-6)
    same_v = normal_bf16(32, 5, (1, d), 1.0).expand(n, d).contiguous()
    K = normal_bf16(32, 6, (n, d), 1.0)
    out = oracle.attention_row(q, K, same_v, n)                      # equal values -> that value
    assert torch.allclose(out.double(), same_v[0].double(), atol=1e-6)
    out = oracle.attention_row(q, K, V, 1)                           # one key -> its value
    assert torch.equal(out, V[0].float())
    big = bf16(torch.zeros(n, d)); big[4, 0] = 100.0                 # one dominant key -> its value
    e0 = torch.zeros(d); e0[0] = 50.0
    out = oracle.attention_row(e0, big, V, n)
    assert torch.allclose(out, V[4].float(), atol=1e-6)


# -------------------------------------------- whole model vs library ops ----
def library_forward(model, tokens, lens, K_old, V_old):
    """Independent fp64 forward of the verify pass built from library routines
    (F.rms_norm, matmul, complex multiply for RoPE, F.scaled_dot_product_attention
    with an explicit boolean mask, F.silu).  K_old/V_old: per layer bf16
    [n_kv, lens, d] for a single sequence.  New K/V are rounded to bf16 like the cache."""
    s = model.shape
    d, g = s.head_dim, s.n_q_heads // s.n_kv_heads
    sq = tokens.numel()
    x = model.g["embed"].double()[tokens.long()]
    pos = lens + torch.arange(sq)
    inv = torch.pow(torch.tensor(s.rope_base, dtype=torch.float64), -2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    rot = torch.polar(torch.ones(sq, d // 2, dtype=torch.float64), pos.double()[:, None] * inv[None, :])

    def rope(t):                                   # t [sq, heads, d]
        z = torch.complex(t[..., : d // 2], t[..., d // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    for l in range(s.n_layers):
        w = {k: v.double() for k, v in model.layers[l].items()}
        a = F.rms_norm(x, (s.hidden,), w["attn_norm"], s.rms_eps)
        q = rope((a @ w["wq"].T).float().double().view(sq, s.n_q_heads, d))
        kn = rope((a @ w["wk"].T).float().double().view(sq, s.n_kv_heads, d))
        vn = (a @ w["wv"].T).view(sq, s.n_kv_heads, d)
        Kall = torch.cat([K_old[l].double(), kn.float().to(torch.bfloat16).double().transpose(0, 1)], 1)
        Vall = torch.cat([V_old[l].double(), vn.float().to(torch.bfloat16).double().transpose(0, 1)], 1)
        mask = torch.zeros(sq, lens + sq, dtype=torch.bool)
        for j in range(sq):
            mask[j, : lens + j + 1] = True
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], Kall.repeat_interleave(g, 0)[None],
                                           Vall.repeat_interleave(g, 0)[None], attn_mask=mask)[0]
        x = x + o.transpose(0, 1).reshape(sq, -1) @ w["wo"].T
        m = F.rms_norm(x, (s.hidden,), w["mlp_norm"], s.rms_eps)
        x = x + (F.silu(m @ w["w_gate"].T) * (m @ w["w_up"].T)) @ w["w_down"].T
    xf = F.rms_norm(x, (s.hidden,), model.g["final_norm"].double(), s.rms_eps)
    return xf @ model.g["lm_head"].double().T


@pytest.mark.parametrize("lens,k", [(0, 0), (0, 4), (37, 4), (64, 1)])
def test_verify_pass_vs_library_forward(tiny_shape, lens, k):
    s = tiny_shape
    model = oracle.build_model(s, seed=1, max_batch=1, max_seq=128, unit_gains=False)
    K_old, V_old = [], []
    for l in range(s.n_layers):
        Kp = normal_bf16(40, 2 * l, (s.n_kv_heads, lens, s.head_dim), 1.0)
        Vp = normal_bf16(40, 2 * l + 1, (s.n_kv_heads, lens, s.head_dim), 1.0)
        model.K[l, 0, :, :lens] = Kp
        model.V[l, 0, :, :lens] = Vp
        K_old.append(Kp); V_old.append(Vp)
    tokens = uniform_int(41, k, (1, k + 1), 0, s.vocab - 1)
    out = model.verify_step(tokens, torch.tensor([lens]))
    ref = library_forward(model, tokens[0], lens, K_old, V_old)
    err = (out["logits"][0].double() - ref).abs().max().item()
    assert err < 2e-4, err                      # bf16 rounding of new K/V can flip by one ulp; else ~1e-6
    assert out["that"][0].tolist() == ref.argmax(-1).tolist()


# --------------------------------- verify pass == sequential decoding ----
@pytest.mark.parametrize("k", [0, 1, 4, 7])
def test_verify_pass_equals_sequential_decode(tiny_shape, k):
    s = tiny_shape
    prompt = 9
    a = oracle.build_model(s, seed=1, max_batch=2, max_seq=64)
    b = oracle.build_model(s, seed=1, max_batch=2, max_seq=64)
    toks = uniform_int(50, k, (2, prompt + k + 1), 0, s.vocab - 1)
    # prefill both caches identically by sequential decode of the prompt
    for m in (a, b):
        for seq in range(2):
            for p in range(prompt):
                m.decode_token(seq, int(toks[seq, p]), p)
    assert torch.equal(a.K.view(torch.int16), b.K.view(torch.int16))
    out = a.verify_step(toks[:, prompt:].contiguous(), torch.tensor([prompt, prompt]))
    for seq in range(2):
        for j in range(k + 1):
            lg = b.decode_token(seq, int(toks[seq, prompt + j]), prompt + j)
            assert torch.equal(lg, out["logits"][seq, j]), (seq, j)      # bit-identical
    assert torch.equal(a.K.view(torch.int16), b.K.view(torch.int16))
    assert torch.equal(a.V.view(torch.int16), b.V.view(torch.int16))


def test_row_j_does_not_depend_on_later_rows_or_other_sequences(tiny_shape):
    s = tiny_shape
    m1 = oracle.build_model(s, seed=1, max_batch=2, max_seq=32)
    m2 = oracle.build_model(s, seed=1, max_batch=2, max_seq=32)
    t = uniform_int(51, 0, (2, 6), 0, s.vocab - 1)
    lens = torch.tensor([0, 0])
    full = m1.verify_step(t, lens)["logits"]
    part = m2.verify_step(t[:1, :3].contiguous(), lens[:1])["logits"]
    assert torch.equal(full[0, :3], part[0])


# ---------------------------------------------------------- acceptance ----
def test_accept_special_cases():
    assert oracle.accept([7], [3]) == (0, 3)                                    # k = 0
    assert oracle.accept([7, 1, 2, 3], [1, 2, 3, 9]) == (3, 9)                  # all drafts right
    assert oracle.accept([7, 5, 2, 3], [1, 2, 3, 9]) == (0, 1)                  # first draft wrong
    assert oracle.accept([7, 1, 2, 8], [1, 2, 3, 9]) == (2, 3)                  # wrong at position 2
    assert oracle.accept([7, 1, 8, 3], [1, 2, 3, 9]) == (1, 2)                  # later match must not count


def test_accept_brute_force_all_match_patterns():
    for k in range(0, 5):
        that = list(range(100, 101 + k))
        for pattern in itertools.product([0, 1], repeat=k):
            tokens = [5] + [that[i] if pattern[i] else 999 for i in range(k)]
            n = 0
            for bit in pattern:
                if not bit:
                    break
                n += 1
            assert oracle.accept(tokens, that) == (n, that[n])


def test_argmax_ties_lowest_index():
    assert oracle.argmax(torch.tensor([1.0, 5.0, 5.0, 2.0])) == 1
    assert oracle.argmax(torch.tensor([-3.0, -3.0])) == 0
    assert oracle.top2(torch.tensor([1.0, 5.0, 4.0, 5.0])) == (5.0, 5.0)


@pytest.mark.parametrize("draft_kind", ["random", "correct", "one_wrong"])
def test_speculative_loop_equals_greedy_loop(tiny_shape, draft_kind):
    """Paper Sec. 2: verification keeps the target's exact output (greedy here)."""
    s = tiny_shape
    k, n_new, prompt_len = 4, 24, 12
    prompt = uniform_int(60, 1, (prompt_len,), 0, s.vocab - 1).tolist()
    g = oracle.build_model(s, seed=1, max_batch=1, max_seq=96)
    greedy = []
    for p, t in enumerate(prompt):
        lg = g.decode_token(0, t, p)
    tok = oracle.argmax(lg)
    while len(greedy) < n_new + k + 2:
        greedy.append(tok)
        tok = oracle.argmax(g.decode_token(0, tok, prompt_len + len(greedy) - 1))

    m = oracle.build_model(s, seed=1, max_batch=1, max_seq=96)
    for p, t in enumerate(prompt[:-1]):
        m.decode_token(0, t, p)
    lens, last, out, step = prompt_len - 1, prompt[-1], [], 0
    while len(out) < n_new:
        done = len(out)                      # greedy[done:] is the true continuation after `last`
        if draft_kind == "random":
            drafts = uniform_int(61, step, (k,), 0, s.vocab - 1).tolist()
        else:
            drafts = list(greedy[done: done + k])
            if draft_kind == "one_wrong":
                wp = step % (k + 1)
                if wp < k:
                    drafts[wp] = (drafts[wp] + 1) % s.vocab
        r = m.verify_step(torch.tensor([[last] + drafts], dtype=torch.int32), torch.tensor([lens]))
        acc, nxt = int(r["accepted_len"][0]), int(r["next_token"][0])
        if draft_kind == "correct":
            assert acc == k
        if draft_kind == "one_wrong":
            assert acc == step % (k + 1)
        out += drafts[:acc] + [nxt]
        lens += acc + 1
        last = nxt
        step += 1
    assert out[:n_new] == greedy[:n_new]
