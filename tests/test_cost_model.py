"""Cost model vs the paper's printed example and vs what the oracle executes."""
import os

import torch

import oracle
from paper_2411_05894_amd import cost_model as cm
from sssd_synth import MODEL_SHAPES, uniform_int

GOLD = os.path.join(os.path.dirname(__file__), "golden", "knee_example.txt")


def test_knee_example_printed_in_paper():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    for h, tf, tb, b, printed_bsq, printed_sq in rows:
        budget = cm.free_budget(float(tf) * 1e12, float(tb) * 1e12)
        assert round(budget) == int(printed_bsq)                     # 173.7 -> "~174"
        assert cm.speculation_length(float(tf) * 1e12, float(tb) * 1e12, int(b)) == int(printed_sq)
        exact = cm.free_budget_exact(int(h), float(tf) * 1e12, float(tb) * 1e12)
        assert 174 < exact < 190                                     # keeping 1/h moves it to ~181
    assert cm.speculation_length(2.5e15, 8e12, 1) == 32              # cap at b = 1


def test_table2_flops_match_executed_macs(tiny_shape):
    s = tiny_shape
    d = cm.Dims.of(s)
    B, k, ctx = 2, 3, 10
    m = oracle.build_model(s, seed=1, max_batch=B, max_seq=32)
    tok = uniform_int(70, 0, (B, k + 1), 0, s.vocab - 1)
    oracle.counters_reset()
    m.verify_step(tok, torch.tensor([ctx, ctx]))
    lin, att = oracle.counters()
    t2 = cm.table2_flops_per_layer(d, B, k + 1, ctx)
    lin_t2 = sum(v for n, v in t2.items() if n != "attention") * s.n_layers + 2.0 * B * (k + 1) * s.hidden * s.vocab
    assert 2 * lin == lin_t2
    # Table 2 charges every query row the full s_kv + s_q keys; the causal chain
    # executes sum_j (s_kv + j + 1) of them.
    full = t2["attention"] * s.n_layers
    causal = sum(4.0 * B * (ctx + j + 1) * d.n_q_heads * d.head_dim for j in range(k + 1)) * s.n_layers
    assert 2 * att == causal and causal <= full
    assert cm.gemm_flops(d, B * (k + 1)) == lin_t2


def test_byte_budget_of_the_8b_and_70b_configs():
    d8, d70 = cm.Dims.of(MODEL_SHAPES["8b"]), cm.Dims.of(MODEL_SHAPES["70b"])
    assert abs(cm.weight_bytes(d8) / 1e9 - 15.009) < 1e-3
    assert abs(cm.weight_bytes(d70) / 1e9 - 139.003) < 1e-3
    assert cm.kv_bytes_per_token(d8) == 128 * 1024 and cm.kv_bytes_per_token(d70) == 320 * 1024
    b = cm.algorithmic_bytes(d8, [2048], 8)
    assert abs(b["total"] / 1e9 - 15.28) < 0.01
    # read bytes of Table 2 at p=1 are dominated by the weights: 2*params per layer
    r = cm.table2_read_bytes_per_layer(d8, 1, 1, 0, mask_bytes=False)
    lin = sum(v for n, v in r.items() if n != "attention")
    per_layer_w = (cm.weight_bytes(d8) - 2 * d8.vocab * d8.hidden) / d8.n_layers
    assert 0 < lin - per_layer_w < 2 * (5 * d8.hidden + d8.ffn) + 1
