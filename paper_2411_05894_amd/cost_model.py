"""Analytic cost of one verification pass (host side, no GPU work).

Restates the per-operation FLOP and byte counts of the paper's Table 2
(App. B) with tensor parallelism p = 1, adds the LM head the table leaves out,
and gives the "free speculation budget" of Sec. 3.2 / App. B:
``1 / (1/h + 1/(b s_q)) = peak FLOPS / peak bandwidth`` and its simplified
form ``b s_q = I_knee``.  bench.py uses ``algorithmic_bytes`` for the HBM
roofline; nothing here touches the device.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Sequence


@dataclass(frozen=True)
class Dims:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int

    @staticmethod
    def of(shape) -> "Dims":
        return Dims(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                    shape.ffn, shape.vocab)


def table2_flops_per_layer(d: Dims, b: int, s_q: int, s_kv: int) -> Dict[str, float]:
    """FLOPs column of Table 2 (p = 1), one entry per row of the table."""
    h, g = d.n_q_heads * d.head_dim, d.n_q_heads // d.n_kv_heads
    hm = d.ffn
    return {
        "Q": 2.0 * b * s_q * h * h,
        "K_new": 2.0 * b * s_q * h * h / g,
        "V_new": 2.0 * b * s_q * h * h / g,
        "attention": 4.0 * b * s_q * (s_kv + s_q) * h,
        "O": 2.0 * b * s_q * h * h,
        "SwiGLU_in": 4.0 * b * s_q * h * hm,
        "down": 2.0 * b * s_q * h * hm,
    }


def table2_read_bytes_per_layer(d: Dims, b: int, s_q: int, s_kv: int, mask_bytes: bool = True) -> Dict[str, float]:
    """Read column of Table 2 (p = 1); 2 bytes per element, 1 per mask element."""
    h, g = d.n_q_heads * d.head_dim, d.n_q_heads // d.n_kv_heads
    hm = d.ffn
    m = b * s_q
    return {
        "Q": 2.0 * (m * h + h * h),
        "K_new": 2.0 * (m * h + h * h / g),
        "V_new": 2.0 * (m * h + h * h / g),
        "attention": 2.0 * (b * h / g) * (2 * (s_kv + s_q) + g * s_q) + (b * s_q * (s_kv + s_q) if mask_bytes else 0),
        "O": 2.0 * (m * h + h * h),
        "SwiGLU_in": 2.0 * (m * h + 2 * h * hm),
        "down": 2.0 * (m * hm + h * hm),
    }


def weight_bytes(d: Dims) -> int:
    """bf16 bytes of every matrix streamed once per step (layers + LM head)."""
    qd, kd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    per_layer = d.hidden * (qd + 2 * kd) + qd * d.hidden + 3 * d.hidden * d.ffn
    return 2 * (d.n_layers * per_layer + d.vocab * d.hidden)


def kv_bytes_per_token(d: Dims) -> int:
    """bf16 K+V bytes of one cached token over all layers."""
    return 4 * d.n_layers * d.n_kv_heads * d.head_dim


def algorithmic_bytes(d: Dims, lens: Sequence[int], k: int) -> Dict[str, int]:
    """Bytes the step has to move through HBM: every weight once, every valid
    KV row once, the new KV rows written once, the embedding rows read once.
    Activations stay on chip; the causal chain needs no mask tensor; logits are
    not materialised."""
    B = len(lens)
    M = B * (k + 1)
    w = weight_bytes(d)
    kv_r = kv_bytes_per_token(d) * int(sum(lens))
    kv_w = kv_bytes_per_token(d) * M
    emb = 2 * M * d.hidden
    return {"weights": w, "kv_read": kv_r, "kv_write": kv_w, "embed": emb, "total": w + kv_r + kv_w + emb}


def gemm_flops(d: Dims, M: int) -> float:
    """2*M*params over every matrix of the step."""
    return float(M) * weight_bytes(d)          # 2 flops per weight per row, 2 bytes per weight


def free_budget_exact(hidden: int, peak_flops: float, peak_bw: float) -> float:
    """b*s_q solving 1/(1/h + 1/(b s_q)) = peak_flops/peak_bw (App. B equation)."""
    knee = peak_flops / peak_bw
    return 1.0 / (1.0 / knee - 1.0 / hidden)


def free_budget(peak_flops: float, peak_bw: float) -> float:
    """Simplified rule of Sec. 3.2: b*s_q = I_knee = peak FLOPS / peak bandwidth."""
    return peak_flops / peak_bw


def speculation_length(peak_flops: float, peak_bw: float, b: int, cap: int = 32) -> int:
    """s_q = I_knee / b, capped (the paper caps at e.g. 32 for b = 1), at least 1."""
    return max(1, min(cap, int(round(free_budget(peak_flops, peak_bw) / b))))
