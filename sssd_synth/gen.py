"""Counter-based seeded generators (see package docstring for the recipe)."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Tuple

import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(u: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit value."""
    u &= _M64
    return u - (1 << 64) if u >= (1 << 63) else u


def _mix_python(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _key(seed: int, tensor_id: int) -> int:
    return _mix_python(_mix_python(seed * _GOLDEN + 0x1234567) ^ (tensor_id * _C1 + 0x89ABCDEF))


def hash_u64_python(seed: int, tensor_id: int, counter: int) -> int:
    """Reference (pure Python integers) of the hash the tensor code computes."""
    return _mix_python(_key(seed, tensor_id) + counter * _GOLDEN)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_tensor(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _hash_tensor(seed: int, tensor_id: int, counter: torch.Tensor) -> torch.Tensor:
    return _mix_tensor(counter * _s64(_GOLDEN) + _s64(_key(seed, tensor_id)))


_IH_SIGMA = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)
_CHUNK = 1 << 24


def _irwin_hall(seed: int, tensor_id: int, start: int, stop: int, device) -> torch.Tensor:
    idx = torch.arange(start, stop, dtype=torch.int64, device=device)
    total = torch.zeros_like(idx)
    for j in range(2):
        h = _hash_tensor(seed, tensor_id, idx * 2 + j)
        for f in range(4):
            total += _lsr(h, 16 * f) & 0xFFFF
    return total - 4 * 65535


def normal_bf16(seed: int, tensor_id: int, shape, std: float, device="cpu",
                out: torch.Tensor | None = None) -> torch.Tensor:
    """bf16 tensor of approximately N(0, std) values (Irwin-Hall, n = 8)."""
    n = 1
    for s in shape:
        n *= int(s)
    if out is None:
        out = torch.empty(n, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    assert flat.numel() == n
    scale = std / _IH_SIGMA
    for start in range(0, n, _CHUNK):
        stop = min(n, start + _CHUNK)
        s = _irwin_hall(seed, tensor_id, start, stop, flat.device)
        flat[start:stop] = (s.to(torch.float64) * scale).to(torch.float32).to(torch.bfloat16)
    return out.view(*shape)


def uniform_int(seed: int, tensor_id: int, shape, low: int, high: int, device="cpu",
                dtype=torch.int32) -> torch.Tensor:
    """Integers uniform on [low, high] (inclusive)."""
    n = 1
    for s in shape:
        n *= int(s)
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h = _hash_tensor(seed, tensor_id, idx) & ((1 << 63) - 1)
    return (h % (high - low + 1) + low).to(dtype).view(*shape)


def uniform_bf16(seed: int, tensor_id: int, shape, low: float, high: float, device="cpu") -> torch.Tensor:
    """bf16 values uniform on [low, high) with 16-bit resolution."""
    n = 1
    for s in shape:
        n *= int(s)
    idx = torch.arange(n, dtype=torch.int64, device=device)
    u = (_hash_tensor(seed, tensor_id, idx) & 0xFFFF).to(torch.float64) / 65536.0
    return (u * (high - low) + low).to(torch.float32).to(torch.bfloat16).view(*shape)


def repetitive_stream(seed: int, tensor_id: int, n: int, vocab: int, n_templates: int = 12, min_len: int = 4,
                      max_len: int = 14, noise: float = 0.05) -> "list[int]":
    """Token stream with the n-gram repetition that retrieval-based drafting feeds on: a seeded
    set of templates (random token runs of min_len..max_len tokens) concatenated in a seeded random
    order, with a fraction `noise` of the tokens replaced by uniform-random ids.  It stands in for
    the prompt / self-output and datastore text of the paper's chat, code and maths workloads."""
    lens = uniform_int(seed, tensor_id * 8 + 1, (n_templates,), min_len, max_len).tolist()
    body = uniform_int(seed, tensor_id * 8 + 2, (n_templates, max_len), 0, vocab - 1).tolist()
    templates = [body[i][: lens[i]] for i in range(n_templates)]
    pick = uniform_int(seed, tensor_id * 8 + 3, (n,), 0, n_templates - 1).tolist()
    flip = uniform_int(seed, tensor_id * 8 + 4, (n,), 0, 999_999).tolist()
    rand = uniform_int(seed, tensor_id * 8 + 5, (n,), 0, vocab - 1).tolist()
    out: "list[int]" = []
    i = 0
    while len(out) < n:
        out += templates[pick[i]]
        i += 1
    out = out[:n]
    thresh = int(noise * 1_000_000)
    return [rand[j] if flip[j] < thresh else out[j] for j in range(n)]


class TensorId:
    """Tensor ids: globals below 16, per-layer tensors at 16 + 16*layer + slot."""
    EMBED, LM_HEAD, FINAL_NORM, TOKENS, LENS, PROMPT, REPLACE_POS, REPLACE_TOK = range(8)
    KV_K, KV_V = 8, 9
    WQ, WK, WV, WO, W_GATE, W_UP, W_DOWN, ATTN_NORM, MLP_NORM = range(9)

    @staticmethod
    def layer(layer: int, slot: int) -> int:
        return 16 + 16 * layer + slot

    @staticmethod
    def kv(layer: int, which: int) -> int:
        return (1 << 20) + 2 * layer + (which - TensorId.KV_K)


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float
    rope_base: float


MODEL_SHAPES: Dict[str, ModelShape] = {
    # The benchmark configurations: tiny parity model, Llama-3-8B shape, Llama-3-70B shape.
    "tiny": ModelShape("tiny", 2, 256, 4, 2, 64, 688, 1024, 1e-5, 10000.0),
    "8b": ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 500000.0),
    "70b": ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 128256, 1e-5, 500000.0),
}


def layer_weight_specs(s: ModelShape) -> List[Tuple[str, int, Tuple[int, ...]]]:
    """(name, slot, shape) of every per-layer tensor; matrices are [out][in]."""
    qd = s.n_q_heads * s.head_dim
    kd = s.n_kv_heads * s.head_dim
    T = TensorId
    return [
        ("wq", T.WQ, (qd, s.hidden)), ("wk", T.WK, (kd, s.hidden)), ("wv", T.WV, (kd, s.hidden)),
        ("wo", T.WO, (s.hidden, qd)),
        ("w_gate", T.W_GATE, (s.ffn, s.hidden)), ("w_up", T.W_UP, (s.ffn, s.hidden)),
        ("w_down", T.W_DOWN, (s.hidden, s.ffn)),
        ("attn_norm", T.ATTN_NORM, (s.hidden,)), ("mlp_norm", T.MLP_NORM, (s.hidden,)),
    ]


def global_weight_specs(s: ModelShape) -> List[Tuple[str, int, Tuple[int, ...]]]:
    T = TensorId
    return [("embed", T.EMBED, (s.vocab, s.hidden)), ("lm_head", T.LM_HEAD, (s.vocab, s.hidden)),
            ("final_norm", T.FINAL_NORM, (s.hidden,))]


def make_weight(seed: int, name: str, tensor_id: int, shape, device="cpu", unit_gains: bool = True,
                std: float = 0.02) -> torch.Tensor:
    """One weight tensor: matrices ~N(0, std); norm gains all-ones, or
    U[0.5, 1.5) when ``unit_gains`` is False (kernel unit tests)."""
    if name.endswith("norm"):
        if unit_gains:
            return torch.ones(shape, dtype=torch.bfloat16, device=device)
        return uniform_bf16(seed, tensor_id, shape, 0.5, 1.5, device)
    return normal_bf16(seed, tensor_id, shape, std, device)


def make_kv_prefill(seed: int, layer: int, shape, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Random 'prefilled' K and V ~N(0,1), bf16, of the given shape."""
    k = normal_bf16(seed, TensorId.kv(layer, TensorId.KV_K), shape, 1.0, device)
    v = normal_bf16(seed, TensorId.kv(layer, TensorId.KV_V), shape, 1.0, device)
    return k, v
