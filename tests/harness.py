"""Shared set-up for the GPU parity tests: the same seeded weights and KV on the
device (for the library) and on the host (for the oracle)."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import torch

import oracle
from paper_2411_05894_amd import binding as sv
from sssd_synth import (MODEL_SHAPES, TensorId, global_weight_specs, layer_weight_specs, make_kv_prefill,
                        make_weight, uniform_int)

LOGIT_TOL = 2e-2      # max abs logit error allowed (bf16 kernels vs fp32 oracle)
MARGIN = 1e-2         # token ids must agree wherever the oracle's top-2 margin exceeds this
MAX_EXEMPT_FRAC = 0.25  # at most this share of the compared rows (and never all of them) may be undecided


def check_exempt(exempt: int, rows: int):
    """The id rule only binds rows the oracle decides by more than MARGIN.  Which rows those are depends
    on the oracle alone, so a kernel fault cannot enlarge the set; the bound keeps a test from passing on
    too few decided rows (seeded inputs at vocab 128256 leave about 4 % of rows undecided)."""
    limit = max(1, int(MAX_EXEMPT_FRAC * rows))
    assert exempt <= limit and (rows == 1 or exempt < rows), f"{exempt} of {rows} rows undecided (limit {limit})"


def check_fused_argmax(that, gl, ref_that, decided, where):
    """`that` is the vector the step's own arg-max kernels produced (never read back from stored logits).
    Every row must pick a maximum of the step's own logits; decided rows must pick the oracle's token."""
    for j, t in enumerate(that):
        assert 0 <= t < gl.shape[-1], f"fused arg-max out of range at {where},{j}"
        assert float(gl[j, t]) == float(gl[j].max()), f"fused arg-max is not a maximum of the logits at ({where},{j})"
        first = int((gl[j] == gl[j].max()).nonzero()[0])
        assert t == first, f"fused arg-max does not take the lowest id among equal logits at ({where},{j})"
        if j < len(decided) and decided[j]:
            assert t == int(ref_that[j]), f"fused arg-max differs from the oracle at ({where},{j})"


def gen_weights(shape, seed: int, device, unit_gains: bool = True):
    layers = [{n: make_weight(seed, n, TensorId.layer(l, slot), shp, device=device, unit_gains=unit_gains)
               for n, slot, shp in layer_weight_specs(shape)} for l in range(shape.n_layers)]
    g = {n: make_weight(seed, n, tid, shp, device=device, unit_gains=unit_gains)
         for n, tid, shp in global_weight_specs(shape)}
    return layers, g


def host_copy(layers, g):
    return [{n: t.cpu() for n, t in l.items()} for l in layers], {n: t.cpu() for n, t in g.items()}


class Pair:
    """A library context and an oracle model over identical weights."""

    def __init__(self, shape, seed: int, max_batch: int, max_k: int, max_seq: int, unit_gains: bool = True,
                 in_place: bool = False, oracle_batch: Optional[int] = None):
        dev = torch.device("cuda:0")
        self.shape = shape
        layers, g = gen_weights(shape, seed, dev, unit_gains)
        hl, hg = host_copy(layers, g)
        self.oracle = oracle.OracleModel(shape, hl, hg, oracle_batch or max_batch, max_seq)
        self.cfg = sv.make_config(shape, max_batch, max_k, max_seq)
        self.ctx = sv.VerifyContext(self.cfg, layers, g, in_place=in_place)
        if not in_place:
            del layers          # the packed copy is what the kernels read
        self.dev = dev
        M = max_batch * (max_k + 1)
        self.logits = torch.zeros(M, shape.vocab, dtype=torch.float32, device=dev)
        self.hidden = torch.zeros(M, shape.hidden, dtype=torch.float32, device=dev)
        self.that = torch.full((M,), -1, dtype=torch.int32, device=dev)
        self.ctx.sssd_debug_outputs(self.logits, self.hidden)
        self.ctx.sssd_debug_argmax(self.that)

    def prefill_random_kv(self, seed: int, b: int, n_rows: int, oracle_slot: Optional[int] = None):
        """Cache rows 0..n_rows-1 of sequence b <- N(0,1) bf16, in both caches."""
        s = self.shape
        if n_rows == 0:
            return
        for l in range(s.n_layers):
            K, V = make_kv_prefill(seed * 1000 + b, l, (s.n_kv_heads, n_rows, s.head_dim), device=self.dev)
            self.ctx.sssd_kv_import(l, b, 0, K, V)
            if oracle_slot is not None:
                self.oracle.K[l, oracle_slot, :, :n_rows] = K.cpu()
                self.oracle.V[l, oracle_slot, :, :n_rows] = V.cpu()

    def step(self, tokens: torch.Tensor, lens: torch.Tensor):
        """Run the library on (tokens [B,k+1], lens [B]) given as CPU int32 tensors."""
        B, sq = tokens.shape
        t = tokens.to(self.dev, torch.int32).contiguous()
        ln = lens.to(self.dev, torch.int32).contiguous()
        acc = torch.empty(B, dtype=torch.int32, device=self.dev)
        nxt = torch.empty(B, dtype=torch.int32, device=self.dev)
        self.ctx.sssd_verify_step(t, ln, acc, nxt)
        rc = self.ctx.sssd_verify_sync()
        assert rc == 0, sv.strerror(rc)
        M = B * sq
        return {"logits": self.logits[:M].cpu().view(B, sq, -1), "hidden": self.hidden[:M].cpu().view(B, sq, -1),
                "that": self.that[:M].cpu().view(B, sq), "accepted_len": acc.cpu(), "next_token": nxt.cpu()}


def step_tree(pair: "Pair", tokens: torch.Tensor, parents: torch.Tensor, lens: torch.Tensor):
    """Run the library's tree step on CPU int32 tensors tokens/parents [B,k+1], lens [B]."""
    B, sq = tokens.shape
    dev = pair.dev
    t = tokens.to(dev, torch.int32).contiguous()
    par = parents.to(dev, torch.int32).contiguous()
    ln = lens.to(dev, torch.int32).contiguous()
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty(B, sq, dtype=torch.int32, device=dev)
    pair.ctx.sssd_verify_step_tree(t, par, ln, acc, nxt, path)
    rc = pair.ctx.sssd_verify_sync()
    assert rc == 0, sv.strerror(rc)
    M = B * sq
    return {"logits": pair.logits[:M].cpu().view(B, sq, -1), "hidden": pair.hidden[:M].cpu().view(B, sq, -1),
            "that": pair.that[:M].cpu().view(B, sq), "accepted_len": acc.cpu(), "next_token": nxt.cpu(), "path": path.cpu(),
            "dev": {"accepted_len": acc, "path": path}}


def walk_tree(tokens: Sequence[int], parents: Sequence[int], that: Sequence[int]) -> List[int]:
    """The accepted path the interface defines, from a given arg-max vector (plain Python)."""
    cur, path = 0, [0]
    while True:
        nxt = [c for c in range(cur + 1, len(tokens)) if parents[c] == cur and tokens[c] == that[cur]]
        if not nxt:
            return path
        cur = nxt[0]
        path.append(cur)


def compare_tree_step(gpu: Dict[str, torch.Tensor], ref: Dict[str, torch.Tensor], tokens: torch.Tensor,
                      parents: torch.Tensor, tol: float = LOGIT_TOL):
    """Logits element by element; arg-max ids where the oracle's margin decides them; the accepted
    path against the oracle's when every row on it is decided, and always against the library's
    own logits.  Returns (max_err, exempt_rows, rows)."""
    B, sq = tokens.shape
    max_err, exempt = 0.0, 0
    for b in range(B):
        rl, gl = ref["logits"][b], gpu["logits"][b]
        err = (rl - gl).abs().max().item()
        max_err = max(max_err, err)
        assert err <= tol, f"sequence {b}: max abs logit error {err}"
        decided = []
        for j in range(sq):
            t1, t2 = oracle.top2(rl[j])
            decided.append((t1 - t2) > MARGIN)
            if decided[-1]:
                assert int(gl[j].argmax()) == int(ref["that"][b, j]), f"argmax differs at ({b},{j})"
            else:
                exempt += 1
        if "that" in gpu:
            check_fused_argmax(gpu["that"][b].tolist(), gl, ref["that"][b], decided, b)
        ref_path = ref["path"][b]
        n = int(gpu["accepted_len"][b])
        g_path = gpu["path"][b].tolist()
        if all(decided[i] for i in ref_path):
            assert g_path[: n + 1] == ref_path, f"accepted path differs for sequence {b}"
            assert int(gpu["next_token"][b]) == int(ref["next_token"][b])
        own = walk_tree(tokens[b].tolist(), parents[b].tolist(), gl.argmax(-1).tolist())
        assert g_path[: n + 1] == own and n == len(own) - 1
        assert all(x == -1 for x in g_path[n + 1:])
        assert int(gpu["next_token"][b]) == int(gl[own[-1]].argmax())
    return max_err, exempt, B * sq


def compare_step(gpu: Dict[str, torch.Tensor], ref: Dict[str, torch.Tensor], tokens: torch.Tensor,
                 seqs: Optional[Sequence[int]] = None, tol: float = LOGIT_TOL):
    """Element-by-element logits check plus the id rule; ``seqs`` maps oracle
    sequence i to library sequence seqs[i].  The oracle may cover only the first
    rows of a sequence (row j never depends on later rows); then the logits and
    ids of those rows are compared.  Returns (max_err, exempt_rows, rows)."""
    B, sq_ref = ref["logits"].shape[:2]
    sq = gpu["logits"].shape[1]
    seqs = list(range(B)) if seqs is None else list(seqs)
    max_err, exempt = 0.0, 0
    for i, b in enumerate(seqs):
        rl, gl = ref["logits"][i], gpu["logits"][b]
        err = (rl - gl[:sq_ref]).abs().max().item()
        max_err = max(max_err, err)
        assert err <= tol, f"sequence {b}: max abs logit error {err}"
        row_ok = []
        for j in range(sq_ref):
            t1, t2 = oracle.top2(rl[j])
            decided = (t1 - t2) > MARGIN
            row_ok.append(decided)
            if decided:
                assert int(gl[j].argmax()) == int(ref["that"][i, j]), f"argmax differs at ({b},{j})"
            else:
                exempt += 1
        if "that" in gpu:
            check_fused_argmax(gpu["that"][b].tolist(), gl, ref["that"][i], row_ok, b)
        # acceptance walks rows 0..acc; it is pinned when the oracle covers those rows and all are decided
        acc_ref = int(ref["accepted_len"][i])
        if (sq_ref == sq or acc_ref < sq_ref - 1) and all(row_ok[: acc_ref + 1]):
            assert int(gpu["accepted_len"][b]) == acc_ref, f"accepted_len differs for sequence {b}"
            assert int(gpu["next_token"][b]) == int(ref["next_token"][i]), f"next_token differs for sequence {b}"
        # whatever the rows, the library's outputs must be consistent with its own logits
        g_that = gl.argmax(-1).tolist()
        n = 0
        while n < sq - 1 and int(tokens[b, n + 1]) == g_that[n]:
            n += 1
        assert int(gpu["accepted_len"][b]) == n and int(gpu["next_token"][b]) == g_that[n]
    return max_err, exempt, len(seqs) * sq_ref
