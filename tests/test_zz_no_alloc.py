"""The GEMM entry point that allocates nothing (its split-K partial sums live in a device array inside
the library image) against the entry point that takes the caller's scratch: same bits, on calls in a
row that share the array, a larger problem first and a smaller one after it."""
import os
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_05894_amd import binding as sv
from sssd_synth import normal_bf16

DEV = "cuda:0"


def _case(seed, M, N, K):
    w = normal_bf16(seed, N * 3 + K, (N, K), 0.02, device=DEV)
    x = normal_bf16(seed + 1, M * 7 + K, (M, K), 1.0, device=DEV).float() * 1.25
    x += 2.0 ** -10 * normal_bf16(seed + 2, M + K, (M, K), 1.0, device=DEV).float()
    hi, lo = sv.sssd_op_pack_activation(x)
    return w, x, hi, lo, sv.sssd_op_pack_weight(w)


def test_static_scratch_gemm_equals_the_workspace_gemm_on_calls_in_a_row():
    limit = sv.sssd_op_gemm_static_scratch_limit()
    # (M, N, K): all split K over workgroups, i.e. all use the scratch array; sizes shrink from call to call
    shapes = [(16, 4096, 14336), (5, 512, 8192), (100, 688, 4096), (3, 256, 8192)]
    cases = [_case(41 + 3 * i, *s) for i, s in enumerate(shapes)]
    needs = [sv.lib().sssd_op_gemm_scratch_bytes(*s) for s in shapes]
    assert all(0 < n <= limit for n in needs), needs
    assert needs[0] > needs[1] and needs[2] > needs[3]
    outs = [torch.full((s[0], s[1]), float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (M, N, K), (w, x, hi, lo, wp), out in zip(shapes, cases, outs):          # back to back on one stream
        sv.sssd_op_gemm_static(hi, lo, wp, M, N, K, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before                              # torch allocated nothing either
    for (M, N, K), (w, x, hi, lo, wp), out in zip(shapes, cases, outs):
        want = sv.sssd_op_gemm(hi, lo, wp, M, N, K)
        assert torch.equal(out, want), (M, N, K)
        ref = oracle.linear(x.cpu(), w.cpu())
        assert (out.cpu() - ref).abs().max().item() <= 3e-5 * ref.abs().max().item() + 1e-6, (M, N, K)
    # and again in the opposite order: the array keeps the last call's contents, which must not matter
    for (M, N, K), (w, x, hi, lo, wp), out in reversed(list(zip(shapes, cases, outs))):
        again = torch.full_like(out, float("nan"))
        sv.sssd_op_gemm_static(hi, lo, wp, M, N, K, again)
        assert torch.equal(again, out), (M, N, K)


def test_static_scratch_gemm_without_a_split_and_beyond_the_limit():
    M, N, K = 7, 512, 256                                                       # K not split: the array is not touched
    w, x, hi, lo, wp = _case(61, M, N, K)
    assert sv.lib().sssd_op_gemm_scratch_bytes(M, N, K) == 0
    out = torch.empty(M, N, dtype=torch.float32, device=DEV)
    sv.sssd_op_gemm_static(hi, lo, wp, M, N, K, out)
    assert torch.equal(out, sv.sssd_op_gemm(hi, lo, wp, M, N, K))
    # a shape whose partial sums do not fit the array is refused before anything is launched
    big = (160, 128256, 4096)
    assert sv.lib().sssd_op_gemm_scratch_bytes(*big) > sv.sssd_op_gemm_static_scratch_limit()
    with pytest.raises(sv.SssdError) as ei:
        sv.sssd_op_gemm_static(hi, lo, wp, *big, out)
    assert ei.value.code == sv.SSSD_ECAPACITY
