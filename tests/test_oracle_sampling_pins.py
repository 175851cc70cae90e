"""Pins of the oracle's target-only sampler (Sec. 4.4: speculative sampling that preserves the target
distribution without draft probabilities): limits that reduce to arg-max, the plain softmax through
a library routine, a nucleus worked by hand, brute-force inverse CDF, frequencies over a grid of
uniforms, and the emitted distribution of the tree walk."""
import itertools

import numpy as np
import torch

import oracle
from sssd_synth import normal_bf16, uniform_int


def row(seed, V, scale=3.0):
    return normal_bf16(seed, 1, (V,), 1.0).float() * scale


def test_limits_reduce_to_argmax():
    z = row(91, 500)
    best = int(z.argmax())
    for u in (0.0, 0.3, 0.999):
        assert oracle.sample_row(z, 1.0, 1, 1.0, u)[0] == best          # top_k = 1
        assert oracle.sample_row(z, 1.0, 0, 1e-9, u)[0] == best         # vanishing nucleus
        assert oracle.sample_row(z, 1e-4, 0, 1.0, u)[0] == best         # temperature -> 0


def test_plain_sampling_is_the_inverse_cdf_of_softmax():
    z = row(92, 64)
    p = torch.softmax(z.double() / 0.7, dim=0).numpy()                  # library softmax
    assert np.allclose(oracle.target_distribution(z, 0.7, 0, 1.0), p, rtol=1e-12, atol=0)
    cdf = np.cumsum(p)
    for u in np.linspace(0.001, 0.999, 97):
        want = int(next(i for i in range(64) if cdf[i] > u))            # brute force, token id order
        assert oracle.sample_row(z, 0.7, 0, 1.0, float(u))[0] == want


def test_nucleus_and_top_k_worked_by_hand():
    # probabilities 0.5, 0.25, 0.15, 0.1 (ids 2, 0, 3, 1) at temperature 1
    p = np.array([0.25, 0.1, 0.5, 0.15])
    z = torch.tensor(np.log(p), dtype=torch.float32)
    d = oracle.target_distribution(z, 1.0, 0, 0.7)                      # 0.5 + 0.25 reaches 0.7
    assert np.allclose(d, [1 / 3, 0, 2 / 3, 0], atol=1e-6)
    d = oracle.target_distribution(z, 1.0, 0, 0.76)                     # needs the third token
    assert np.allclose(d, [0.25 / 0.9, 0, 0.5 / 0.9, 0.15 / 0.9], atol=1e-6)
    d = oracle.target_distribution(z, 1.0, 3, 1.0)                      # top-3
    assert np.allclose(d, [0.25 / 0.9, 0, 0.5 / 0.9, 0.15 / 0.9], atol=1e-6)
    d = oracle.target_distribution(z, 1.0, 3, 0.6)                      # top-3, then 0.6 of the 0.9 kept = 0.54 -> two tokens
    assert np.allclose(d, [1 / 3, 0, 2 / 3, 0], atol=1e-6)
    # inverse CDF in token-id order over S = {0, 2} with masses 1/3, 2/3
    assert oracle.sample_row(z, 1.0, 0, 0.7, 0.30)[0] == 0
    assert oracle.sample_row(z, 1.0, 0, 0.7, 0.34)[0] == 2
    # equal logits: the lower token id comes first in the order
    z2 = torch.tensor([1.0, 2.0, 2.0, 2.0, 0.5])
    assert np.allclose(oracle.target_distribution(z2, 1.0, 2, 1.0), [0, 0.5, 0.5, 0, 0])


def test_frequencies_over_a_grid_of_uniforms_match_the_distribution():
    z = row(93, 40, scale=2.0)
    for T, k, p in ((1.0, 0, 1.0), (0.6, 0, 0.95), (0.7, 20, 0.8), (1.3, 7, 1.0)):
        d = oracle.target_distribution(z, T, k, p)
        N = 4000
        counts = np.zeros(40)
        for i in range(N):
            counts[oracle.sample_row(z, T, k, p, (i + 0.5) / N)[0]] += 1
        assert np.abs(counts / N - d).max() <= 1.0 / N + 1e-12
        assert abs(d.sum() - 1) < 1e-12


def test_margin_reports_the_distance_to_the_nearest_decision():
    p = np.array([0.25, 0.1, 0.5, 0.15])
    z = torch.tensor(np.log(p), dtype=torch.float32)
    _, m = oracle.sample_row(z, 1.0, 0, 1.0, 0.2500001)
    assert m < 1e-6
    _, m = oracle.sample_row(z, 1.0, 0, 1.0, 0.6)
    assert abs(m - 0.25) < 1e-6                                         # cdf 0.25 | 0.35 | 0.85: 0.6 is 0.25 from both
    # nucleus cut within 1e-7 of a threshold: token 3 (mass 0.15) may or may not be in S
    t, m = oracle.sample_row(z, 1.0, 0, 0.7500001, 0.1, w_noise=1e-6)
    # S = {0, 2, 3} (Z_S = 0.9), r = 0.09 lies 0.16 below the first step; token 3's 0.15 is uncertain
    assert t == 0 and abs(m - (0.16 - 0.15) / 0.9) < 1e-5
    _, m0 = oracle.sample_row(z, 1.0, 0, 0.7500001, 0.1)
    assert m0 > 0.09                                                    # without noise the cut is a plain decision
    # a logit within the noise of the top-k threshold makes that token's membership uncertain
    z3 = torch.tensor([2.0, 1.0, 0.99995, 0.0])
    t, m = oracle.sample_row(z3, 1.0, 2, 1.0, 0.99, logit_noise=1e-4)
    assert t == 1 and m == 0.0
    t, m = oracle.sample_row(z3, 1.0, 2, 1.0, 0.99)
    assert t == 1 and m > 0.0


def test_tree_walk_emits_exact_samples_of_the_target():
    """One node with two children: over a grid of uniforms the first emitted token is distributed as
    the target, whatever the drafts are (accepted child or bonus token)."""
    p = np.array([0.4, 0.3, 0.2, 0.1])
    that_for = lambda u: int(np.searchsorted(np.cumsum(p), u, side="right"))
    tokens, parents = [9, 1, 3], [0, 0, 0]
    N, counts, accepted = 2000, np.zeros(4), 0
    for i in range(N):
        t = that_for((i + 0.5) / N)
        acc, nxt, path = oracle.accept_tree(tokens, parents, [t, 0, 0])
        first = tokens[path[1]] if acc else nxt
        counts[first] += 1
        accepted += acc
    assert np.abs(counts / N - p).max() <= 1.0 / N
    assert abs(accepted / N - (p[1] + p[3])) <= 2.0 / N               # a draft is accepted with its target probability
