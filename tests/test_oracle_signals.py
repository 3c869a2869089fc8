"""Pins for the checker's Appendix-B signals and the two-clause gate (Appendix E, Eq. 3).

Every expected value here comes from the paper's definitions worked by hand, from closed forms, from a
library routine (scipy's entropy) or from a second, independent evaluation written in this file with
Python sets, exact fractions and a memoised recursion -- never from the checker itself.
"""
import functools
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.stats import entropy as scipy_entropy

import oracle

RUNNING = 10 ** 6


def lev_rec(a, b):
    a, b = tuple(a), tuple(b)

    @functools.lru_cache(maxsize=None)
    def f(i, j):
        if i == 0:
            return j
        if j == 0:
            return i
        return min(f(i - 1, j) + 1, f(i, j - 1) + 1, f(i - 1, j - 1) + (a[i - 1] != b[j - 1]))

    return f(len(a), len(b))


def brute(actions, obs, end, K):
    """Appendix B, straight from the prose, in exact arithmetic where the quantity is rational."""
    G = len(actions)
    pre = [tuple(actions[i][:min(K, end[i])]) for i in range(G)]
    pairs = [(i, j) for i in range(G) for j in range(i + 1, G)]
    d = Fraction(0)
    jac = Fraction(0)
    plain = 0
    for i, j in pairs:
        longer = max(len(pre[i]), len(pre[j]))
        plain += lev_rec(pre[i], pre[j])
        if longer:
            d += Fraction(lev_rec(pre[i], pre[j]), longer)
        A = set(zip(pre[i][:-1], pre[i][1:]))
        B = set(zip(pre[j][:-1], pre[j][1:]))
        jac += 1 - Fraction(len(A & B), len(A | B)) if A | B else 0
    at = [i for i in range(G) if len(pre[i]) == K]
    acts = [actions[i][K - 1] for i in at]
    counts = [acts.count(v) for v in sorted(set(acts))]
    return {
        "d": d / len(pairs), "jac": jac / len(pairs), "lev_sum": plain, "unique_prefix": len(set(pre)),
        "n_at_step": len(at),
        "unique_action": len(set(acts)), "unique_obs": len({obs[i][K - 1] for i in at}),
        "entropy": float(scipy_entropy(counts)) if counts else 0.0, "n_done": sum(e <= K for e in end),
    }


def one(actions, K, d_L=0.3, tau_H=2.0, obs=None, end=None):
    a = np.asarray(actions, dtype=np.int32)[None]
    o = None if obs is None else np.asarray(obs, dtype=np.int32)[None]
    e = None if end is None else np.asarray(end, dtype=np.int32)[None]
    return oracle.signals_batch(a, [K], d_L, tau_H, obs=o, end_step=e)[0, 0]


def test_lcm_constant():
    assert oracle.lcm32() == math.lcm(*range(1, 33))


def test_identical_members_are_zero_everywhere():
    # Appendix B: every signal is 0 (unique ratios at their minimum 1/G) when the trajectories coincide
    r = one([[3, 1, 4, 1, 5]] * 6, 5, obs=[[7, 7, 7, 7, 7]] * 6)
    assert r["d_K"] == 0.0 and r["lev_scaled"] == 0 and r["bigram_jaccard"] == 0.0
    assert r["unique_prefix"] == 1 and r["unique_action"] == 1 and r["unique_obs"] == 1
    assert r["action_entropy"] == 0.0 and r["n_at_step"] == 6 and r["n_done"] == 0
    assert r["cut_d"] == 1


def test_disjoint_members_are_maximal():
    # Section 3.2: d_K = 1 when no two trajectories share any action; entropy of G distinct symbols is ln G
    G, K = 5, 4
    acts = [[100 * i + t for t in range(K)] for i in range(G)]
    r = one(acts, K, obs=acts)
    assert r["d_K"] == 1.0 and r["bigram_jaccard"] == 1.0
    assert r["lev_scaled"] == oracle.lcm32() * (G * (G - 1) // 2)
    assert r["unique_prefix"] == G and r["unique_action"] == G and r["unique_obs"] == G
    assert abs(r["action_entropy"] - math.log(G)) < 1e-15
    assert r["cut_d"] == 0


def test_longer_length_normalises_each_pair():
    # a = 123, b = 1234 (b still running at K = 4, a finished after 3 steps): lev 1, longer 4 -> 1/4
    r = one([[1, 2, 3, 9], [1, 2, 3, 4]], 4, end=[3, RUNNING])
    assert r["d_K"] == 0.25 and r["lev_scaled"] == oracle.lcm32() // 4
    assert r["n_at_step"] == 1 and r["n_done"] == 1 and r["unique_prefix"] == 2
    # dividing by the shorter length would give 1/3; by K for a pair that both stopped at 2 would give 0
    r = one([[1, 2, 7, 7], [1, 5, 8, 8]], 4, end=[2, 2])
    assert r["d_K"] == 0.5                      # lev(12, 15) = 1, both lengths 2


def test_strict_threshold_with_unequal_lengths():
    acts, end = [[1, 2, 3, 9], [1, 2, 3, 4]], [3, RUNNING]       # d_K = 0.25 exactly
    assert one(acts, 4, d_L=0.25, end=end)["cut_d"] == 0          # Eq. 2 is strict
    assert one(acts, 4, d_L=0.250001, end=end)["cut_d"] == 1
    assert one(acts, 4, d_L=0.249999, end=end)["cut_d"] == 0
    # thirds are not representable in binary: 123, 124, 156 -> pairs 1/3, 2/3, 2/3 -> mean 5/9
    acts = [[1, 2, 3], [1, 2, 4], [1, 5, 6]]
    assert one(acts, 3, d_L=0.555555)["cut_d"] == 0               # 5/9 = 0.5555555...
    assert one(acts, 3, d_L=0.555556)["cut_d"] == 1


def test_bigram_sets_not_multisets():
    # A = {(1,2),(2,1)}, B = {(1,2),(2,9)}: overlap 1 of 3 -> distance 2/3
    r = one([[1, 2, 1, 2, 1], [1, 2, 9, 0, 0]], 5, end=[RUNNING, 3])
    assert abs(r["bigram_jaccard"] - 2 / 3) < 1e-15
    # one-step prefixes have no bigram: two empty sets count as identical
    assert one([[1, 5], [2, 6]], 1)["bigram_jaccard"] == 0.0


def test_entropy_is_in_nats_and_over_step_k_only():
    r = one([[9, 1], [9, 1], [9, 2], [9, 2]], 2)
    assert abs(r["action_entropy"] - math.log(2)) < 1e-15 and r["unique_action"] == 2
    assert abs(one([[1, 1], [2, 1], [3, 1], [4, 1]], 2)["action_entropy"]) == 0.0   # step-2 action is shared


def test_termination_fraction_and_or_rule():
    acts = [[i, 10 + i, 20 + i, 30 + i] for i in range(8)]        # all different: the d clause never fires
    end = [2, 3, 3, 4, RUNNING, RUNNING, RUNNING, RUNNING]
    for K, done in ((1, 0), (2, 1), (3, 3), (4, 4)):
        r = one(acts, K, d_L=0.12, tau_H=0.5, end=end)
        assert r["n_done"] == done and r["cut_d"] == 0
        assert r["cut_or"] == (1 if done * 2 >= 8 else 0)          # tau_K >= 0.5, not strict (Eq. 3)
    assert one(acts, 4, d_L=0.12, tau_H=0.500001, end=end)["cut_or"] == 0
    # the d clause alone also fires the two-clause gate
    assert one([[1, 2]] * 4, 2, d_L=0.12, tau_H=0.9)["cut_or"] == 1


def test_equal_lengths_reduce_to_the_pinned_gate():
    rng = np.random.default_rng(5)
    acts = rng.integers(0, 4, size=(200, 8, 12)).astype(np.int32)
    acts[::3, 1:] = acts[::3, :1]                                  # some converging groups
    lens = [3, 7, 12]
    sums, cut = oracle.gate_batch(acts, lens, 0.3)
    sig = oracle.signals_batch(acts, lens, 0.3)
    for li, K in enumerate(lens):
        assert np.array_equal(sig["lev_scaled"][li], sums[li].astype(np.int64) * (oracle.lcm32() // K))
        assert np.array_equal(sig["cut_d"][li], cut[li]) and np.array_equal(sig["lev_sum"][li], sums[li])
        assert np.allclose(sig["d_K"][li], sums[li] / (28 * K), rtol=0, atol=1e-15)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_the_definitions_worked_in_python(seed):
    rng = np.random.default_rng(seed)
    n_groups, G, stride = 60, int(rng.integers(2, 7)), 7
    acts = rng.integers(0, 3, size=(n_groups, G, stride)).astype(np.int32)
    obs = rng.integers(0, 2, size=(n_groups, G, stride)).astype(np.int32)
    end = np.where(rng.random((n_groups, G)) < 0.4, rng.integers(1, stride + 1, size=(n_groups, G)), RUNNING)
    acts[::4, 1:] = acts[::4, :1]
    lens = [1, 2, 4, 7]
    sig = oracle.signals_batch(acts, lens, 0.3, 0.5, obs=obs, end_step=end)
    P = G * (G - 1) // 2
    for li, K in enumerate(lens):
        for g in range(n_groups):
            ref = brute(acts[g].tolist(), obs[g].tolist(), end[g].tolist(), K)
            r = sig[li, g]
            assert Fraction(int(r["lev_scaled"]), oracle.lcm32() * P) == ref["d"]
            assert abs(r["d_K"] - float(ref["d"])) < 1e-14
            assert abs(r["bigram_jaccard"] - float(ref["jac"])) < 1e-14
            for k in ("unique_prefix", "n_at_step", "unique_action", "unique_obs", "n_done", "lev_sum"):
                assert r[k] == ref[k], (k, K, g)
            assert abs(r["action_entropy"] - ref["entropy"]) < 1e-14
            assert r["cut_d"] == (ref["d"] < Fraction(3, 10))
            assert r["cut_or"] == (ref["d"] < Fraction(3, 10) or Fraction(ref["n_done"], G) >= Fraction(1, 2))
