"""Pins for the CPU checker's gate arithmetic (Section 3.2 signal d_K, Eq. 2 gate, Eq. 1 advantage).

Each pin is something fixed by the paper or by mathematics, not by the checker itself:
shortest-edit-path search on tiny strings, metric axioms, textbook worked values, the
paper's operating point worked by hand, exact rational comparison, and Table 1's printed
step-token percentages.
"""
import itertools
import os
from collections import deque
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- edit distance by breadth-first search over single edits (the definition itself) ----
def _neighbours(s, alphabet, max_len):
    out = set()
    for i in range(len(s)):
        out.add(s[:i] + s[i + 1:])                       # delete
        for c in alphabet:
            if c != s[i]:
                out.add(s[:i] + (c,) + s[i + 1:])        # substitute
    if len(s) < max_len:
        for i in range(len(s) + 1):
            for c in alphabet:
                out.add(s[:i] + (c,) + s[i:])            # insert
    return out


def _bfs_all(alphabet, max_len):
    nodes = [t for n in range(max_len + 1) for t in itertools.product(alphabet, repeat=n)]
    dist = {}
    for src in nodes:
        d = {src: 0}
        q = deque([src])
        while q:
            u = q.popleft()
            for v in _neighbours(u, alphabet, max_len):
                if v not in d:
                    d[v] = d[u] + 1
                    q.append(v)
        dist[src] = d
    return nodes, dist


@pytest.fixture(scope="module")
def bfs3():
    return _bfs_all((0, 1, 2), 4)


def test_lev_matches_shortest_edit_path_on_all_tiny_strings(bfs3):
    nodes, dist = bfs3
    assert len(nodes) == 121
    for a in nodes:
        for b in nodes:
            assert oracle.lev(a, b) == dist[a][b], (a, b)


def _s(word):
    return [ord(c) for c in word]


@pytest.mark.parametrize("a,b,d", [("kitten", "sitting", 3), ("flaw", "lawn", 2), ("saturday", "sunday", 3),
                                   ("", "abc", 3), ("abc", "", 3), ("", "", 0), ("intention", "execution", 5)])
def test_lev_textbook_values(a, b, d):
    assert oracle.lev(_s(a), _s(b)) == d


def test_lev_metric_axioms_and_bounds():
    rng = np.random.default_rng(1)
    for _ in range(300):
        m, n, k = rng.integers(0, 12, size=3)
        a, b, c = (rng.integers(0, 4, size=x) for x in (m, n, k))
        dab, dba = oracle.lev(a, b), oracle.lev(b, a)
        assert dab == dba
        assert oracle.lev(a, a) == 0
        assert (dab == 0) == (list(a) == list(b))
        assert dab <= oracle.lev(a, c) + oracle.lev(c, b)
        assert abs(int(m) - int(n)) <= dab <= max(m, n)
        if m == n:
            assert dab <= int(np.sum(a != b))
        # disjoint alphabets: nothing can be matched, distance is the longer length
        assert oracle.lev(a, b + 100) == max(m, n)


# ---- the signal d_K and the gate ----
def test_d_K_extremes():
    """d_K = 0 iff all G prefixes identical; d_K = 1 when no two members share an action (Section 3.2)."""
    G, K = 8, 10
    same = np.tile(np.arange(K, dtype=np.int32), (G, 1))
    assert oracle.pair_sum(same, K) == 0 and oracle.mean_prefix_distance(same, K) == 0.0
    disjoint = (np.arange(G)[:, None] * 1000 + np.arange(K)[None, :]).astype(np.int32)
    assert oracle.pair_sum(disjoint, K) == 28 * K and oracle.mean_prefix_distance(disjoint, K) == 1.0
    one_off = same.copy()
    one_off[3, 4] = 99           # one member differs in one step: 7 pairs at distance 1
    assert oracle.pair_sum(one_off, K) == 7
    assert oracle.mean_prefix_distance(one_off, K) == pytest.approx(7 / 280)


def test_gate_bounds_golden():
    for line in open(os.path.join(GOLDEN, "gate_bounds.txt")):
        if line.startswith("#") or not line.strip():
            continue
        G, K, dL, T = line.split()
        assert oracle.gate_bound(float(dL), int(G), int(K)) == int(T), line


def test_gate_is_exact_strict_inequality():
    """cut <=> S/(P*K) < d_L with d_L an exact decimal; compared with Fractions."""
    rng = np.random.default_rng(2)
    for _ in range(2000):
        G = int(rng.integers(2, 17))
        K = int(rng.integers(1, 31))
        P = G * (G - 1) // 2
        micro = int(rng.integers(0, 1_000_001))
        if rng.random() < 0.3:      # land exactly on attainable ratios to exercise the strict '<'
            micro = int(Fraction(int(rng.integers(0, P * K + 1)), P * K) * 1_000_000)
        dL = micro / 1e6
        T = oracle.gate_bound(dL, G, K)
        for S in {0, max(T - 1, 0), T, min(T + 1, P * K), P * K}:
            assert (S < T) == (Fraction(S, P * K) < Fraction(micro, 1_000_000)), (G, K, micro, S)
    assert oracle.gate_bound(0.0, 8, 10) == 0          # d_L = 0 never fires
    assert oracle.gate_bound(0.25, 8, 10) == 70         # 0.25*280 = 70 exactly: S = 70 is NOT cut


def test_pair_sum_invariances():
    rng = np.random.default_rng(3)
    for _ in range(50):
        G, K = int(rng.integers(2, 9)), int(rng.integers(1, 16))
        a = rng.integers(0, 5, size=(G, 20)).astype(np.int32)
        s = oracle.pair_sum(a, K)
        assert oracle.pair_sum(a[rng.permutation(G)], K) == s           # members are unordered
        relabel = rng.permutation(5).astype(np.int32)
        assert oracle.pair_sum(relabel[a], K) == s                      # only equality of symbols matters
        b = a.copy()
        b[:, K:] = rng.integers(0, 5, size=b[:, K:].shape)
        assert oracle.pair_sum(b, K) == s                               # only the first K actions count


def test_gate_enumeration_small(bfs3):
    """Every group with G=3, K=3 over a binary alphabet, against the search-based distance."""
    _, dist = bfs3
    seqs = list(itertools.product((0, 1), repeat=3))
    for d_L in (0.0, 0.2, 1 / 3, 0.34, 0.5, 1.0):
        T = oracle.gate_bound(d_L, 3, 3)
        for trip in itertools.product(seqs, repeat=3):
            S = dist[trip[0]][trip[1]] + dist[trip[0]][trip[2]] + dist[trip[1]][trip[2]]
            acts = np.array(trip, dtype=np.int32)
            assert oracle.pair_sum(acts, 3) == S
            sums, cut = oracle.gate_batch(acts[None], [3], d_L)
            assert sums[0, 0] == S
            assert bool(cut[0, 0]) == (Fraction(S, 9) < Fraction(int(round(d_L * 1e6)), 10 ** 6))
            assert bool(cut[0, 0]) == (S < T)


def test_gate_batch_matches_single_group_calls():
    import synth
    acts, _ = synth.gate_actions(64, 8, 30, 64, seed=5)
    lens = [5, 10, 15]
    sums, cut = oracle.gate_batch(acts, lens, 0.3)
    for li, K in enumerate(lens):
        for g in range(64):
            assert sums[li, g] == oracle.pair_sum(acts[g], K)
            assert cut[li, g] == (sums[li, g] < oracle.gate_bound(0.3, 8, K))


# ---- Table 1 step-token accounting ----
def test_step_token_accounting_reproduces_table1():
    T_max, K, N = 30, 10, 100
    for line in open(os.path.join(GOLDEN, "table1_step_tokens.txt")):
        if line.startswith("#") or not line.strip():
            continue
        dL, cut, tp, safe, raw = line.split()
        assert round(100 * int(tp) * (T_max - K) / (N * T_max), 1) == float(safe)
        assert round(100 * int(cut) * (T_max - K) / (N * T_max), 1) == float(raw)


# ---- Eq. 1 ----
def test_zero_variance_group_has_exactly_zero_advantage():
    for G in (2, 3, 8, 16):
        for r in (0.0, 1.0, 0.1, 1 / 3, -2.7):
            A = oracle.advantage([r] * G)
            assert np.all(A == 0.0) and not np.any(np.signbit(A))


def test_advantage_is_a_z_score():
    rng = np.random.default_rng(4)
    for _ in range(20):
        r = rng.random(8)
        A = oracle.advantage(r, eps=0.0)
        assert abs(A.sum()) < 1e-12
        assert np.mean(A * A) == pytest.approx(1.0, rel=1e-12)
        assert np.all(np.argsort(A) == np.argsort(r))
    A = oracle.advantage([1, 0, 0, 0], eps=0.0)       # mean .25, sigma sqrt(3)/4
    assert A[0] == pytest.approx(0.75 / (np.sqrt(3) / 4)) and A[1] == pytest.approx(-0.25 / (np.sqrt(3) / 4))
