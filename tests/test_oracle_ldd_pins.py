"""Pins for the logit-distance oracle (oracle/ldd.py): hand-computed values, identities of the
two divergences, and for the top-K distance an independent linear-programming solution of its
defining minimisation plus the brute-force evaluation and the Lipschitz property.  CPU only."""
import math

import numpy as np
import pytest
from scipy.optimize import linprog

from oracle import ldd
from tests.test_oracle_pins import G


def test_tv_kl_hand_values():
    g = G["LDD"]
    l = np.array(g["tv_l"])
    lref = np.log(np.array(g["tv_lref_ratio"]))
    assert ldd.tv_distance(l, lref) == pytest.approx(g["tv"], abs=1e-15)
    assert math.exp(2 * ldd.kl_divergence(l, lref)) == pytest.approx(g["kl_times_2_exp"], rel=1e-14)


def test_tv_kl_identities():
    rng = np.random.default_rng(0)
    for n in (2, 17, 1000):
        x, y = rng.normal(0, 3, n), rng.normal(0, 3, n)
        tv, kl = ldd.tv_distance(x, y), ldd.kl_divergence(x, y)
        assert 0.0 <= tv <= 1.0 and kl >= 0.0
        assert tv <= math.sqrt(kl / 2) + 1e-12                       # Pinsker
        assert ldd.tv_distance(x, x) == 0.0 and abs(ldd.kl_divergence(x, x)) < 1e-15
        assert ldd.tv_distance(x + 7.5, y - 2.0) == pytest.approx(tv, abs=1e-14)   # shift invariance
        assert ldd.kl_divergence(x + 7.5, y - 2.0) == pytest.approx(kl, abs=1e-12)
        assert ldd.tv_distance(x, y) == pytest.approx(ldd.tv_distance(y, x), abs=1e-15)
        # TV = 1 - sum_i min(p_i, q_i)
        p, q = ldd.softmax64(x), ldd.softmax64(y)
        assert tv == pytest.approx(1.0 - np.minimum(p, q).sum(), abs=1e-14)
    # nearly disjoint supports
    a = np.array([50.0, 0.0]); b = np.array([0.0, 50.0])
    assert ldd.tv_distance(a, b) == pytest.approx(1.0, abs=1e-20 + 4e-22 * 1e22 * 1e-21 + 1e-15)
    # large logits do not overflow
    assert math.isfinite(ldd.kl_divergence(np.array([1e4, 0.0]), np.array([0.0, 1e4])))


def test_tail_density():
    d = np.array([0.05, 0.11, 0.3, 0.1, 0.09])
    assert ldd.tail_density(d, 0.1) == 2 / 5
    assert ldd.tail_density(d, 1.0) == 0.0 and ldd.tail_density(d, 0.0) == 1.0


def test_topk_hand_values():
    g = G["TOPK"]
    x = np.array(g["logits"])
    for c in ("case1", "case2", "case3"):
        assert ldd.topk_distance(x, g[c + "_idx"]) == g[c]
        assert ldd.topk_distance_bruteforce(x, g[c + "_idx"]) == g[c]


def lp_topk(x, idx):
    """min sum |l' - l|  s.t.  l'_i >= t (i in I), l'_j <= t (j not in I);  variables l', t, slacks."""
    n = len(x)
    member = np.zeros(n, dtype=bool); member[idx] = True
    # variables: l'(n), t(1), s(n) with s_i >= |l'_i - x_i|
    c = np.concatenate([np.zeros(n + 1), np.ones(n)])
    A, b = [], []
    for i in range(n):
        row = np.zeros(2 * n + 1); row[i] = 1; row[n + 1 + i] = -1; A.append(row); b.append(x[i])      # l' - s <= x
        row = np.zeros(2 * n + 1); row[i] = -1; row[n + 1 + i] = -1; A.append(row); b.append(-x[i])    # -l' - s <= -x
        row = np.zeros(2 * n + 1)
        if member[i]:
            row[i] = -1; row[n] = 1      # t - l'_i <= 0
        else:
            row[i] = 1; row[n] = -1      # l'_j - t <= 0
        A.append(row); b.append(0.0)
    res = linprog(c, A_ub=np.array(A), b_ub=np.array(b), bounds=[(None, None)] * (n + 1) + [(0, None)] * n,
                  method="highs")
    assert res.status == 0
    return res.fun


def test_topk_matches_linear_program_and_bruteforce():
    rng = np.random.default_rng(1)
    for trial in range(40):
        n = int(rng.integers(3, 12)); K = int(rng.integers(1, n))
        x = np.round(rng.normal(0, 2, n), 2)
        if trial % 4 == 0:
            x[rng.integers(0, n)] = x[rng.integers(0, n)]          # ties
        idx = rng.choice(n, K, replace=False)
        want = lp_topk(x, idx)
        assert ldd.topk_distance_bruteforce(x, idx) == pytest.approx(want, abs=1e-8)
        assert ldd.topk_distance(x, idx) == pytest.approx(want, abs=1e-8)


def test_topk_zero_iff_valid_and_lipschitz():
    rng = np.random.default_rng(2)
    for _ in range(20):
        n, K = 200, 7
        x = rng.normal(0, 3, n)
        top = np.argsort(-x)[:K]
        assert ldd.topk_distance(x, top) == 0.0
        bad = top.copy(); bad[0] = np.argsort(-x)[K + 3]
        d = ldd.topk_distance(x, bad)
        assert d > 0 and d == pytest.approx(ldd.topk_distance_bruteforce(x, bad), rel=1e-12)
        # swapping in the runner-up costs exactly the gap between the two values
        sw = top.copy(); sw[K - 1] = np.argsort(-x)[K]
        gap = np.sort(x)[::-1][K - 1] - np.sort(x)[::-1][K]
        assert ldd.topk_distance(x, sw) == pytest.approx(gap, rel=1e-12)
        delta = rng.normal(0, 0.05, n)
        assert abs(ldd.topk_distance(x + delta, bad) - d) <= np.abs(delta).sum() + 1e-12


def test_topk_linear_equals_bruteforce_medium():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 4, 1500).astype(np.float32)
    idx = np.argsort(-(x + rng.normal(0, 0.5, x.size)))[:20]
    assert ldd.topk_distance(x, idx) == pytest.approx(ldd.topk_distance_bruteforce(x, idx), rel=1e-12)
