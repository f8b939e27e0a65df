"""Pins for the oracle's top-k retention and cache update (Sec. 3.4; Alg. 2)."""
import itertools

import numpy as np
import pytest

from oracle.pafu_oracle import compact_kv, select_topk


def _brute(scores, k):
    """k rounds of 'take the best remaining token' under the stated total order."""
    n = len(scores)
    alive = list(range(n))
    taken = []

    def better(i, j):  # is token i strictly preferred over token j?
        a, b = scores[i], scores[j]
        an, bn = a != a, b != b
        if an or bn:
            if an and bn:
                return i < j
            return bn
        if a > b:
            return True
        if a < b:
            return False
        return i < j   # equal (covers -0.0 == +0.0)

    for _ in range(min(k, n)):
        best = alive[0]
        for j in alive[1:]:
            if better(j, best):
                best = j
        taken.append(best)
        alive.remove(best)
    return sorted(taken)


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_small(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 65))
    # few distinct values -> many ties across the threshold
    s = rng.integers(-3, 4, size=n).astype(np.float32) * np.float32(0.5)
    for k in (0, 1, n // 2, max(n - 1, 0), n, n + 5):
        got = select_topk(s, k)
        assert got.dtype == np.int32
        assert got.tolist() == _brute(s.tolist(), k)


def test_special_values_order():
    s = np.array([np.nan, -np.inf, -0.0, 0.0, 1.0, np.inf, -1.0, np.nan, 0.0], dtype=np.float32)
    full_order = [5, 4, 2, 3, 8, 6, 1, 0, 7]   # inf, 1, zeros by index, -1, -inf, NaNs by index
    for k in range(len(s) + 1):
        assert select_topk(s, k).tolist() == sorted(full_order[:k])
        assert select_topk(s, k).tolist() == _brute(s.tolist(), k)


def test_monotone_and_constant_inputs():
    n, k = 50, 17
    assert select_topk(np.zeros(n, np.float32), k).tolist() == list(range(k))
    assert select_topk(-np.arange(n, dtype=np.float32), k).tolist() == list(range(k))
    assert select_topk(np.arange(n, dtype=np.float32), k).tolist() == list(range(n - k, n))


def test_fifo_is_a_special_case():
    # score := -age keeps the newest k tokens = the sliding-window policy of Sec. 3.1
    n, k = 40, 12
    age = np.arange(n, 0, -1).astype(np.float32)      # token 0 is the oldest
    assert select_topk(-age, k).tolist() == list(range(n - k, n))


def test_budget_at_least_cache_keeps_everything():
    s = np.random.default_rng(0).standard_normal(9).astype(np.float32)
    for k in (9, 10, 1000):
        assert select_topk(s, k).tolist() == list(range(9))
    assert select_topk(np.zeros(0, np.float32), 3).tolist() == []


def test_agrees_with_full_sort_on_distinct_scores():
    rng = np.random.default_rng(11)
    s = rng.permutation(2000).astype(np.float32)   # all distinct
    for k in (1, 999, 1500):
        want = np.sort(np.argsort(-s, kind="stable")[:k])
        assert np.array_equal(select_topk(s, k), want)


def test_permutation_moves_the_selected_set():
    rng = np.random.default_rng(12)
    n, k = 300, 77
    s = rng.permutation(n).astype(np.float32)
    perm = rng.permutation(n)
    a = set(select_topk(s, k).tolist())
    b = set(select_topk(s[perm], k).tolist())
    assert {int(perm[i]) for i in b} == a


def test_threshold_property_exhaustive_tiny():
    # every 3-valued score vector of length 5, every k
    for s in itertools.product((-1.0, 0.0, 2.0), repeat=5):
        arr = np.array(s, dtype=np.float32)
        for k in range(6):
            ids = select_topk(arr, k).tolist()
            assert ids == _brute(list(s), k)


def test_compact_identity_composition_and_sync():
    rng = np.random.default_rng(2)
    n, N, D = 23, 2, 4
    K = rng.standard_normal((n, N, D)).astype(np.float32)
    V = rng.standard_normal((n, N, D)).astype(np.float32)
    SL = rng.standard_normal(n).astype(np.float32)
    Ki, Vi, SLi = compact_kv(K, V, SL, np.arange(n))
    assert np.array_equal(Ki, K) and np.array_equal(Vi, V) and np.array_equal(SLi, SL)
    a = np.sort(rng.permutation(n)[:15])
    b = np.sort(rng.permutation(15)[:6])
    K1, V1, S1 = compact_kv(K, V, SL, a)
    K2, V2, S2 = compact_kv(K1, V1, S1, b)
    K3, V3, S3 = compact_kv(K, V, SL, a[b])
    assert np.array_equal(K2, K3) and np.array_equal(V2, V3) and np.array_equal(S2, S3)
    # scores travel with their rows, rows are whole, K and V are not swapped
    for r, i in enumerate(a):
        assert np.array_equal(K1[r], K[i]) and np.array_equal(V1[r], V[i]) and S1[r] == SL[i]
    assert K1.dtype == K.dtype and K1.shape == (15, N, D)
    # bit copy also for integer payloads (bf16 bit patterns)
    Kb = rng.integers(0, 65536, size=(n, N, D)).astype(np.uint16)
    assert np.array_equal(compact_kv(Kb, Kb, SL, a)[0], Kb[a])


# ---------------------------------------------------------------------- pinned prefix (frame sink)
def _brute_pinned(scores, k, n_pinned):
    """k rounds of 'take the best remaining token'; a pinned token beats any other, pinned tokens rank by index."""
    n = len(scores)
    alive = list(range(n))
    taken = []

    def better(i, j):
        pi, pj = i < n_pinned, j < n_pinned
        if pi or pj:
            if pi and pj:
                return i < j
            return pi
        a, b = scores[i], scores[j]
        an, bn = a != a, b != b
        if an or bn:
            if an and bn:
                return i < j
            return bn
        if a != b:
            return a > b
        return i < j

    for _ in range(min(k, n)):
        best = alive[0]
        for j in alive[1:]:
            if better(j, best):
                best = j
        taken.append(best)
        alive.remove(best)
    return sorted(taken)


@pytest.mark.parametrize("seed", range(6))
def test_pinned_prefix_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 50))
    s = rng.integers(-3, 4, size=n).astype(np.float32)
    s[rng.integers(0, n)] = np.inf          # a +inf outside or inside the prefix must not change the rule
    s[rng.integers(0, n)] = np.nan
    for n_pinned in (0, 1, n // 3, n - 1, n, n + 3):
        for k in (0, 1, n // 2, n - 1, n, n + 2):
            assert select_topk(s, k, n_pinned).tolist() == _brute_pinned(s.tolist(), k, n_pinned)


def test_pinned_prefix_invariants():
    rng = np.random.default_rng(7)
    n, k, p = 200, 60, 25
    s = rng.standard_normal(n).astype(np.float32)
    s[:p] = -10.0                                         # the prefix would all be evicted on its scores
    ids = select_topk(s, k, p)
    assert ids[:p].tolist() == list(range(p)) and len(ids) == k
    # the rest is the plain top-(k - p) of the other tokens
    assert (ids[p:] - p).tolist() == select_topk(s[p:], k - p).tolist()
    # no prefix: the plain rule
    assert select_topk(s, k, 0).tolist() == select_topk(s, k).tolist()
    # same as raising the prefix above every finite score
    t = s.copy()
    t[:p] = np.inf
    assert select_topk(t, k).tolist() == ids.tolist()
    # a budget inside the prefix keeps its first k tokens; a budget covering the cache keeps everything
    assert select_topk(s, 10, p).tolist() == list(range(10))
    assert select_topk(s, n, p).tolist() == list(range(n))
