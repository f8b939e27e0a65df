"""Pins for the oracle's teacher-side salience score (Sec. 3.2, Eq. 4-5)."""
import math

import numpy as np
import pytest

from oracle.pafu_oracle import sse_score


def _loops(Q, K, L_B):
    """Eq. 4-5 with explicit loops: the index sets written as the paper defines them (l(i), h(i))."""
    L, N, D = Q.shape
    P = np.zeros((N, L, L))
    for h in range(N):
        for i in range(L):
            z = [sum(Q[i, h, d] * K[j, h, d] for d in range(D)) / math.sqrt(D) for j in range(L)]
            m = max(z)
            e = [math.exp(v - m) for v in z]
            t = sum(e)
            for j in range(L):
                P[h, i, j] = e[j] / t
    s = np.zeros(L)
    for j in range(L):
        sets = {"low": [], "diag": [], "up": []}
        for i in range(L):
            lo = (i // L_B) * L_B
            hi = lo + L_B
            if j < lo:
                sets["low"].append(i)
            elif j < hi:
                sets["diag"].append(i)
            else:
                sets["up"].append(i)
        part = {name: sum(max(P[h, i, j] for i in idx) for h in range(N)) / N for name, idx in sets.items() if idx}
        if 0 <= j < L_B and L >= 2 * L_B:
            want = (part["diag"] + part["low"]) / 2
        elif L_B <= j < L - L_B:
            want = (part["up"] + part["diag"] + part["low"]) / 3
        elif L - L_B <= j < L and L >= 2 * L_B and L % L_B == 0:
            want = (part["diag"] + part["up"]) / 2
        else:
            want = sum(part.values()) / len(part)          # outside Eq. 5's cases: the parts that exist
        s[j] = want
    return s


@pytest.mark.parametrize("L,L_B,N,D", [(12, 4, 2, 3), (8, 4, 1, 2), (9, 3, 2, 4), (6, 6, 2, 3), (10, 4, 2, 3)])
def test_matches_explicit_loops(L, L_B, N, D):
    rng = np.random.default_rng(L * 10 + L_B)
    Q = rng.standard_normal((L, N, D)) * 2.0
    K = rng.standard_normal((L, N, D)) * 2.0
    assert np.allclose(sse_score(Q, K, L_B), _loops(Q, K, L_B), rtol=1e-12, atol=1e-14)


def test_uniform_attention_closed_form():
    # Q = 0: every row of P is 1/L, so every part that exists is 1/L and so is the score
    L, N, D = 24, 3, 4
    K = np.random.default_rng(0).standard_normal((L, N, D))
    s, low, diag, up = sse_score(np.zeros((L, N, D)), K, 8, return_parts=True)
    assert np.allclose(s, 1.0 / L) and np.allclose(diag, 1.0 / L)
    assert np.allclose(low[:16], 1.0 / L) and np.all(low[16:] == 0)      # the last block has no later queries
    assert np.allclose(up[8:], 1.0 / L) and np.all(up[:8] == 0)


def test_parts_partition_the_queries():
    # the largest of the three parts (per head) is the plain column maximum of P
    rng = np.random.default_rng(1)
    L, D, L_B = 20, 5, 5
    Q = rng.standard_normal((L, 1, D)) * 3
    K = rng.standard_normal((L, 1, D)) * 3
    _, low, diag, up = sse_score(Q, K, L_B, return_parts=True)
    z = Q[:, 0] @ K[:, 0].T / math.sqrt(D)
    P = np.exp(z - z.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    assert np.allclose(np.maximum(np.maximum(low, diag), up), P.max(axis=0), rtol=1e-12)


def test_single_block_is_the_plain_max_and_one_hot_attention():
    rng = np.random.default_rng(2)
    L, N, D = 10, 2, 4
    Q = rng.standard_normal((L, N, D))
    K = rng.standard_normal((L, N, D))
    s, low, diag, up = sse_score(Q, K, L, return_parts=True)
    assert np.array_equal(s, diag) and np.all(low == 0) and np.all(up == 0)
    # every query attends (almost) only to key 7: that key scores ~1 in every part, the others ~0
    K2 = np.zeros((12, 1, 2))
    K2[7, 0] = [40.0, 0.0]
    Q2 = np.tile(np.array([[[40.0, 0.0]]]), (12, 1, 1))
    s2 = sse_score(Q2, K2, 4)
    assert abs(s2[7] - 1.0) < 1e-9 and np.all(np.delete(s2, 7) < 1e-9)


def test_block_relation_follows_the_query_not_the_key():
    # queries of the LAST block look only at key 0, all others only at their own position:
    # key 0 gets its large weight in the "low" part (queries in later blocks), not in "up"
    L, L_B = 12, 4
    K = np.eye(L)[:, None, :] * 30.0
    Q = np.eye(L)[:, None, :] * 30.0
    Q[8:] = 0
    Q[8:, 0, 0] = 30.0
    _, low, diag, up = sse_score(Q, K, L_B, return_parts=True)
    assert low[0] > 0.99 and up[0] == 0.0 and diag[0] > 0.99
    assert low[5] < 1e-6 and diag[5] > 0.99


def test_scale_argument_and_head_mean():
    rng = np.random.default_rng(3)
    L, N, D = 9, 3, 4
    Q = rng.standard_normal((L, N, D))
    K = rng.standard_normal((L, N, D))
    assert np.allclose(sse_score(Q, K, 3), sse_score(Q * 2, K, 3, scale=0.5 / math.sqrt(D)))
    per_head = [sse_score(Q[:, h:h + 1], K[:, h:h + 1], 3, return_parts=True) for h in range(N)]
    _, low, diag, up = sse_score(Q, K, 3, return_parts=True)
    assert np.allclose(diag, np.mean([p[2] for p in per_head], axis=0))
    assert np.allclose(low, np.mean([p[1] for p in per_head], axis=0))
