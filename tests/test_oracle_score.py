"""Pins for the oracle's S-MLP score (App. A "S-MLP"; Sec. 3.3-3.4).

The paper prints no worked example, so the pins are closed forms, a brute-force
scalar loop, an independent library composition, and invariants."""
import math

import numpy as np
import pytest
import torch

from oracle.pafu_oracle import smlp_score

SILU_1 = 0.7310585786300049      # 1 / (1 + e^-1)
SILU_M1 = -0.2689414213699951    # -1 / (1 + e)
GELU_1 = 0.8413447460685429      # Phi(1)
GELU_M1 = -0.15865525393145707   # -Phi(-1)


def test_scalar_closed_forms():
    one = np.ones((1, 1))
    for x, want in ((0.0, 0.0), (1.0, SILU_1), (-1.0, SILU_M1)):
        got = smlp_score(np.array([[x]]), one, None, one, None)
        assert got.shape == (1,)
        assert abs(got[0] - want) < 1e-15
    # w1, b1, w2, b2 each enter where they should: s = w2*silu(w1*x+b1)+b2
    got = smlp_score(np.array([[2.0]]), np.array([[0.5]]), np.array([0.0]), np.array([[3.0]]), np.array([0.25]))
    assert abs(got[0] - (3.0 * SILU_1 + 0.25)) < 1e-15
    got = smlp_score(np.array([[2.0]]), np.array([[-1.0]]), np.array([1.0]), np.array([[-2.0]]), np.array([0.5]))
    assert abs(got[0] - (-2.0 * SILU_M1 + 0.5)) < 1e-15


def test_gelu_closed_forms():
    one = np.ones((1, 1))
    for x, want in ((0.0, 0.0), (1.0, GELU_1), (-1.0, GELU_M1)):
        got = smlp_score(np.array([[x]]), one, None, one, None, act="gelu_erf")
        assert abs(got[0] - want) < 1e-15


def test_zero_first_layer_closed_form():
    rng = np.random.default_rng(1)
    T, F, M, n_out = 5, 7, 4, 3
    X = rng.standard_normal((T, F))
    W2 = rng.standard_normal((n_out, M))
    b1 = rng.standard_normal(M)
    b2 = rng.standard_normal(n_out)
    got = smlp_score(X, np.zeros((M, F)), b1, W2, b2)
    silu_b1 = [b / (1.0 + math.exp(-b)) for b in b1]
    want = sum(b2) / n_out + sum(W2[o, m] * silu_b1[m] for o in range(n_out) for m in range(M)) / n_out
    assert np.allclose(got, want, rtol=0, atol=1e-14)


def _loops(X, W1, b1, W2, b2):
    T, F = len(X), len(X[0])
    M, n_out = len(W1), len(W2)
    out = []
    for t in range(T):
        a = []
        for m in range(M):
            h = b1[m]
            for f in range(F):
                h += W1[m][f] * X[t][f]
            a.append(h / (1.0 + math.exp(-h)))
        tot = 0.0
        for o in range(n_out):
            y = b2[o]
            for m in range(M):
                y += W2[o][m] * a[m]
            tot += y
        out.append(tot / n_out)
    return out


@pytest.mark.parametrize("T,F,M,n_out", [(3, 5, 4, 1), (6, 9, 7, 12), (1, 2, 3, 5)])
def test_brute_force_loops(T, F, M, n_out):
    rng = np.random.default_rng(T * 100 + F)
    X = rng.standard_normal((T, F))
    W1 = rng.standard_normal((M, F))
    W2 = rng.standard_normal((n_out, M))
    b1 = rng.standard_normal(M)
    b2 = rng.standard_normal(n_out)
    got = smlp_score(X, W1, b1, W2, b2)
    want = _loops(X.tolist(), W1.tolist(), b1.tolist(), W2.tolist(), b2.tolist())
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("act", ["silu", "gelu_erf"])
def test_library_composition(act):
    rng = np.random.default_rng(7)
    T, F, M, n_out = 33, 48, 20, 12
    X = rng.standard_normal((T, F))
    W1 = rng.standard_normal((M, F)) * 0.3
    W2 = rng.standard_normal((n_out, M))
    b1 = rng.standard_normal(M)
    b2 = rng.standard_normal(n_out)
    tX, tW1, tW2, tb1, tb2 = (torch.from_numpy(a) for a in (X, W1, W2, b1, b2))
    h = torch.nn.functional.linear(tX, tW1, tb1)
    a = torch.nn.functional.silu(h) if act == "silu" else torch.nn.functional.gelu(h)
    want = torch.nn.functional.linear(a, tW2, tb2).mean(dim=1).numpy()
    got = smlp_score(X, W1, b1, W2, b2, act=act)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_output_mean_folds_into_one_output():
    # mean over outputs of a linear layer == one output with averaged weights and bias
    rng = np.random.default_rng(3)
    T, F, M, n_out = 17, 24, 10, 12
    X = rng.standard_normal((T, F))
    W1 = rng.standard_normal((M, F)) * 0.2
    W2 = rng.standard_normal((n_out, M))
    b1 = rng.standard_normal(M)
    b2 = rng.standard_normal(n_out)
    full = smlp_score(X, W1, b1, W2, b2)
    folded = smlp_score(X, W1, b1, W2.mean(axis=0, keepdims=True), np.array([b2.mean()]))
    assert np.allclose(full, folded, rtol=1e-13, atol=1e-14)


def test_rows_are_independent_and_permutation_equivariant():
    rng = np.random.default_rng(5)
    T, F, M = 12, 16, 8
    X = rng.standard_normal((T, F))
    W1 = rng.standard_normal((M, F))
    W2 = rng.standard_normal((2, M))
    base = smlp_score(X, W1, None, W2, None)
    X2 = X.copy()
    X2[4] += 1.0
    moved = smlp_score(X2, W1, None, W2, None)
    changed = np.nonzero(moved != base)[0]
    assert changed.tolist() == [4]
    perm = rng.permutation(T)
    assert np.array_equal(smlp_score(X[perm], W1, None, W2, None), base[perm])


def test_segmented_input_equals_concatenated():
    # the paper-form input is [Q | K | V] along the feature axis
    rng = np.random.default_rng(9)
    T, Hh, M = 10, 6, 5
    q, k, v = (rng.standard_normal((T, Hh)) for _ in range(3))
    W1 = rng.standard_normal((M, 3 * Hh))
    W2 = rng.standard_normal((3, M))
    whole = smlp_score(np.concatenate([q, k, v], axis=1), W1, None, W2, None)
    # linear in the pre-activation: sum of the three segment products
    h = q @ W1[:, :Hh].T + k @ W1[:, Hh:2 * Hh].T + v @ W1[:, 2 * Hh:].T
    a = h / (1 + np.exp(-h))
    assert np.allclose(whole, (a @ W2.T).mean(axis=1), rtol=1e-13, atol=1e-14)
