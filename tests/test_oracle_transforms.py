"""Pins of the oracle's alternative transforms (App. B, the nine feature-amplification methods)
against library routines and closed forms in fp64, the value the paper prints, and the properties
the threshold relies on (monotone in the mean map, minimum attained at the clamp)."""
import os

import numpy as np
import pytest
import scipy.stats

import oracle

EPS = 1e-10                                  # App. B states 1e-10
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def softmax_map(rng, H, L, sharp=2.0):
    s = rng.standard_normal((H, L, L)) * sharp
    s[:, ~np.tril(np.ones((L, L), bool))] = -np.inf
    e = np.exp(s - s.max(-1, keepdims=True))
    return (e / e.sum(-1, keepdims=True)).astype(np.float32)


def stabilised(A, C, eps):
    """X of App. B in fp64, from the stored fp32 inputs (never-valid pairs: A = 0, C = 0)."""
    L = A.shape[-1]
    tri = np.tril(np.ones((L, L)))
    a = A.astype(np.float64) * tri if C is None else A.astype(np.float64)
    c = np.broadcast_to(tri, A.shape) if C is None else C.astype(np.float64)
    return a, a / (c + eps), np.maximum(a / (c + eps), eps)


REF = {
    "raw_sum": lambda a, abar, X, lam, eps: a,
    "average": lambda a, abar, X, lam, eps: abar,
    "log": lambda a, abar, X, lam, eps: np.log(X),
    "yeo_johnson": lambda a, abar, X, lam, eps: scipy.stats.yeojohnson(X, lmbda=lam),
    "zscore": lambda a, abar, X, lam, eps: (X - X.mean()) / (X.std() + eps),
    "minmax": lambda a, abar, X, lam, eps: (X - X.min()) / (X.max() - X.min() + eps),
    "sqrt": lambda a, abar, X, lam, eps: np.sqrt(X),
    "arcsinh": lambda a, abar, X, lam, eps: np.arcsinh(X),
}


@pytest.mark.parametrize("kind", sorted(REF))
@pytest.mark.parametrize("with_counts", [False, True])
def test_against_library_and_closed_forms(kind, with_counts):
    rng = np.random.default_rng(11)
    A = softmax_map(rng, 3, 23)
    C = None
    if with_counts:
        C = np.tril(rng.integers(1, 4, (3, 23, 23)).astype(np.float32))
        A = A * C                                                  # sums over C captures
    lam = 0.7
    T, tmin = oracle.transform(A, C, kind, lam, EPS)
    a, abar, X = stabilised(A, C, EPS)
    want = REF[kind](a, abar, X, lam, EPS)
    scale = max(1.0, float(np.abs(want).max()))
    np.testing.assert_allclose(T, want, rtol=0, atol=4e-6 * scale)   # a few fp32 ulp of the largest value
    assert tmin == T.min()
    # after the shift the minimum is 0 and sits on the never-valid pairs (X = eps there), as in the table
    # of App. B where all but the attended entries are exactly zero
    assert (T - tmin)[0, 0, 5] == 0.0


def test_yeo_johnson_lambda_zero_and_one():
    rng = np.random.default_rng(12)
    A = softmax_map(rng, 1, 9)
    _, _, X = stabilised(A, None, EPS)
    T0, _ = oracle.transform(A, None, "yeo_johnson", 0.0, EPS)
    np.testing.assert_allclose(T0, np.log1p(X), atol=1e-6)
    T1, _ = oracle.transform(A, None, "yeo_johnson", 1.0, EPS)
    np.testing.assert_allclose(T1, X, atol=1e-6)                   # lambda = 1 is the identity on X >= 0


def test_square_root_printed_relation_to_box_cox():
    # lambda = 0.5: Box-Cox = 2 (sqrt X - 1), so the shifted Box-Cox map is twice the shifted square-root map;
    # App. B's table prints max 2.00 for Box-Cox, i.e. 1.00 for the square root of a probability of one.
    A = np.zeros((1, 2, 2), np.float32)
    A[0, 0, 0], A[0, 1, 0], A[0, 1, 1] = 1.0, 0.25, 0.75
    Ts, smin = oracle.transform(A, None, "sqrt", 0.5, EPS)
    Tb, bmin = oracle.transform(A, None, "boxcox", 0.5, EPS)
    np.testing.assert_allclose(2.0 * (Ts - smin), Tb - bmin, atol=1e-6)
    line = [l for l in open(os.path.join(GOLDEN, "boxcox_table_appB.txt")) if l.startswith("max_value")][0]
    assert f"{2.0 * float((Ts - smin).max()):.2f}" == line.split()[1]


@pytest.mark.parametrize("kind", ["average", "log", "yeo_johnson", "zscore", "minmax", "sqrt", "arcsinh"])
def test_monotone_in_the_mean_map(kind):
    # the threshold on the transformed map is a threshold on the mean map: sorting by Abar sorts by T
    rng = np.random.default_rng(13)
    A = softmax_map(rng, 2, 31, sharp=3.0)
    T, _ = oracle.transform(A, None, kind, 0.5, 1e-8)
    tri = np.tril(np.ones((31, 31), bool))
    a, t = A[:, tri].reshape(-1), T[:, tri].reshape(-1)
    order = np.argsort(a, kind="stable")
    assert (np.diff(t[order]) >= 0).all()


def test_derive_with_a_transform_reduces_to_a_threshold_on_the_mean():
    rng = np.random.default_rng(14)
    A = softmax_map(rng, 2, 40, sharp=3.0)
    art = oracle.derive(A, None, 0.5, 1e-8, 0.1, 0.8, kind="sqrt")
    # sqrt(X) - sqrt(eps) >= tau  <=>  X >= (tau + sqrt(eps))^2, away from the rounding boundary
    theta = (0.1 + np.sqrt(1e-8)) ** 2
    _, _, X = stabilised(A, None, 1e-8)
    far = np.abs(X - theta) > 1e-6
    tri = np.tril(np.ones((40, 40), bool))[None]
    assert np.array_equal((art.true_mask == 1)[far & tri], (X >= theta)[far & tri])
    assert not art.true_mask[:, ~tri[0]].any()
