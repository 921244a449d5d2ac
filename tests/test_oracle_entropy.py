"""Pins for the oracle's truncated matrix entropy (Sec. 3.1-3.2; Lemmas 2-4).

None of these re-call the oracle's own formula: expected values are closed forms
worked out from a *constructed* spectrum, the paper's printed special cases, a
2x2 analytic eigen-decomposition, bounds from Lemma 4, and invariances."""
import math
import os

import numpy as np
import pytest

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(20241003)


def _orthonormal_centered(N, D, rng):
    """N x D matrix with orthonormal columns that are all orthogonal to the ones vector."""
    A = rng.standard_normal((N, D + 1))
    A[:, 0] = 1.0
    Q, _ = np.linalg.qr(A)
    return Q[:, 1:]


def _with_spectrum(sigma, N, rng, offset=None):
    """Token matrix whose centred covariance has exactly the eigenvalues sigma."""
    D = len(sigma)
    U = _orthonormal_centered(N, D, rng)
    W, _ = np.linalg.qr(rng.standard_normal((D, D)))
    X = math.sqrt(N - 1) * (U * np.sqrt(sigma)) @ W.T
    if offset is not None:
        X = X + offset
    return X


def _plogp(v):
    return -sum(x * math.log(x) for x in v if x > 0)


def test_paper_closed_forms(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_entropy_closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        D, k, kind, exp = line.split()
        D, k = int(D), int(k)
        p = np.zeros(D)
        if kind == "onehot":
            p[0] = 1.0
        else:
            p[:] = 1.0 / D
        want = 0.0 if exp == "0" else math.log(int(exp[3:]))
        for renorm in (True, False):
            assert O.truncated_entropy(p, k, renorm) == pytest.approx(want, abs=1e-12)


def test_geometric_spectrum_closed_form():
    # sigma_i = 2^-i (i = 1..D) -> unit-trace p_i = 2^-i / (1 - 2^-D)
    D, N, k = 16, 200, 5
    sigma = np.array([2.0 ** -(i + 1) for i in range(D)])
    X = _with_spectrum(sigma, N, RNG, offset=RNG.standard_normal(D) * 3.0)
    H, eig = O.head_entropy(X[None], k_trunc=k, flags=O.FLAG_CENTER)          # literal Eq. 5
    Z = 1.0 - 2.0 ** -D
    p = [2.0 ** -(i + 1) / Z for i in range(D)]
    assert np.allclose(eig[0], p, rtol=1e-9, atol=1e-14)
    assert H[0] == pytest.approx(_plogp(p[:k]), rel=1e-10)
    Hr, _ = O.head_entropy(X[None], k_trunc=k, flags=O.FLAG_CENTER | O.FLAG_TRUNC_RENORM)
    Zk = sum(p[:k])
    assert Hr[0] == pytest.approx(_plogp([x / Zk for x in p[:k]]), rel=1e-10)
    # full (k = D) entropy against the closed form of a truncated geometric law
    Hf, _ = O.head_entropy(X[None], k_trunc=D, flags=O.FLAG_CENTER)
    want = math.log(Z) + math.log(2.0) * sum((i + 1) * 2.0 ** -(i + 1) for i in range(D)) / Z
    assert Hf[0] == pytest.approx(want, rel=1e-10)


def test_isotropic_gives_log_of_truncation_rank():
    D, N = 128, 512
    X = _with_spectrum(np.full(D, 0.37), N, RNG)
    for k in (1, 16, 32, 64, 128):
        Hr, _ = O.head_entropy(X[None], k_trunc=k)
        assert Hr[0] == pytest.approx(math.log(k), abs=1e-9)
        Hl, _ = O.head_entropy(X[None], k_trunc=k, flags=O.FLAG_CENTER)
        assert Hl[0] == pytest.approx(k / D * math.log(D), abs=1e-9)


def test_rank_k_isotropic_gives_log_k_under_both_readings():
    D, N, k = 128, 400, 32
    sigma = np.zeros(D)
    sigma[:k] = 2.5
    X = _with_spectrum(sigma, N, RNG)
    for flags in (O.FLAG_CENTER, O.FLAG_CENTER | O.FLAG_TRUNC_RENORM):
        H, _ = O.head_entropy(X[None], k_trunc=k, flags=flags)
        assert H[0] == pytest.approx(math.log(k), abs=1e-8)


def test_rank_one_gives_zero():
    N, D = 300, 128
    u = RNG.standard_normal(N)
    v = RNG.standard_normal(D)
    X = np.outer(u, v)
    for flags in (0, O.FLAG_CENTER, O.FLAG_TRUNC_RENORM, O.DEFAULT_FLAGS):
        H, eig = O.head_entropy(X[None], flags=flags)
        assert abs(H[0]) < 1e-9
        assert eig[0, 0] == pytest.approx(1.0, abs=1e-12)


def test_two_by_two_analytic():
    # D = 2: eigenvalues of [[a, b], [b, c]] are (a+c)/2 +- sqrt(((a-c)/2)^2 + b^2)
    N = 50
    X = RNG.standard_normal((N, 2)) @ np.array([[1.3, 0.4], [0.0, 0.6]])
    xb = X.sum(0) / N
    a = sum((x[0] - xb[0]) ** 2 for x in X) / (N - 1)
    c = sum((x[1] - xb[1]) ** 2 for x in X) / (N - 1)
    b = sum((x[0] - xb[0]) * (x[1] - xb[1]) for x in X) / (N - 1)
    rad = math.sqrt(((a - c) / 2) ** 2 + b * b)
    l1, l2 = (a + c) / 2 + rad, (a + c) / 2 - rad
    p1, p2 = l1 / (l1 + l2), l2 / (l1 + l2)
    H, eig = O.head_entropy(X[None], k_trunc=2)
    assert eig[0] == pytest.approx([p1, p2], rel=1e-10)
    assert H[0] == pytest.approx(_plogp([p1, p2]), rel=1e-10)
    H1, _ = O.head_entropy(X[None], k_trunc=1, flags=O.FLAG_CENTER)
    assert H1[0] == pytest.approx(_plogp([p1]), rel=1e-10)
    # uncentred reading: second moments instead of central moments
    a0 = sum(x[0] ** 2 for x in X) / (N - 1)
    c0 = sum(x[1] ** 2 for x in X) / (N - 1)
    b0 = sum(x[0] * x[1] for x in X) / (N - 1)
    rad0 = math.sqrt(((a0 - c0) / 2) ** 2 + b0 * b0)
    q1 = ((a0 + c0) / 2 + rad0) / (a0 + c0)
    Hu, _ = O.head_entropy(X[None], k_trunc=2, flags=O.FLAG_TRUNC_RENORM)
    assert Hu[0] == pytest.approx(_plogp([q1, 1 - q1]), rel=1e-10)


def test_centering_removes_a_constant_offset_and_flag_matters():
    N, D = 256, 32
    X = RNG.standard_normal((N, D)) * np.linspace(0.2, 2.0, D)
    off = RNG.standard_normal(D) * 50.0
    Hc, _ = O.head_entropy(np.stack([X, X + off]), k_trunc=8)
    assert Hc[0] == pytest.approx(Hc[1], rel=1e-9)
    Hu, _ = O.head_entropy(np.stack([X, X + off]), k_trunc=8, flags=O.FLAG_TRUNC_RENORM)
    assert abs(Hu[0] - Hu[1]) > 0.1          # uncentred: the offset becomes a dominant direction
    # constant rows: centred covariance is zero (H = 0), uncentred is rank one (H = 0 too)
    C = np.tile(np.round(off * 4.0) / 4.0, (N, 1))   # quarter-integers: the mean of 256 rows is exact
    assert O.head_entropy(C[None])[0][0] == 0.0
    assert np.all(O.head_entropy(C[None])[1] == 0.0)


def test_invariances_permutation_rotation_scale():
    N, D, k = 384, 64, 16
    X = RNG.standard_normal((N, 12)) @ RNG.standard_normal((12, D)) + 0.1 * RNG.standard_normal((N, D))
    H0 = O.head_entropy(X[None], k_trunc=k)[0][0]
    perm = RNG.permutation(N)
    Q, _ = np.linalg.qr(RNG.standard_normal((D, D)))
    for Y in (X[perm], X @ Q, 7.5 * X, -X):
        assert O.head_entropy(Y[None], k_trunc=k)[0][0] == pytest.approx(H0, rel=1e-9)


def test_lemma4_bounds_on_random_inputs():
    for trial in range(20):
        N = int(RNG.integers(8, 200))
        D = int(RNG.integers(2, 48))
        r = int(RNG.integers(1, D + 1))
        k = int(RNG.integers(1, D + 1))
        X = RNG.standard_normal((N, r)) @ RNG.standard_normal((r, D))
        Hlit, eig = O.head_entropy(X[None], k_trunc=k, flags=O.FLAG_CENTER)
        Hren, _ = O.head_entropy(X[None], k_trunc=k)
        Hfull, _ = O.head_entropy(X[None], k_trunc=D, flags=O.FLAG_CENTER)
        rank = int((eig[0] > 1e-10).sum())
        assert rank <= min(r, N - 1, D)                       # rank(Sigma) <= rank(X)
        assert eig[0].sum() == pytest.approx(1.0, abs=1e-12)  # unit trace
        assert np.all(np.diff(eig[0]) <= 1e-15)               # descending
        assert -1e-12 <= Hlit[0] <= Hfull[0] + 1e-12 <= math.log(D) + 1e-12
        assert Hlit[0] <= math.log(k) + 1e-12 and Hren[0] <= math.log(k) + 1e-12
        assert math.exp(Hfull[0]) <= rank + 1e-8               # erank <= rank
        if k >= rank:                                          # nothing is cut off
            assert Hlit[0] == pytest.approx(Hfull[0], abs=1e-8)
            assert Hren[0] == pytest.approx(Hfull[0], abs=1e-8)


def test_degenerate_shapes():
    assert O.head_entropy(np.zeros((1, 5, 8)))[0][0] == 0.0
    assert O.head_entropy(RNG.standard_normal((1, 1, 8)))[0][0] == 0.0          # one token, centred
    H, _ = O.head_entropy(RNG.standard_normal((1, 1, 8)), flags=O.FLAG_TRUNC_RENORM)
    assert H[0] == 0.0
    H, _ = O.head_entropy(RNG.standard_normal((1, 40, 8)), k_trunc=100)         # k > D behaves as k = D
    H2, _ = O.head_entropy(RNG.standard_normal((1, 40, 8)), k_trunc=8)
    assert np.isfinite(H[0]) and np.isfinite(H2[0])
