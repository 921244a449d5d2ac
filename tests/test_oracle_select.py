"""Pins for the oracle's per-head top-k and compaction (Sec. 3.3.3; Alg. 2 prefill)."""
import itertools

import numpy as np

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(1487)


def _best_subset(score, k):
    """Exhaustive search: the k-subset of maximal total score; among equal totals the
    lexicographically smallest index tuple (= lower positions win ties)."""
    best, best_key = None, None
    for comb in itertools.combinations(range(len(score)), k):
        key = (-sum(score[i] for i in comb), comb)
        if best_key is None or key < best_key:
            best, best_key = comb, key
    return list(best)


def test_exhaustive_subset_search_tiny():
    for trial in range(30):
        P = int(RNG.integers(3, 11))
        w = int(RNG.integers(1, 4))
        N = P + w
        # few distinct values (exactly representable) so ties are common
        score = RNG.integers(0, 4, size=P).astype(np.float64) * 0.25
        for budget in range(0, N + 2):
            sel = O.select_indices(score, budget, N, w)
            b = min(max(budget, min(w, N)), N)
            kp = min(max(b - w, 0), P)
            want = _best_subset(score, kp) + list(range(N - min(b, w), N))
            assert sel.tolist() == want, (score, budget, w)


def test_structure_random():
    B, H, N, D, w, cap = 2, 3, 200, 8, 16, 64
    P = N - w
    score = RNG.random((B, H, P))
    budget = RNG.integers(0, 80, size=(B, H))
    budget[0, 0] = 5          # below the window
    budget[1, 2] = 64
    K = RNG.standard_normal((B, H, N, D)).astype(np.float32)
    V = RNG.standard_normal((B, H, N, D)).astype(np.float32)
    budget = np.minimum(budget, cap)
    Ko, Vo, idx, ln = O.select_gather(score, budget, K, V, w, cap)
    for b in range(B):
        for h in range(H):
            n = ln[b, h]
            assert n == min(max(budget[b, h], w), N)
            ids = idx[b, h, :n]
            assert np.all(np.diff(ids) > 0)
            assert ids[-w:].tolist() == list(range(P, N))
            assert np.all(idx[b, h, n:] == -1)
            kept = ids[:-w]
            if len(kept) and len(kept) < P:
                dropped = np.setdiff1d(np.arange(P), kept)
                assert score[b, h, kept].min() >= score[b, h, dropped].max()
            assert Ko[b, h, :n].tobytes() == K[b, h][ids].tobytes()
            assert Vo[b, h, :n].tobytes() == V[b, h][ids].tobytes()
            assert not Ko[b, h, n:].any() and not Vo[b, h, n:].any()


def test_plateau_ties_take_lowest_positions():
    score = np.array([0.1, 0.7, 0.7, 0.7, 0.7, 0.2, 0.9])
    sel = O.select_indices(score, budget=3 + 2, N=9, w=2)
    assert sel.tolist() == [1, 2, 6, 7, 8]
