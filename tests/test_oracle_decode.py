"""Pins for the oracle's decode-time eviction step (Sec. 3.3.3 "Dynamic KV Cache
Eviction", last sentence; Alg. 2 "Decoding")."""

import numpy as np
from scipy.special import softmax

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(1494)


def _run(K, V, Q, n0, budget, w, cum0=None):
    """Feeds tokens n0.. of K/V/Q ([N,D], [N,D], [N,G,D]) one by one into a cache that
    starts with tokens 0..n0-1.  Returns the final state and the per-step records."""
    Kc, Vc = K[:n0].copy(), V[:n0].copy()
    idx = np.arange(n0, dtype=np.int32)
    cum = np.zeros(n0) if cum0 is None else np.asarray(cum0, dtype=np.float64).copy()
    steps = []
    for t in range(n0, K.shape[0]):
        before = (idx.copy(), cum.copy())
        Kc, Vc, idx, cum, out, ev = O.decode_step(Kc, Vc, idx, cum, Q[t], K[t], V[t], t, budget, w)
        steps.append((before, out, ev, idx.copy(), cum.copy()))
    return (Kc, Vc, idx, cum), steps


def test_no_eviction_equals_unpooled_window_score():
    """With room for everything, T decode steps accumulate exactly the attention that the
    last T queries pay to the earlier tokens: the prefill window score with pool 1."""
    N, T, D, G = 57, 9, 16, 3
    K = RNG.standard_normal((N, D))
    V = RNG.standard_normal((N, D))
    Q = RNG.standard_normal((N, G, D)) * 1.5
    (Kc, Vc, idx, cum), _ = _run(K, V, Q, N - T, budget=N + 5, w=1)
    assert idx.tolist() == list(range(N))
    Qwin = np.transpose(Q[N - T:], (1, 0, 2))[None]            # [1, G, T, D]
    want = O.window_score(Qwin, K[None, None], G, pool=1)[0, 0]
    np.testing.assert_allclose(cum[: N - T], want, rtol=1e-12, atol=1e-14)
    # the rows themselves were stored untouched, in position order
    assert np.array_equal(Kc, K) and np.array_equal(Vc, V)


def test_attention_output_matches_library_softmax():
    N, n0, D, G = 20, 12, 8, 4
    K = RNG.standard_normal((N, D))
    V = RNG.standard_normal((N, D))
    Q = RNG.standard_normal((N, G, D)) * 2.0
    _, steps = _run(K, V, Q, n0, budget=N, w=2)
    for s, t in zip(steps, range(n0, N)):
        prob = softmax(Q[t] @ K[: t + 1].T / np.sqrt(D), axis=1)   # [G, t+1]
        np.testing.assert_allclose(s[1], prob @ V[: t + 1], rtol=1e-12, atol=1e-14)


def test_equal_keys_closed_form():
    """All keys equal: every query head spreads its unit mass evenly, each of the n+1
    entries gains G/(n+1) and the output is the mean value row."""
    n, D, G = 10, 4, 4
    k = RNG.standard_normal(D)
    Kc = np.tile(k, (n, 1))
    Vc = RNG.standard_normal((n, D))
    v_new = RNG.standard_normal(D)
    cum0 = RNG.random(n)
    q = RNG.standard_normal((G, D))
    _, _, idx, cum, out, ev = O.decode_step(Kc, Vc, np.arange(n), cum0, q, k, v_new, n, budget=n + 1, w=1)
    assert ev == -1 and idx.tolist() == list(range(n + 1))
    np.testing.assert_allclose(cum, np.concatenate([cum0, [0.0]]) + G / (n + 1), rtol=1e-13)
    mean_v = np.concatenate([Vc, v_new[None]]).mean(axis=0)
    np.testing.assert_allclose(out, np.tile(mean_v, (G, 1)), rtol=1e-12, atol=1e-14)


def test_mass_per_step_is_G():
    N, n0, D, G = 40, 25, 8, 2
    K = RNG.standard_normal((N, D))
    V = RNG.standard_normal((N, D))
    Q = RNG.standard_normal((N, G, D)) * 3.0
    _, steps = _run(K, V, Q, n0, budget=N, w=3)
    prev = 0.0
    for s in steps:
        now = s[4].sum()
        assert abs((now - prev) - G) < 1e-12
        prev = now


def test_dominant_key_takes_the_step():
    n, D, G = 12, 8, 2
    Kc = RNG.standard_normal((n, D)) * 0.1
    q = RNG.standard_normal((G, D))
    q[1] = 2.0 * q[0]
    Kc[5] = 40.0 * q[0] / np.linalg.norm(q[0])                 # far ahead for both query heads
    Vc = RNG.standard_normal((n, D))
    _, _, _, cum, out, _ = O.decode_step(Kc, Vc, np.arange(n), np.zeros(n), q, np.zeros(D), np.zeros(D), n,
                                         budget=n + 1, w=1)
    assert abs(cum[5] - G) < 1e-9 and cum.sum() - cum[5] < 1e-9
    np.testing.assert_allclose(out, np.tile(Vc[5], (G, 1)), atol=1e-8)


# Hand-worked evictions.  The query is zero, so every entry gains the same G/(n+1) and the
# order of the starting scores decides.  Columns: start scores | positions | pos | budget | w
# | position that must leave (-1: none).
HAND = [
    ([5.0, 1.0, 3.0, 0.5], [0, 1, 2, 3], 4, 4, 1, 3),        # lowest score leaves
    ([5.0, 1.0, 3.0, 0.5], [0, 1, 2, 3], 4, 4, 2, 1),        # position 3 is inside the recent window (3, 4)
    ([5.0, 1.0, 3.0, 0.5], [0, 1, 2, 3], 4, 5, 1, -1),       # room left
    ([2.0, 1.0, 1.0, 7.0], [0, 4, 6, 9], 10, 4, 1, 4),       # equal scores: the older one leaves
    ([2.0, 1.0, 1.0, 7.0], [0, 4, 6, 9], 10, 4, 5, -1),      # a budget below w counts as w: room left
    ([2.0, 0.5, 1.0, 7.0], [0, 7, 8, 9], 10, 4, 4, 0),       # window = positions 7..10: only 0 may leave
    ([0.0, 0.0, 0.0], [0, 1, 2], 3, 3, 3, 0),                # budget == w: the one outside the window
    ([9.0, 8.0, 7.0], [0, 1, 2], 3, 3, 1, 2),                # the new token (score 0 + share) is exempt
]


def test_hand_worked_evictions():
    D, G = 4, 2
    for cum0, where, pos, budget, w, leaves in HAND:
        n = len(cum0)
        Kc = RNG.standard_normal((n, D))
        Vc = RNG.standard_normal((n, D))
        k_new, v_new = RNG.standard_normal(D), RNG.standard_normal(D)
        Ko, Vo, idx, cum, out, ev = O.decode_step(Kc, Vc, np.array(where), np.array(cum0), np.zeros((G, D)),
                                                  k_new, v_new, pos, budget, w)
        assert ev == leaves, (cum0, where, pos, budget, w)
        want_pos = [p for p in where + [pos] if p != leaves]
        assert idx.tolist() == want_pos
        rows = {p: r for p, r in zip(where + [pos], list(Kc) + [k_new])}
        vrows = {p: r for p, r in zip(where + [pos], list(Vc) + [v_new])}
        for r, p in enumerate(idx.tolist()):
            assert np.array_equal(Ko[r], rows[p]) and np.array_equal(Vo[r], vrows[p])
        share = G / (n + 1)
        start = dict(zip(where + [pos], cum0 + [0.0]))
        np.testing.assert_allclose(cum, [start[p] + share for p in want_pos], rtol=1e-14)


def test_eviction_exhaustive_tiny():
    """Direct search over the entries that may leave (outside the recent window): the
    oracle's choice must be the one of smallest score, older position first among equals."""
    D, G = 4, 1
    for trial in range(200):
        n = int(RNG.integers(2, 8))
        w = int(RNG.integers(1, n + 1))
        where = sorted(RNG.choice(20, size=n, replace=False).tolist())
        pos = 20 + int(RNG.integers(0, 3))
        cum0 = (RNG.integers(0, 4, size=n) * 0.5).tolist()     # ties are common, values exact in fp32
        _, _, idx, cum, _, ev = O.decode_step(RNG.standard_normal((n, D)), RNG.standard_normal((n, D)),
                                              np.array(where), np.array(cum0), np.zeros((G, D)),
                                              np.zeros(D), np.zeros(D), pos, budget=max(n, w), w=w)
        allowed = [p for p in where if p <= pos - w]
        if n + 1 <= max(n, w):
            assert ev == -1
            continue
        assert allowed, "more entries than the window holds: something must be removable"
        start = dict(zip(where, cum0))
        best = min(allowed, key=lambda p: (start[p], p))
        assert ev == best, (where, cum0, pos, w)


def test_long_run_invariants():
    N, n0, D, G, budget, w = 300, 40, 8, 2, 48, 8
    K = RNG.standard_normal((N, D))
    V = RNG.standard_normal((N, D))
    Q = RNG.standard_normal((N, G, D)) * 2.0
    (Kc, Vc, idx, cum), steps = _run(K, V, Q, n0, budget, w, cum0=RNG.random(n0) * 4)
    for (before, out, ev, idx_t, cum_t), t in zip(steps, range(n0, N)):
        assert len(idx_t) <= budget
        assert len(idx_t) == min(len(before[0]) + 1, budget)
        assert np.all(np.diff(idx_t) > 0)
        assert set(range(t - w + 1, t + 1)) <= set(idx_t.tolist())
        if ev >= 0:
            assert ev <= t - w and ev in before[0].tolist() and ev not in idx_t.tolist()
        assert np.all(cum_t >= 0)
    # rows still are the original rows of their positions
    assert np.array_equal(Kc, K[idx]) and np.array_equal(Vc, V[idx])


def test_decode_init_hand_case():
    score = np.array([0.5, 4.0, 1.5, 2.5, 0.25, 3.0])          # P = 6 prefix positions
    idx = np.array([1, 3, 5, 6, 7])                            # N = 8, w = 2: window = 6, 7
    got = O.decode_init(score, idx, N=8, w=2)
    assert got.tolist() == [4.0, 2.5, 3.0, 0.0, 0.0]


def test_decode_follows_prefill_selection():
    """End to end on one head: prefill score -> selection -> decode_init -> steps.  The
    first eviction must be the kept prefix token of smallest prefill score plus decode
    gains, found here by direct search."""
    N, D, G, w, budget = 64, 8, 2, 4, 16
    K = RNG.standard_normal((N + 3, D))
    V = RNG.standard_normal((N + 3, D))
    Q = RNG.standard_normal((N + 3, G, D))
    Qwin = np.transpose(Q[N - w:N], (1, 0, 2))[None]
    score = O.window_score(Qwin, K[None, None, :N], G, pool=3)[0, 0]
    sel = O.select_indices(score, budget, N, w)
    cum = O.decode_init(score, sel, N, w)
    Kc, Vc, idx = K[sel], V[sel], sel
    for t in range(N, N + 3):
        prob = softmax(Q[t] @ np.concatenate([Kc, K[t][None]]).T / np.sqrt(D), axis=1).sum(axis=0)
        after = (np.concatenate([cum, [0.0]]) + prob).astype(np.float32)
        cand = [(after[j], int(p)) for j, p in enumerate(idx.tolist()) if p <= t - w]
        Kc, Vc, idx, cum, _, ev = O.decode_step(Kc, Vc, idx, cum, Q[t], K[t], V[t], t, budget, w)
        assert ev == min(cand)[1]
        assert len(idx) == budget
