"""Pins for the oracle's stage-1 hidden-state eviction (Sec. 3.3.2 "Hidden State Eviction")."""
import itertools

import numpy as np

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(404)


def test_score_is_head_sum_of_one_token_window_score():
    """The last token's attention over the earlier positions is the observation-window score with a
    window of one token and no pooling, summed over the KV heads."""
    H, G, N, D = 3, 2, 41, 16
    K = RNG.standard_normal((H, N, D))
    q = RNG.standard_normal((H * G, D)) * 2.0
    got = O.last_token_score(q, K, G)
    win = O.window_score(q[None, :, None, :], K[None], G, pool=1)[0]        # [H, N-1]
    np.testing.assert_allclose(got[: N - 1], win.sum(axis=0), rtol=1e-12, atol=1e-15)


def test_zero_queries_closed_form_and_tie_rule():
    H, G, N, D, Dm = 2, 2, 12, 8, 6
    K = RNG.standard_normal((1, H, N, D))
    Hs = RNG.standard_normal((1, N, Dm))
    rows, idx, score = O.hidden_evict(np.zeros((1, H * G, D)), K, Hs, n_keep=5, w=2, G=G)
    np.testing.assert_allclose(score[0], np.full(N, H * G / N), rtol=1e-14)
    assert idx[0].tolist() == [0, 1, 2, 10, 11]                 # all equal: the lowest positions, then the window
    assert np.array_equal(rows[0], Hs[0, [0, 1, 2, 10, 11]])


def test_total_mass_is_number_of_query_heads():
    H, G, N, D = 4, 4, 100, 32
    score = O.last_token_score(RNG.standard_normal((H * G, D)) * 3, RNG.standard_normal((H, N, D)), G)
    assert abs(score.sum() - H * G) < 1e-12 and np.all(score > 0)


def test_dominant_key_survives():
    H, G, N, D, Dm = 2, 1, 30, 8, 4
    K = RNG.standard_normal((1, H, N, D)) * 0.1
    q = RNG.standard_normal((1, H * G, D))
    K[0, 0, 7] = 30.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    K[0, 1, 19] = 30.0 * q[0, 1] / np.linalg.norm(q[0, 1])
    _, idx, score = O.hidden_evict(q, K, RNG.standard_normal((1, N, Dm)), n_keep=3, w=1, G=G)
    assert idx[0].tolist() == [7, 19, 29]
    assert abs(score[0, 7] - 1) < 1e-6 and abs(score[0, 19] - 1) < 1e-6


def test_exhaustive_subset_search_tiny():
    H, G, D, Dm = 1, 2, 4, 3
    for trial in range(40):
        N = int(RNG.integers(3, 9))
        w = int(RNG.integers(1, 3))
        K = RNG.integers(-1, 2, size=(1, H, N, D)).astype(np.float64)      # few distinct logits: ties happen
        q = RNG.integers(-1, 2, size=(1, H * G, D)).astype(np.float64)
        Hs = RNG.standard_normal((1, N, Dm))
        for n_keep in range(0, N + 2):
            rows, idx, score = O.hidden_evict(q, K, Hs, n_keep, w, G)
            nk = min(max(n_keep, min(w, N)), N)
            kp = max(nk - w, 0)
            P = N - w
            best = min(itertools.combinations(range(P), kp),
                       key=lambda cmb: (-sum(score[0, j] for j in cmb), cmb)) if kp <= P else ()
            want = list(best) + list(range(N - min(nk, w), N))
            assert idx[0].tolist() == want, (N, w, n_keep)
            assert np.array_equal(rows[0], Hs[0, want])


def test_rows_copied_verbatim_any_dtype():
    B, H, G, N, D, Dm = 2, 2, 2, 50, 16, 24
    K = RNG.standard_normal((B, H, N, D))
    q = RNG.standard_normal((B, H * G, D))
    Hs = RNG.integers(-30000, 30000, size=(B, N, Dm)).astype(np.int16)      # stands for bf16 bit patterns
    rows, idx, _ = O.hidden_evict(q, K, Hs, n_keep=20, w=4, G=G)
    assert rows.dtype == np.int16 and rows.shape == (B, 20, Dm)
    for b in range(B):
        assert np.all(np.diff(idx[b]) > 0) and idx[b, -4:].tolist() == [46, 47, 48, 49]
        assert np.array_equal(rows[b], Hs[b, idx[b]])
