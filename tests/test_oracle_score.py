"""Pins for the oracle's observation-window score (Sec. 3.3.3, "Dynamic KV Cache Eviction")."""
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(472)


def test_zero_queries_give_causal_harmonic_sums():
    # q = 0 -> every causal row is uniform: p_ij = 1/(P+i+1); vote = sum_i 1/(P+i+1) for all j < P
    B, H, G, N, D, w = 1, 2, 3, 40, 16, 5
    K = RNG.standard_normal((B, H, N, D))
    Q = np.zeros((B, H * G, w, D))
    s = O.window_score(Q, K, G=G, pool=7)
    P = N - w
    want = G * sum(1.0 / (P + i + 1) for i in range(w))
    assert s.shape == (B, H, P)
    assert np.allclose(s, want, rtol=1e-12)


def test_single_row_reduces_to_library_softmax():
    B, H, G, N, D, w = 1, 1, 1, 33, 8, 1
    K = RNG.standard_normal((B, H, N, D))
    Q = RNG.standard_normal((B, 1, w, D)) * 2.0
    s = O.window_score(Q, K, G=1, pool=1)
    logits = np.array([sum(Q[0, 0, 0, d] * K[0, 0, j, d] for d in range(D)) for j in range(N)]) / math.sqrt(D)
    want = softmax(logits)[: N - 1]
    assert np.allclose(s[0, 0], want, rtol=1e-12)


def test_mass_conservation_pool1():
    # with pool = 1 and G = 1: sum_j score[j] + (mass on window keys) = w; the window part is
    # recomputed here from a library softmax per causal row
    B, H, N, D, w = 2, 2, 64, 16, 6
    K = RNG.standard_normal((B, H, N, D))
    Q = RNG.standard_normal((B, H, w, D)) * 3.0
    s = O.window_score(Q, K, G=1, pool=1)
    P = N - w
    for b in range(B):
        for h in range(H):
            win_mass = 0.0
            for i in range(w):
                row = softmax((K[b, h, : P + i + 1] @ Q[b, h, i]) / math.sqrt(D))
                win_mass += row[P:].sum()
            assert s[b, h].sum() + win_mass == pytest.approx(w, rel=1e-12)


def test_spike_becomes_plateau_and_group_sum():
    # one key aligned with the query and scaled up: attention concentrates on it, the max-pool
    # spreads it to the +-3 neighbours, clipped at the prefix boundary
    B, H, G, N, D, w, pool = 1, 1, 2, 50, 8, 3, 7
    P = N - w
    for j0 in (0, 1, 20, P - 1):
        K = np.zeros((B, H, N, D))
        K[0, 0, j0, 0] = 40.0
        Q = np.zeros((B, G, w, D))
        Q[:, :, :, 0] = 40.0
        s = O.window_score(Q, K, G=G, pool=pool)[0, 0]
        plateau = np.arange(max(0, j0 - 3), min(P, j0 + 4))
        assert np.allclose(s[plateau], G * w, rtol=1e-9)        # each of G*w rows puts ~all mass on j0
        rest = np.setdiff1d(np.arange(P), plateau)
        assert np.all(s[rest] < 1e-9)
    # pool = 1 leaves the spike alone
    s1 = O.window_score(Q, K, G=G, pool=1)[0, 0]
    assert s1[P - 1] == pytest.approx(G * w, rel=1e-9) and np.all(s1[: P - 1] < 1e-9)


def test_query_heads_map_to_their_kv_head():
    # KV head 1 has the spike, KV head 0 does not; only query heads 2,3 (G = 2) read head 1
    B, H, G, N, D, w = 1, 2, 2, 30, 4, 2
    K = np.zeros((B, H, N, D))
    K[0, 1, 5, 0] = 30.0
    Q = np.zeros((B, H * G, w, D))
    Q[:, :, :, 0] = 30.0
    s = O.window_score(Q, K, G=G, pool=1)
    P = N - w
    uniform = G * sum(1.0 / (P + i + 1) for i in range(w))
    assert np.allclose(s[0, 0], uniform, rtol=1e-12)
    assert s[0, 1, 5] == pytest.approx(G * w, rel=1e-9)


def test_pool_is_per_query_head_before_group_sum():
    # two query heads of one KV head spike at tokens 10 and 13 (pool 7: plateaus 7..13 and 10..16).
    # pooling each head first gives 2*w on the overlap 10..13 and w on 7..9, 14..16.
    B, H, G, N, D, w = 1, 1, 2, 40, 4, 2
    K = np.zeros((B, H, N, D))
    K[0, 0, 10, 0] = 50.0
    K[0, 0, 13, 1] = 50.0
    Q = np.zeros((B, G, w, D))
    Q[0, 0, :, 0] = 50.0
    Q[0, 1, :, 1] = 50.0
    s = O.window_score(Q, K, G=G, pool=7)[0, 0]
    assert np.allclose(s[10:14], 2 * w, rtol=1e-9)
    assert np.allclose(s[7:10], w, rtol=1e-9) and np.allclose(s[14:17], w, rtol=1e-9)
    assert np.all(s[:7] < 1e-9) and np.all(s[17:] < 1e-9)


def test_scale_is_one_over_sqrt_d():
    # two keys, logits differ by exactly delta/sqrt(D): p ratio = exp(delta/sqrt(D))
    D, N, w = 16, 3, 1
    K = np.zeros((1, 1, N, D))
    K[0, 0, 0, 0] = 1.0
    Q = np.zeros((1, 1, w, D))
    Q[0, 0, 0, 0] = 8.0
    s = O.window_score(Q, K, G=1, pool=1)[0, 0]
    assert s[0] / s[1] == pytest.approx(math.exp(8.0 / 4.0), rel=1e-12)


def test_window_lse_closed_form_library_and_consistency():
    # zero queries: every logit is 0, the normaliser of row i is ln(number of causal keys)
    B, H, G, N, D, w = 1, 2, 2, 37, 8, 4
    P = N - w
    K = RNG.standard_normal((B, H, N, D))
    lse0 = O.window_lse(np.zeros((B, H * G, w, D)), K, G)
    for i in range(w):
        assert np.allclose(lse0[:, :, i], math.log(P + i + 1), rtol=0, atol=1e-13)
    # random queries: a library logsumexp over each causal row, with the query head -> KV head map
    from scipy.special import logsumexp
    Q = RNG.standard_normal((B, H * G, w, D)) * 3.0
    lse = O.window_lse(Q, K, G)
    for q in range(H * G):
        for i in range(w):
            row = (K[0, q // G, : P + i + 1] @ Q[0, q, i]) / math.sqrt(D)
            assert lse[0, q, i] == pytest.approx(logsumexp(row), rel=1e-13)
    # exp(logit - lse) summed over the window rows and the query heads is the unpooled score
    s = O.window_score(Q, K, G=G, pool=1)
    for h in range(H):
        want = np.zeros(P)
        for q in range(h * G, (h + 1) * G):
            for i in range(w):
                want += np.exp((K[0, h, :P] @ Q[0, q, i]) / math.sqrt(D) - lse[0, q, i])
        assert np.allclose(s[0, h], want, rtol=1e-12)
