"""Pins for the oracle's offline preparation (Sec. 3.3.1 Eq. 7; App. Alg. 1)."""
import numpy as np

from oracle import uncomp_oracle as O

RNG = np.random.default_rng(500)


def test_hand_worked_two_samples():
    """One layer, four heads, two groups.  Sample 1 entropies ln(8, 4, 2, 1): groups 0 0 1 1.
    Sample 2 entropies ln(1, 9, 8, 2): groups 1 0 0 1.  Mean erank (4.5, 6.5, 5, 1.5): groups
    1 0 0 1.  Votes: head 0 has one vote each way -> lower label 0; head 2 likewise -> 0."""
    st = O.prepare_new(1, 4, 2)
    O.prepare_accumulate(st, np.log(np.array([[[8.0, 4, 2, 1]]])), 2)
    O.prepare_accumulate(st, np.log(np.array([[[1.0, 9, 8, 2]]])), 2)
    lm, lv, mean = O.prepare_finish(st, 2)
    np.testing.assert_allclose(mean[0], [4.5, 6.5, 5.0, 1.5], rtol=1e-14)
    assert lm[0].tolist() == [1, 0, 0, 1]
    assert st["votes"][0].tolist() == [[1, 1], [2, 0], [1, 1], [0, 2]]
    assert lv[0].tolist() == [0, 0, 0, 1]
    assert st["count"] == 2


def test_one_sample_reproduces_online_groups():
    L, B, H, M = 5, 1, 8, 4
    ent = RNG.random((L, B, H)).astype(np.float32) * 3
    st = O.prepare_new(L, H, M)
    O.prepare_accumulate(st, ent, M)
    lm, lv, _ = O.prepare_finish(st, M)
    _, group, _, _ = O.assign_budgets(ent, M, 640, 74, 8192, 32, 0.4, 512)
    assert np.array_equal(lm, group[:, 0]) and np.array_equal(lv, group[:, 0])


def test_batch_and_order_do_not_matter():
    L, H, M, d = 3, 8, 8, 11
    ent = RNG.random((L, d, H)) * 3
    a = O.prepare_new(L, H, M)
    O.prepare_accumulate(a, ent, M)
    b = O.prepare_new(L, H, M)
    for i in RNG.permutation(d):
        O.prepare_accumulate(b, ent[:, i:i + 1], M)
    assert np.array_equal(a["votes"], b["votes"]) and a["count"] == b["count"] == d
    np.testing.assert_allclose(a["erank_sum"], b["erank_sum"], rtol=1e-13)
    assert a["votes"].sum() == L * H * d and np.all(a["votes"].sum(axis=2) == d)
    assert np.all(a["votes"].sum(axis=1) == d * (H // M))         # every sample fills every group of a layer


def test_mean_is_of_erank_not_of_entropy():
    """Two heads, two samples, entropies (0, 1.3) and (2.5, 1.3): the mean entropy ranks head 1 first
    (1.3 > 1.25), the mean erank of Eq. 7 ranks head 0 first (6.59 > 3.67)."""
    st = O.prepare_new(1, 2, 2)
    O.prepare_accumulate(st, np.array([[[0.0, 1.3]]]), 2)
    O.prepare_accumulate(st, np.array([[[2.5, 1.3]]]), 2)
    lm, _, mean = O.prepare_finish(st, 2)
    np.testing.assert_allclose(mean[0], [(1 + np.exp(2.5)) / 2, np.exp(1.3)], rtol=1e-14)
    assert lm[0].tolist() == [0, 1]


def test_budgets_from_labels_paper_vector():
    """Labels 0..7 with the paper's N_1 = 640 and step 74 (Sec. 4.2 'Main Results') give its
    printed per-group sizes."""
    import os
    golden = os.path.join(os.path.dirname(__file__), "golden", "paper_budget_vectors.txt")
    line = next(ln for ln in open(golden) if ln.startswith("8 640 74 |"))
    want = [int(x) for x in line.split("|")[1].split()]
    assert want == [640, 566, 492, 418, 344, 270, 196, 122]
    got = O.budgets_from_labels(np.arange(8)[None], 2, 640, 74, 8192, 32)
    assert got.shape == (1, 2, 8) and got[0, 0].tolist() == want and got[0, 1].tolist() == want
    assert O.budgets_from_labels(np.array([[0, 7]]), 1, 100, 20, 50, 8)[0, 0].tolist() == [50, 8]    # clamps


def test_budgets_from_labels_match_online_budgets():
    L, B, H, M = 4, 3, 8, 8
    ent = RNG.random((L, B, H)).astype(np.float32)
    hb, hg, _, _ = O.assign_budgets(ent, M, 640, 74, 8192, 32, 0.4, 512)
    for b in range(B):
        assert np.array_equal(O.budgets_from_labels(hg[:, b], 1, 640, 74, 8192, 32)[:, 0], hb[:, b])
