"""Pins for the oracle's budget assignment (Sec. 3.3.3 Eq. 11; Sec. 3.3.2 Eq. 8-10)."""
import os

import numpy as np

from oracle import uncomp_oracle as O


def _paper_rows(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_budget_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        left, right = line.split("|")
        M, n_max, step = (int(x) for x in left.split())
        yield M, n_max, step, [int(x) for x in right.split()]


def test_paper_printed_budget_vectors(golden_dir):
    rows = list(_paper_rows(golden_dir))
    assert len(rows) == 7
    for M, n_max, step, want in rows:
        # one head per group, entropies strictly decreasing with head index
        ent = np.linspace(3.0, 1.0, M, dtype=np.float32)[None, None, :]
        hb, hg, _, _ = O.assign_budgets(ent, M, n_max, step, N=4096, w=8, eps=0.3, delta_n=512)
        assert hb[0, 0].tolist() == want
        assert hg[0, 0].tolist() == list(range(M))


def test_main_setting_mean_is_about_384(golden_dir):
    M, n_max, step, want = next(_paper_rows(golden_dir))
    assert (M, n_max, step) == (8, 640, 74)
    assert abs(sum(want) / M - 384) <= 3          # the paper's "average KV size 384"


def test_highest_entropy_gets_largest_budget_hand_example():
    # 8 heads, M = 4 groups of 2.  Ranking by entropy (desc): h5 h2 | h7 h0 | h3 h6 | h1 h4
    ent = np.array([2.0, 0.5, 3.0, 1.5, 0.1, 3.5, 1.0, 2.5], dtype=np.float32)[None, None]
    hb, hg, _, _ = O.assign_budgets(ent, M=4, n_max=100, step=20, N=1000, w=8, eps=0.3, delta_n=512)
    assert hg[0, 0].tolist() == [1, 3, 0, 2, 3, 0, 2, 1]
    assert hb[0, 0].tolist() == [80, 40, 100, 60, 40, 100, 60, 80]


def test_ties_go_to_lower_head_index_and_batches_rank_separately():
    ent = np.array([[[1.0, 2.0, 2.0, 1.0]], ], dtype=np.float32)           # L=1,B=1,H=4
    hb, hg, _, _ = O.assign_budgets(ent, M=4, n_max=40, step=10, N=100, w=4, eps=0.3, delta_n=10)
    assert hg[0, 0].tolist() == [2, 0, 1, 3]
    ent2 = np.array([[[1.0, 2.0], [2.0, 1.0]]], dtype=np.float32)           # L=1,B=2,H=2
    hb2, _, _, _ = O.assign_budgets(ent2, M=2, n_max=40, step=10, N=100, w=4, eps=0.3, delta_n=10)
    assert hb2[0].tolist() == [[30, 40], [40, 30]]


def test_budget_clamps():
    ent = np.array([3.0, 2.0, 1.0, 0.5], dtype=np.float32)[None, None]
    hb, _, _, _ = O.assign_budgets(ent, M=4, n_max=70, step=30, N=64, w=16, eps=0.3, delta_n=10)
    assert hb[0, 0].tolist() == [64, 40, 16, 16]       # 70->N, 40, 10->w, -20->w


def test_layer_stages_hand_worked():
    # PARITY UNPINNED in the paper (no worked example for Eq. 8-10): this fixes only the
    # arithmetic of the chosen reading.  erank per layer = 10, 9, 9.5, 8, 8 (single head).
    er = np.array([10.0, 9.0, 9.5, 8.0, 8.0])
    ent = np.log(er).astype(np.float32)[:, None, None]
    _, _, lg, lt = O.assign_budgets(ent, M=1, n_max=64, step=0, N=4096, w=8, eps=0.4, delta_n=512)
    # reductions 1.0, -0.5, 1.5, 0.0 -> boundaries after layers 0 and 2
    assert lg.tolist() == [0, 1, 1, 2, 2]
    assert lt.tolist() == [4096, 3584, 3584, 3072, 3072]
    _, _, lg2, lt2 = O.assign_budgets(ent, M=1, n_max=64, step=0, N=4096, w=8, eps=0.4, delta_n=512,
                                      flags=O.DEFAULT_FLAGS | O.FLAG_LAYER_DELTA_INCREASE)
    assert lg2.tolist() == [0, 0, 1, 1, 1]             # only the +0.5 increase exceeds eps
    # monotone, first stage full, floor at w
    _, _, lg3, lt3 = O.assign_budgets(ent, M=1, n_max=64, step=0, N=600, w=100, eps=0.4, delta_n=512)
    assert lt3.tolist() == [600, 100, 100, 100, 100]
    assert all(a >= b for a, b in zip(lt3[:-1], lt3[1:]))


def test_layer_mean_is_over_erank_not_entropy():
    # two heads: eranks (1, 9) -> mean 5;  next layer (4, 4) -> mean 4.  Mean-of-erank drop = 1.0;
    # a mean-of-entropy reading would give exp(mean H): 3 -> 4, i.e. an increase.
    ent = np.log(np.array([[[1.0, 9.0]], [[4.0, 4.0]]])).astype(np.float32)
    _, _, lg, _ = O.assign_budgets(ent, M=1, n_max=8, step=0, N=64, w=4, eps=0.5, delta_n=8)
    assert lg.tolist() == [0, 1]
