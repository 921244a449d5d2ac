"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp32/bf16 tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def raw_bits(t: torch.Tensor) -> np.ndarray:
    """The storage bits of a tensor as an integer numpy array (for bit-exact compares)."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy()
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy()
    return t.numpy()


def check_index_sets(idx_gpu, len_gpu, idx_ref, len_ref, score_ref, w, rel_band=1e-5):
    """Kept-position sets must agree except for positions whose oracle score lies within
    rel_band (relative) of the oracle's k-th largest score.  Returns the number of such
    near-tie swaps.  idx_* [cap] int arrays, score_ref [P] float64."""
    assert int(len_gpu) == int(len_ref), (len_gpu, len_ref)
    n = int(len_ref)
    a = np.asarray(idx_gpu[:n]).astype(np.int64)
    b = np.asarray(idx_ref[:n]).astype(np.int64)
    assert np.all(np.diff(a) > 0), "GPU indices not strictly ascending"
    if np.array_equal(a, b):
        return 0
    k = n - w
    assert np.array_equal(a[k:], b[k:]), "window suffix differs"
    only_gpu = np.setdiff1d(a[:k], b[:k])
    only_ref = np.setdiff1d(b[:k], a[:k])
    assert len(only_gpu) == len(only_ref)
    kth = np.sort(score_ref)[::-1][k - 1]
    band = rel_band * abs(kth)
    for j in np.concatenate([only_gpu, only_ref]):
        assert abs(score_ref[j] - kth) <= band, (
            f"position {j}: score {score_ref[j]!r} differs from k-th {kth!r} by more than the tie band")
    return len(only_gpu)


def tie_band_count(idx_ref, n, score_ref, w, rel_band=1e-5):
    """How many of the kept prefix positions of one head have an oracle score within rel_band
    (relative) of the oracle's k-th largest score, i.e. could legitimately be swapped for a
    rejected position of (almost) the same score.  idx_ref: the oracle's kept positions."""
    k = int(n) - w
    if k <= 0 or k >= len(score_ref):
        return 0
    kth = np.sort(score_ref)[::-1][k - 1]
    kept = np.asarray(idx_ref[:k]).astype(np.int64)
    return int(np.sum(np.abs(score_ref[kept] - kth) <= rel_band * abs(kth)))


def check_budgets_against_oracle_entropy(budget_gpu, ent_ref, budget_ref, rel_gap=2e-4):
    """Budgets of the H heads of one (layer, batch) against the budgets the oracle derives from its
    OWN entropies (rounded to fp32 before ranking).  They must be equal, except that two heads whose
    oracle entropies differ by less than rel_gap (relative) may have traded places: every pair that
    the GPU orders against the oracle's entropies must be such a near-tie, and the multiset of
    budgets must be the oracle's.  Returns the number of heads whose budget differs (0 or more,
    all of them inside near-ties)."""
    bg = np.asarray(budget_gpu).astype(np.int64)
    br = np.asarray(budget_ref).astype(np.int64)
    e = np.asarray(ent_ref, dtype=np.float64)
    assert np.array_equal(np.sort(bg), np.sort(br)), (bg, br)
    if np.array_equal(bg, br):
        return 0
    H = len(bg)
    for a in range(H):
        for b in range(H):
            if bg[a] > bg[b] and not (e[a] > e[b] or (e[a] == e[b] and a < b)):
                # the GPU ranked a above b although the oracle's entropies say otherwise
                gap = abs(e[a] - e[b]) / max(abs(e[a]), abs(e[b]), 1e-300)
                assert gap < rel_gap, (
                    f"heads {a},{b}: budgets {bg[a]},{bg[b]} against oracle entropies {e[a]!r},{e[b]!r} "
                    f"(relative gap {gap:.3e} is no near-tie)")
    return int(np.sum(bg != br))
