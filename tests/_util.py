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
