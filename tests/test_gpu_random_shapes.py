"""Seeded sweep of small random shapes through the four prefill calls, against the oracle: sequence
lengths that are not multiples of any tile, windows of every parity, query-head counts that do and do not
fill 16-row blocks, budgets below the window and above the capacity, padded key rows."""
import numpy as np
import pytest
import torch

from oracle import uncomp_oracle as O
from paper_2410_03090_amd import synth
from tests._util import check_index_sets, raw_bits, to_f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D = 128


@pytest.fixture(scope="module")
def ctx():
    from paper_2410_03090_amd import binding
    c = binding.Context(0, 256 << 20)
    yield c
    c.close()


def _cases():
    rng = np.random.default_rng(20241003)
    out = []
    for i in range(24):
        w = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 32, 48, 64]))
        G = int(rng.choice([1, 2, 3, 4, 7, 8]))
        while G * w > 512:
            G = max(1, G // 2)
        N = int(w + 1 + rng.integers(1, 2600))
        H = int(rng.choice([1, 2, 3, 4]))
        M = int(rng.choice([m for m in (1, 2, 3, 4) if H % m == 0]))
        pool = int(rng.choice([1, 3, 7, 15]))
        out.append((i, "bf16" if i % 3 else "f32", H, G, N, w, M, pool, int(rng.integers(0, 3)) * 8))
    return out


@pytest.mark.parametrize("case,dtype,H,G,N,w,M,pool,pad", _cases())
def test_random_shape(ctx, case, dtype, H, G, N, w, M, pool, pad):
    cfg = synth.tiny_config(dtype=dtype, B=2, H=H, G=G, N=N, w=w, M=M, pool=pool, rank_lo=2, rank_hi=30)
    K, V, Q = synth.gen_all(cfg, seed0=900 + case)
    K, V, Q = K[0], V[0], Q[0]
    if pad:                                                              # key / value rows with a gap after the 128 features
        Kp = torch.zeros(2, H, N, D + pad, dtype=K.dtype)
        Vp = torch.zeros_like(Kp)
        Kp[..., :D], Vp[..., :D] = K, V
        Kd, Vd = Kp.to(DEV)[..., :D], Vp.to(DEV)[..., :D]
    else:
        Kd, Vd = K.to(DEV), V.to(DEV)
    Qd = Q.to(DEV)
    k_trunc = 32
    ent = torch.stack([ctx.head_entropy(Kd[b], k_trunc=k_trunc) for b in range(2)])      # [B, H]: strided matrices per batch entry
    n_max, step = max(w + 5, N // 3), max(1, N // 12)
    hb, hg, lg, lt = ctx.assign_budgets(ent.reshape(1, 2, H), M, n_max, step, N, w)
    score = ctx.window_score(Qd, Kd, G, pool)
    cap = min(N, n_max)
    budget = hb[0].clone()
    budget[0, 0] = 0                                                    # below the window
    budget[1, -1] = N + 10                                              # above the capacity
    Ko, Vo, idx, ln = ctx.select_gather(score, budget, Kd, Vd, w, cap)
    torch.cuda.synchronize()

    Href, _ = O.head_entropy(to_f64(K.reshape(-1, N, D)), k_trunc=k_trunc)
    np.testing.assert_allclose(ent.cpu().numpy().ravel(), Href, rtol=1e-4, atol=5e-5)
    rb = O.assign_budgets(ent.cpu().numpy().reshape(1, 2, H), M, n_max, step, N, w, 0.4, 512)
    assert np.array_equal(hb.cpu().numpy(), rb[0]) and np.array_equal(hg.cpu().numpy(), rb[1])
    sref = O.window_score(to_f64(Q), to_f64(K), G, pool)
    np.testing.assert_allclose(score.cpu().numpy(), sref, rtol=2e-5, atol=1e-9)
    bud_h = np.minimum(budget.cpu().numpy(), cap)
    idx_h, ln_h = idx.cpu().numpy(), ln.cpu().numpy()
    Kb, Vb, Kob, Vob = raw_bits(K), raw_bits(V), raw_bits(Ko), raw_bits(Vo)
    for b in range(2):
        for h in range(H):
            sel = O.select_indices(sref[b, h], int(bud_h[b, h]), N, w)
            check_index_sets(idx_h[b, h], ln_h[b, h], sel, len(sel), sref[b, h], w)
            n = int(ln_h[b, h])
            assert np.array_equal(Kob[b, h, :n], Kb[b, h][idx_h[b, h, :n]])
            assert np.array_equal(Vob[b, h, :n], Vb[b, h][idx_h[b, h, :n]])
