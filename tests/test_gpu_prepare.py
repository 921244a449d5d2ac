"""GPU parity of the offline-preparation calls (Sec. 3.3.1 Eq. 7; App. Alg. 1) against the oracle:
votes, counts, labels and budgets exact; erank sums to fp64 rounding."""
import numpy as np
import pytest
import torch

from oracle import uncomp_oracle as O
from paper_2410_03090_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    from paper_2410_03090_amd import binding
    c = binding.Context(0, 64 << 20)
    yield c
    c.close()


@pytest.mark.parametrize("L,H,M", [(1, 8, 8), (5, 8, 2), (3, 32, 8), (2, 12, 1), (4, 64, 16), (2, 1024, 8)])
def test_prepare_matches_oracle(ctx, L, H, M):
    g = torch.Generator().manual_seed(L * 100 + H)
    st = ctx.prepare_new(L, H, M)
    ref = O.prepare_new(L, H, M)
    for B in (1, 3, 7):
        # quantised so that equal entropies (ties) occur
        ent = (torch.randint(0, 12, (L, B, H), generator=g).float() * 0.25 + 0.1).contiguous()
        ctx.prepare_accumulate(st, ent.to(DEV))
        O.prepare_accumulate(ref, ent.numpy(), M)
    lm, lv, mean = ctx.prepare_finish(st, want_mean=True)
    torch.cuda.synchronize()
    rlm, rlv, rmean = O.prepare_finish(ref, M)
    assert int(st[2][0]) == ref["count"] == 11
    assert np.array_equal(st[1].cpu().numpy(), ref["votes"])
    np.testing.assert_allclose(st[0].cpu().numpy(), ref["erank_sum"], rtol=1e-13)
    assert np.array_equal(lm.cpu().numpy(), rlm) and np.array_equal(lv.cpu().numpy(), rlv)
    np.testing.assert_allclose(mean.cpu().numpy(), rmean, rtol=1e-6)
    for labels, rl in ((lm, rlm), (lv, rlv)):
        hb = ctx.budgets_from_labels(labels, 3, 640, 74, 8192, 32)
        assert np.array_equal(hb.cpu().numpy(), O.budgets_from_labels(rl, 3, 640, 74, 8192, 32))
    hb = ctx.budgets_from_labels(lm, 2, 100, 30, 60, 8)                     # both clamps
    assert np.array_equal(hb.cpu().numpy(), O.budgets_from_labels(rlm, 2, 100, 30, 60, 8))


def test_prepare_from_entropy_call_and_reset(ctx):
    """d = 6 synthetic prompts through uncomp_head_entropy; the statistics of the GPU's own entropies
    match the oracle's; a reset starts over."""
    cfg = synth.tiny_config(dtype="bf16", L=3, B=2, H=8, G=1, N=512, w=8, M=4, rank_lo=2, rank_hi=40)
    st = ctx.prepare_new(cfg.L, cfg.H, cfg.M)
    ref = O.prepare_new(cfg.L, cfg.H, cfg.M)
    for seed in (1, 2, 3):
        K, _, _ = synth.gen_all(cfg, seed0=1000 * seed)
        ent = ctx.head_entropy(K.reshape(-1, cfg.N, cfg.D).to(DEV), k_trunc=cfg.k_trunc).reshape(cfg.L, cfg.B, cfg.H)
        ctx.prepare_accumulate(st, ent)
        torch.cuda.synchronize()
        O.prepare_accumulate(ref, ent.cpu().numpy(), cfg.M)
    lm, lv = ctx.prepare_finish(st)
    rlm, rlv, _ = O.prepare_finish(ref, cfg.M)
    assert int(st[2][0]) == 6
    assert np.array_equal(lm.cpu().numpy(), rlm) and np.array_equal(lv.cpu().numpy(), rlv)
    # the online call on one of the prompts uses the same ranking
    _, hg, _, _ = ctx.assign_budgets(ent, cfg.M, cfg.n_max, cfg.step, cfg.N, cfg.w)
    one = ctx.prepare_new(cfg.L, cfg.H, cfg.M)
    ctx.prepare_accumulate(one, ent[:, :1].contiguous())
    lm1, lv1 = ctx.prepare_finish(one)
    assert torch.equal(lm1, hg[:, 0]) and torch.equal(lv1, hg[:, 0])
    ctx.lib.uncomp_prepare_reset(ctx.handle, cfg.L, cfg.H, cfg.M, st[0].data_ptr(), st[1].data_ptr(), st[2].data_ptr(), None)
    torch.cuda.synchronize()
    assert int(st[2][0]) == 0 and float(st[0].abs().sum()) == 0.0 and int(st[1].abs().sum()) == 0


def test_prepare_argument_errors(ctx):
    from paper_2410_03090_amd import binding
    st = ctx.prepare_new(2, 8, 4)
    ent = torch.zeros(2, 1, 8, device=DEV)
    lib = ctx.lib
    code = lib.uncomp_prepare_accumulate(ctx.handle, ent.data_ptr(), 2, 1, 8, 3, st[0].data_ptr(), st[1].data_ptr(),
                                         st[2].data_ptr(), None)
    assert code == binding.ERR_UNSUPPORTED                                  # M does not divide H
    code = lib.uncomp_prepare_accumulate(ctx.handle, None, 2, 1, 8, 4, st[0].data_ptr(), st[1].data_ptr(),
                                         st[2].data_ptr(), None)
    assert code == binding.ERR_INVALID_ARG
    code = lib.uncomp_prepare_finish(ctx.handle, 2, 2048, 4, st[0].data_ptr(), st[1].data_ptr(), st[2].data_ptr(),
                                     st[1].data_ptr(), st[1].data_ptr(), None, None)
    assert code == binding.ERR_UNSUPPORTED                                  # H above the limit
    code = lib.uncomp_budgets_from_labels(ctx.handle, st[1].data_ptr(), 2, 1, 8, 100, 10, 50, 50, st[1].data_ptr(), None)
    assert code == binding.ERR_UNSUPPORTED                                  # w >= N
    torch.cuda.synchronize()
    assert int(st[2][0]) == 0
