"""Sizes at the far ends of what the calls accept: a million-token head, tens of thousands of short
matrices, the widest head count of the budget call, a compacted cache of half a million rows."""
import numpy as np
import pytest
import torch

from oracle import uncomp_oracle as O
from tests._util import check_index_sets, raw_bits, to_f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D = 128


def test_million_token_head():
    from paper_2410_03090_amd import binding
    B, H, G, N, w, pool = 1, 1, 4, 1_000_003, 64, 7
    g = torch.Generator(device=DEV).manual_seed(1)
    r = 24
    Vf = torch.randn(D, r, generator=g, device=DEV) / r ** 0.5
    K = ((torch.randn(N, r, generator=g, device=DEV) / r ** 0.5) @ Vf.T + 0.1 * torch.randn(N, D, generator=g, device=DEV))
    K = K.to(torch.bfloat16).view(B, H, N, D)
    V = torch.randn(B, H, N, D, generator=g, device=DEV).to(torch.bfloat16)
    Q = ((torch.randn(G * w, r, generator=g, device=DEV) / r ** 0.5) @ Vf.T).to(torch.bfloat16).view(B, H * G, w, D)
    ctx = binding.Context(0, binding.Context.workspace_bytes(1, N, D, B, H, G, w))
    ent, eig = ctx.head_entropy(K.view(1, N, D), k_trunc=32, want_eig=True)
    score = ctx.window_score(Q, K, G, pool)
    budget = torch.tensor([[500_000]], dtype=torch.int32, device=DEV)
    cap = 500_000
    Ko, Vo, idx, ln = ctx.select_gather(score, budget, K, V, w, cap)
    torch.cuda.synchronize()
    Href, eref = O.head_entropy(to_f64(K.view(1, N, D)), k_trunc=32)
    np.testing.assert_allclose(ent.cpu().numpy(), Href, rtol=1e-4)
    np.testing.assert_allclose(eig.cpu().numpy(), eref, rtol=0, atol=2e-5)
    sref = O.window_score(to_f64(Q), to_f64(K), G, pool)
    np.testing.assert_allclose(score.cpu().numpy(), sref, rtol=2e-5, atol=1e-12)
    sel = O.select_indices(sref[0, 0], cap, N, w)
    check_index_sets(idx.cpu().numpy()[0, 0], int(ln[0, 0]), sel, len(sel), sref[0, 0], w)
    assert torch.equal(Ko[0, 0].view(torch.int16), K[0, 0][idx[0, 0].long()].view(torch.int16))
    assert torch.equal(Vo[0, 0].view(torch.int16), V[0, 0][idx[0, 0].long()].view(torch.int16))
    ctx.close()


def test_many_short_matrices_and_widest_budget_call():
    from paper_2410_03090_amd import binding
    n_mat, N = 40_960, 48
    g = torch.Generator(device=DEV).manual_seed(2)
    X = (torch.randn(n_mat, N, 6, generator=g, device=DEV) @ torch.randn(6, D, generator=g, device=DEV)
         + 0.05 * torch.randn(n_mat, N, D, generator=g, device=DEV)).to(torch.bfloat16)
    ctx = binding.Context(0, binding.Context.workspace_bytes(n_mat, N, D, 0, 0, 0, 0))
    ent = ctx.head_entropy(X, k_trunc=32)
    torch.cuda.synchronize()
    pick = list(range(0, n_mat, 4099)) + [n_mat - 1]
    Href, _ = O.head_entropy(to_f64(X[pick]), k_trunc=32)
    np.testing.assert_allclose(ent.cpu().numpy()[pick], Href, rtol=1e-4)
    assert torch.isfinite(ent).all() and float(ent.min()) >= 0 and float(ent.max()) <= np.log(32) + 1e-5
    # the budget call at its limits: 1024 heads per layer, 40 layers
    L, B, H, M = 40, 1, 1024, 8
    e3 = ent[: L * B * H].reshape(L, B, H).contiguous()
    hb, hg, lg, lt = ctx.assign_budgets(e3, M, 640, 74, 8192, 32)
    torch.cuda.synchronize()
    rb = O.assign_budgets(e3.cpu().numpy(), M, 640, 74, 8192, 32, 0.4, 512)
    for a, b in zip((hb, hg, lg, lt), rb):
        assert np.array_equal(a.cpu().numpy(), b)
    ctx.close()


def test_decode_cache_beyond_the_merge_tables_is_refused_before_any_launch():
    """bf16 decode: the per-head merge tables of the update kernel live in 64 KiB of LDS.  A cache beyond that is
    UNSUPPORTED (status code, nothing launched, state untouched); one just inside works and matches the oracle."""
    from paper_2410_03090_amd import binding
    G, w = 16, 8
    g = torch.Generator(device=DEV).manual_seed(3)
    for cap, ok in ((50_000, False), (40_000, True)):
        n = cap - 5
        Kc = torch.randn(1, cap, D, generator=g, device=DEV).to(torch.bfloat16)
        Vc = torch.randn(1, cap, D, generator=g, device=DEV).to(torch.bfloat16)
        idx = torch.arange(cap, dtype=torch.int32, device=DEV).view(1, cap).contiguous()
        cum = torch.rand(1, cap, generator=g, device=DEV)
        ln = torch.tensor([n], dtype=torch.int32, device=DEV)
        q = (0.3 * torch.randn(1, G, D, generator=g, device=DEV)).to(torch.bfloat16)
        kn = torch.randn(1, D, generator=g, device=DEV).to(torch.bfloat16)
        vn = torch.randn(1, D, generator=g, device=DEV).to(torch.bfloat16)
        pos = torch.tensor([n], dtype=torch.int32, device=DEV)
        bud = torch.tensor([n], dtype=torch.int32, device=DEV)          # full: the step evicts
        ctx = binding.Context(0, binding.Context.decode_workspace_bytes(1, G, cap))
        before = [t.clone() for t in (Kc, Vc, idx, cum, ln)]
        if not ok:
            with pytest.raises(binding.UncompError) as e:
                ctx.decode_step(q, kn, vn, pos, bud, w, Kc, Vc, idx, cum, ln)
            assert e.value.status == binding.ERR_UNSUPPORTED
            torch.cuda.synchronize()
            for a, b in zip(before, (Kc, Vc, idx, cum, ln)):
                assert torch.equal(a, b)
        else:
            out, ev = ctx.decode_step(q, kn, vn, pos, bud, w, Kc, Vc, idx, cum, ln)
            torch.cuda.synchronize()
            r = O.decode_step(to_f64(before[0][0, :n]), to_f64(before[1][0, :n]), before[2][0, :n].cpu().numpy(),
                              before[3][0, :n].cpu().numpy().astype(np.float64), to_f64(q[0]), to_f64(kn[0]), to_f64(vn[0]),
                              n, n, w)
            np.testing.assert_allclose(out[0].cpu().numpy(), r[4], atol=2e-5)
            assert int(ev[0]) == r[5] and int(ln[0]) == len(r[2])
        ctx.close()


def test_budget_arithmetic_beyond_32_bits():
    """group index times step may exceed 2^31: the budget is still the clamped arithmetic value."""
    from paper_2410_03090_amd import binding
    ctx = binding.Context(0, 1 << 20)
    ent = torch.tensor([[[3.0, 2.5, 2.0, 1.5, 1.0, 0.9, 0.8, 0.1]]], device=DEV)
    n_max, step, N, w = 2_000_000_000, 1_000_000_000, 2_100_000_000, 8
    hb, hg, _, _ = ctx.assign_budgets(ent, 8, n_max, step, N, w)
    torch.cuda.synchronize()
    ref = O.assign_budgets(ent.cpu().numpy(), 8, n_max, step, N, w, 0.4, 512)
    assert np.array_equal(hb.cpu().numpy(), ref[0]) and np.array_equal(hg.cpu().numpy(), ref[1])
    assert hb.cpu().numpy().ravel().tolist() == [2_000_000_000, 1_000_000_000] + [8] * 6
    ctx.close()
