"""GPU parity of uncomp_hidden_evict (Sec. 3.3.2 "Hidden State Eviction") against the oracle.
Tolerances as for the prefill selection: scores 2e-5 relative, kept positions exact except ties
within 1e-5 of the last kept score, rows bit-exact."""
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
    c = binding.Context(0, 512 << 20)
    yield c
    c.close()


def _inputs(B, H, G, N, Dm, dtype, seed, row_pad=0):
    g = torch.Generator().manual_seed(seed)
    K = (torch.randn(B, H, N, D, generator=g) * 1.5).to(dtype)
    q = (torch.randn(B, H * G, D, generator=g) * 1.5).to(dtype)
    Hs_full = torch.randn(B, N, Dm + row_pad, generator=g).to(dtype)
    return q, K, Hs_full


def _compare(ctx, q, K, Hs_full, Dm, G, n_keep, w, cap):
    B, H, N, _ = K.shape
    Hs = Hs_full[:, :, :Dm]
    nk = torch.tensor([n_keep], dtype=torch.int32, device=DEV)
    Ho, idx, ln, score = ctx.hidden_evict(q.to(DEV), K.to(DEV), G, nk, w, Hs_full.to(DEV)[:, :, :Dm], cap, want_score=True)
    torch.cuda.synchronize()
    rows_ref, idx_ref, score_ref = O.hidden_evict(to_f64(q), to_f64(K), raw_bits(Hs), min(n_keep, cap), w, G)
    np.testing.assert_allclose(score.cpu().numpy(), score_ref[:, : N - w], rtol=2e-5, atol=1e-9)
    idx, ln, Ho = idx.cpu().numpy(), ln.cpu().numpy(), Ho.cpu()
    for b in range(B):
        n = idx_ref.shape[1]
        check_index_sets(idx[b], ln[b], idx_ref[b], n, score_ref[b, : N - w], w)
        assert np.array_equal(raw_bits(Ho[b, :n]), raw_bits(Hs[b])[idx[b, :n]])       # rows of the GPU's own choice, bit for bit
        assert np.all(raw_bits(Ho[b, n:]) == 0) and np.all(idx[b, n:] == -1)          # untouched beyond len


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("H,G,N,w,Dm", [(2, 1, 33, 1, 64), (3, 4, 300, 4, 256), (2, 4, 1027, 1, 4096), (8, 4, 2050, 8, 512)])
def test_hidden_evict_matches_oracle(ctx, dtype, H, G, N, w, Dm):
    q, K, Hs = _inputs(2, H, G, N, Dm, dtype, seed=N + H)
    for n_keep in (0, w, N // 3, N - 1, N, N + 7):
        _compare(ctx, q, K, Hs, Dm, G, n_keep, w, cap=N)


def test_hidden_evict_bf16_general_path(ctx):
    """bf16 through the general scoring kernels (the path fp32 always takes) instead of the MFMA pass."""
    q, K, Hs = _inputs(2, 3, 4, 700, 128, torch.bfloat16, seed=77)
    ctx.set_kernel_path(True)
    try:
        _compare(ctx, q, K, Hs, 128, 4, 300, 4, cap=700)
    finally:
        ctx.set_kernel_path(False)
    _compare(ctx, q, K, Hs, 128, 4, 300, 4, cap=700)


def test_hidden_evict_strided_rows_and_small_cap(ctx):
    q, K, Hs = _inputs(2, 2, 2, 500, 128, torch.bfloat16, seed=5, row_pad=64)        # row stride 192 elements
    _compare(ctx, q, K, Hs, 128, 2, 400, 2, cap=120)                                  # n_keep above cap: clamped to cap
    _compare(ctx, q, K, Hs, 128, 2, 50, 2, cap=120)


def test_hidden_evict_indices_only_and_budget_from_layer_tokens(ctx):
    """n_keep read from the layer_tokens array that uncomp_assign_budgets wrote."""
    B, H, G, N, w = 1, 4, 2, 600, 4
    q, K, _ = _inputs(B, H, G, N, 64, torch.float32, seed=9)
    ent = torch.tensor([[[3.0] * H], [[2.0] * H], [[1.2] * H]], device=DEV)           # erank falls by > eps twice
    _, _, lg, lt = ctx.assign_budgets(ent, M=2, n_max=200, step=20, N=N, w=w, eps=0.4, delta_n=100)
    _, idx, ln, score = ctx.hidden_evict(q.to(DEV), K.to(DEV), G, lt[2:3], w, None, cap=N, want_score=True)
    torch.cuda.synchronize()
    assert lt.cpu().tolist() == [600, 500, 400] and int(ln[0]) == 400
    _, idx_ref, score_ref = O.hidden_evict(to_f64(q), to_f64(K), np.zeros((B, N, 1)), 400, w, G)
    check_index_sets(idx.cpu().numpy()[0], 400, idx_ref[0], 400, score_ref[0, : N - w], w)


def test_hidden_evict_full_size_llama3_8b_128k(ctx):
    """One layer of the 128K workload: 8 KV heads x 4 query heads over 131072 positions, hidden rows of
    4096 bf16; N - 512 rows survive (Eq. 10 with the paper's increment)."""
    cfg = synth.CONFIGS[3]
    K, V, Q = synth.gen_layers(cfg, 2410, [5], device=DEV)
    N, w, Dm = cfg.N, 8, 4096
    q = Q[0][:, :, -1, :].contiguous()                                                 # [B, Hq, D]: the last window query
    g = torch.Generator(device=DEV).manual_seed(3)
    Hs = torch.randn(cfg.B, N, Dm, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    n_keep = N - 512
    nk = torch.tensor([n_keep], dtype=torch.int32, device=DEV)
    Ho, idx, ln, score = ctx.hidden_evict(q, K[0], cfg.G, nk, w, Hs, cap=n_keep, want_score=True)
    torch.cuda.synchronize()
    score_ref = O.last_token_score(to_f64(q[0]), to_f64(K[0, 0]), cfg.G)
    np.testing.assert_allclose(score.cpu().numpy()[0], score_ref[: N - w], rtol=2e-5, atol=1e-12)
    sel_ref = O.select_indices(score_ref[: N - w], n_keep, N, w)
    check_index_sets(idx.cpu().numpy()[0], int(ln[0]), sel_ref, n_keep, score_ref[: N - w], w)
    pick = torch.from_numpy(np.linspace(0, n_keep - 1, 200).astype(np.int64)).to(DEV)
    assert torch.equal(Ho[0, pick].view(torch.int16), Hs[0, idx[0, pick].long()].view(torch.int16))
    assert torch.equal(Ho[0].view(torch.int16), Hs[0, idx[0, :n_keep].long()].view(torch.int16))


@pytest.mark.parametrize("N,w", [(40007, 4), (36872, 8), (75000, 1)])
def test_hidden_evict_long_rows_split_over_workgroups(ctx, N, w):
    """Rows of 32768 scores or more are selected by many workgroups per row.  The keys are drawn from 40
    distinct vectors, so thousands of scores are exactly equal and the threshold falls inside a run of
    ties: the kept positions must be those of the one-workgroup selection on the same scores (the earliest
    positions among equals), and agree with the oracle up to its tie band."""
    B, H, G = 2, 1, 2
    g = torch.Generator().manual_seed(N)
    pool = torch.randn(40, D, generator=g) * 1.2
    pick = torch.randint(0, 40, (B, H, N), generator=g)
    K = pool[pick].to(torch.float32)
    K[:, :, ::7] += 0.05 * torch.randn(B, H, (N + 6) // 7, D, generator=g)            # some distinct scores in between
    q = (torch.randn(B, H * G, D, generator=g) * 1.2).to(torch.float32)
    P = N - w
    for n_keep in (0, w, w + 1, 17, N // 3, N - 5000, N - 1, N, N + 3):
        nk = torch.tensor([n_keep], dtype=torch.int32, device=DEV)
        _, idx, ln, score = ctx.hidden_evict(q.to(DEV), K.to(DEV), G, nk, w, None, cap=N, want_score=True)
        bud = torch.full((B, 1), n_keep, dtype=torch.int32, device=DEV)
        _, _, idx_one, ln_one = ctx.select_gather(score.view(B, 1, P).contiguous(), bud, None, None, w, cap=N, N=N)
        torch.cuda.synchronize()
        assert torch.equal(ln.view(-1), ln_one.view(-1))
        assert torch.equal(idx.view(B, -1), idx_one.view(B, -1)), f"n_keep {n_keep}"
    _, idx_ref, score_ref = O.hidden_evict(to_f64(q), to_f64(K), np.zeros((B, N, 1)), N // 3, w, G)
    nk = torch.tensor([N // 3], dtype=torch.int32, device=DEV)
    _, idx, ln, _ = ctx.hidden_evict(q.to(DEV), K.to(DEV), G, nk, w, None, cap=N)
    torch.cuda.synchronize()
    for b in range(B):
        check_index_sets(idx.cpu().numpy()[b], int(ln[b]), idx_ref[b], N // 3, score_ref[b, :P], w)


def test_hidden_evict_argument_errors(ctx):
    from paper_2410_03090_amd import binding
    q, K, Hs = _inputs(1, 2, 2, 100, 64, torch.bfloat16, seed=1)
    nk = torch.tensor([10], dtype=torch.int32, device=DEV)
    with pytest.raises(binding.UncompError) as e:
        ctx.hidden_evict(q.to(DEV), K.to(DEV), 2, nk, 0, Hs.to(DEV), cap=50)           # w < 1
    assert e.value.status == binding.ERR_UNSUPPORTED
    with pytest.raises(binding.UncompError) as e:
        ctx.hidden_evict(q.to(DEV), K.to(DEV), 2, nk, 8, Hs.to(DEV), cap=4)            # cap < w
    assert e.value.status == binding.ERR_INVALID_ARG
    with pytest.raises(binding.UncompError) as e:
        ctx.hidden_evict(q.to(DEV), K.to(DEV), 2, nk, 2, Hs.to(DEV)[:, :, :60], cap=50)   # 120-byte rows
    assert e.value.status == binding.ERR_INVALID_ARG
    need = binding.Context.hidden_workspace_bytes(1, 2, 2, 100, 2)
    small = binding.Context(0, need - 512)
    with pytest.raises(binding.UncompError) as e:
        small.hidden_evict(q.to(DEV), K.to(DEV), 2, nk, 2, Hs.to(DEV), cap=50)
    assert e.value.status == binding.ERR_WORKSPACE
    small.close()
    exact = binding.Context(0, need)
    exact.hidden_evict(q.to(DEV), K.to(DEV), 2, nk, 2, Hs.to(DEV), cap=50)
    torch.cuda.synchronize()
    exact.close()
