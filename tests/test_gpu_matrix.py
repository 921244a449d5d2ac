"""GPU parity of uncomp_matrix_entropy (the entropy of Sec. 3.1-3.2 for wide token matrices, by
subspace iteration) against the float64 oracle (full eigendecomposition).  Entropy 1e-4 relative
after 8 rounds on spectra that fall off before the 129th eigenvalue; the leading Ritz values to
2e-5 of the trace."""
import math

import numpy as np
import pytest
import torch

from oracle import uncomp_oracle as O
from tests._util import to_f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    from paper_2410_03090_amd import binding
    c = binding.Context(0, 1 << 30)
    yield c
    c.close()


def _lowrank(n_mat, N, D, r, dtype, seed, offset=0.0):
    g = torch.Generator().manual_seed(seed)
    U = torch.randn(n_mat, N, r, generator=g) / math.sqrt(r)
    V = torch.randn(n_mat, D, r, generator=g) / math.sqrt(r)
    X = U @ V.transpose(1, 2) + 0.1 * math.sqrt(128.0 / D) * torch.randn(n_mat, N, D, generator=g) + offset
    return X.to(dtype)


def _powerlaw(n_mat, N, D, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    Qm, _ = torch.linalg.qr(torch.randn(D, D, generator=g, dtype=torch.float64))
    scale = torch.arange(1, D + 1, dtype=torch.float64) ** -0.75
    X = (torch.randn(n_mat, N, D, generator=g, dtype=torch.float64) * scale) @ Qm.T
    return X.float().to(dtype)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N,D,r", [(300, 256, 40), (2000, 1024, 64), (777, 512, 100)])
def test_matrix_entropy_lowrank(ctx, dtype, N, D, r):
    X = _lowrank(2, N, D, r, dtype, seed=N + D, offset=0.25)
    for flags in (O.DEFAULT_FLAGS, O.FLAG_CENTER, O.FLAG_TRUNC_RENORM, 0):
        for k in (8, 32):            # the paper's k = 32 leaves the block 96 spare directions; k near 128 has none
            H, eig = ctx.matrix_entropy(X.to(DEV), k_trunc=k, flags=flags, n_iter=8, want_eig=True)
            torch.cuda.synchronize()
            Href, eref = O.head_entropy(to_f64(X), k_trunc=k, flags=flags)
            np.testing.assert_allclose(H.cpu().numpy(), Href, rtol=1e-4)
            np.testing.assert_allclose(eig.cpu().numpy()[:, :k], eref[:, :k], rtol=0, atol=2e-5)


def test_matrix_entropy_rounds_close_a_flat_stretch(ctx):
    """24 strong directions over a flat noise floor: the top 32 reach into the flat part, where the
    rounds gain slowly; the error falls with the number of rounds."""
    X = _lowrank(1, 300, 256, 24, torch.bfloat16, seed=556)
    Href, _ = O.head_entropy(to_f64(X), k_trunc=32)
    err = []
    for n_iter in (2, 8, 32):
        H = ctx.matrix_entropy(X.to(DEV), k_trunc=32, n_iter=n_iter)
        err.append(abs(float(H[0]) / Href[0] - 1))
    assert err[0] > err[1] > err[2] or err[2] < 1e-6
    assert err[1] < 1e-3 and err[2] < 2e-5


def test_matrix_entropy_powerlaw_and_strided(ctx):
    N, D = 1500, 1024
    X = _powerlaw(1, N, D, torch.bfloat16, seed=3)
    pad = torch.zeros(1, N, D + 64, dtype=torch.bfloat16)
    pad[:, :, :D] = X
    H = ctx.matrix_entropy(pad.to(DEV)[:, :, :D], k_trunc=32, n_iter=8)
    Href, _ = O.head_entropy(to_f64(X), k_trunc=32)
    np.testing.assert_allclose(H.cpu().numpy(), Href, rtol=1e-4)
    # more rounds do not move a converged value
    H16 = ctx.matrix_entropy(X.to(DEV), k_trunc=32, n_iter=16)
    np.testing.assert_allclose(H16.cpu().numpy(), H.cpu().numpy(), rtol=2e-5)


def test_matrix_entropy_isotropic_bound_and_degenerate(ctx):
    N, D = 4000, 512
    g = torch.Generator().manual_seed(11)
    iso = torch.randn(N, D, generator=g)
    const = torch.randn(1, D, generator=g).repeat(N, 1)
    u = 2.0 ** torch.randint(-2, 3, (N, 1), generator=g).float() * (torch.randint(0, 2, (N, 1), generator=g) * 2 - 1)
    rank1 = u @ torch.randint(1, 16, (1, D), generator=g).float()
    X = torch.stack([iso, const, rank1, torch.zeros(N, D)]).to(torch.bfloat16)
    H = ctx.matrix_entropy(X.to(DEV), k_trunc=32, n_iter=12).cpu().numpy()
    Href, _ = O.head_entropy(to_f64(X), k_trunc=32)
    assert abs(H[0] - Href[0]) < 2e-3 * Href[0] and H[0] <= math.log(32) + 1e-6      # flat spectrum: slow, still close to log k
    assert H[1] == 0.0 and H[3] == 0.0                                            # no spread
    assert abs(H[2]) < 1e-4 and abs(Href[2]) < 1e-9                               # rank one (Lemma 4)


def test_matrix_entropy_hidden_state_width(ctx):
    """D = 4096 (the model width of the 8B configurations), 4096 tokens, one matrix."""
    N, D = 4096, 4096
    X = _lowrank(1, N, D, 80, torch.bfloat16, seed=4096)
    H, eig = ctx.matrix_entropy(X.to(DEV), k_trunc=32, n_iter=8, want_eig=True)
    torch.cuda.synchronize()
    Href, eref = O.head_entropy(to_f64(X), k_trunc=32)
    np.testing.assert_allclose(H.cpu().numpy(), Href, rtol=1e-4)
    np.testing.assert_allclose(eig.cpu().numpy()[:, :32], eref[:, :32], rtol=0, atol=2e-5)


def test_matrix_entropy_maximum_width(ctx):
    """D = 16384, the widest matrix the call takes.  Only 384 columns, scattered over the width, are non-zero:
    the covariance is then the 384 x 384 covariance of those columns bordered by zeros, so the oracle on the
    columns alone gives the same eigenvalues, trace and entropy without a 16384 x 16384 eigendecomposition."""
    from paper_2410_03090_amd import binding
    N, D, live = 1500, 16384, 384
    g = torch.Generator().manual_seed(16384)
    cols = torch.randperm(D, generator=g)[:live].sort().values
    Xs = _lowrank(1, N, live, 48, torch.bfloat16, seed=77, offset=0.2)
    X = torch.zeros(1, N, D, dtype=torch.bfloat16)
    X[:, :, cols] = Xs
    wide = binding.Context(0, binding.Context.matrix_workspace_bytes(N, D) + (16 << 20))
    try:
        for flags in (O.DEFAULT_FLAGS, 0):
            H, eig = wide.matrix_entropy(X.to(DEV), k_trunc=32, flags=flags, n_iter=8, want_eig=True)
            torch.cuda.synchronize()
            Href, eref = O.head_entropy(to_f64(Xs), k_trunc=32, flags=flags)
            np.testing.assert_allclose(H.cpu().numpy(), Href, rtol=1e-4)
            np.testing.assert_allclose(eig.cpu().numpy()[:, :32], eref[:, :32], rtol=0, atol=2e-5)
    finally:
        wide.close()


def test_matrix_entropy_is_deterministic(ctx):
    """Fixed start block, fixed-order reductions, no atomics: two runs give the same bits."""
    X = _lowrank(2, 1500, 768, 50, torch.bfloat16, seed=12).to(DEV)
    a = ctx.matrix_entropy(X, k_trunc=32, n_iter=6, want_eig=True)
    b = ctx.matrix_entropy(X, k_trunc=32, n_iter=6, want_eig=True)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_matrix_entropy_argument_errors(ctx):
    from paper_2410_03090_amd import binding
    X = torch.zeros(1, 64, 256, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.UncompError) as e:
        ctx.matrix_entropy(X[:, :, :128].contiguous())                  # D = 128: the other call's job
    assert e.value.status == binding.ERR_UNSUPPORTED
    with pytest.raises(binding.UncompError) as e:
        ctx.matrix_entropy(X, k_trunc=129)
    assert e.value.status == binding.ERR_UNSUPPORTED
    with pytest.raises(binding.UncompError) as e:
        ctx.matrix_entropy(X, n_iter=0)
    assert e.value.status == binding.ERR_INVALID_ARG
    small = binding.Context(0, 1 << 20)
    with pytest.raises(binding.UncompError) as e:
        small.matrix_entropy(torch.zeros(1, 4096, 1024, dtype=torch.bfloat16, device=DEV))
    assert e.value.status == binding.ERR_WORKSPACE
    small.close()
