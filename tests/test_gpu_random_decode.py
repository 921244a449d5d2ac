"""Seeded sweep of random decode states and steps against the oracle (every step from the GPU's own state,
as in test_gpu_decode.py): head counts, query heads per KV head, capacities, windows, lengths and budgets
drawn at random, both cache dtypes."""
import numpy as np
import pytest
import torch

from tests.test_gpu_decode import DEV, D, _check_step, _random_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2410_03090_amd import binding
    c = binding.Context(0, 256 << 20)
    yield c
    c.close()


def _cases():
    rng = np.random.default_rng(1503)
    out = []
    for i in range(14):
        cap = int(rng.choice([17, 64, 129, 257, 500, 1030]))
        w = int(rng.integers(1, min(cap, 40) + 1))
        out.append((i, "bf16" if i % 4 else "f32", int(rng.integers(1, 9)), int(rng.integers(1, 17)), cap, w))
    return out


@pytest.mark.parametrize("case,dtype,n_heads,G,cap,w", _cases())
def test_random_decode(ctx, case, dtype, n_heads, G, cap, w):
    rng = np.random.default_rng(7000 + case)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    lens = [int(rng.integers(0, cap + 1)) for _ in range(n_heads)]
    pos0 = [int(cap + 50 + rng.integers(0, 100)) for _ in range(n_heads)]
    budget = torch.tensor([int(rng.integers(0, cap + 30)) for _ in range(n_heads)], dtype=torch.int32)
    st = _random_state(n_heads, cap, lens, pos0, tdt, seed=300 + case, w=w)
    g = torch.Generator().manual_seed(case)
    swaps = 0
    for t in range(6):
        q = (torch.randn(n_heads, G, D, generator=g) * 2.0).to(tdt)
        kn = torch.randn(n_heads, D, generator=g).to(tdt)
        vn = torch.randn(n_heads, D, generator=g).to(tdt)
        pos = torch.tensor([p + t for p in pos0], dtype=torch.int32)
        before = st.host()
        out, ev = ctx.decode_step(q.to(DEV), kn.to(DEV), vn.to(DEV), pos.to(DEV), budget.to(DEV), w,
                                  st.Kc, st.Vc, st.idx, st.cum, st.ln)
        torch.cuda.synchronize()
        swaps += _check_step(before, st.host(), out.cpu().numpy(), ev.cpu().numpy(), q, kn, vn, pos.numpy(),
                             budget.numpy(), w, cap)
    assert swaps <= 1
