"""GPU parity of the decode-time eviction calls against the float64 oracle.

Every step is checked from the GPU's own state before the step (the oracle is fed that
state, sorted by position), so rounding differences cannot pile up over steps; separate
tests let both sides run freely from the prefill result.  Tolerances: cumulative scores
and attention output 2e-5 relative to their scale (fp32 logits and exp, as for the
prefill score); evicted position exact unless the two candidates' oracle scores lie
within 1e-5 relative (a tie at fp32 resolution); cache rows bit-exact."""
import numpy as np
import pytest
import torch

from oracle import uncomp_oracle as O
from paper_2410_03090_amd import synth
from tests._util import raw_bits, to_f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D = 128


@pytest.fixture(scope="module")
def ctx():
    from paper_2410_03090_amd import binding
    c = binding.Context(0, 256 << 20)
    yield c
    c.close()


class State:
    """A decode state on the GPU plus a host snapshot helper."""

    def __init__(self, Kc, Vc, idx, cum, ln):
        self.Kc, self.Vc, self.idx, self.cum, self.ln = Kc, Vc, idx, cum, ln

    def host(self):
        return (self.Kc.cpu(), self.Vc.cpu(), self.idx.cpu().numpy(), self.cum.cpu().numpy().astype(np.float64),
                self.ln.cpu().numpy())


def _check_step(before, after, out, evicted, q, kn, vn, pos, budget, w, cap, heads=None):
    """before / after: host snapshots; q, kn, vn, pos, budget: host tensors / arrays of the step.
    Returns the number of near-tie disagreements (each verified to be inside the band)."""
    Kb, Vb, idxb, cumb, lnb = before
    Ka, Va, idxa, cuma, lna = after
    n_heads = lnb.shape[0]
    swaps = 0
    for h in (range(n_heads) if heads is None else heads):
        n = int(lnb[h])
        order = np.argsort(idxb[h, :n], kind="stable")
        b_eff = min(int(budget[h]), cap)
        args = (to_f64(Kb[h, :n])[order], to_f64(Vb[h, :n])[order], idxb[h, :n][order], cumb[h, :n][order],
                to_f64(q[h]), to_f64(kn[h]), to_f64(vn[h]), int(pos[h]))
        Kr, Vr, idxr, cumr, outr, evr = O.decode_step(*args, budget=b_eff, w=w)
        scale_v = max(1.0, float(np.abs(args[1]).max()) if n else 1.0)
        np.testing.assert_allclose(out[h], outr, rtol=0, atol=2e-5 * scale_v, err_msg=f"head {h}: attention output")
        n2 = int(lna[h])
        assert n2 == len(idxr), (h, n2, len(idxr))
        order2 = np.argsort(idxa[h, :n2], kind="stable")
        got_idx = idxa[h, :n2][order2]
        assert np.all(np.diff(got_idx) > 0), f"head {h}: duplicate positions"
        if int(evicted[h]) != evr:
            # both must be removable and tied at fp32 resolution in the oracle's own totals
            _, _, idx_all, cum_all, _, _ = O.decode_step(*args, budget=10 ** 9, w=w)
            tot = dict(zip(idx_all.tolist(), cum_all.tolist()))
            a, b = tot[int(evicted[h])], tot[evr]
            assert int(evicted[h]) <= int(pos[h]) - w
            assert abs(a - b) <= 1e-5 * max(abs(a), abs(b)), (h, evicted[h], evr, a, b)
            swaps += 1
            continue
        assert np.array_equal(got_idx, idxr), f"head {h}: kept positions"
        np.testing.assert_allclose(cuma[h, :n2][order2], cumr, rtol=2e-5, atol=2e-6, err_msg=f"head {h}: cum")
        assert np.array_equal(to_f64(Ka[h, :n2])[order2], Kr), f"head {h}: K rows"
        assert np.array_equal(to_f64(Va[h, :n2])[order2], Vr), f"head {h}: V rows"
    return swaps


def _random_state(n_heads, cap, lens, pos0, dtype, seed, w):
    g = torch.Generator().manual_seed(seed)
    Kc = torch.randn(n_heads, cap, D, generator=g).to(dtype)
    Vc = torch.randn(n_heads, cap, D, generator=g).to(dtype)
    idx = torch.full((n_heads, cap), -1, dtype=torch.int32)
    cum = torch.zeros(n_heads, cap)
    for h, n in enumerate(lens):
        # the most recent min(n, w-1) positions plus older ones picked at random, in shuffled slot order
        recent = list(range(pos0[h] - min(n, w - 1), pos0[h]))
        older = torch.randperm(pos0[h] - len(recent), generator=g)[: n - len(recent)].tolist()
        allp = torch.tensor(recent + older, dtype=torch.int32)
        idx[h, :n] = allp[torch.randperm(n, generator=g)] if n else allp
        cum[h, :n] = torch.rand(n, generator=g) * 3
    ln = torch.tensor(lens, dtype=torch.int32)
    return State(Kc.to(DEV), Vc.to(DEV), idx.to(DEV), cum.to(DEV), ln.to(DEV))


@pytest.mark.parametrize("dtype,plain_alu", [(torch.bfloat16, False), (torch.bfloat16, True), (torch.float32, False)])
@pytest.mark.parametrize("G", [1, 4, 7, 16])
def test_decode_step_matches_oracle_every_step(ctx, dtype, plain_alu, G):
    """bf16 through the two-kernel MFMA path and through the one-kernel path, fp32 through the latter.
    cap = 300 spans three 128-row wave parts with a ragged last one."""
    cap, w, steps = 300, 8, 28
    lens = [0, 5, 127, 128, 299, 300, 200]
    budgets = [300, 3, 127, 300, 300, 500, 150]   # below w, equal to len, above cap, below len
    ctx.set_kernel_path(plain_alu)
    try:
        n_heads = len(lens)
        pos0 = [500 + 10 * h for h in range(n_heads)]
        st = _random_state(n_heads, cap, lens, pos0, dtype, seed=100 + G, w=w)
        budget = torch.tensor(budgets, dtype=torch.int32)
        g = torch.Generator().manual_seed(7 * G + (1 if dtype == torch.float32 else 0))
        swaps = 0
        for t in range(steps):
            q = (torch.randn(n_heads, G, D, generator=g) * 2.5).to(dtype)
            kn = torch.randn(n_heads, D, generator=g).to(dtype)
            vn = torch.randn(n_heads, D, generator=g).to(dtype)
            pos = torch.tensor([p + t for p in pos0], dtype=torch.int32)
            before = st.host()
            out, ev = ctx.decode_step(q.to(DEV), kn.to(DEV), vn.to(DEV), pos.to(DEV), budget.to(DEV), w,
                                      st.Kc, st.Vc, st.idx, st.cum, st.ln)
            torch.cuda.synchronize()
            swaps += _check_step(before, st.host(), out.cpu().numpy(), ev.cpu().numpy(), q, kn, vn, pos.numpy(),
                                 budget.numpy(), w, cap)
    finally:
        ctx.set_kernel_path(False)
    assert swaps <= 2
    # occupancy: never above max(start, clamp(budget)); heads with room grew by one per step
    ln = st.ln.cpu().numpy()
    for h in range(n_heads):
        b = min(max(budgets[h], w), cap)
        assert ln[h] == (min(lens[h] + steps, b) if lens[h] < b else lens[h])


def test_decode_init_matches_oracle(ctx):
    n_heads, N, w, cap = 7, 300, 16, 64
    g = torch.Generator().manual_seed(3)
    score = torch.rand(n_heads, N - w, generator=g)
    budget = torch.randint(10, 80, (n_heads,), generator=g, dtype=torch.int32)
    _, _, idx, ln = ctx.select_gather(score.view(1, n_heads, -1).to(DEV), budget.view(1, n_heads).to(DEV), None, None,
                                      w=w, cap=cap, N=N)
    cum = ctx.decode_init(score.to(DEV), idx, ln, N, w)
    torch.cuda.synchronize()
    idx, ln, cum = idx.cpu().numpy()[0], ln.cpu().numpy()[0], cum.cpu().numpy()[0]
    for h in range(n_heads):
        ref = O.decode_init(score[h].numpy().astype(np.float64), idx[h, : ln[h]], N, w)
        assert np.array_equal(cum[h, : ln[h]].astype(np.float64), ref)          # a gather: exact
        assert np.all(cum[h, ln[h]:] == 0)
        assert np.all(cum[h, ln[h] - w: ln[h]] == 0)                           # the window rows


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prefill_then_decode_free_running(ctx, dtype):
    """Prefill calls, decode_init, then both sides run 40 tokens on their own state."""
    cfg = synth.tiny_config(dtype=dtype, H=4, G=4, N=700, w=16, avg_budget=96, M=4)
    T = 40
    K, V, Q = synth.gen_all(cfg, seed0=77)
    Kd, Vd, Qd = K[0].to(DEV), V[0].to(DEV), Q[0].to(DEV)
    score = ctx.window_score(Qd, Kd, G=cfg.G, pool=cfg.pool)
    ent = ctx.head_entropy(Kd.reshape(-1, cfg.N, D), k_trunc=cfg.k_trunc).reshape(1, cfg.B, cfg.H)
    budget = ctx.assign_budgets(ent, cfg.M, cfg.n_max, cfg.step, cfg.N, cfg.w)[0][0]
    Kc, Vc, idx, ln = ctx.select_gather(score, budget, Kd, Vd, w=cfg.w, cap=cfg.cap)
    n_heads = cfg.B * cfg.H
    cum = ctx.decode_init(score, idx, ln, cfg.N, cfg.w)
    torch.cuda.synchronize()
    # the oracle starts from the GPU's prefill result (prefill parity is tested elsewhere)
    score_h = score.cpu().numpy().astype(np.float64).reshape(n_heads, -1)
    idx_h, ln_h, bud_h = idx.cpu().numpy().reshape(n_heads, -1), ln.cpu().numpy().reshape(-1), budget.cpu().numpy().reshape(-1)
    ref = []
    for h in range(n_heads):
        sel = idx_h[h, : ln_h[h]]
        ref.append([to_f64(K[0, 0, h])[sel], to_f64(V[0, 0, h])[sel], sel.copy(), O.decode_init(score_h[h], sel, cfg.N, cfg.w)])
    toks = [synth.gen_decode_tokens(cfg, 77, 0, 0, h, T) for h in range(n_heads)]
    kn_all = torch.stack([t[0] for t in toks], 1)          # [T, heads, D]
    vn_all = torch.stack([t[1] for t in toks], 1)
    q_all = torch.stack([t[2] for t in toks], 1)           # [T, heads, G, D]
    st = State(Kc.view(n_heads, cfg.cap, D), Vc.view(n_heads, cfg.cap, D), idx.view(n_heads, -1),
               cum.view(n_heads, -1), ln.view(-1))
    bud_d = budget.reshape(-1).contiguous()
    alive = [True] * n_heads
    for t in range(T):
        pos = torch.full((n_heads,), cfg.N + t, dtype=torch.int32)
        out, ev = ctx.decode_step(q_all[t].to(DEV), kn_all[t].to(DEV), vn_all[t].to(DEV), pos.to(DEV), bud_d, cfg.w,
                                  st.Kc, st.Vc, st.idx, st.cum, st.ln)
        torch.cuda.synchronize()
        out, ev = out.cpu().numpy(), ev.cpu().numpy()
        for h in range(n_heads):
            if not alive[h]:
                continue
            r = ref[h]
            r[0], r[1], r[2], r[3], outr, evr = O.decode_step(r[0], r[1], r[2], r[3], to_f64(q_all[t, h]), to_f64(kn_all[t, h]),
                                                              to_f64(vn_all[t, h]), cfg.N + t, min(int(bud_h[h]), cfg.cap), cfg.w)
            if ev[h] != evr:
                alive[h] = False          # a tie at fp32 resolution sends the two runs apart; checked per step elsewhere
                continue
            np.testing.assert_allclose(out[h], outr, rtol=0, atol=1e-4)
    assert sum(alive) >= n_heads - 1
    _, _, idxa, cuma, lna = st.host()
    for h in range(n_heads):
        if alive[h]:
            order = np.argsort(idxa[h, : lna[h]])
            assert np.array_equal(idxa[h, : lna[h]][order], ref[h][2])
            np.testing.assert_allclose(cuma[h, : lna[h]][order], ref[h][3], rtol=1e-4, atol=1e-5)


def test_decode_state_that_cannot_evict(ctx):
    """Positions in the cache lie in the future of `pos`: nothing is old enough to leave."""
    dtype, G, w = torch.bfloat16, 2, 4
    for cap, n, want_len, want_ev in ((8, 8, 8, -2), (16, 6, 7, -1)):
        st = _random_state(1, cap, [n], [100], dtype, seed=cap, w=w)
        st.idx[0, :n] = torch.arange(200, 200 + n, dtype=torch.int32, device=DEV)
        before = st.host()
        g = torch.Generator().manual_seed(cap)
        q = torch.randn(1, G, D, generator=g).to(dtype).to(DEV)
        kn = torch.randn(1, D, generator=g).to(dtype).to(DEV)
        vn = torch.randn(1, D, generator=g).to(dtype).to(DEV)
        out, ev = ctx.decode_step(q, kn, vn, torch.tensor([100], dtype=torch.int32, device=DEV),
                                  torch.tensor([4], dtype=torch.int32, device=DEV), w, st.Kc, st.Vc, st.idx, st.cum, st.ln)
        torch.cuda.synchronize()
        after = st.host()
        assert int(after[4][0]) == want_len and int(ev[0]) == want_ev
        assert np.array_equal(raw_bits(after[0][0, :n]), raw_bits(before[0][0, :n]))      # old rows untouched
        if want_ev == -1:
            assert int(after[2][0, n]) == 100
            assert np.array_equal(raw_bits(after[0][0, n]), raw_bits(kn[0]))
            assert np.array_equal(raw_bits(after[1][0, n]), raw_bits(vn[0]))


def test_decode_argument_errors(ctx):
    from paper_2410_03090_amd import binding
    n_heads, G, cap, w = 2, 4, 32, 8
    st = _random_state(n_heads, cap, [10, 12], [50, 50], torch.bfloat16, seed=1, w=w)
    q = torch.zeros(n_heads, G, D, dtype=torch.bfloat16, device=DEV)
    kn = torch.zeros(n_heads, D, dtype=torch.bfloat16, device=DEV)
    pos = torch.full((n_heads,), 50, dtype=torch.int32, device=DEV)
    bud = torch.full((n_heads,), 16, dtype=torch.int32, device=DEV)
    before = st.host()
    with pytest.raises(binding.UncompError) as e:
        ctx.decode_step(q, kn, kn, pos, bud, 0, st.Kc, st.Vc, st.idx, st.cum, st.ln)          # w < 1
    assert e.value.status == binding.ERR_INVALID_ARG
    with pytest.raises(binding.UncompError) as e:
        ctx.decode_step(q, kn, kn, pos, bud, cap + 1, st.Kc, st.Vc, st.idx, st.cum, st.ln)    # w > cap
    assert e.value.status == binding.ERR_INVALID_ARG
    q17 = torch.zeros(n_heads, 17, D, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.UncompError) as e:
        ctx.decode_step(q17, kn, kn, pos, bud, w, st.Kc, st.Vc, st.idx, st.cum, st.ln)        # G > 16
    assert e.value.status == binding.ERR_UNSUPPORTED
    lib = ctx.lib
    st_code = lib.uncomp_decode_step(ctx.handle, q.data_ptr(), kn.data_ptr(), kn.data_ptr(), binding.BF16, n_heads, G, 64,
                                     pos.data_ptr(), bud.data_ptr(), w, cap, st.Kc.data_ptr(), st.Vc.data_ptr(),
                                     st.idx.data_ptr(), st.cum.data_ptr(), st.ln.data_ptr(), None, None, None)
    assert st_code == binding.ERR_UNSUPPORTED                                                   # D != 128
    st_code = lib.uncomp_decode_step(ctx.handle, q.data_ptr(), kn.data_ptr(), kn.data_ptr(), binding.F32, n_heads, G, D,
                                     pos.data_ptr(), bud.data_ptr(), w, 20000, st.Kc.data_ptr(), st.Vc.data_ptr(),
                                     st.idx.data_ptr(), st.cum.data_ptr(), st.ln.data_ptr(), None, None, None)
    assert st_code == binding.ERR_UNSUPPORTED                                 # fp32: probability table too large for LDS
    small = binding.Context(0, 1 << 20)
    st_code = lib.uncomp_decode_step(small.handle, q.data_ptr(), kn.data_ptr(), kn.data_ptr(), binding.BF16, 4096, G, D,
                                     pos.data_ptr(), bud.data_ptr(), w, 4096, st.Kc.data_ptr(), st.Vc.data_ptr(),
                                     st.idx.data_ptr(), st.cum.data_ptr(), st.ln.data_ptr(), None, None, None)
    assert st_code == binding.ERR_WORKSPACE                                   # bf16: partial results do not fit
    assert binding.Context.decode_workspace_bytes(4096, G, 4096) > (1 << 20)
    small.close()
    st_code = lib.uncomp_decode_step(ctx.handle, None, kn.data_ptr(), kn.data_ptr(), binding.BF16, n_heads, G, D,
                                     pos.data_ptr(), bud.data_ptr(), w, cap, st.Kc.data_ptr(), st.Vc.data_ptr(),
                                     st.idx.data_ptr(), st.cum.data_ptr(), st.ln.data_ptr(), None, None, None)
    assert st_code == binding.ERR_INVALID_ARG
    torch.cuda.synchronize()
    after = st.host()
    for a, b in zip(before, after):
        assert np.array_equal(raw_bits(a) if isinstance(a, torch.Tensor) else a, raw_bits(b) if isinstance(b, torch.Tensor) else b)


def test_decode_without_output_buffers(ctx):
    """out == NULL and evicted == NULL: the state update is the same."""
    dtype, G, cap, w = torch.bfloat16, 4, 64, 8
    sa = _random_state(3, cap, [64, 30, 64], [300, 300, 300], dtype, seed=9, w=w)
    sb = _random_state(3, cap, [64, 30, 64], [300, 300, 300], dtype, seed=9, w=w)
    g = torch.Generator().manual_seed(2)
    q = (torch.randn(3, G, D, generator=g) * 2).to(dtype).to(DEV)
    kn = torch.randn(3, D, generator=g).to(dtype).to(DEV)
    vn = torch.randn(3, D, generator=g).to(dtype).to(DEV)
    pos = torch.full((3,), 300, dtype=torch.int32, device=DEV)
    bud = torch.tensor([64, 64, 32], dtype=torch.int32, device=DEV)
    ctx.decode_step(q, kn, vn, pos, bud, w, sa.Kc, sa.Vc, sa.idx, sa.cum, sa.ln)
    from paper_2410_03090_amd import binding
    code = ctx.lib.uncomp_decode_step(ctx.handle, q.data_ptr(), kn.data_ptr(), vn.data_ptr(), binding.BF16, 3, G, D,
                                      pos.data_ptr(), bud.data_ptr(), w, cap, sb.Kc.data_ptr(), sb.Vc.data_ptr(),
                                      sb.idx.data_ptr(), sb.cum.data_ptr(), sb.ln.data_ptr(), None, None,
                                      torch.cuda.current_stream().cuda_stream)
    assert code == 0
    torch.cuda.synchronize()
    for a, b in zip(sa.host(), sb.host()):
        assert np.array_equal(raw_bits(a) if isinstance(a, torch.Tensor) else a, raw_bits(b) if isinstance(b, torch.Tensor) else b)


def test_decode_steps_replayed_from_a_hip_graph(ctx):
    """Four decode steps captured in a HIP graph (the calls only enqueue kernels: no allocation, no
    memset, no synchronisation) give, on every replay, exactly the state and outputs of the eager calls.
    Replays alternate with eager work and synchronisations."""
    dtype, G, cap, w, n_heads, T = torch.bfloat16, 4, 300, 8, 12, 4
    lens = [300, 299, 150, 0, 300, 257, 256, 255, 40, 300, 7, 128]
    g = torch.Generator().manual_seed(5)
    q = (torch.randn(T, n_heads, G, D, generator=g) * 2).to(dtype).to(DEV)
    kn = torch.randn(T, n_heads, D, generator=g).to(dtype).to(DEV)
    vn = torch.randn(T, n_heads, D, generator=g).to(dtype).to(DEV)
    pos = [torch.full((n_heads,), 600 + t, dtype=torch.int32, device=DEV) for t in range(T)]
    bud = torch.randint(w, cap + 20, (n_heads,), generator=g, dtype=torch.int32).to(DEV)
    start = _random_state(n_heads, cap, lens, [600] * n_heads, dtype, seed=8, w=w)
    init = [t.clone() for t in (start.Kc, start.Vc, start.idx, start.cum, start.ln)]
    outs = [torch.empty(n_heads, G, D, device=DEV) for _ in range(T)]
    evs = [torch.empty(n_heads, dtype=torch.int32, device=DEV) for _ in range(T)]

    def reset():
        for dst, src in zip((start.Kc, start.Vc, start.idx, start.cum, start.ln), init):
            dst.copy_(src)

    def run_steps():
        for t in range(T):
            ctx.decode_step(q[t], kn[t], vn[t], pos[t], bud, w, start.Kc, start.Vc, start.idx, start.cum, start.ln,
                            out=outs[t], evicted=evs[t])

    run_steps()                                                   # eager reference (also warms everything up)
    torch.cuda.synchronize()
    want = [t.clone() for t in (start.Kc, start.Vc, start.idx, start.cum, start.ln)] + [o.clone() for o in outs] + \
           [e.clone() for e in evs]
    reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run_steps()
    torch.cuda.synchronize()
    for replay in range(3):
        reset()
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [start.Kc, start.Vc, start.idx, start.cum, start.ln] + outs + evs
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"replay {replay}"
        # eager work between the replays
        reset()
        run_steps()
        torch.cuda.synchronize()


def test_decode_many_heads(ctx):
    """1024 heads with 8 query heads each: enough waves for the 256-rows-per-wave variant (two parts
    per head, the second ragged).  Sampled heads against the oracle."""
    n_heads, G, cap, w = 1024, 8, 300, 8
    g = torch.Generator(device=DEV).manual_seed(21)
    Kc = torch.randn(n_heads, cap, D, generator=g, device=DEV).to(torch.bfloat16)
    Vc = torch.randn(n_heads, cap, D, generator=g, device=DEV).to(torch.bfloat16)
    ln = torch.randint(0, cap + 1, (n_heads,), generator=g, device=DEV).to(torch.int32)
    ln[:4] = torch.tensor([0, 255, 256, 300], dtype=torch.int32, device=DEV)
    budget = torch.randint(w, cap + 40, (n_heads,), generator=g, device=DEV).to(torch.int32)
    idx = torch.argsort(torch.rand(n_heads, 1000, generator=g, device=DEV), dim=1)[:, :cap].to(torch.int32).contiguous()
    cum = torch.rand(n_heads, cap, generator=g, device=DEV) * 2
    st = State(Kc, Vc, idx, cum, ln)
    sample = [0, 1, 2, 3, 500, 1023]
    for t in range(3):
        q = (torch.randn(n_heads, G, D, generator=g, device=DEV) * 2).to(torch.bfloat16)
        kn = torch.randn(n_heads, D, generator=g, device=DEV).to(torch.bfloat16)
        vn = torch.randn(n_heads, D, generator=g, device=DEV).to(torch.bfloat16)
        pos = torch.full((n_heads,), 1000 + t, dtype=torch.int32, device=DEV)
        before = st.host()
        out, ev = ctx.decode_step(q, kn, vn, pos, budget, w, st.Kc, st.Vc, st.idx, st.cum, st.ln)
        torch.cuda.synchronize()
        after = st.host()
        _check_step(before, after, out.cpu().numpy(), ev.cpu().numpy(), q.cpu(), kn.cpu(), vn.cpu(), pos.cpu().numpy(),
                    budget.cpu().numpy(), w, cap, heads=sample)
        b = np.clip(budget.cpu().numpy(), w, cap)
        assert np.all(after[4] == np.where(before[4] + 1 > b, before[4], before[4] + 1))
        assert np.isfinite(out.cpu().numpy()).all() and np.isfinite(after[3]).all()


def test_decode_full_size_llama3_8b_128k(ctx):
    """All 256 KV heads of the 128K workload's compacted cache (budgets 858..3238 rows, the
    configuration's arithmetic progression), 4 query heads each: sampled heads against
    the oracle, whole-state properties for every head."""
    cfg = synth.CONFIGS[3]
    n_heads, G, cap, w = cfg.L * cfg.B * cfg.H, cfg.G, cfg.cap, cfg.w
    g = torch.Generator(device=DEV).manual_seed(11)
    grp = torch.arange(n_heads, device=DEV) % cfg.M
    budget = (cfg.n_max - grp * cfg.step).to(torch.int32)
    ln0 = budget.clone()
    ln0[::5] -= 3                                           # some heads still have room
    Kc = torch.randn(n_heads, cap, D, generator=g, device=DEV).to(torch.bfloat16)
    Vc = torch.randn(n_heads, cap, D, generator=g, device=DEV).to(torch.bfloat16)
    N = cfg.N
    idx = torch.empty(n_heads, cap, dtype=torch.int32, device=DEV)
    for h in range(n_heads):
        n = int(ln0[h])
        older = torch.randperm(N - w, generator=g, device=DEV)[: n - w].sort().values
        idx[h, :n] = torch.cat([older, torch.arange(N - w, N, device=DEV)]).to(torch.int32)
        idx[h, n:] = -1
    cum = torch.rand(n_heads, cap, generator=g, device=DEV) * 2
    st = State(Kc, Vc, idx, cum, ln0.clone())
    sample = [0, 7, 100, 255]
    for t in range(3):
        q = (torch.randn(n_heads, G, D, generator=g, device=DEV) * 2).to(torch.bfloat16)
        kn = torch.randn(n_heads, D, generator=g, device=DEV).to(torch.bfloat16)
        vn = torch.randn(n_heads, D, generator=g, device=DEV).to(torch.bfloat16)
        pos = torch.full((n_heads,), N + t, dtype=torch.int32, device=DEV)
        before = st.host()
        out, ev = ctx.decode_step(q, kn, vn, pos, budget, w, st.Kc, st.Vc, st.idx, st.cum, st.ln)
        torch.cuda.synchronize()
        after = st.host()
        _check_step(before, after, out.cpu().numpy(), ev.cpu().numpy(), q.cpu(), kn.cpu(), vn.cpu(), pos.cpu().numpy(),
                    budget.cpu().numpy(), w, cap, heads=sample)
        lnb, lna, evh = before[4], after[4], ev.cpu().numpy()
        bud = budget.cpu().numpy()
        assert np.all(lna == np.minimum(lnb + 1, bud))
        assert np.all((evh >= 0) == (lnb + 1 > bud))
        assert np.all(evh[evh >= 0] <= N + t - w)
        # every query head hands out one unit of attention
        gain = np.array([after[3][h, : lna[h]].sum() - before[3][h, : lnb[h]].sum() for h in range(n_heads)])
        lost = np.array([before[3][h, : lnb[h]][before[2][h, : lnb[h]] == evh[h]].sum() for h in range(n_heads)])
        # (the entry that left takes its own share of this step with it, hence the one-sided slack)
        assert np.all(gain + lost <= G + 1e-3) and np.all(gain + lost >= G - 0.25)
        assert np.isfinite(out.cpu().numpy()).all()
