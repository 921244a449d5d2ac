"""Benchmark of libuncomp's compression hot path on one MI355X.

One step = the four C-ABI calls (entropy -> budgets -> window score -> select+gather) over
ALL layers of one synthetic prefill, inputs resident in HBM.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

PROFILES = os.path.join(ROOT, "profiles")
CSRC = os.path.join(ROOT, "paper_2410_03090_amd", "csrc")


def kernel_sources_hash():
    """sha256 over the kernel sources, in name order: identifies the kernels a stored measurement belongs to."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch of each kernel from the stored rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of
    this workload (profiles/hbm_traffic_<workload>.txt: lines `traffic_bytes <kernel> <fetched> <written>`,
    already scaled by what the counters read for a plain copy of known size).  Returns ({kernel: bytes},
    commit, stale): stale is True when the kernel sources have changed since the counters were read, and
    then no figure is reported."""
    path = os.path.join(PROFILES, f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return {}, None, None
    table, commit, src_hash = {}, None, None
    with open(path) as f:
        for line in f:
            t = line.split()
            if len(t) == 4 and t[0] == "traffic_bytes":
                table[t[1]] = int(t[2]) + int(t[3])
            elif len(t) == 2 and t[0] == "measured_at_commit":
                commit = t[1]
            elif len(t) == 2 and t[0] == "kernel_sources_sha256":
                src_hash = t[1]
    stale = src_hash != kernel_sources_hash()
    return ({} if stale else table), commit, stale


def algorithmic_work(cfg, name):
    """(bytes, flops) one launch of kernel `name` must move / compute, over all L*B*H heads.
    Per (layer, batch, KV head): N tokens of D features at e bytes each."""
    e = 2 if cfg.dtype == "bf16" else 4
    heads = cfg.L * cfg.B * cfg.H
    N, D, w, G = cfg.N, cfg.D, cfg.w, cfg.G
    P = N - w
    R = G * w
    if name.startswith("gram"):
        return heads * N * D * e, heads * 2.0 * N * D * D
    if name.startswith("score_stats"):
        return heads * N * D * e, heads * 2.0 * R * D * N
    if name.startswith("score_vote"):
        return heads * (P * D * e + 4 * P), heads * 2.0 * R * D * P
    if name.startswith("score_pool"):
        return heads * (G * P * 4 + 4 * P), 0.0
    if name == "select":
        return heads * 4 * P, 0.0
    if name == "gather":
        return heads * 4 * cfg.avg_budget * D * e, 0.0
    return 0, 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 0-4 (default 3: the 128K-token prefill)")
    ap.add_argument("--seed", type=int, default=2410)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="run the eigen stage and the budgets on the context's side stream beside the scoring kernels")
    ap.add_argument("--no-overlap", action="store_true", help="(default) keep every kernel on one stream")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for HBM byte counters)")
    ap.add_argument("--cpu-heads", type=int, default=0, help="heads in the oracle sample (0 = auto)")
    ap.add_argument("--zero-keys", action="store_true",
                    help="all keys zero: same instructions, no switching activity in the matrix operands (shows what the "
                         "chip's clock management costs the kernels on live data); results are degenerate, timing only")
    ap.add_argument("--no-with-lse", action="store_true", help="skip the leg that hands the row normalisers to uncomp_window_score")
    ap.add_argument("--no-prepare", action="store_true", help="skip the offline-preparation leg")
    ap.add_argument("--no-matrix-entropy", action="store_true", help="skip the wide-matrix (hidden-state) entropy leg")
    ap.add_argument("--no-hidden-evict", action="store_true", help="skip the stage-1 hidden-state eviction leg")
    ap.add_argument("--decode-steps", type=int, default=64,
                    help="generated tokens to run through uncomp_decode_step after the timed prefill steps (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2410_03090_amd import binding, synth

    cfg = synth.CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t_gen = time.time()
    K, V, Q = synth.gen_all(cfg, args.seed, device=dev)
    if args.zero_keys:
        K.zero_()
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    L, B, H, N, D, G, w = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D, cfg.G, cfg.w
    LB = L * B
    Kf, Vf, Qf = K.reshape(LB, H, N, D), V.reshape(LB, H, N, D), Q.reshape(LB, H * G, w, D)

    ws = binding.Context.workspace_bytes(LB * H, N, D, LB, H, G, w)
    if args.decode_steps > 0:
        ws = max(ws, binding.Context.decode_workspace_bytes(LB * H, G, cfg.cap))
    if not args.no_hidden_evict:
        ws = max(ws, binding.Context.hidden_workspace_bytes(B, H, G, N, w))
    if not args.no_matrix_entropy:
        ws = max(ws, binding.Context.matrix_workspace_bytes(N, 4096))
    ctx = binding.Context(0, ws)
    ctx.set_overlap(args.overlap and not args.no_overlap)
    i32 = dict(dtype=torch.int32, device=dev)
    ent = torch.empty(L, B, H, dtype=torch.float32, device=dev)
    bud = (torch.empty(L, B, H, **i32), torch.empty(L, B, H, **i32), torch.empty(L, **i32), torch.empty(L, **i32))
    score = torch.empty(LB, H, N - w, dtype=torch.float32, device=dev)
    cap = cfg.cap
    outs = (torch.zeros(LB, H, cap, D, dtype=K.dtype, device=dev), torch.zeros(LB, H, cap, D, dtype=K.dtype, device=dev),
            torch.full((LB, H, cap), -1, **i32), torch.zeros(LB, H, **i32))

    def step():
        ctx.head_entropy(Kf.reshape(LB * H, N, D), k_trunc=cfg.k_trunc, entropy_out=ent.reshape(-1))
        ctx.assign_budgets(ent, cfg.M, cfg.n_max, cfg.step, N, w, 0.4, 512, out=bud)
        ctx.window_score(Qf, Kf, G, cfg.pool, out=score)
        ctx.select_gather(score, bud[0].reshape(LB, H), Kf, Vf, w, cap, out=outs)

    if args.calib_copy_mib:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    recs = ctx.profile_read()
    ctx.profile(False)

    ms_per_step = elapsed * 1e3 / args.steps
    value = B * N / (elapsed / args.steps)

    # per-kernel averages from the HIP events recorded inside the timed region
    per = {}
    for name, ms in recs:
        per.setdefault(name, []).append(ms)
    kernels = {}
    for name, v in per.items():
        avg = sum(v) / len(v)
        byt, flops = algorithmic_work(cfg, name)
        kernels[name] = {"ms": round(avg, 4), "launches": len(v),
                         "GBps": round(byt / avg / 1e6, 1) if byt else None,
                         "TFLOPs": round(flops / avg / 1e9, 1) if flops else None}
    # what this machine sustains: a plain streaming read and the bf16 MFMA loop (live and zero operands)
    peak_buf = Kf if Kf.numel() * Kf.element_size() >= (256 << 20) else torch.zeros(256 << 20, dtype=torch.uint8, device=Kf.device)
    read_peak, mfma_live, mfma_zero = ctx.measure_peaks(peak_buf)      # the keys, or 256 MiB of its own for a small workload
    peaks = {"stream_read_GBps": round(read_peak, 1), "mfma_bf16_loop_TFLOPs_live_operands": round(mfma_live, 1),
             "mfma_bf16_loop_TFLOPs_zero_operands": round(mfma_zero, 1),
             "note": "measured by uncomp_measure_peaks on this device; the data-sheet peaks are 8000 GB/s and 2500 TFLOP/s"}
    traffic, traffic_commit, traffic_stale = measured_traffic(cfg.name)
    for name, k in kernels.items():
        if k["GBps"]:
            k["hbm_frac"] = round(k["GBps"] / HBM_PEAK_GBS, 4)
            k["hbm_frac_of_measured"] = round(k["GBps"] / read_peak, 4)
        if k["TFLOPs"]:
            issued = 36.0 / 64.0 if name == "gram_mfma" else 1.0          # the Gram kernel computes 36 of 64 symmetric blocks
            k["mfma_frac_issued"] = round(k["TFLOPs"] * issued / MFMA_BF16_PEAK_TFLOPS, 4)
            k["mfma_frac_issued_of_measured"] = round(k["TFLOPs"] * issued / mfma_live, 4)
    dominant = max(kernels, key=lambda n: kernels[n]["ms"]) if kernels else None
    roofline = None
    if dominant is not None:
        byt, flops = algorithmic_work(cfg, dominant)
        avg_ms = kernels[dominant]["ms"]
        if byt:
            ach = byt / avg_ms / 1e6
            roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                        "traffic": traffic.get(dominant),
                        "traffic_measured_at_commit": traffic_commit, "traffic_stale": traffic_stale,
                        "algorithmic_bytes": int(byt),
                        "peak_measured": round(read_peak, 1), "frac_of_measured": round(ach / read_peak, 4),
                        "mfma_TFLOPs": round(flops / avg_ms / 1e9, 1) if flops else None,
                        "mfma_frac": round(flops / avg_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4) if flops else None,
                        "mfma_frac_of_measured": round(flops / avg_ms / 1e9 / mfma_live, 4) if flops else None}
        else:
            roofline = {"kernel": dominant, "bound": "alu", "achieved": None, "peak": None, "unit": "TFLOP/s",
                        "frac": None, "traffic": None}

    with_lse = None if args.no_with_lse else with_lse_leg(cfg, ctx, Kf, Vf, Qf, ent, bud, score, outs, args)
    gram_resident = gram_resident_leg(cfg, ctx, Kf) if cfg.dtype == "bf16" else None
    decode = decode_leg(cfg, ctx, score, bud[0], outs, args) if args.decode_steps > 0 else None
    hidden = None if args.no_hidden_evict else hidden_leg(cfg, ctx, K, Q, args)
    prepare = None if args.no_prepare else prepare_leg(cfg, ctx, Kf, ent, args)
    matrix = None if args.no_matrix_entropy else matrix_leg(cfg, ctx, args)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, K, V, Q, args)

    kept = float(outs[3].float().mean().item())
    out = {
        "metric": "kv_tokens_compressed_per_sec", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic" if not args.zero_keys else "all-zero keys (timing experiment, not a result)",
        "config": {"workload": cfg.name, "layers": L, "batch": B, "kv_heads": H, "q_per_kv": G, "seq_len": N,
                   "head_dim": D, "window": w, "pool": cfg.pool, "k_trunc": cfg.k_trunc,
                   "avg_budget": cfg.avg_budget, "mean_kept": round(kept, 1), "rho": round(kept / N, 5),
                   "head_tokens_per_s": round(value * L * H, 1)},
        "roofline": roofline, "cpu_baseline": cpu, "peaks": peaks, "kernels": kernels, "with_lse": with_lse, "gram_cache_resident": gram_resident, "decode": decode, "hidden_evict": hidden, "prepare": prepare, "matrix_entropy": matrix,
        "gen_seconds": round(t_gen, 1),
    }
    print(json.dumps(out))


def with_lse_leg(cfg, ctx, Kf, Vf, Qf, ent, bud, score, outs, args):
    """Not part of `value`: the same step when the caller hands uncomp_window_score the row normalisers its
    attention kernel already has (lse_opt), so the library's statistics pass over the keys is skipped.  The
    normalisers are formed here once, outside the timed region, with library fp32 matrix products (they stand
    in for the model's attention kernel)."""
    import math

    import torch
    L, B, H, N, D, G, w = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D, cfg.G, cfg.w
    LB, P = L * B, N - w
    lse = torch.empty(LB, H * G, w, dtype=torch.float32, device=Kf.device)
    causal = torch.arange(N, device=Kf.device)[None, :] > (P + torch.arange(w, device=Kf.device))[:, None]      # [w, N]
    for lb in range(LB):
        for h in range(H):
            q = Qf[lb, h * G:(h + 1) * G].reshape(G * w, D).float()
            logits = (q @ Kf[lb, h].float().T) * (1.0 / math.sqrt(D))
            logits.view(G, w, N).masked_fill_(causal[None], float("-inf"))
            lse[lb, h * G:(h + 1) * G] = torch.logsumexp(logits, dim=1).view(G, w)
    del logits

    def step():
        ctx.head_entropy(Kf.reshape(LB * H, N, D), k_trunc=cfg.k_trunc, entropy_out=ent.reshape(-1))
        ctx.assign_budgets(ent, cfg.M, cfg.n_max, cfg.step, N, w, 0.4, 512, out=bud)
        ctx.window_score(Qf, Kf, G, cfg.pool, out=score, lse=lse)
        ctx.select_gather(score, bud[0].reshape(LB, H), Kf, Vf, w, cfg.cap, out=outs)

    ref = score.clone()
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    dev = float(((score - ref).abs() / ref.abs().clamp_min(1e-30)).max().item())
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    return {"ms_per_step": round(dt * 1e3, 4), "tokens_per_s": round(B * N / dt, 1),
            "max_rel_dev_of_score_from_the_full_step": float(f"{dev:.3e}"),
            "note": "uncomp_window_score given lse_opt: no statistics pass; not the headline"}


def gram_resident_leg(cfg, ctx, Kf):
    """The Gram kernel with its input resident in cache: the same launch shape as the timed step, but every
    matrix is the same 8192 tokens of one head (2 MiB, stride 0 between matrices), so HBM delivers
    almost nothing and the MFMA rate shows what the kernel does when memory is out of the way.  The streamed
    figure is the `gram_mfma` entry of `kernels`."""
    import torch
    L, B, H, N, D = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D
    n_tok = min(N, 8192)
    n_mat = L * B * H * (N // n_tok)                             # same number of tokens as the real step
    X = Kf[0, 0, :n_tok].unsqueeze(0).expand(n_mat, n_tok, D)
    ent = torch.empty(n_mat, dtype=torch.float32, device=Kf.device)
    ctx.head_entropy(X, k_trunc=cfg.k_trunc, entropy_out=ent)
    torch.cuda.synchronize()
    ctx.profile(True)
    for _ in range(3):
        ctx.head_entropy(X, k_trunc=cfg.k_trunc, entropy_out=ent)
    torch.cuda.synchronize()
    ms = [m for name, m in ctx.profile_read() if name == "gram_mfma"]
    ctx.profile(False)
    if not ms:
        return None
    avg = sum(ms) / len(ms)
    flops = n_mat * 2.0 * n_tok * D * D
    return {"matrices": n_mat, "tokens_each": n_tok, "ms": round(avg, 4), "TFLOPs_nominal": round(flops / avg / 1e9, 1),
            "mfma_frac_nominal": round(flops / avg / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
            "mfma_frac_issued": round(flops * 36 / 64 / avg / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
            "note": "nominal = 2*N*D*D flop per matrix; issued = the 36 of 64 output blocks the kernel computes (symmetry)"}


def matrix_leg(cfg, ctx, args):
    """Not part of `value`: truncated entropy of one [N, 4096] hidden-state matrix (low rank plus noise, as the
    keys) by uncomp_matrix_entropy, 8 rounds of two tall-skinny products each (matrix cores for bf16).
    HBM-bound in principle: reports the time and the rate at which the matrix is streamed."""
    import math

    import torch
    dev = "cuda:0"
    N, D, r, n_iter = cfg.N, 4096, 80, 8
    g = torch.Generator(device=dev).manual_seed(args.seed + 4096)
    X = ((torch.randn(N, r, generator=g, device=dev) / math.sqrt(r)) @ (torch.randn(r, D, generator=g, device=dev) / math.sqrt(r))
         + 0.1 * math.sqrt(128.0 / D) * torch.randn(N, D, generator=g, device=dev)).to(torch.bfloat16 if cfg.dtype == "bf16" else torch.float32)[None]
    ctx.matrix_entropy(X, k_trunc=cfg.k_trunc, n_iter=n_iter)
    torch.cuda.synchronize()
    ctx.profile(True)
    t0 = time.perf_counter()
    H = ctx.matrix_entropy(X, k_trunc=cfg.k_trunc, n_iter=n_iter)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per = {}
    for name, m in ctx.profile_read():
        per[name] = per.get(name, 0.0) + m
    ctx.profile(False)
    flops = (2 * n_iter + 1) * 2.0 * N * D * 128
    e = 2 if cfg.dtype == "bf16" else 4
    return {"tokens": N, "width": D, "rounds": n_iter, "entropy": round(float(H[0]), 5), "ms": round(dt * 1e3, 2),
            "TFLOPs": round(flops / dt / 1e12, 1), "x_read_GBps": round((2 * n_iter + 2) * N * D * e / dt / 1e9, 1),
            "hbm_frac": round((2 * n_iter + 2) * N * D * e / dt / 1e9 / HBM_PEAK_GBS, 4),
            "stages_ms": {k: round(v, 3) for k, v in per.items()}}


def prepare_leg(cfg, ctx, Kf, ent, args):
    """Not part of `value`: the offline preparation (Eq. 7 / Alg. 1).  Every sampled prompt costs one
    entropy pass over all its layers plus the accumulation of the statistics; the resident prompt stands
    for each of the samples.  Reports prompts per second at this sequence length."""
    import torch
    L, B, H, N, D = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D
    st = ctx.prepare_new(L, H, cfg.M)
    reps = 4
    X = Kf.reshape(L * B * H, N, D)

    def one():
        ctx.head_entropy(X, k_trunc=cfg.k_trunc, entropy_out=ent.reshape(-1))
        ctx.prepare_accumulate(st, ent)

    one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        one()
    labels = ctx.prepare_finish(st)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    groups = torch.bincount(labels[0].reshape(-1).long(), minlength=cfg.M).tolist()
    return {"ms_per_batch_of_prompts": round(dt * 1e3, 3), "prompts_per_s": round(B / dt, 1), "seq_len": N,
            "samples_accumulated": int(st[2][0]), "heads_per_group": groups}


def hidden_leg(cfg, ctx, K, Q, args):
    """Not part of `value`: one stage-1 hidden-state eviction (uncomp_hidden_evict) at a layer-group
    boundary: the last token's attention over one layer's keys picks the N - 512 rows (Eq. 10 with the
    paper's increment) of the [N, 4096] hidden states that enter the next group.  HBM-bound on the row
    copy; reports per-kernel times and the rate on the bytes that must move."""
    import torch
    dev = K.device
    B, H, N, D, G, w = cfg.B, cfg.H, cfg.N, cfg.D, cfg.G, cfg.w
    Dm = 4096 if cfg.H * cfg.G * D <= 4096 else 8192                    # model width of the config's family
    n_keep = max(N - 512, w + 1)
    e = 2 if cfg.dtype == "bf16" else 4
    g = torch.Generator(device=dev).manual_seed(args.seed + 404)
    Hs = torch.randn(B, N, Dm, generator=g, device=dev, dtype=torch.float32).to(K.dtype)
    q = Q[0][:, :, -1, :].contiguous()
    nk = torch.tensor([n_keep], dtype=torch.int32, device=dev)
    out = ctx.hidden_evict(q, K[0], G, nk, w, Hs, cap=n_keep)[:3]
    torch.cuda.synchronize()
    reps = 5
    ctx.profile(True)
    for _ in range(reps):
        ctx.hidden_evict(q, K[0], G, nk, w, Hs, cap=n_keep, out=out)
    torch.cuda.synchronize()
    per = {}
    for name, m in ctx.profile_read():
        per.setdefault(name, []).append(m)
    ctx.profile(False)
    kern = {name: sum(v) / len(v) for name, v in per.items()}
    total = sum(kern.values())
    byt = B * ((1 if cfg.dtype == "bf16" else 2) * H * N * D * e + 2 * n_keep * Dm * e)   # keys (once for bf16), rows in and out
    return {"layer_tokens_in": N, "layer_tokens_out": n_keep, "hidden_width": Dm, "kernel_us": round(total * 1e3, 1),
            "algorithmic_bytes": int(byt), "GBps": round(byt / total / 1e6, 1),
            "hbm_frac": round(byt / total / 1e6 / HBM_PEAK_GBS, 4),
            "kernels_us": {k: round(v * 1e3, 1) for k, v in kern.items()}}


def decode_leg(cfg, ctx, score, head_budget, outs, args):
    """Not part of `value`: the tokens generated after the prefill.  Every KV head of every
    layer takes one uncomp_decode_step per token (attention over its compacted cache, score
    update, eviction), all heads in one launch.  Reports the kernel's time per generated
    token and its HBM rate on the bytes it has to read (the cached K and V rows once)."""
    import torch

    from paper_2410_03090_amd import synth
    dev = score.device
    L, B, H, N, D, G, w = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D, cfg.G, cfg.w
    heads, T, cap = L * B * H, args.decode_steps, cfg.cap
    Kc, Vc, idx, ln = (outs[0].view(heads, cap, D), outs[1].view(heads, cap, D), outs[2].view(heads, cap),
                       outs[3].view(heads))
    scales = synth.layer_scales(cfg, args.seed)
    kn = torch.empty(T, heads, D, dtype=Kc.dtype, device=dev)
    vn = torch.empty_like(kn)
    qn = torch.empty(T, heads, G, D, dtype=Kc.dtype, device=dev)
    for l in range(L):
        for b in range(B):
            for h in range(H):
                u = (l * B + b) * H + h
                kn[:, u], vn[:, u], qn[:, u] = synth.gen_decode_tokens(cfg, args.seed, l, b, h, T, device=dev,
                                                                       scale=float(scales[l]))
    budget = head_budget.reshape(heads).contiguous()
    cum = ctx.decode_init(score.view(heads, N - w), idx, ln, N, w)
    out = torch.empty(heads, G, D, dtype=torch.float32, device=dev)
    ev = torch.empty(heads, dtype=torch.int32, device=dev)
    pos = [torch.full((heads,), N + t, dtype=torch.int32, device=dev) for t in range(T)]
    rows = float(ln.float().sum().item()) + heads            # entries read per step (cache is full: stays constant)
    torch.cuda.synchronize()
    ctx.profile(True)
    t0 = time.perf_counter()
    for t in range(T):
        ctx.decode_step(qn[t], kn[t], vn[t], pos[t], budget, w, Kc, Vc, idx, cum, ln, out=out, evicted=ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = {}
    for name, m in ctx.profile_read():
        per.setdefault(name, []).append(m)
    ctx.profile(False)
    # per kernel: mean over the last three quarters of the steps (first-touch, clocks)
    kern = {name: sum(v[len(v) // 4:]) / len(v[len(v) // 4:]) for name, v in per.items()}
    avg = sum(kern.values())
    # the same T steps replayed from a HIP graph (the calls only enqueue kernels): no launch overhead per step
    graph_us = None
    try:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for t in range(T):
                    ctx.decode_step(qn[t], kn[t], vn[t], pos[t], budget, w, Kc, Vc, idx, cum, ln, out=out, evicted=ev)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / T * 1e6
    except Exception as exc:                                   # a torch build without graph support: report, do not fail the bench
        graph_us = f"unavailable: {exc}"
    e = 2 if cfg.dtype == "bf16" else 4
    byt = rows * 2 * D * e
    return {"steps": T, "kv_heads_per_step": heads, "cache_rows": int(rows), "kernel_us_per_token": round(avg * 1e3, 2),
            "wall_us_per_token": round(wall / T * 1e6, 2),
            "graph_replay_us_per_token": round(graph_us, 2) if isinstance(graph_us, float) else graph_us,
            "algorithmic_bytes": int(byt),
            "GBps": round(byt / avg / 1e6, 1), "hbm_frac": round(byt / avg / 1e6 / HBM_PEAK_GBS, 4),
            "kernels_us": {k: round(v * 1e3, 2) for k, v in kern.items()},
            "evicting_heads": int((ev >= 0).sum().item())}


def cpu_baseline(cfg, K, V, Q, args):
    """Times the float64 oracle, as it stands, on a few (layer, batch, head) units of the same inputs and
    scales to the whole job: once with every host thread the numerical library takes, once limited to one
    thread (a quarter of the sample).  Also counts, on the sampled heads, how many kept positions lie within
    1e-5 (relative) of the k-th largest score: the band inside which two correct selections may differ.
    Baseline only."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info, threadpool_limits

    from oracle import uncomp_oracle as O
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    L, B, H, N, D, G, w = cfg.L, cfg.B, cfg.H, cfg.N, cfg.D, cfg.G, cfg.w
    units = L * B * H
    # one head of the 128K config costs the oracle about 0.65 s: take enough heads for ~15 s
    est = 0.65 * (N / 131072.0) * (G * w / 256.0)
    n_heads = args.cpu_heads or int(max(1, min(units, 64, round(15.0 / est))))
    n_single = max(1, n_heads // 4)
    f64 = lambda t: t.detach().cpu().to(torch.float64).numpy()
    bits = lambda t: t.detach().cpu().contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()
    band = {"kept_prefix_positions": 0, "within_1e-5_of_kth_score": 0}

    def run_unit(u, count_band):
        l, b, h = (u * 7) % L, u % B, (u * 3) % H
        Kh, Vh = K[l, b, h], V[l, b, h]
        Qh = Q[l, b, h * G:(h + 1) * G]
        Kn, Qn = f64(Kh)[None, None], f64(Qh)[None]
        Kb, Vb = bits(Kh)[None, None], bits(Vh)[None, None]
        t0 = time.perf_counter()
        Hh, _ = O.head_entropy(Kn[0], k_trunc=cfg.k_trunc)
        e = np.repeat(Hh.astype(np.float32)[None, None], 1, axis=2)
        hb, _, _, _ = O.assign_budgets(e.reshape(1, 1, 1), 1, cfg.avg_budget, 0, N, w, 0.4, 512)
        s = O.window_score(Qn, Kn, G, cfg.pool)
        _, _, idx, ln = O.select_gather(s, hb[0], Kb, Vb, w, cfg.cap)
        dt = time.perf_counter() - t0
        if count_band:
            k = int(ln[0, 0]) - w
            if 0 < k < N - w:
                row = s[0, 0]
                kth = np.sort(row)[::-1][k - 1]
                band["kept_prefix_positions"] += k
                band["within_1e-5_of_kth_score"] += int(np.sum(np.abs(row[idx[0, 0, :k]] - kth) <= 1e-5 * abs(kth)))
        return dt

    t_all = sum(run_unit(u, True) for u in range(n_heads))
    with threadpool_limits(limits=1):
        t_one = sum(run_unit(u, False) for u in range(n_single))
    t_job, t_job1 = t_all / n_heads * units, t_one / n_single * units
    return {"value": round(B * N / t_job, 2), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "value_1_thread": round(B * N / t_job1, 2),
            "sample": f"{n_heads} of {units} (layer,batch,head) units of {cfg.name}, all four stages, "
                      f"{t_all:.1f} s measured with {threads} threads; {n_single} units, {t_one:.1f} s, with one thread; "
                      f"both scaled linearly to the whole job",
            "tie_band": dict(band, units=n_heads)}


if __name__ == "__main__":
    main()
