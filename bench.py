#!/usr/bin/env python3
"""Throughput of the Power-SMC per-token step on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic logits with the KV cache resident in
HBM: smc_step (boundary reweight, vocabulary pass, increment) -> smc_resample (ESS, trigger, ancestors) ->
smc_kv_reindex (KV / history / cumulative-log-p gather for the prompts that resampled).  Resampling fires
whenever the weights say so; how often is an observed quantity and is reported.

Prints ONE JSON line.  `value` is particle-steps/s over the timed steps.  `roofline` describes the kernel that
took the most time in a second, instrumented run of the same number of steps (HIP events recorded by the library
on its own stream around each launch); `roofline_other` the other dominant kernel.  `cpu_baseline` times the CPU
oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0: per-workload default)")
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kv", action="store_true", help="vocabulary pass + weights only (no cache bound)")
    ap.add_argument("--n-split", type=int, default=0)
    ap.add_argument("--mode", default="step", choices=["step", "reindex", "attention"],
                    help="step: the whole hot path (default); reindex: the KV reorder alone, every prompt resampled "
                         "with synthetic ancestors (sorted draws from Dirichlet(0.5) weights); attention: decode "
                         "attention of every layer over the full cache (dense, or paged with --paged P)")
    ap.add_argument("--q-heads", type=int, default=0, help="query heads for --mode attention (default 7 per KV head)")
    ap.add_argument("--paged", type=int, default=0, metavar="P",
                    help="paged cache with P positions per page: the reorder copies page numbers, appends copy on write")
    ap.add_argument("--in-place", action="store_true",
                    help="ancestor order 1: surviving ancestors keep their slot, only the other copies move")
    return ap.parse_args()


def cpu_baseline(w, seed, gpu_resample_frac):
    """The oracle as it stands, on the host cores: a few full-width steps on all rows, plus the KV gather of one
    prompt's rows scaled to the number of prompts that resample per step."""
    import numpy as np
    from oracle import reference as orc
    from paper_2602_10273_amd import synth

    threads = orc.threads()
    o = orc.OracleSMC(w.B, w.N, w.V, 4096, w.kappa, seed, w.dtype)
    n_buf = 2 if w.R * w.V > 1e8 else 3
    x = [synth.logits_torch(w, 1000 + i, seed, device="cpu") for i in range(n_buf)]
    if w.dtype == "bf16":
        import torch
        x = [t.view(torch.int16).numpy().view(np.uint16) for t in x]
    else:
        x = [t.numpy() for t in x]
    # full-width steps on all rows until about 10 s of CPU work have been timed (at least 3 steps)
    t0 = time.perf_counter()
    n_res = n_steps = 0
    while n_steps < 3 or (time.perf_counter() - t0 < 10.0 and n_steps < 4000):
        i = n_steps
        o.step(x[i % n_buf], i + 1, w.alpha_at(i + 1), w.alpha_at(i), -1.0)
        _, flag, _ = o.resample(i + 1)
        n_res += int(flag.sum())
        n_steps += 1
    t_step = (time.perf_counter() - t0) / n_steps
    # KV gather: one prompt (N rows) of a few tensors, timed and scaled linearly to all tensors
    n_t = max(1, min(w.kv_tensors, int(1.5e9 // (w.N * w.kv_row_bytes))))
    rng = np.random.default_rng(seed)
    src = [rng.integers(0, 65535, size=(w.N, w.H, w.S, w.D), dtype=np.uint16) for _ in range(n_t)]
    dst = [np.empty_like(a) for a in src]
    anc = np.sort(rng.integers(0, w.N, w.N)).astype(np.int32)
    flag = np.ones(1, np.int32)
    t0 = time.perf_counter()
    for a, d in zip(src, dst):
        orc.gather_kv(a, anc, flag, w.N, w.S, d)
    t_gather_prompt = (time.perf_counter() - t0) * (w.kv_tensors / n_t)
    t_total = t_step + t_gather_prompt * gpu_resample_frac * w.B
    return {
        "value": w.R / t_total, "unit": "particle-steps/s", "cores": threads, "kind": "oracle",
        "sample": (f"{n_steps} full-width steps (vocabulary pass + ESS + resampling) on all {w.R} rows; KV gather of one "
                   f"prompt ({w.N} rows x {n_t} of {w.kv_tensors} tensors) scaled to all tensors and to the "
                   f"{gpu_resample_frac * w.B:.2f} prompts/step that resampled on the GPU"),
        "step_s": t_step, "gather_prompt_s": t_gather_prompt,
    }


def measured_ceilings(smc, torch, dev):
    """Plain streaming kernels of the library on a 4 GiB buffer: the device's own ceilings for four read:write mixes."""
    nbytes = 4 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    out = {name: smc.smc_hbm_probe(kind, buf, nbytes, stream)
           for kind, name in enumerate(("read", "write", "copy_1r1w", "fanout_1r3w"))}
    del buf
    return out


def reindex_only(args, w, K, W, smc, synth, Session, np, torch):
    """The KV reorder alone at the workload's full cache: K launches with distinct synthetic ancestor vectors."""
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, args.seed, kv_geom=(w.kv_tensors, w.H, w.S, w.D))
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed + 12345)
    for t in s.kvA:
        t.normal_(generator=g)
    ancs = [synth.ancestors_numpy(w, args.seed + i) for i in range(W + K)]
    d_anc = [torch.as_tensor(a).cuda() for a in ancs]
    flag = torch.ones(w.B, dtype=torch.int32, device="cuda")
    for i in range(W):
        s.reindex(w.S, 4, d_anc[i], flag)
    torch.cuda.synchronize()
    smc.smc_profile_enable(s.ctx, 1)
    t0 = time.perf_counter()
    for i in range(W, W + K):
        s.reindex(w.S, 4, d_anc[i], flag)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_gather, n_gather = smc.smc_profile_read(s.ctx, 1)
    smc.smc_profile_enable(s.ctx, 0)
    ident = np.arange(w.R)
    rows_written = rows_read = 0
    for a in ancs[W:]:
        moved = a != ident
        rows_written += int(moved.sum())
        rows_read += sum(len(np.unique(a[b * w.N:(b + 1) * w.N][moved[b * w.N:(b + 1) * w.N]])) for b in range(w.B))
    total_bytes = float(rows_written + rows_read) * w.kv_row_bytes * w.kv_tensors
    gbps = total_bytes / (ms_gather * 1e-3) / 1e9
    s.close()
    del s
    torch.cuda.empty_cache()
    out = {
        "metric": "particle-steps/s (KV reindex only), 1 MI355X",
        "value": w.R * K / elapsed, "unit": "particle-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": w.name, "mode": "reindex", "B": w.B, "N": w.N,
                   "kv": f"{w.layers}x2 tensors [{w.R},{w.H},{w.S},{w.D}] bf16 x2 buffers", "valid_len": w.S,
                   "ancestors": "sorted draws from Dirichlet(0.5) weights, every prompt resampled",
                   "rows_read_per_row_written": rows_read / max(rows_written, 1)},
        "roofline": {"kernel": "gather_kernel", "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "traffic": None, "launches": int(n_gather),
                     "avg_launch_ms": ms_gather / max(n_gather, 1), "algorithmic_bytes_per_launch": total_bytes / max(n_gather, 1)},
    }
    out["measured_ceilings_GBps"] = measured_ceilings(smc, torch, "cuda")
    print(json.dumps(out))


def attention_only(args, w, K, W, smc, synth, Session, np, torch):
    """Decode attention of all layers over the workload's full cache: one step = one call per layer."""
    P = args.paged
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, args.seed, kv_geom=(w.kv_tensors, w.H, w.S, w.D), with_hist=False,
                page_len=P, len0=w.S)
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed + 12345)
    for t in (s.pools if P else s.kvA):
        t.normal_(generator=g)
    if not P:                                           # rows in both buffers, as after a few reorders
        flag = torch.ones(w.B, dtype=torch.int32, device="cuda")
        for i in range(2):
            s.reindex(w.S, 0, torch.as_tensor(synth.ancestors_numpy(w, args.seed + i)).cuda(), flag)
    Hq = args.q_heads or 7 * w.H
    q = torch.randn((w.R, Hq, w.D), device="cuda", generator=g).to(torch.bfloat16)
    scale = float(w.D) ** -0.5

    def one_step():
        for layer in range(w.layers):
            s.attention(2 * layer, 2 * layer + 1, q, w.S, scale)

    for _ in range(W):
        one_step()
    torch.cuda.synchronize()
    smc.smc_profile_enable(s.ctx, 1)
    t0 = time.perf_counter()
    for _ in range(K):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms, n = smc.smc_profile_read(s.ctx, 3)
    smc.smc_profile_enable(s.ctx, 0)
    bytes_per_call = 2.0 * w.R * w.H * w.S * w.D * 2            # K and V of one layer, every position read once
    gbps = bytes_per_call * n / (ms * 1e-3) / 1e9
    s.close()
    del s
    torch.cuda.empty_cache()
    out = {
        "metric": "particle-steps/s (decode attention of all layers only), 1 MI355X",
        "value": w.R * K / elapsed, "unit": "particle-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "mode": "attention", "rows": w.R, "kv_heads": w.H, "q_heads": Hq, "head_dim": w.D,
                   "positions": w.S, "layers": w.layers, "cache": f"paged, {P} positions per page" if P else "dense, double-buffered rows"},
        "roofline": {"kernel": "attn_decode_kernel", "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "traffic": None, "launches": int(n), "avg_launch_ms": ms / max(n, 1),
                     "algorithmic_bytes_per_launch": bytes_per_call},
    }
    try:
        ratio = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic_ratio.json"))).get(args.workload, {}).get("attn_decode_kernel")
        if ratio and not P:
            out["roofline"]["traffic"] = ratio * bytes_per_call
            out["roofline"]["traffic_source"] = "profiles/hbm_traffic_ratio.json x algorithmic bytes of this run"
    except OSError:
        pass
    out["measured_ceilings_GBps"] = measured_ceilings(smc, torch, "cuda")
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by prompt with no communication); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2602_10273_amd import binding as smc
    from paper_2602_10273_amd import synth
    from paper_2602_10273_amd.harness import Session

    w = synth.WORKLOADS[args.workload]
    K = args.steps or {"cfg2": 48, "cfg3": 16, "cfg4": 12, "cfg5": 16}[args.workload]
    W = args.warmup
    if args.mode == "reindex":
        torch.cuda.set_device(0)
        return reindex_only(args, w, K, min(W, 2), smc, synth, Session, np, torch)
    if args.mode == "attention":
        torch.cuda.set_device(0)
        return attention_only(args, w, K, min(W, 2), smc, synth, Session, np, torch)
    dev = "cuda"
    torch.cuda.set_device(0)
    T_max = (W + 2 * K + 8 + 3) // 4 * 4

    kv_geom = None if args.no_kv else (w.kv_tensors, w.H, w.S, w.D)
    P = 0 if args.no_kv else args.paged
    len0 = max(0, w.S - (W + 2 * K) - 1)           # paged runs: the cache is this full when the run starts
    s = Session(w.B, w.N, w.V, T_max, w.dtype, w.kappa, args.seed, kv_geom=kv_geom, page_len=P, len0=len0)
    if args.n_split:
        smc.smc_set_tuning(s.ctx, args.n_split, 0)
    if args.in_place:
        smc.smc_set_ancestor_order(s.ctx, 1)
    if not args.no_kv:
        g = torch.Generator(device=dev); g.manual_seed(args.seed + 12345)
        for t in (s.pools if P else s.kvA):
            t.normal_(generator=g)
    n_ring = 4 if w.dtype == "f32" else 16       # distinct logits buffers: more bytes than the 256 MB last-level cache
    ring = [synth.logits_torch(w, i, args.seed) for i in range(n_ring)]
    torch.cuda.synchronize()

    step_no = [0]

    def reorder(t):
        if P:
            s.paged_reindex(t)
        else:
            s.reindex(w.S, t)

    def one_step():
        step_no[0] += 1
        t = step_no[0]
        if P:
            s.prepare_append(len0 + t - 1)          # the decoder would now write position len0+t-1 and emit logits
        s.step(ring[t % n_ring], t, w.alpha_at(t), w.alpha_at(t - 1), -1.0)
        s.resample(t)
        reorder(t)

    for _ in range(W):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- instrumented run of the same length: per-kernel event timing + what was gathered -------------------
    anc_log = torch.zeros((K, w.R), dtype=torch.int32, device=dev)
    flag_log = torch.zeros((K, w.B), dtype=torch.int32, device=dev)
    smc.smc_profile_enable(s.ctx, 1)
    for i in range(K):
        step_no[0] += 1
        t = step_no[0]
        if P:
            s.prepare_append(len0 + t - 1)
        s.step(ring[t % n_ring], t, w.alpha_at(t), w.alpha_at(t - 1), -1.0)
        s.resample(t)
        anc_log[i].copy_(s.anc); flag_log[i].copy_(s.resampled)
        reorder(t)
    first_t = step_no[0] - K + 1
    ms_vocab, n_vocab = smc.smc_profile_read(s.ctx, 0)
    ms_gather, n_gather = smc.smc_profile_read(s.ctx, 2 if P else 1)
    smc.smc_profile_enable(s.ctx, 0)
    anc_h = anc_log.cpu().numpy().reshape(K, w.B, w.N)
    flag_h = flag_log.cpu().numpy()
    esz = 2 if w.dtype == "bf16" else 4
    vocab_bytes = float(w.R) * w.V * esz                              # per launch: every logit read once
    # per resampled prompt: rows whose ancestor is another row are written once; their distinct ancestors are read once
    local = anc_h - (np.arange(w.B)[None, :, None] * w.N)
    moved = (local != np.arange(w.N)[None, None, :]) & (flag_h[:, :, None] != 0)
    rows_moved = int(moved.sum()) + sum(len(np.unique(local[i, b][moved[i, b]])) for i in range(K) for b in range(w.B))
    gather_bytes_total = float(rows_moved) * w.kv_row_bytes * w.kv_tensors
    if P:
        # an append at offset o = pos % P copies o positions (read + write) for every sharer of a page but one: the
        # rows of the prompts that resampled at the previous step, minus their distinct ancestors
        gather_bytes_total = 0.0
        pos_bytes = w.kv_row_bytes // w.S
        for i in range(1, K):
            o = (len0 + first_t + i - 1) % P
            needy = sum(w.N - len(np.unique(local[i - 1, b])) for b in range(w.B) if flag_h[i - 1, b])
            gather_bytes_total += 2.0 * needy * o * pos_bytes * w.kv_tensors
    resample_frac = float(flag_h.mean())

    def roof(name, total_bytes, ms, launches):
        if launches == 0 or ms <= 0:
            return {"kernel": name, "bound": "hbm", "achieved": 0.0, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": 0.0, "traffic": None, "launches": int(launches)}
        gbps = total_bytes / (ms * 1e-3) / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gbps / HBM_PEAK_GBPS, "traffic": None, "launches": int(launches),
                "avg_launch_ms": ms / launches, "algorithmic_bytes_per_launch": total_bytes / launches}

    # HBM traffic per launch: measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (calibrated on a copy of
    # known size) as a multiple of the algorithmic bytes; the committed ratio is applied to this run's bytes.
    ratios = {}
    try:
        ratios = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic_ratio.json"))).get(args.workload, {})
    except OSError:
        pass

    r_vocab = roof("vocab_pass_kernel", vocab_bytes * n_vocab, ms_vocab, n_vocab)
    r_gather = roof("paged_copy_kernel" if P else "gather_kernel", gather_bytes_total, ms_gather,
                    n_gather if not args.no_kv else 0)
    for r in (r_vocab, r_gather):
        if r["kernel"] in ratios and r.get("algorithmic_bytes_per_launch"):
            r["traffic"] = ratios[r["kernel"]] * r["algorithmic_bytes_per_launch"]
            r["traffic_source"] = "profiles/hbm_traffic_ratio.json x algorithmic bytes of this run"
    dominant, other = (r_gather, r_vocab) if ms_gather >= ms_vocab else (r_vocab, r_gather)

    out = {
        "metric": "particle-steps/s (SMC step + KV reindex), 1 MI355X",
        "value": w.R * K / elapsed, "unit": "particle-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "N": w.N, "V": w.V, "logits_dtype": w.dtype, "alpha": w.alpha,
                   "kappa": w.kappa, "ancestor_order": "survivors-in-place" if args.in_place else "as-drawn", "kv": None if args.no_kv else (f"{w.layers}x2 paged pools [{w.B}x{s.Q},{w.H},{P},{w.D}] bf16, {len0} positions filled at start"
                                                 if P else f"{w.layers}x2 tensors [{w.R},{w.H},{w.S},{w.D}] bf16 x2 buffers"),
                   "valid_len": w.S, "resampled_prompt_fraction": resample_frac,
                   "logits_ring": n_ring},
        "roofline": dominant, "roofline_other": other,
    }
    s.close()
    del s
    torch.cuda.empty_cache()
    # the device's own ceilings (plain streaming kernels) as a second, measured denominator
    out["measured_ceilings_GBps"] = measured_ceilings(smc, torch, dev)
    out["device_copy_GBps"] = out["measured_ceilings_GBps"]["copy_1r1w"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.seed, resample_frac if not args.no_kv else 0.0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
