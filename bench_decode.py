#!/usr/bin/env python3
"""Latency of Power-SMC decoding relative to plain decoding on one MI355X, with the KV cache in the library's layouts.

The paper's headline is a latency ratio over standard decoding (Sec. 7, Table 1).  No model weights exist in this
environment, so the language model here is a RANDOM-INIT decoder of the Qwen2.5-7B shape (28 layers, d = 3584,
28 query / 4 KV heads of 128, d_ff = 18944, V = 152064; bf16) written in plain PyTorch-ROCm: its tokens mean nothing,
its per-step cost (weight reads, attention over the cache, the LM head) is that of the real model.  Attention reads the
cache in place through smc_attn_decode, new keys and values are stored by smc_kv_append, and the logits go straight
from the LM head into smc_step.

Three loops over the same model, rows and cache length are timed:
  plain  : one token per row per step by Gumbel-max sampling at temperature 1/alpha in PyTorch, no weights, no reorder;
  dense  : Power-SMC with the double-buffered cache (smc_step, smc_resample, smc_kv_reindex);
  paged  : Power-SMC with the paged cache (smc_paged_prepare_append, smc_step, smc_resample, smc_paged_reindex).
Prints ONE JSON line with the three step times and the ratios.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

SHAPES = {
    # name: layers, d_model, q heads, kv heads, head dim, d_ff, vocabulary
    "qwen2.5-7b": (28, 3584, 28, 4, 128, 18944, 152064),
    "llama-3-8b": (32, 4096, 32, 8, 128, 14336, 128256),
    "tiny": (2, 256, 4, 2, 64, 512, 4096),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="qwen2.5-7b", choices=sorted(SHAPES))
    ap.add_argument("--prompts", type=int, default=16)
    ap.add_argument("--particles", type=int, default=8)
    ap.add_argument("--positions", type=int, default=2048, help="cache capacity per row")
    ap.add_argument("--start", type=int, default=-1, help="positions already in the cache when timing starts (default: capacity - steps - warmup - 1)")
    ap.add_argument("--steps", type=int, default=24)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--alpha", type=float, default=4.0)
    ap.add_argument("--kappa", type=float, default=0.5)
    ap.add_argument("--page", type=int, default=16)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--modes", default="plain,dense,paged")
    ap.add_argument("--in-place", action="store_true", help="ancestor vectors permuted so that survivors keep their rows")
    return ap.parse_args()


class RandomInitDecoder:
    """Pre-norm decoder-only transformer with grouped-query attention, rotary embeddings and a SwiGLU MLP."""

    def __init__(self, shape, device, seed):
        import torch
        self.L, self.d, self.Hq, self.Hkv, self.D, self.dff, self.V = shape
        g = torch.Generator(device=device); g.manual_seed(seed)

        def w(*s):
            return (torch.randn(*s, device=device, dtype=torch.float32, generator=g) * 0.02).to(torch.bfloat16)

        self.emb = w(self.V, self.d)
        self.layers = []
        for _ in range(self.L):
            self.layers.append(dict(
                wqkv=w(self.d, (self.Hq + 2 * self.Hkv) * self.D), wo=w(self.Hq * self.D, self.d),
                wgu=w(self.d, 2 * self.dff), wd=w(self.dff, self.d),
                n1=torch.ones(self.d, device=device, dtype=torch.bfloat16), n2=torch.ones(self.d, device=device, dtype=torch.bfloat16)))
        self.nf = torch.ones(self.d, device=device, dtype=torch.bfloat16)
        self.head = w(self.d, self.V)
        half = self.D // 2
        self.inv_freq = 1.0 / (1.0e6 ** (torch.arange(0, half, device=device, dtype=torch.float32) / half))
        self.n_params = sum(t.numel() for l in self.layers for t in l.values()) + self.emb.numel() + self.head.numel()

    @staticmethod
    def _norm(x, wt):
        import torch
        xf = x.float()
        return (xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + 1e-6)).to(torch.bfloat16) * wt

    def _rope(self, x, pos):
        import torch
        ang = pos * self.inv_freq                                  # [D/2]
        cos, sin = torch.cos(ang), torch.sin(ang)
        xf = x.float()
        a, b = xf[..., : self.D // 2], xf[..., self.D // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1).to(torch.bfloat16)

    def step(self, tokens, pos, write_kv, attend):
        """One decode step: tokens int64 [R] at position pos -> logits bf16 [R, V].
        write_kv(layer, k, v) stores bf16 [R, Hkv, D] at position pos; attend(layer, q, pos + 1) returns f32 [R, Hq, D]."""
        import torch
        x = self.emb[tokens]
        R = x.shape[0]
        for i, l in enumerate(self.layers):
            h = self._norm(x, l["n1"])
            qkv = h @ l["wqkv"]
            q, k, v = torch.split(qkv, [self.Hq * self.D, self.Hkv * self.D, self.Hkv * self.D], dim=-1)
            q = self._rope(q.view(R, self.Hq, self.D), pos).contiguous()
            k = self._rope(k.view(R, self.Hkv, self.D), pos)
            write_kv(i, k, v.view(R, self.Hkv, self.D))
            a = attend(i, q, pos + 1).to(torch.bfloat16).view(R, self.Hq * self.D)
            x = x + a @ l["wo"]
            h = self._norm(x, l["n2"])
            gu = h @ l["wgu"]
            x = x + (torch.nn.functional.silu(gu[:, : self.dff]) * gu[:, self.dff:]) @ l["wd"]
        return self._norm(x, self.nf) @ self.head


def run_mode(mode, args, model, torch, smc, Session):
    B, N = args.prompts, args.particles
    R = B * N
    S, P = args.positions, args.page
    W, K = args.warmup, args.steps
    start = args.start if args.start >= 0 else S - (W + K) - 1
    assert 0 <= start and start + W + K <= S
    paged = mode == "paged"
    T_max = (W + K + 3) // 4 * 4
    s = Session(B, N, model.V, T_max, "bf16", args.kappa if mode != "plain" else 0.0, args.seed,
                kv_geom=(2 * model.L, model.Hkv, S, model.D), page_len=P if paged else 0, len0=start if paged else 0)
    if args.in_place and mode != "plain":
        smc.smc_set_ancestor_order(s.ctx, 1)
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed + 1)
    for t in (s.pools if paged else s.kvA):                       # the cache as start positions of earlier decoding left it
        t.normal_(generator=g)
    scale = 1.0 / math.sqrt(model.D)
    pos_state = dict(pos=start)

    def write_kv(layer, k, v):
        s.append(2 * layer, 2 * layer + 1, k, v, pos_state["pos"])     # one launch: each row's live buffer or page

    def attend(layer, q, length):
        return s.attention(2 * layer, 2 * layer + 1, q, length, scale)

    tokens = torch.zeros(R, dtype=torch.int64, device="cuda")
    n_resampled = torch.zeros((), dtype=torch.int64, device="cuda")
    beta = args.alpha

    def one_step(t):
        nonlocal tokens
        pos = pos_state["pos"]
        if paged:
            s.prepare_append(pos)
        logits = model.step(tokens, pos, write_kv, attend)
        if mode == "plain":                                       # low-temperature sampling, tau = 1/alpha, by Gumbel-max
            u = torch.rand(logits.shape, device="cuda", generator=g).clamp_(1e-20, 1.0)
            tokens = (logits.float() * beta - torch.log(-torch.log(u))).argmax(dim=-1)
        else:
            s.step(logits, t, args.alpha, args.alpha, -1.0)
            s.resample(t)
            n_resampled.add_(s.resampled.sum())
            if paged:
                s.paged_reindex(t)
            else:
                s.reindex(pos + 1, t)
            tokens = s.tokens.long()
        pos_state["pos"] = pos + 1

    for i in range(W):
        one_step(i + 1)
    torch.cuda.synchronize()
    n_resampled.zero_()
    t0 = time.perf_counter()
    for i in range(K):
        one_step(W + i + 1)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / K * 1e3
    frac = float(n_resampled.item()) / (K * B)
    s.close()
    del s
    torch.cuda.empty_cache()
    return ms, frac, start


def main():
    args = parse()
    import torch
    from paper_2602_10273_amd import binding as smc
    from paper_2602_10273_amd.harness import Session
    torch.cuda.set_device(0)
    shape = SHAPES[args.shape]
    model = RandomInitDecoder(shape, "cuda", args.seed)
    out = {"metric": "decode step latency, Power-SMC relative to plain decoding (random-init model), 1 MI355X",
           "unit": "ms per step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic (random-init weights)",
           "config": {"shape": args.shape, "parameters": model.n_params, "prompts": args.prompts, "particles": args.particles,
                      "rows": args.prompts * args.particles, "positions": args.positions, "alpha": args.alpha,
                      "kappa": args.kappa, "page": args.page,
                      "ancestor_order": "survivors-in-place" if args.in_place else "as-drawn"}}
    for mode in args.modes.split(","):
        ms, frac, start = run_mode(mode, args, model, torch, smc, Session)
        out[f"{mode}_ms_per_step"] = ms
        if mode != "plain":
            out[f"{mode}_resampled_prompt_fraction"] = frac
        out["config"]["cache_positions_at_start"] = start
    if "plain_ms_per_step" in out:
        for mode in ("dense", "paged"):
            if f"{mode}_ms_per_step" in out:
                out[f"{mode}_latency_ratio"] = out[f"{mode}_ms_per_step"] / out["plain_ms_per_step"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
