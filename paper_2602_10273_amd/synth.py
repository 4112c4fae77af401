"""Seeded synthetic inputs shaped like the paper's workloads (LLM decode logits and KV caches).

Input generation only: nothing of the method's arithmetic lives here, so both the CPU checker and the
HIP path may be fed from this module.  The paper evaluates on MATH500 with 7-8B models (Sec. 7); neither
the dataset nor weights are used here -- logits and caches are random with the stated shapes and value
distributions.

numpy generators (CPU, for parity inputs) and torch generators (on device, for throughput runs) follow the
same recipe but are different random streams.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int
    V: int
    dtype: str            # "bf16" | "f32"   storage type of the logits
    alpha: float
    kappa: float
    layers: int
    H: int                # KV heads
    D: int                # head dim
    S: int                # cache positions
    steps: int
    ramp: int = 0         # >0: alpha_t ramps linearly from 1 to alpha over this many steps (Sec. 5.3)
    kind: str = "gauss_boost"
    sigma: float = 3.0

    @property
    def R(self):
        return self.B * self.N

    @property
    def kv_tensors(self):
        return 2 * self.layers

    @property
    def kv_row_bytes(self):
        return self.H * self.S * self.D * 2

    def alpha_at(self, t):
        """Exponent used for token t (1-based): one bridging stage per token while ramping, alpha_0 = 1."""
        if self.ramp <= 0:
            return float(self.alpha)
        if t <= 0:
            return 1.0
        return 1.0 + (self.alpha - 1.0) * min(t, self.ramp) / self.ramp


WORKLOADS = {
    "cfg1": Workload("cfg1_tiny_enumerable", 1, 4, 8, "f32", 4.0, 0.5, 2, 2, 16, 6, 6, kind="bigram", sigma=2.0),
    "cfg2": Workload("cfg2_qwen2.5-7b_decode", 16, 8, 152064, "bf16", 4.0, 0.5, 28, 4, 128, 2048, 512),
    "cfg3": Workload("cfg3_llama3-8b_decode", 8, 16, 128256, "bf16", 4.0, 0.5, 32, 8, 128, 4096, 1024,
                     kind="gauss_zipf", sigma=2.5),
    "cfg4": Workload("cfg4_alpha_ramp_stress", 64, 32, 152064, "f32", 4.0, 0.5, 28, 4, 128, 1024, 256,
                     ramp=128, kind="student_t", sigma=3.0),
    "cfg5": Workload("cfg5_large_particle_set", 4, 64, 152064, "bf16", 6.0, 0.7, 28, 4, 128, 4096, 2048),
}


def scaled(w: Workload, **kw) -> Workload:
    """Same recipe at other sizes (tests use reduced shapes that still span several tiles and a ragged tail)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


# ----------------------------------------------------------------------------- bf16 storage helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- numpy (CPU) generators
def bigram_table(V, sigma, seed):
    return (np.random.default_rng([seed, 11]).standard_normal((V, V)) * sigma).astype(np.float32)


def logits_numpy(w: Workload, step: int, seed: int, prev_tokens=None, table=None) -> np.ndarray:
    """Logits of one decode step, [R, V]; uint16 (bf16 bits) or float32 by w.dtype."""
    rng = np.random.default_rng([seed, 7, step])
    R, V = w.R, w.V
    if w.kind == "bigram":
        prev = np.zeros(R, np.int64) if prev_tokens is None else np.asarray(prev_tokens, np.int64)
        x = table[prev].astype(np.float32)
    elif w.kind == "gauss_boost":
        x = (rng.standard_normal((R, V), dtype=np.float32) * np.float32(w.sigma))
        nb = min(20, V)
        for r in range(R):
            idx = rng.choice(V, size=nb, replace=False)
            x[r, idx] += np.float32(8.0)
    elif w.kind == "gauss_zipf":
        x = (rng.standard_normal((R, V), dtype=np.float32) * np.float32(w.sigma))
        boost = (10.0 * np.arange(1, V + 1, dtype=np.float64) ** -1.1).astype(np.float32)
        for r in range(R):
            x[r, rng.permutation(V)] += boost
    elif w.kind == "student_t":
        x = (rng.standard_t(3.0, size=(R, V)) * w.sigma).astype(np.float32)
    else:
        raise ValueError(w.kind)
    return f32_to_bf16_bits(x) if w.dtype == "bf16" else x


def kv_numpy(w: Workload, seed: int):
    """List of 2*layers arrays [R, H, S, D] of bf16 bit patterns ~ N(0,1)."""
    rng = np.random.default_rng([seed, 13])
    return [f32_to_bf16_bits(rng.standard_normal((w.R, w.H, w.S, w.D), dtype=np.float32))
            for _ in range(w.kv_tensors)]


# ----------------------------------------------------------------------------- torch (device) generators
def logits_torch(w: Workload, step: int, seed: int, device="cuda"):
    """Same recipe generated on the device (a different random stream than logits_numpy)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + step) & 0x7FFFFFFF)
    R, V = w.R, w.V
    if w.kind == "gauss_boost":
        x = torch.randn((R, V), generator=g, device=device, dtype=torch.float32) * w.sigma
        idx = torch.rand((R, V), generator=g, device=device).topk(min(20, V), dim=1).indices
        x.scatter_add_(1, idx, torch.full_like(idx, 8.0, dtype=torch.float32))
    elif w.kind == "gauss_zipf":
        x = torch.randn((R, V), generator=g, device=device, dtype=torch.float32) * w.sigma
        rank = torch.rand((R, V), generator=g, device=device).argsort(dim=1).argsort(dim=1).to(torch.float32) + 1.0
        x += 10.0 * rank.pow(-1.1)
    elif w.kind == "student_t":
        z = torch.randn((R, V), generator=g, device=device, dtype=torch.float32)
        c = torch.randn((3, R, V), generator=g, device=device, dtype=torch.float32).square_().sum(0)
        x = z * torch.rsqrt(c / 3.0) * w.sigma
    else:
        raise ValueError(w.kind)
    return x.to(torch.bfloat16) if w.dtype == "bf16" else x


def kv_torch(w: Workload, seed: int, device="cuda"):
    """2*layers tensors [R, H, S, D] bf16 ~ N(0,1), filled on the device tensor by tensor."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed + 12345)
    out = []
    for _ in range(w.kv_tensors):
        t = torch.empty((w.R, w.H, w.S, w.D), device=device, dtype=torch.bfloat16)
        t.normal_(generator=g)
        out.append(t)
    return out


def ancestors_numpy(w: "Workload", seed: int, concentration: float = 0.5):
    """Synthetic ancestor vector [R] (global rows) for a stand-alone reorder: per prompt, N sorted draws from weights
    ~ Dirichlet(concentration) -- sorted with duplicates, as resampling of a moderately degenerate weight vector
    gives.  Every prompt counts as resampled."""
    rng = np.random.default_rng([seed, 777])
    anc = np.empty(w.R, np.int32)
    for b in range(w.B):
        p = rng.dirichlet(np.full(w.N, concentration))
        anc[b * w.N:(b + 1) * w.N] = b * w.N + np.sort(rng.choice(w.N, size=w.N, p=p))
    return anc
