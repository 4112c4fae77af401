"""Device-memory plumbing around the C ABI: a Session owns the torch buffers a context needs and forwards calls.

No arithmetic of the method happens here -- every step runs in the HIP kernels behind `binding`.
"""
import numpy as np
import torch

from . import binding as smc


class Session:
    def __init__(self, B, N, V, T_max, dtype, kappa, seed, kv_geom=None, kv=None, with_hist=True, device="cuda",
                 stream=None, eos_id=-1, page_len=0, len0=0):
        """kv_geom = (kv_tensors, H, S, D) allocates zeroed double buffers; kv = list of [R,H,S,D] bf16/uint16
        tensors (numpy or torch) to copy into buffer A instead.  page_len > 0 (with kv_geom): the cache is paged
        instead -- one zeroed pool [B*Q, H, page_len, D] per tensor, the table as after len0 appends."""
        self.B, self.N, self.V, self.T_max, self.R = B, N, V, T_max, B * N
        self.dtype, self.device = dtype, device
        dev = torch.device(device)
        self.kvA, self.kvB = [], []
        if kv is not None:
            for t in kv:
                a = torch.as_tensor(np.ascontiguousarray(t).view(np.int16)) if isinstance(t, np.ndarray) else t
                a = a.to(dev).contiguous()
                self.kvA.append(a)
                self.kvB.append(torch.zeros_like(a))
            kv_geom = (len(kv),) + tuple(self.kvA[0].shape[1:])
        elif kv_geom is not None and page_len == 0:
            n, H, S, D = kv_geom
            for _ in range(n):
                self.kvA.append(torch.zeros((self.R, H, S, D), dtype=torch.bfloat16, device=dev))
                self.kvB.append(torch.zeros((self.R, H, S, D), dtype=torch.bfloat16, device=dev))
        n, H, S, D = kv_geom if kv_geom is not None else (0, 0, 0, 0)
        self.kv_geom = (n, H, S, D)
        self.cfg = smc.make_config(B, N, V, T_max, dtype, kappa, seed, n, H, S, D, 2, eos_id)
        nbytes = smc.smc_workspace_bytes(self.cfg)
        if nbytes == 0:
            raise ValueError("invalid configuration")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) & ~255
        self.stream = stream
        sptr = stream.cuda_stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
        self.ctx = smc.smc_init(self.cfg, self._ws_ptr, nbytes, sptr)
        self.tokens = torch.zeros(self.R, dtype=torch.int32, device=dev)
        self.ess = torch.zeros(B, dtype=torch.float64, device=dev)
        self.lognormw = torch.zeros(self.R, dtype=torch.float64, device=dev)
        self.anc = torch.zeros(self.R, dtype=torch.int32, device=dev)
        self.resampled = torch.zeros(B, dtype=torch.int32, device=dev)
        self.choice = torch.zeros(B, dtype=torch.int32, device=dev)
        self.histA = self.histB = None
        if with_hist:
            self.histA = torch.zeros((self.R, T_max), dtype=torch.int32, device=dev)
            self.histB = torch.zeros((self.R, T_max), dtype=torch.int32, device=dev)
        if n > 0 or with_hist:
            smc.smc_kv_bind(self.ctx, self.kvA, self.kvB, self.histA, self.histB)
        self.page_len = page_len
        if page_len > 0:
            self.M = (S + page_len - 1) // page_len
            self.Q = N * self.M
            self.pools = [torch.zeros((B * self.Q, H, page_len, D), dtype=torch.bfloat16, device=dev) for _ in range(n)]
            assert self.pools[0].numel() * 2 == smc.smc_paged_pool_bytes(self.cfg, page_len)
            pbytes = smc.smc_paged_workspace_bytes(self.cfg, page_len)
            self.paged_ws = torch.empty(pbytes + 256, dtype=torch.uint8, device=dev)
            smc.smc_paged_bind(self.ctx, self.pools, page_len, (self.paged_ws.data_ptr() + 255) & ~255, pbytes, len0)
            self.slot = torch.zeros(self.R, dtype=torch.int32, device=dev)

    def close(self):
        if self.ctx is not None:
            smc.smc_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- forwards -----------------------------------------------------------------------------------------
    def step(self, logits, t, alpha_t, alpha_prev, tau_t=-1.0):
        smc.smc_step(self.ctx, logits, logits.stride(0), t, alpha_t, alpha_prev, tau_t, self.tokens)

    def step_resample(self, logits, t, alpha_t, alpha_prev, tau_t=-1.0):
        """a0..a4 in one launch (the same results as step() followed by resample())."""
        smc.smc_step_resample(self.ctx, logits, logits.stride(0), t, alpha_t, alpha_prev, tau_t, self.tokens, self.anc,
                              self.resampled, self.ess)

    def step_resample_reindex(self, logits, t, alpha_t, alpha_prev, valid_len, tau_t=-1.0):
        """a0..a5 in one call (the same results as step_resample() followed by reindex())."""
        smc.smc_step_resample_reindex(self.ctx, logits, logits.stride(0), t, alpha_t, alpha_prev, tau_t, valid_len,
                                      self.tokens, self.anc, self.resampled, self.ess)

    def compute_ess(self):
        smc.smc_ess(self.ctx, self.ess, self.lognormw)

    def resample(self, t):
        smc.smc_resample(self.ctx, t, self.anc, self.resampled, self.ess)

    def reindex(self, valid_len, t, anc=None, resampled=None):
        smc.smc_kv_reindex(self.ctx, self.anc if anc is None else anc,
                           self.resampled if resampled is None else resampled, valid_len, t)

    def prepare_append(self, pos):
        smc.smc_paged_prepare_append(self.ctx, pos, self.slot)

    def paged_reindex(self, t, anc=None, resampled=None):
        smc.smc_paged_reindex(self.ctx, self.anc if anc is None else anc,
                              self.resampled if resampled is None else resampled, t)

    def paged_reindex_prepare(self, t, next_pos, anc=None, resampled=None):
        smc.smc_paged_reindex_prepare(self.ctx, self.anc if anc is None else anc,
                                      self.resampled if resampled is None else resampled, t, next_pos, self.slot)

    def paged_state(self):
        """(table [R, M], refcnt [B*Q]) as numpy, after synchronising."""
        torch.cuda.synchronize()
        tab, ref, M, Q, _ = smc.smc_paged_view(self.ctx)
        base = (self.paged_ws.data_ptr() + 255) & ~255
        flat = self.paged_ws[base - self.paged_ws.data_ptr():]
        t0 = tab - base
        r0 = ref - base
        table = flat[t0:t0 + self.R * M * 4].view(torch.int32).reshape(self.R, M).cpu().numpy()
        refcnt = flat[r0:r0 + self.B * Q * 4].view(torch.int32).cpu().numpy()
        return table, refcnt

    def parity_view(self):
        """int32 [R] device tensor aliasing the context's parity words (no copy, no synchronisation)."""
        off = smc.smc_kv_parity(self.ctx) - self.workspace.data_ptr()
        return self.workspace[off:off + 4 * self.R].view(torch.int32)

    def append(self, k_tensor, v_tensor, k_new, v_new, pos):
        """k_new / v_new: [R, H, D] bf16 views whose rows may be strided; v_tensor = -1 writes K only."""
        assert k_new.stride(-1) == 1 and k_new.stride(1) == k_new.shape[2]
        if v_tensor >= 0:
            assert v_new.stride(-1) == 1 and v_new.stride(1) == v_new.shape[2]
        smc.smc_kv_append(self.ctx, k_tensor, v_tensor, k_new, k_new.stride(0), v_new if v_tensor >= 0 else None,
                          v_new.stride(0) if v_tensor >= 0 else 0, pos)

    def attention(self, k_tensor, v_tensor, q, length, scale):
        """Decode attention over the context's cache; q: bf16 [R, Hq, D] device tensor; returns float32 [R, Hq, D]."""
        Hq = q.shape[1]
        nbytes = smc.smc_attn_workspace_bytes(self.cfg, Hq)
        if nbytes == 0:
            raise ValueError("invalid attention geometry")
        if getattr(self, "_attn_ws", None) is None or self._attn_ws.numel() < nbytes:
            self._attn_ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        smc.smc_attn_decode(self.ctx, k_tensor, v_tensor, q, Hq, length, scale, self._attn_ws, nbytes, out)
        return out

    def final_draw(self, t):
        smc.smc_final_draw(self.ctx, t, self.choice)

    def log_Zhat(self):
        """log of the normalising-constant estimate per prompt (numpy [B]), computed by the library."""
        out = np.empty(self.B, np.float64)
        smc.smc_get_log_zhat(self.ctx, out)
        return out

    def banked_log_Zhat(self):
        """The part of the estimate accumulated at the resampling times so far (what a resumed run restores)."""
        out = np.empty(self.B, np.float64)
        smc.smc_get_log_zhat(self.ctx, None, out)
        return out

    def set_banked_log_Zhat(self, x):
        smc.smc_set_log_zhat(self.ctx, np.ascontiguousarray(x, np.float64))

    def done(self):
        d = np.empty(self.R, np.int32)
        smc.smc_get_done(self.ctx, d)
        return d

    def set_done(self, d):
        smc.smc_set_done(self.ctx, np.ascontiguousarray(d, np.int32))

    # ---- inspection ---------------------------------------------------------------------------------------
    def state(self):
        logW = np.empty(self.R, np.float64); cum = np.empty(self.R, np.float64); par = np.empty(self.R, np.int32)
        smc.smc_get_state(self.ctx, logW, cum, par)
        return logW, cum, par

    def set_state(self, logW=None, cumlogp=None):
        smc.smc_set_state(self.ctx, None if logW is None else np.ascontiguousarray(logW, np.float64),
                          None if cumlogp is None else np.ascontiguousarray(cumlogp, np.float64))

    def diag(self):
        R = self.R
        d = dict(delta=np.empty(R), logZ1=np.empty(R), logZb=np.empty(R), second=np.empty(R, np.int32),
                 gap=np.empty(R), counters=np.zeros(4, np.uint64))
        smc.smc_get_diag(self.ctx, d["delta"], d["logZ1"], d["logZb"], d["second"], d["gap"], d["counters"])
        return d

    def live_hist(self):
        """[R, T_max] numpy: each row taken from its live buffer."""
        _, _, par = self.state()
        A, Bh = self.histA.cpu().numpy(), self.histB.cpu().numpy()
        sel = par.astype(bool)
        return np.where(sel[:, None], Bh, A)

    def live_kv(self, tensor, rows=None):
        """numpy uint16 view of the live rows of one KV tensor (all rows, or the given ones)."""
        _, _, par = self.state()
        rows = np.arange(self.R) if rows is None else np.asarray(rows)
        out = []
        for r in rows:
            src = self.kvB[tensor] if par[r] else self.kvA[tensor]
            out.append(src[int(r)].view(torch.int16).cpu().numpy().view(np.uint16))
        return np.stack(out)


def to_device_logits(x, dtype, device="cuda"):
    """numpy logits (uint16 bf16 bits or float32) -> torch tensor on the device with the same bits."""
    if dtype == "bf16":
        return torch.as_tensor(np.ascontiguousarray(x).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.as_tensor(np.ascontiguousarray(x, np.float32)).to(device)
