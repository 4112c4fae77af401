"""Python face of the CPU oracle (TEST INFRASTRUCTURE, not the product).

Thin ctypes calls into power_smc_oracle.c plus a small state machine that strings the
steps of Algorithm 1 together in the paper's order.  Only tests, the smoke check and
the bench's cpu_baseline leg may import this module; it never imports the HIP package.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_uniform.restype = C.c_double
        L.orc_uniform.argtypes = [C.c_uint32]
        L.orc_gumbel.restype = C.c_double
        L.orc_gumbel.argtypes = [C.c_uint32]
        L.orc_random_word.restype = C.c_uint32
        L.orc_random_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_logsumexp.restype = C.c_double
        L.orc_logsumexp.argtypes = [C.c_void_p, C.c_int64, C.c_double]
        _lib = L
    return _lib


_DT = {"bf16": 0, "f32": 1, "f64": 2}
_NP = {"bf16": np.uint16, "f32": np.float32, "f64": np.float64}


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def threads():
    return int(lib().orc_threads())


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) for x in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def random_word(seed, t, r, v, domain=0):
    return int(lib().orc_random_word(int(seed), int(t), int(r), int(v), int(domain)))


def uniform(x):
    return float(lib().orc_uniform(int(x)))


def gumbel(x):
    return float(lib().orc_gumbel(int(x)))


def logsumexp(x, scale=1.0):
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(lib().orc_logsumexp(_p(x), x.size, float(scale)))


def beta_of(alpha_t, tau_t):
    """beta = 1/tau; tau <= 0 selects the locally optimal proposal tau = 1/alpha (Thm 1), i.e. beta = alpha exactly."""
    return float(alpha_t) if tau_t <= 0 else 1.0 / float(tau_t)


def vocab_row(logits, dtype, beta, alpha, seed, t, r, forced=-1):
    """One particle's vocabulary pass; returns a dict (token, second, logZ1, logZb, logp, logq, delta, gap)."""
    logits = np.ascontiguousarray(logits, dtype=_NP[dtype])
    out = (C.c_int32 * 2)()
    res = (C.c_double * 6)()
    lib().orc_vocab_row(_p(logits), _DT[dtype], C.c_int32(logits.size), C.c_double(beta), C.c_double(alpha),
                        C.c_uint64(int(seed)), C.c_int32(t), C.c_int32(r), C.c_int32(forced), out, res)
    return dict(token=out[0], second=out[1], logZ1=res[0], logZb=res[1], logp=res[2], logq=res[3],
                delta=res[4], gap=res[5])


def ess(logW, B, N):
    logW = np.ascontiguousarray(logW, dtype=np.float64)
    e = np.empty(B, np.float64)
    lnw = np.empty(B * N, np.float64)
    lib().orc_ess(_p(logW), C.c_int32(B), C.c_int32(N), _p(e), _p(lnw))
    return e, lnw


def systematic(w, u0):
    w = np.ascontiguousarray(w, dtype=np.float64)
    A = np.empty(w.size, np.int32)
    lib().orc_systematic(_p(w), C.c_int32(w.size), C.c_double(u0), _p(A))
    return A


SCHEMES = {"systematic": 0, "stratified": 1, "multinomial": 2, "residual": 3}


def resample_scheme(w, scheme, seed, t, b):
    """Ancestors (local indices) of one prompt with normalised weights w under the named scheme."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    A = np.empty(w.size, np.int32)
    scratch = np.empty(w.size, np.float64)
    lib().orc_resample_scheme(_p(w), C.c_int32(w.size), C.c_int32(SCHEMES.get(scheme, scheme)), C.c_uint64(int(seed)),
                              C.c_int32(t), C.c_int32(b), _p(A), _p(scratch))
    return A


def survivors_in_place(A):
    """The permutation of an ancestor vector (local indices) in which every distinct ancestor keeps its own slot."""
    A = np.ascontiguousarray(A, np.int32)
    out = np.empty_like(A)
    lib().orc_survivors_in_place(_p(A), C.c_int32(A.size), _p(out))
    return out


def resample(logW, B, N, kappa, seed, t, scheme=0, in_place=False):
    """Returns (anc[R] global rows, resampled[B], ess[B], logW after reset)."""
    lw = np.array(logW, dtype=np.float64).copy()
    anc = np.empty(B * N, np.int32)
    flag = np.empty(B, np.int32)
    e = np.empty(B, np.float64)
    scratch = np.empty(2 * N, np.float64)
    lib().orc_resample(_p(lw), C.c_int32(B), C.c_int32(N), C.c_double(kappa), C.c_uint64(int(seed)),
                       C.c_int32(t), _p(anc), _p(flag), _p(e), _p(scratch), C.c_int32(SCHEMES.get(scheme, scheme)),
                       C.c_int32(1 if in_place else 0))
    return anc, flag, e, lw


def final_draw(logW, B, N, seed, t):
    logW = np.ascontiguousarray(logW, np.float64)
    out = np.empty(B, np.int32)
    lib().orc_final_draw(_p(logW), C.c_int32(B), C.c_int32(N), C.c_uint64(int(seed)), C.c_int32(t), _p(out))
    return out


def gather_kv(src, anc, resampled, N, valid_len, dst=None):
    """src: [R,H,S,D] array (any 1/2/4/8-byte dtype). Returns dst with resampled prompts' rows gathered."""
    R, H, S, D = src.shape
    if dst is None:
        dst = np.zeros_like(src)
    anc = np.ascontiguousarray(anc, np.int32)
    resampled = np.ascontiguousarray(resampled, np.int32)
    lib().orc_gather_kv(_p(src), _p(dst), _p(anc), _p(resampled), C.c_int32(R), C.c_int32(N), C.c_int32(H),
                        C.c_int32(S), C.c_int32(D), C.c_int32(src.dtype.itemsize), C.c_int32(valid_len))
    return dst


class OracleSMC:
    """Algorithm 1 for B independent prompts, state held in fp64 / numpy, one call per step of the path."""

    def __init__(self, B, N, V, T_max, kappa, seed, dtype="f32", kv=None, eos_id=-1, scheme="systematic",
                 in_place=False, skip_terminated_kv=False):
        self.B, self.N, self.V, self.T_max, self.R = B, N, V, T_max, B * N
        self.kappa, self.seed, self.dtype = float(kappa), int(seed), dtype
        self.logW = np.zeros(self.R, np.float64)          # Alg. 1: W~_0 = 1
        self.cumlogp = np.zeros(self.R, np.float64)       # log p(y_{1:t}) (Sec. 5.3)
        self.hist = np.zeros((self.R, T_max), np.int32)   # prefixes y_{1:t}
        self.kv = kv                                      # list of [R,H,S,D] arrays or None
        self.log_Zhat = np.zeros(B, np.float64)           # running log of the normalising-constant estimate
        self.scheme = scheme                              # resampling scheme (App. E); the paper uses systematic
        self.in_place = bool(in_place)                    # survivors keep their slot (same particle system)
        self.eos_id = int(eos_id)                         # -1: EOS is not special
        self.done = np.zeros(self.R, np.int32)            # Alg. 1 termination flags
        # Reading of App. D ("skipping cache updates" for terminated particles) as an option: when on, the reorder is
        # not required to move the KV rows of a terminated ancestor (nothing reads them again), so the KV content of a
        # row that continues one is unspecified from then on.  kv_specified[r] says whether row r's KV bytes are
        # defined by the gather; with the option off (the default: Alg. 1 "reorder KV cache by A" as written) all are.
        self.skip_terminated_kv = bool(skip_terminated_kv) and self.eos_id >= 0
        self.kv_specified = np.ones(self.R, bool)

    def step(self, logits, t, alpha_t, alpha_prev, tau_t=-1.0, row_stride=None):
        """a0..a2. logits: [R, >=V] array of self.dtype storage. Returns dict of per-row arrays."""
        logits = np.ascontiguousarray(logits, dtype=_NP[self.dtype])
        stride = logits.shape[1] if row_stride is None else row_stride
        R = self.R
        tokens = np.empty(R, np.int32); second = np.empty(R, np.int32)
        gap = np.empty(R, np.float64); delta = np.empty(R, np.float64)
        beta = beta_of(alpha_t, tau_t)
        lib().orc_step(_p(logits), C.c_int32(_DT[self.dtype]), C.c_int64(stride), C.c_int32(R), C.c_int32(self.V),
                       C.c_double(alpha_t), C.c_double(alpha_prev), C.c_double(beta), C.c_uint64(self.seed),
                       C.c_int32(t), _p(self.logW), _p(self.cumlogp), _p(self.hist), C.c_int32(self.T_max),
                       _p(tokens), _p(second), _p(gap), _p(delta), C.c_int32(self.eos_id), _p(self.done))
        return dict(tokens=tokens, second=second, gap=gap, delta=delta)

    def ess(self):
        return ess(self.logW, self.B, self.N)

    def resample(self, t):
        """a4; also accumulates log Zhat += L1 - log N for prompts that resample."""
        L1 = np.array([logsumexp(self.logW[b * self.N:(b + 1) * self.N]) for b in range(self.B)])
        anc, flag, e, lw = resample(self.logW, self.B, self.N, self.kappa, self.seed, t, self.scheme, self.in_place)
        self.log_Zhat += np.where(flag != 0, L1 - np.log(self.N), 0.0)
        self.logW = lw
        return anc, flag, e

    def log_Z_estimate(self):
        """log of the SMC estimate of Z_alpha: resampling-time factors times the current mean weight."""
        L1 = np.array([logsumexp(self.logW[b * self.N:(b + 1) * self.N]) for b in range(self.B)])
        return self.log_Zhat + L1 - np.log(self.N)

    def final_draw(self, t):
        """Output line of Alg. 1: one particle per prompt drawn from the final weights (global row indices)."""
        return final_draw(self.logW, self.B, self.N, self.seed, t)

    def reindex(self, anc, resampled, valid_len, t):
        """a5: prefixes, cumulative log p and every KV tensor gathered by ancestor for resampled prompts."""
        R, N = self.R, self.N
        hist2 = self.hist.copy(); cum2 = self.cumlogp.copy(); done2 = self.done.copy()
        anc = np.ascontiguousarray(anc, np.int32); resampled = np.ascontiguousarray(resampled, np.int32)
        # which rows hold gather-defined KV bytes afterwards: a row that receives another row's data inherits that
        # row's status, except that data of a terminated ancestor need not be moved when the option is on
        spec2 = self.kv_specified.copy()
        for k in range(R):
            a = int(anc[k])
            if resampled[k // N] and a != k and (k // N) * N <= a < (k // N + 1) * N:
                spec2[k] = self.kv_specified[a] and not (self.skip_terminated_kv and self.done[a] != 0)
        self.kv_specified = spec2
        lib().orc_gather_state(_p(self.hist), _p(hist2), C.c_int32(self.T_max), C.c_int32(t),
                               _p(self.cumlogp), _p(cum2), _p(anc), _p(resampled), C.c_int32(R), C.c_int32(N),
                               _p(self.done), _p(done2))
        self.hist, self.cumlogp, self.done = hist2, cum2, done2
        if self.kv is not None:
            new = []
            for ten in self.kv:
                dst = ten.copy()
                gather_kv(ten, anc, resampled, N, valid_len, dst)
                new.append(dst)
            self.kv = new
