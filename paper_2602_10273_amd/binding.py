"""ctypes binding of libpower_smc.so: the same names as the C ABI, argument marshalling only.

PyTorch is used by callers for device memory and streams; this module only turns tensors into pointers.
If the HIP library has not been built the import of the library fails loudly -- there is no fallback path.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpower_smc.so")

SMC_OK = 0
SMC_BF16, SMC_F32 = 0, 1
STATUS = {0: "SMC_OK", 1: "SMC_E_NULL", 2: "SMC_E_SHAPE", 3: "SMC_E_DTYPE", 4: "SMC_E_ALIGN", 5: "SMC_E_RANGE",
          6: "SMC_E_STATE", 7: "SMC_E_HIP"}

EXPORTS = ["smc_workspace_bytes", "smc_init", "smc_destroy", "smc_kv_bind", "smc_step", "smc_ess", "smc_resample",
           "smc_kv_reindex", "smc_final_draw", "smc_get_done", "smc_set_done", "smc_ess_from", "smc_resample_from", "smc_get_state", "smc_set_state", "smc_get_diag",
           "smc_set_tuning", "smc_set_resampler", "smc_set_ancestor_order", "smc_set_gather_tuning", "smc_profile_enable", "smc_profile_read", "smc_status_str",
           "smc_paged_workspace_bytes", "smc_paged_pool_bytes", "smc_paged_bind", "smc_paged_prepare_append",
           "smc_paged_reindex", "smc_paged_reindex_prepare", "smc_paged_view", "smc_paged_check", "smc_hbm_probe",
           "smc_attn_workspace_bytes", "smc_attn_decode", "smc_kv_parity", "smc_kv_append", "smc_step_noalloc",
           "smc_get_log_zhat", "smc_set_log_zhat", "smc_set_kv_skip_terminated",
           "smc_step_resample", "smc_step_resample_reindex", "smc_set_schedule", "smc_set_device_step", "smc_advance_step", "smc_get_device_step"]


class smc_config(C.Structure):
    _fields_ = [("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32), ("T_max", C.c_int32),
                ("logits_dtype", C.c_int32), ("eos_id", C.c_int32), ("kappa", C.c_double), ("seed", C.c_uint64),
                ("kv_tensors", C.c_int32), ("kv_H", C.c_int32), ("kv_S", C.c_int32), ("kv_D", C.c_int32),
                ("kv_elem_bytes", C.c_int32), ("reserved1", C.c_int32)]


class SMCError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn} -> {STATUS.get(status, status)}")


_lib = None


def lib():
    """The loaded library; raises if it was not built (python -c 'import __graft_entry__ as g; g.build()')."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build the HIP library first (no CPU fallback exists)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double, C.c_uint64
        L.smc_workspace_bytes.restype = C.c_size_t
        L.smc_workspace_bytes.argtypes = [C.POINTER(smc_config)]
        L.smc_init.argtypes = [C.POINTER(smc_config), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.smc_destroy.argtypes = [vp]
        L.smc_kv_bind.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, vp]
        L.smc_step.argtypes = [vp, vp, i64, i32, f64, f64, f64, vp]
        L.smc_step_noalloc.argtypes = [C.POINTER(smc_config), vp, vp, i64, i32, f64, f64, f64, vp, vp, vp, vp]
        L.smc_step_resample.argtypes = [vp, vp, i64, i32, f64, f64, f64, vp, vp, vp, vp]
        L.smc_step_resample_reindex.argtypes = [vp, vp, i64, i32, f64, f64, f64, i32, vp, vp, vp, vp]
        L.smc_set_schedule.argtypes = [vp, vp, i32]
        L.smc_set_device_step.argtypes = [vp, i32, i32]
        L.smc_advance_step.argtypes = [vp]
        L.smc_get_device_step.argtypes = [vp, C.POINTER(i32)]
        L.smc_ess.argtypes = [vp, vp, vp]
        L.smc_resample.argtypes = [vp, i32, vp, vp, vp]
        L.smc_kv_reindex.argtypes = [vp, vp, vp, i32, i32]
        L.smc_final_draw.argtypes = [vp, i32, vp]
        L.smc_get_log_zhat.argtypes = [vp, vp, vp]
        L.smc_set_log_zhat.argtypes = [vp, vp]
        L.smc_set_kv_skip_terminated.argtypes = [vp, i32]
        L.smc_get_done.argtypes = [vp, vp]
        L.smc_set_done.argtypes = [vp, vp]
        L.smc_ess_from.argtypes = [vp, vp, vp, vp]
        L.smc_resample_from.argtypes = [vp, vp, i32, vp, vp, vp]
        L.smc_get_state.argtypes = [vp, vp, vp, vp]
        L.smc_set_state.argtypes = [vp, vp, vp]
        L.smc_get_diag.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.smc_set_tuning.argtypes = [vp, i32, i32, i32]
        L.smc_set_resampler.argtypes = [vp, i32]
        L.smc_set_ancestor_order.argtypes = [vp, i32]
        L.smc_set_gather_tuning.argtypes = [vp, i32, i32]
        L.smc_profile_enable.argtypes = [vp, i32]
        L.smc_profile_read.argtypes = [vp, i32, C.POINTER(f64), C.POINTER(i64)]
        L.smc_paged_workspace_bytes.restype = C.c_size_t
        L.smc_paged_workspace_bytes.argtypes = [C.POINTER(smc_config), i32]
        L.smc_paged_pool_bytes.restype = C.c_size_t
        L.smc_paged_pool_bytes.argtypes = [C.POINTER(smc_config), i32]
        L.smc_paged_bind.argtypes = [vp, C.POINTER(vp), i32, vp, C.c_size_t, i32]
        L.smc_paged_prepare_append.argtypes = [vp, i32, vp]
        L.smc_paged_reindex.argtypes = [vp, vp, vp, i32]
        L.smc_paged_reindex_prepare.argtypes = [vp, vp, vp, i32, i32, vp]
        L.smc_paged_view.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.smc_paged_check.argtypes = [vp, C.POINTER(i32)]
        L.smc_attn_workspace_bytes.restype = C.c_size_t
        L.smc_attn_workspace_bytes.argtypes = [C.POINTER(smc_config), i32]
        L.smc_attn_decode.argtypes = [vp, i32, i32, vp, i32, i32, C.c_float, vp, C.c_size_t, vp]
        L.smc_kv_append.argtypes = [vp, i32, i32, vp, C.c_int64, vp, C.c_int64, i32]
        L.smc_kv_parity.argtypes = [vp, C.POINTER(vp)]
        L.smc_hbm_probe.argtypes = [i32, vp, C.c_size_t, vp, C.POINTER(f64)]
        L.smc_status_str.restype = C.c_char_p
        L.smc_status_str.argtypes = [C.c_int]
        for name in EXPORTS:
            if name not in ("smc_workspace_bytes", "smc_paged_workspace_bytes", "smc_paged_pool_bytes", "smc_attn_workspace_bytes",
                            "smc_status_str"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(x):
    """torch tensor / numpy array / int / None -> address."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _check(fn, st):
    if st != SMC_OK:
        raise SMCError(fn, st)


def make_config(B, N, V, T_max, logits_dtype, kappa, seed, kv_tensors=0, kv_H=0, kv_S=0, kv_D=0, kv_elem_bytes=2,
                eos_id=-1):
    dt = {"bf16": SMC_BF16, "f32": SMC_F32}.get(logits_dtype, logits_dtype)
    return smc_config(B, N, V, T_max, dt, int(eos_id), float(kappa), int(seed) & 0xFFFFFFFFFFFFFFFF, kv_tensors, kv_H, kv_S,
                      kv_D, kv_elem_bytes, 0)


# ---- one function per C entry point, same names --------------------------------------------------------------
def smc_workspace_bytes(cfg):
    return int(lib().smc_workspace_bytes(C.byref(cfg)))


def smc_init(cfg, d_workspace, workspace_bytes, hip_stream=None):
    ctx = C.c_void_p()
    _check("smc_init", lib().smc_init(C.byref(cfg), _ptr(d_workspace), workspace_bytes, hip_stream, C.byref(ctx)))
    return ctx


def smc_destroy(ctx):
    _check("smc_destroy", lib().smc_destroy(ctx))


def smc_kv_bind(ctx, bufA, bufB, d_histA=None, d_histB=None):
    n = len(bufA)
    A = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in bufA])
    Bp = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in bufB])
    _check("smc_kv_bind", lib().smc_kv_bind(ctx, A if n else None, Bp if n else None, _ptr(d_histA), _ptr(d_histB)))


def smc_step(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out):
    _check("smc_step", lib().smc_step(ctx, _ptr(d_logits), row_stride_elems, t, alpha_t, alpha_prev, tau_t,
                                      _ptr(d_tokens_out)))


def smc_step_noalloc(cfg, hip_stream, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_logW_inout,
                     d_cumlogp_inout, d_done_inout, d_tokens_out):
    _check("smc_step_noalloc", lib().smc_step_noalloc(C.byref(cfg), hip_stream, _ptr(d_logits), row_stride_elems, t, alpha_t,
                                                      alpha_prev, tau_t, _ptr(d_logW_inout), _ptr(d_cumlogp_inout),
                                                      _ptr(d_done_inout), _ptr(d_tokens_out)))


def smc_step_resample(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out, d_anc_out,
                      d_resampled_out, d_ess_out=None):
    _check("smc_step_resample", lib().smc_step_resample(ctx, _ptr(d_logits), row_stride_elems, t, alpha_t, alpha_prev, tau_t,
                                                        _ptr(d_tokens_out), _ptr(d_anc_out), _ptr(d_resampled_out),
                                                        _ptr(d_ess_out)))


def smc_step_resample_reindex(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, valid_len, d_tokens_out,
                              d_anc_out, d_resampled_out, d_ess_out=None):
    _check("smc_step_resample_reindex",
           lib().smc_step_resample_reindex(ctx, _ptr(d_logits), row_stride_elems, t, alpha_t, alpha_prev, tau_t, valid_len,
                                           _ptr(d_tokens_out), _ptr(d_anc_out), _ptr(d_resampled_out), _ptr(d_ess_out)))


def smc_set_schedule(ctx, h_alpha):
    import numpy as np
    a = np.ascontiguousarray(h_alpha, np.float64)
    _check("smc_set_schedule", lib().smc_set_schedule(ctx, _ptr(a), a.size))


def smc_set_device_step(ctx, enable=1, t=1):
    _check("smc_set_device_step", lib().smc_set_device_step(ctx, enable, t))


def smc_advance_step(ctx):
    _check("smc_advance_step", lib().smc_advance_step(ctx))


def smc_get_device_step(ctx):
    t = C.c_int32()
    _check("smc_get_device_step", lib().smc_get_device_step(ctx, C.byref(t)))
    return t.value


def smc_ess(ctx, d_ess_out, d_lognormw_out=None):
    _check("smc_ess", lib().smc_ess(ctx, _ptr(d_ess_out), _ptr(d_lognormw_out)))


def smc_resample(ctx, t, d_anc_out, d_resampled_out, d_ess_out=None):
    _check("smc_resample", lib().smc_resample(ctx, t, _ptr(d_anc_out), _ptr(d_resampled_out), _ptr(d_ess_out)))


def smc_kv_reindex(ctx, d_anc, d_resampled, valid_len, t):
    _check("smc_kv_reindex", lib().smc_kv_reindex(ctx, _ptr(d_anc), _ptr(d_resampled), valid_len, t))


def smc_final_draw(ctx, t, d_choice_out):
    _check("smc_final_draw", lib().smc_final_draw(ctx, t, _ptr(d_choice_out)))


def smc_get_log_zhat(ctx, h_logZhat=None, h_banked=None):
    _check("smc_get_log_zhat", lib().smc_get_log_zhat(ctx, _ptr(h_logZhat), _ptr(h_banked)))


def smc_set_log_zhat(ctx, h_banked):
    _check("smc_set_log_zhat", lib().smc_set_log_zhat(ctx, _ptr(h_banked)))


def smc_set_kv_skip_terminated(ctx, enable=1):
    _check("smc_set_kv_skip_terminated", lib().smc_set_kv_skip_terminated(ctx, enable))


def smc_get_done(ctx, h_done):
    _check("smc_get_done", lib().smc_get_done(ctx, _ptr(h_done)))


def smc_set_done(ctx, h_done):
    _check("smc_set_done", lib().smc_set_done(ctx, _ptr(h_done)))


def smc_ess_from(ctx, d_logW, d_ess_out, d_lognormw_out=None):
    _check("smc_ess_from", lib().smc_ess_from(ctx, _ptr(d_logW), _ptr(d_ess_out), _ptr(d_lognormw_out)))


def smc_resample_from(ctx, d_logW_inout, t, d_anc_out, d_resampled_out, d_ess_out=None):
    _check("smc_resample_from", lib().smc_resample_from(ctx, _ptr(d_logW_inout), t, _ptr(d_anc_out),
                                                        _ptr(d_resampled_out), _ptr(d_ess_out)))


def smc_get_state(ctx, h_logW=None, h_cumlogp=None, h_parity=None):
    _check("smc_get_state", lib().smc_get_state(ctx, _ptr(h_logW), _ptr(h_cumlogp), _ptr(h_parity)))


def smc_set_state(ctx, h_logW=None, h_cumlogp=None):
    _check("smc_set_state", lib().smc_set_state(ctx, _ptr(h_logW), _ptr(h_cumlogp)))


def smc_get_diag(ctx, h_delta=None, h_logZ1=None, h_logZb=None, h_second=None, h_gap=None, h_counters=None):
    _check("smc_get_diag", lib().smc_get_diag(ctx, _ptr(h_delta), _ptr(h_logZ1), _ptr(h_logZb), _ptr(h_second),
                                              _ptr(h_gap), _ptr(h_counters)))


def smc_set_tuning(ctx, n_split=0, dense=0, wg_waves=0):
    _check("smc_set_tuning", lib().smc_set_tuning(ctx, n_split, dense, wg_waves))


def smc_set_resampler(ctx, scheme=0):
    _check("smc_set_resampler", lib().smc_set_resampler(ctx, scheme))


def smc_set_ancestor_order(ctx, order=0):
    _check("smc_set_ancestor_order", lib().smc_set_ancestor_order(ctx, order))


def smc_set_gather_tuning(ctx, wgs_per_cu=8, variant=0):
    _check("smc_set_gather_tuning", lib().smc_set_gather_tuning(ctx, wgs_per_cu, variant))


def smc_profile_enable(ctx, enable=1):
    _check("smc_profile_enable", lib().smc_profile_enable(ctx, enable))


def smc_profile_read(ctx, kind):
    """Returns (total_ms, launches) of kernel kind 0 (vocabulary pass) or 1 (KV gather) since the last read."""
    ms, n = C.c_double(), C.c_int64()
    _check("smc_profile_read", lib().smc_profile_read(ctx, kind, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def smc_status_str(status):
    return lib().smc_status_str(status).decode()


def smc_paged_workspace_bytes(cfg, page_len):
    return int(lib().smc_paged_workspace_bytes(C.byref(cfg), page_len))


def smc_paged_pool_bytes(cfg, page_len):
    return int(lib().smc_paged_pool_bytes(C.byref(cfg), page_len))


def smc_paged_bind(ctx, pools, page_len, d_workspace, workspace_bytes, len0=0):
    P = (C.c_void_p * max(len(pools), 1))(*[_ptr(t) for t in pools])
    _check("smc_paged_bind", lib().smc_paged_bind(ctx, P, page_len, _ptr(d_workspace), workspace_bytes, len0))


def smc_paged_prepare_append(ctx, pos, d_slot_out):
    _check("smc_paged_prepare_append", lib().smc_paged_prepare_append(ctx, pos, _ptr(d_slot_out)))


def smc_paged_reindex(ctx, d_anc, d_resampled, t):
    _check("smc_paged_reindex", lib().smc_paged_reindex(ctx, _ptr(d_anc), _ptr(d_resampled), t))


def smc_paged_reindex_prepare(ctx, d_anc, d_resampled, t, next_pos, d_slot_out):
    _check("smc_paged_reindex_prepare",
           lib().smc_paged_reindex_prepare(ctx, _ptr(d_anc), _ptr(d_resampled), t, next_pos, _ptr(d_slot_out)))


def smc_paged_view(ctx):
    """(table device address, refcnt device address, pages per row, pages per prompt, positions appended)."""
    tab, ref = C.c_void_p(), C.c_void_p()
    M, Q, n = C.c_int32(), C.c_int32(), C.c_int32()
    _check("smc_paged_view", lib().smc_paged_view(ctx, C.byref(tab), C.byref(ref), C.byref(M), C.byref(Q), C.byref(n)))
    return tab.value, ref.value, M.value, Q.value, n.value


def smc_paged_check(ctx):
    n = C.c_int32()
    _check("smc_paged_check", lib().smc_paged_check(ctx, C.byref(n)))
    return n.value


def smc_hbm_probe(kind, d_buf, nbytes, hip_stream=None):
    g = C.c_double()
    _check("smc_hbm_probe", lib().smc_hbm_probe(kind, _ptr(d_buf), nbytes, hip_stream, C.byref(g)))
    return g.value


def smc_attn_workspace_bytes(cfg, n_q_heads):
    return int(lib().smc_attn_workspace_bytes(C.byref(cfg), n_q_heads))


def smc_attn_decode(ctx, k_tensor, v_tensor, d_q, n_q_heads, length, scale, d_workspace, workspace_bytes, d_out):
    _check("smc_attn_decode", lib().smc_attn_decode(ctx, k_tensor, v_tensor, _ptr(d_q), n_q_heads, length, scale,
                                                    _ptr(d_workspace), workspace_bytes, _ptr(d_out)))


def smc_kv_append(ctx, k_tensor, v_tensor, d_k_new, k_row_stride, d_v_new, v_row_stride, pos):
    _check("smc_kv_append", lib().smc_kv_append(ctx, k_tensor, v_tensor, _ptr(d_k_new), k_row_stride,
                                                None if d_v_new is None else _ptr(d_v_new), v_row_stride, pos))


def smc_kv_parity(ctx):
    """Device address of the parity words (int32 [R])."""
    p = C.c_void_p()
    _check("smc_kv_parity", lib().smc_kv_parity(ctx, C.byref(p)))
    return p.value
