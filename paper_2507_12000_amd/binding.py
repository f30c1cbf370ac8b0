"""ctypes binding of libdssd.so (include/dssd.h, include/dssd_aux.h).  Argument marshalling only: every step of
the verification path runs in the library's HIP kernels.  PyTorch tensors are used for device
memory and the launch stream, nothing else.  There is no CPU fallback: if the library is not
built, or no GPU is present, the calls raise.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdssd.so")

DSSD_F32, DSSD_BF16, DSSD_F16 = 0, 1, 2
DSSD_OK, DSSD_EINVAL, DSSD_EALIGN, DSSD_ENOMEM, DSSD_EHIP, DSSD_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
SESSION_BAD_TOKEN, SESSION_ZERO_RESIDUAL, SESSION_BAD_OFFSETS, SESSION_BAD_ROW = 1, 2, 4, 8
SESSION_SUPPORT_OVERFLOW = 16
FLAG_SPARSE_SUPPORT = 1
FLAG_EARLY_EXIT = 2
MAX_SUPPORT = 64
STATIC_SCRATCH_BYTES = 8 << 20
K_ROW_STATS, K_ACCEPT, K_RESID_MASS, K_RESID_PICK, K_BONUS_PICK = 0, 1, 2, 3, 4
K_EXPORT_P, K_DEVICE_MASS, K_DEVICE_PICK, K_FUSED_STEP, K_READ_PROBE, K_ROW_STATS_BLOCK, K_TOPK_STEP, K_COUNT = 5, 6, 7, 8, 9, 10, 11, 12

# every symbol include/dssd.h and include/dssd_aux.h declare
EXPORTS = ("dssd_workspace_bytes", "dssd_create", "dssd_destroy", "dssd_verify_batch",
           "dssd_residual_sample", "dssd_bonus_sample", "dssd_export_p_rows",
           "dssd_residual_sample_from_p", "dssd_step_fused", "dssd_step_static", "dssd_set_fused_limit", "dssd_set_fused_pair_limit", "dssd_set_stream_occupancy", "dssd_set_early_exit_schedule", "dssd_random_words", "dssd_step_topk", "dssd_status_str", "dssd_profile_enable",
           "dssd_profile_read", "dssd_profile_reset", "dssd_kernel_name", "dssd_probe_read")


class dssd_batch(C.Structure):
    _fields_ = [("B", C.c_int32), ("V", C.c_int32), ("gamma", C.c_int32), ("logits_dtype", C.c_int32),
                ("total_drafts", C.c_int64), ("draft_offsets", C.c_void_p), ("logits", C.c_void_p),
                ("draft_probs", C.c_void_p), ("draft_tokens", C.c_void_p),
                ("inv_temperature", C.c_void_p), ("seed", C.c_uint64), ("step", C.c_uint64),
                ("session_base", C.c_uint32), ("flags", C.c_uint32), ("draft_q_tok", C.c_void_p),
                ("step_counter", C.c_void_p)]


class dssd_device_batch(C.Structure):
    _fields_ = [("B", C.c_int32), ("V", C.c_int32), ("gamma", C.c_int32), ("p_dtype", C.c_int32),
                ("total_drafts", C.c_int64), ("draft_offsets", C.c_void_p), ("draft_probs", C.c_void_p),
                ("p_rows", C.c_void_p), ("accepted_len", C.c_void_p), ("rejected", C.c_void_p),
                ("seed", C.c_uint64), ("step", C.c_uint64), ("session_base", C.c_uint32),
                ("reserved", C.c_uint32), ("out_token", C.c_void_p), ("status", C.c_void_p),
                ("step_counter", C.c_void_p)]


class dssd_topk_batch(C.Structure):
    _fields_ = [("B", C.c_int32), ("k", C.c_int32), ("gamma", C.c_int32), ("V", C.c_int32),
                ("total_drafts", C.c_int64), ("draft_offsets", C.c_void_p), ("p_idx", C.c_void_p),
                ("p_logit", C.c_void_p), ("q_idx", C.c_void_p), ("q_prob", C.c_void_p),
                ("draft_tokens", C.c_void_p), ("inv_temperature", C.c_void_p), ("seed", C.c_uint64),
                ("step", C.c_uint64), ("session_base", C.c_uint32), ("reserved", C.c_uint32),
                ("step_counter", C.c_void_p)]


class dssd_out(C.Structure):
    _fields_ = [("accepted_len", C.c_void_p), ("rejected", C.c_void_p), ("out_token", C.c_void_p),
                ("row_stats", C.c_void_p), ("p_tok", C.c_void_p), ("q_tok", C.c_void_p),
                ("status", C.c_void_p)]


class DssdError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_str(code)} ({code})")


_lib = None


def load():
    """Load libdssd.so, compiling it first if it has never been built.  Raises if neither works."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        # nothing built yet: compile it now (hipcc); if that is impossible there is nothing to run
        try:
            from . import build as _build
            _build.build()
        except Exception as e:
            raise RuntimeError(f"{LIB_PATH} is missing and could not be built ({e}); build it with "
                               "`python paper_2507_12000_amd/build.py` (there is no CPU fallback)") from e
    L = C.CDLL(LIB_PATH)
    P = C.c_void_p
    L.dssd_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
    L.dssd_workspace_bytes.restype = C.c_size_t
    L.dssd_create.argtypes = [C.POINTER(P), C.c_int, C.c_int64, C.c_int32]
    L.dssd_create.restype = C.c_int
    L.dssd_destroy.argtypes = [P]
    L.dssd_destroy.restype = None
    L.dssd_set_fused_limit.argtypes = [P, C.c_int64]
    L.dssd_set_fused_limit.restype = C.c_int
    L.dssd_random_words.argtypes = [P, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32, P, P]
    L.dssd_random_words.restype = C.c_int
    L.dssd_set_early_exit_schedule.argtypes = [P, C.POINTER(C.c_int32), C.c_int32]
    L.dssd_set_early_exit_schedule.restype = C.c_int
    L.dssd_set_stream_occupancy.argtypes = [P, C.c_int32, C.c_int32]
    L.dssd_set_stream_occupancy.restype = C.c_int
    L.dssd_set_fused_pair_limit.argtypes = [P, C.c_int64]
    L.dssd_set_fused_pair_limit.restype = C.c_int
    for name in ("dssd_verify_batch", "dssd_residual_sample", "dssd_bonus_sample", "dssd_step_fused"):
        f = getattr(L, name)
        f.argtypes = [P, C.POINTER(dssd_batch), C.POINTER(dssd_out), P]
        f.restype = C.c_int
    L.dssd_step_static.argtypes = [C.POINTER(dssd_batch), C.POINTER(dssd_out), P]
    L.dssd_step_static.restype = C.c_int
    L.dssd_step_topk.argtypes = [P, C.POINTER(dssd_topk_batch), C.POINTER(dssd_out), P]
    L.dssd_step_topk.restype = C.c_int
    L.dssd_export_p_rows.argtypes = [P, C.POINTER(dssd_batch), P, C.c_int32, P]
    L.dssd_export_p_rows.restype = C.c_int
    L.dssd_residual_sample_from_p.argtypes = [P, C.POINTER(dssd_device_batch), P]
    L.dssd_residual_sample_from_p.restype = C.c_int
    L.dssd_probe_read.argtypes = [P, P, C.c_size_t, C.c_int32, C.c_int32, P]
    L.dssd_probe_read.restype = C.c_int
    L.dssd_status_str.argtypes = [C.c_int]
    L.dssd_status_str.restype = C.c_char_p
    L.dssd_kernel_name.argtypes = [C.c_int]
    L.dssd_kernel_name.restype = C.c_char_p
    L.dssd_profile_enable.argtypes = [P, C.c_uint32]
    L.dssd_profile_enable.restype = C.c_int
    L.dssd_profile_reset.argtypes = [P]
    L.dssd_profile_reset.restype = C.c_int
    L.dssd_profile_read.argtypes = [P, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.dssd_profile_read.restype = C.c_int
    _lib = L
    return L


def status_str(code):
    return load().dssd_status_str(int(code)).decode()


def kernel_name(k):
    return load().dssd_kernel_name(int(k)).decode()


def dssd_workspace_bytes(max_rows, max_V, logits_dtype=DSSD_F32):
    return load().dssd_workspace_bytes(int(max_rows), int(max_V), int(logits_dtype))


def dssd_create(device, max_rows, max_V):
    h = C.c_void_p()
    rc = load().dssd_create(C.byref(h), int(device), int(max_rows), int(max_V))
    if rc != DSSD_OK:
        raise DssdError(rc, "dssd_create")
    return h


def dssd_destroy(ctx):
    load().dssd_destroy(ctx)


def _call(name, ctx, batch, out, stream, check=True):
    rc = getattr(load(), name)(ctx, C.byref(batch) if batch is not None else None,
                               C.byref(out) if out is not None else None, C.c_void_p(stream or 0))
    if check and rc != DSSD_OK:
        raise DssdError(rc, name)
    return rc


def dssd_verify_batch(ctx, batch, out, stream=0, check=True):
    return _call("dssd_verify_batch", ctx, batch, out, stream, check)


def dssd_residual_sample(ctx, batch, out, stream=0, check=True):
    return _call("dssd_residual_sample", ctx, batch, out, stream, check)


def dssd_bonus_sample(ctx, batch, out, stream=0, check=True):
    return _call("dssd_bonus_sample", ctx, batch, out, stream, check)


def dssd_step_fused(ctx, batch, out, stream=0, check=True):
    return _call("dssd_step_fused", ctx, batch, out, stream, check)


def dssd_step_static(batch, out, stream=0, check=True):
    rc = load().dssd_step_static(C.byref(batch) if batch is not None else None,
                                 C.byref(out) if out is not None else None, C.c_void_p(stream or 0))
    if check and rc != DSSD_OK:
        raise DssdError(rc, "dssd_step_static")
    return rc


def dssd_set_fused_limit(ctx, max_blocks):
    return load().dssd_set_fused_limit(ctx, int(max_blocks))


def dssd_random_words(ctx, seed, step, session_first, position_first, n_sessions, n_positions, words_ptr, stream):
    return load().dssd_random_words(ctx, seed, step, session_first, position_first, n_sessions, n_positions,
                                    words_ptr, stream)


def dssd_step_topk(ctx, batch, out, stream=0, check=True):
    return _call("dssd_step_topk", ctx, batch, out, stream, check)


def dssd_set_early_exit_schedule(ctx, begin):
    """begin: first rows of the blocks, e.g. (0, 2, 6); () returns to the automatic choice."""
    arr = (C.c_int32 * max(len(begin), 1))(*begin)
    return load().dssd_set_early_exit_schedule(ctx, arr, len(begin))


def dssd_set_stream_occupancy(ctx, stats_waves_per_cu, resid_waves_per_cu):
    return load().dssd_set_stream_occupancy(ctx, int(stats_waves_per_cu), int(resid_waves_per_cu))


def dssd_set_fused_pair_limit(ctx, max_blocks):
    return load().dssd_set_fused_pair_limit(ctx, int(max_blocks))


def dssd_export_p_rows(ctx, batch, p_rows_ptr, p_dtype, stream=0, check=True):
    rc = load().dssd_export_p_rows(ctx, C.byref(batch), C.c_void_p(p_rows_ptr), int(p_dtype), C.c_void_p(stream or 0))
    if check and rc != DSSD_OK:
        raise DssdError(rc, "dssd_export_p_rows")
    return rc


def dssd_residual_sample_from_p(ctx, device_batch, stream=0, check=True):
    rc = load().dssd_residual_sample_from_p(ctx, C.byref(device_batch), C.c_void_p(stream or 0))
    if check and rc != DSSD_OK:
        raise DssdError(rc, "dssd_residual_sample_from_p")
    return rc


def dssd_probe_read(ctx, ptr, nbytes, loads_per_lane=8, waves_per_cu=0, stream=0):
    rc = load().dssd_probe_read(ctx, C.c_void_p(ptr), int(nbytes), int(loads_per_lane), int(waves_per_cu),
                                C.c_void_p(stream or 0))
    if rc != DSSD_OK:
        raise DssdError(rc, "dssd_probe_read")
    return rc


def dssd_profile_enable(ctx, enable=True):
    """enable: True = every kernel, False = off, or an int bit mask (bit k = kernel k)."""
    mask = (0xFFFFFFFF if enable else 0) if isinstance(enable, bool) else int(enable)
    return load().dssd_profile_enable(ctx, mask)


def dssd_profile_reset(ctx):
    return load().dssd_profile_reset(ctx)


def dssd_profile_read(ctx, kernel_id):
    ms, n = C.c_double(), C.c_int64()
    rc = load().dssd_profile_read(ctx, int(kernel_id), C.byref(ms), C.byref(n))
    if rc != DSSD_OK:
        raise DssdError(rc, "dssd_profile_read")
    return ms.value, n.value


# ------------------------------------------------------------------ torch-tensor marshalling
def _dp(t):
    return None if t is None else t.data_ptr()


def make_device_batch(inputs, p_rows, accepted_len, rejected, out_token, status=None, seed=0, step=0,
                      session_base=0, step_counter=None):
    """dssd_device_batch: the device side's view (Q rows, received P rows and j)."""
    import torch
    assert p_rows.is_contiguous() and p_rows.dtype in (torch.float32, torch.float16)
    off = inputs.get("draft_offsets")
    return dssd_device_batch(B=inputs["B"], V=inputs["V"], gamma=inputs["gamma"],
                             p_dtype=DSSD_F32 if p_rows.dtype == torch.float32 else DSSD_F16,
                             total_drafts=inputs["R_Q"], draft_offsets=_dp(off),
                             draft_probs=_dp(inputs["draft_probs"]), p_rows=_dp(p_rows),
                             accepted_len=_dp(accepted_len), rejected=_dp(rejected), seed=seed, step=step,
                             session_base=session_base, reserved=0, out_token=_dp(out_token),
                             status=_dp(status), step_counter=_dp(step_counter))


def make_batch(inputs, seed=0, step=0, session_base=0, q_scalars=None, flags=0, step_counter=None):
    """dssd_batch from a dict of device tensors as `synth.generate` returns them.  With
    `q_scalars` ([R_Q] fp32) the batch carries those instead of the Q rows (the edge's view).
    `step_counter`: a one-element int64 device tensor the kernels add to `step` when they run."""
    import torch
    lg = inputs["logits"]
    assert lg.is_contiguous() and inputs["draft_probs"].is_contiguous()
    assert lg.dtype in (torch.float32, torch.bfloat16) and inputs["draft_probs"].dtype == torch.float32
    assert inputs["draft_tokens"].dtype == torch.int32
    off = inputs.get("draft_offsets")
    it = inputs.get("inv_temperature")
    assert off is None or off.dtype == torch.int32
    assert it is None or it.dtype == torch.float32
    return dssd_batch(B=inputs["B"], V=inputs["V"], gamma=inputs["gamma"],
                      logits_dtype=DSSD_F32 if lg.dtype == torch.float32 else DSSD_BF16,
                      total_drafts=inputs["R_Q"], draft_offsets=_dp(off), logits=_dp(lg),
                      draft_probs=None if q_scalars is not None else _dp(inputs["draft_probs"]),
                      draft_tokens=_dp(inputs["draft_tokens"]),
                      inv_temperature=_dp(it), seed=seed, step=step, session_base=session_base, flags=flags,
                      draft_q_tok=_dp(q_scalars), step_counter=_dp(step_counter))


def alloc_out(inputs, device, debug=True):
    """Output tensors for a batch and the dssd_out that points at them."""
    import torch
    B, R_L, R_Q = inputs["B"], inputs["R_L"], inputs["R_Q"]
    t = dict(accepted_len=torch.full((B,), -7, dtype=torch.int32, device=device),
             rejected=torch.full((B,), -7, dtype=torch.int32, device=device),
             out_token=torch.full((B,), -7, dtype=torch.int32, device=device))
    if debug:
        t.update(row_stats=torch.zeros((R_L, 2), dtype=torch.float32, device=device),
                 p_tok=torch.zeros(R_Q, dtype=torch.float32, device=device),
                 q_tok=torch.zeros(R_Q, dtype=torch.float32, device=device),
                 status=torch.zeros(B, dtype=torch.int32, device=device))
    out = dssd_out(accepted_len=_dp(t["accepted_len"]), rejected=_dp(t["rejected"]),
                   out_token=_dp(t["out_token"]), row_stats=_dp(t.get("row_stats")),
                   p_tok=_dp(t.get("p_tok")), q_tok=_dp(t.get("q_tok")), status=_dp(t.get("status")))
    return t, out


class Context:
    """Owns a dssd_ctx; `step` runs the three calls back to back on torch's current stream."""

    def __init__(self, device, max_rows, max_V):
        import torch
        self.device = torch.device(device)
        idx = self.device.index if self.device.index is not None else 0
        self.handle = dssd_create(idx, max_rows, max_V)

    def close(self):
        if self.handle is not None:
            dssd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def stream(self):
        import torch
        return torch.cuda.current_stream(self.device).cuda_stream

    def step_fused(self, batch, out):
        dssd_step_fused(self.handle, batch, out, self.stream())

    def step(self, batch, out):
        s = self.stream()
        dssd_verify_batch(self.handle, batch, out, s)
        dssd_residual_sample(self.handle, batch, out, s)
        dssd_bonus_sample(self.handle, batch, out, s)
