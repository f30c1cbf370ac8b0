"""ctypes view of the C++ oracle (oracle/dssd_oracle.cpp).  Test infrastructure only.

Argument marshalling, nothing else: every number returned here was computed by the
C++ file.  Arrays are numpy; bf16 logits are passed as uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1


class Result(C.Structure):
    _fields_ = [("n", C.c_int32), ("rejected", C.c_int32), ("token", C.c_int32),
                ("status", C.c_int32), ("resid_mass", C.c_double), ("cdf_margin", C.c_double),
                ("accept_margin", C.c_double)]


RESULT_DTYPE = np.dtype([("n", "<i4"), ("rejected", "<i4"), ("token", "<i4"), ("status", "<i4"),
                         ("resid_mass", "<f8"), ("cdf_margin", "<f8"), ("accept_margin", "<f8")])
assert RESULT_DTYPE.itemsize == C.sizeof(Result)

_lib = None


def lib():
    global _lib
    if _lib is None:
        # DSSD_ORACLE_LIB lets the tests load a deliberately broken build to prove the pins bite
        path = os.environ.get("DSSD_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        vp, dp, ip = C.c_void_p, C.c_void_p, C.c_void_p
        L.dssd_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.dssd_oracle_philox4x32_10.restype = None
        L.dssd_oracle_u01.argtypes = [C.c_uint32]
        L.dssd_oracle_u01.restype = C.c_double
        L.dssd_oracle_random_block.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, vp]
        L.dssd_oracle_random_block.restype = None
        L.dssd_oracle_softmax_row.argtypes = [vp, C.c_int, C.c_int32, C.c_double, dp, dp, dp]
        L.dssd_oracle_softmax_row.restype = None
        L.dssd_oracle_accept.argtypes = [C.c_double] * 3
        L.dssd_oracle_accept.restype = C.c_int
        L.dssd_oracle_accept_margin.argtypes = [C.c_double] * 3
        L.dssd_oracle_accept_margin.restype = C.c_double
        L.dssd_oracle_accept_prob.argtypes = [C.c_double] * 2
        L.dssd_oracle_accept_prob.restype = C.c_double
        L.dssd_oracle_residual.argtypes = [dp, vp, C.c_int32, dp]
        L.dssd_oracle_residual.restype = C.c_double
        L.dssd_oracle_inverse_cdf.argtypes = [dp, C.c_int32, C.c_double, dp]
        L.dssd_oracle_inverse_cdf.restype = C.c_int32
        L.dssd_oracle_inverse_cdf_many.argtypes = [dp, C.c_int32, dp, C.c_int64, ip]
        L.dssd_oracle_inverse_cdf_many.restype = None
        L.dssd_oracle_accept_count.argtypes = [dp, C.c_int64, C.c_double, C.c_double]
        L.dssd_oracle_accept_count.restype = C.c_int64
        L.dssd_oracle_verify_batch.argtypes = [
            C.c_int32, C.c_int32, C.c_int32, vp, vp, C.c_int, vp, vp, vp,
            C.c_uint64, C.c_uint64, C.c_uint32, vp, dp, dp, dp, dp, dp, dp]
        L.dssd_oracle_verify_batch.restype = None
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _logits_array(logits, dtype):
    want = np.float32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(logits)
    if a.dtype != want:
        raise TypeError(f"logits must be {want} for dtype {dtype}, got {a.dtype}")
    return a


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().dssd_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def u01(w):
    return lib().dssd_oracle_u01(int(w))


def random_block(seed, step, session, position):
    out = np.zeros(4, dtype=np.uint32)
    lib().dssd_oracle_random_block(int(seed), int(step), int(session), int(position), _ptr(out))
    return out


def softmax_row(logits_row, dtype=F32, inv_temperature=1.0):
    a = _logits_array(logits_row, dtype)
    V = a.shape[0]
    P = np.zeros(V, dtype=np.float64)
    m = C.c_double()
    Z = C.c_double()
    lib().dssd_oracle_softmax_row(_ptr(a), dtype, V, float(inv_temperature), _ptr(P),
                                  C.byref(m), C.byref(Z))
    return P, m.value, Z.value


def accept(r, p, q):
    return lib().dssd_oracle_accept(float(r), float(p), float(q))


def accept_margin(r, p, q):
    return lib().dssd_oracle_accept_margin(float(r), float(p), float(q))


def accept_prob(p, q):
    return lib().dssd_oracle_accept_prob(float(p), float(q))


def accept_count(r, p, q):
    r = np.ascontiguousarray(r, dtype=np.float64)
    return lib().dssd_oracle_accept_count(_ptr(r), r.size, float(p), float(q))


def residual(P, Q):
    P = np.ascontiguousarray(P, dtype=np.float64)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    w = np.zeros_like(P)
    R = lib().dssd_oracle_residual(_ptr(P), _ptr(Q), P.shape[0], _ptr(w))
    return w, R


def inverse_cdf(w, r):
    w = np.ascontiguousarray(w, dtype=np.float64)
    margin = C.c_double()
    k = lib().dssd_oracle_inverse_cdf(_ptr(w), w.shape[0], float(r), C.byref(margin))
    return k, margin.value


def inverse_cdf_many(w, r):
    w = np.ascontiguousarray(w, dtype=np.float64)
    r = np.ascontiguousarray(r, dtype=np.float64)
    tok = np.zeros(r.size, dtype=np.int32)
    lib().dssd_oracle_inverse_cdf_many(_ptr(w), w.shape[0], _ptr(r), r.size, _ptr(tok))
    return tok


def verify_batch(logits, dtype, draft_probs, draft_tokens, V, gamma=0, draft_offsets=None,
                 inv_temperature=None, seed=0, step=0, session_base=0, want_beta=False):
    """Run the oracle over a batch laid out like the GPU library's input.

    Returns a dict: 'res' (structured array, one record per session), 'p_tok', 'q_tok',
    'r_acc' [R_Q], 'row_m', 'row_Z' [R_L] and, if asked for, 'beta' [R_Q].
    """
    lg = _logits_array(logits, dtype)
    if draft_offsets is not None:
        off = np.ascontiguousarray(draft_offsets, dtype=np.int32)
        B = off.shape[0] - 1
        R_Q = int(off[-1])
    else:
        off = None
        R_Q = int(np.asarray(draft_tokens).size)
        B = R_Q // gamma if gamma > 0 else lg.size // V
    R_L = R_Q + B
    assert lg.size == R_L * V, (lg.size, R_L, V)
    dq = np.ascontiguousarray(draft_probs, dtype=np.float32)
    assert dq.size == R_Q * V
    tk = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    it = None if inv_temperature is None else np.ascontiguousarray(inv_temperature, dtype=np.float32)
    res = np.zeros(B, dtype=RESULT_DTYPE)
    p_tok = np.zeros(R_Q); q_tok = np.zeros(R_Q); r_acc = np.zeros(R_Q)
    row_m = np.zeros(R_L); row_Z = np.zeros(R_L)
    beta = np.zeros(R_Q) if want_beta else None
    lib().dssd_oracle_verify_batch(B, V, gamma, _ptr(off), _ptr(lg), dtype, _ptr(dq), _ptr(tk),
                                   _ptr(it), int(seed), int(step), int(session_base), _ptr(res),
                                   _ptr(p_tok), _ptr(q_tok), _ptr(r_acc), _ptr(row_m), _ptr(row_Z),
                                   _ptr(beta))
    return dict(res=res, p_tok=p_tok, q_tok=q_tok, r_acc=r_acc, row_m=row_m, row_Z=row_Z, beta=beta)


# ------------------------------------------------------------------ the edge / device split
P_F32, P_F16, P_F64 = 0, 2, 3
_P_NP = {P_F32: np.float32, P_F16: np.uint16, P_F64: np.float64}


def _split_lib():
    L = lib()
    if not getattr(L, "_split_ready", False):
        vp = C.c_void_p
        L.dssd_oracle_f32_to_f16.argtypes = [C.c_float]
        L.dssd_oracle_f32_to_f16.restype = C.c_uint16
        L.dssd_oracle_f16_to_f64.argtypes = [C.c_uint16]
        L.dssd_oracle_f16_to_f64.restype = C.c_double
        L.dssd_oracle_quantize_p_row.argtypes = [vp, C.c_int32, C.c_int, vp]
        L.dssd_oracle_quantize_p_row.restype = None
        L.dssd_oracle_edge_batch.argtypes = [C.c_int32, C.c_int32, C.c_int32, vp, vp, C.c_int, vp, vp, vp,
                                             C.c_uint64, C.c_uint64, C.c_uint32, C.c_int, vp, vp, vp]
        L.dssd_oracle_edge_batch.restype = None
        L.dssd_oracle_device_batch.argtypes = [C.c_int32, C.c_int32, C.c_int32, vp, vp, vp, C.c_int, vp, vp,
                                               C.c_uint64, C.c_uint64, C.c_uint32, vp, vp, vp, vp]
        L.dssd_oracle_device_batch.restype = None
        L._split_ready = True
    return L


def f32_to_f16(x):
    return _split_lib().dssd_oracle_f32_to_f16(float(x))


def f16_to_f64(h):
    return _split_lib().dssd_oracle_f16_to_f64(int(h))


def quantize_p_row(P, p_dtype):
    P = np.ascontiguousarray(P, dtype=np.float64)
    out = np.zeros(P.shape[0], dtype=_P_NP[p_dtype])
    _split_lib().dssd_oracle_quantize_p_row(_ptr(P), P.shape[0], p_dtype, _ptr(out))
    return out


def _layout(draft_offsets, draft_tokens, gamma):
    if draft_offsets is not None:
        off = np.ascontiguousarray(draft_offsets, dtype=np.int32)
        return off, off.shape[0] - 1, int(off[-1])
    R_Q = int(np.asarray(draft_tokens).size)
    return None, (R_Q // gamma if gamma > 0 else None), R_Q


def edge_batch(logits, dtype, q_scalars, draft_tokens, V, p_dtype, gamma=0, draft_offsets=None,
               inv_temperature=None, seed=0, step=0, session_base=0, B=None):
    """Edge side of the split.  Returns dict: 'res' (token = bonus token or -1), 'p_rows' [B, V]
    in p_dtype (rows of rejected sessions only are meaningful), 'p_tok'."""
    lg = _logits_array(logits, dtype)
    off, B2, R_Q = _layout(draft_offsets, draft_tokens, gamma)
    B = B2 if B2 is not None else (B if B is not None else lg.size // V)
    qs = np.ascontiguousarray(q_scalars, dtype=np.float32)
    tk = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    it = None if inv_temperature is None else np.ascontiguousarray(inv_temperature, dtype=np.float32)
    res = np.zeros(B, dtype=RESULT_DTYPE)
    p_rows = np.zeros((B, V), dtype=_P_NP[p_dtype])
    p_tok = np.full(R_Q, np.nan)
    _split_lib().dssd_oracle_edge_batch(B, V, gamma, _ptr(off), _ptr(lg), dtype, _ptr(qs), _ptr(tk), _ptr(it),
                                        int(seed), int(step), int(session_base), p_dtype, _ptr(res),
                                        _ptr(p_rows), _ptr(p_tok))
    return dict(res=res, p_rows=p_rows, p_tok=p_tok)


def device_batch(draft_probs, p_rows, p_dtype, accepted_len, rejected, V, gamma=0, draft_offsets=None,
                 seed=0, step=0, session_base=0):
    """Device side of the split.  Returns dict: 'token' (-1 where not rejected), 'resid_mass',
    'cdf_margin', 'status'."""
    off = None if draft_offsets is None else np.ascontiguousarray(draft_offsets, dtype=np.int32)
    al = np.ascontiguousarray(accepted_len, dtype=np.int32)
    rj = np.ascontiguousarray(rejected, dtype=np.int32)
    B = al.shape[0]
    dq = np.ascontiguousarray(draft_probs, dtype=np.float32)
    pr = np.ascontiguousarray(p_rows, dtype=_P_NP[p_dtype])
    assert pr.size == B * V
    token = np.zeros(B, dtype=np.int32)
    R = np.zeros(B); margin = np.zeros(B); status = np.zeros(B, dtype=np.int32)
    _split_lib().dssd_oracle_device_batch(B, V, gamma, _ptr(off), _ptr(dq), _ptr(pr), p_dtype, _ptr(al), _ptr(rj),
                                          int(seed), int(step), int(session_base), _ptr(token), _ptr(R),
                                          _ptr(margin), _ptr(status))
    return dict(token=token, resid_mass=R, cdf_margin=margin, status=status)
