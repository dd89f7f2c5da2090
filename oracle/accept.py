"""ctypes front end of oracle/accept.c (CPU oracle, test infrastructure only).

The arithmetic lives in the C file; this module only widens the inputs to
fp64 and marshals pointers.
"""
import ctypes
import os

import numpy as np

from . import build as _build

FLAG_NEAR_TIE = 1
FLAG_ZERO_RESIDUAL = 2

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_spec_accept.restype = ctypes.c_int
        lib.oracle_spec_accept.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_double, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_greedy_accept.restype = ctypes.c_int
        lib.oracle_greedy_accept.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def spec_accept(p_logits, q_logits, draft_tokens, uniforms, temperature=1.0, tie_eps=1e-5,
                return_rho=False):
    """Speculative-sampling acceptance for `rows` independent sequences.

    p_logits [rows, n_p_rows, V] with n_p_rows in {gamma, gamma+1}; q_logits
    [rows, gamma, V]; draft_tokens int [rows, gamma]; uniforms [rows, gamma+1].
    Any float dtype; everything is widened to fp64 first.
    Returns (accept_len int32[rows], token int32[rows], flags int32[rows]) and,
    if asked, rho float64[rows, gamma] (NaN where the position was not tested).
    """
    lp = np.ascontiguousarray(p_logits, dtype=np.float64)
    lq = np.ascontiguousarray(q_logits, dtype=np.float64)
    x = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    u = np.ascontiguousarray(uniforms, dtype=np.float64)
    if lp.ndim != 3 or lq.ndim != 3:
        raise ValueError("logits must be [rows, positions, V]")
    rows, n_p_rows, V = lp.shape
    gamma = lq.shape[1]
    if lq.shape[0] != rows or lq.shape[2] != V:
        raise ValueError("p and q disagree on rows or vocab")
    if x.shape != (rows, gamma) or u.shape != (rows, gamma + 1):
        raise ValueError("draft_tokens must be [rows,gamma], uniforms [rows,gamma+1]")
    out_n = np.empty(rows, np.int32)
    out_tok = np.empty(rows, np.int32)
    out_flags = np.empty(rows, np.int32)
    rho = np.empty((rows, gamma), np.float64)
    rc = _load().oracle_spec_accept(
        lp.ctypes.data, lq.ctypes.data, x.ctypes.data, u.ctypes.data,
        rows, gamma, n_p_rows, V, float(temperature), float(tie_eps),
        out_n.ctypes.data, out_tok.ctypes.data, out_flags.ctypes.data, rho.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_spec_accept rejected its arguments")
    if return_rho:
        return out_n, out_tok, out_flags, rho
    return out_n, out_tok, out_flags


def sample(logits, uniforms, temperature=1.0):
    """Inverse-CDF draw from softmax(logits/T): the gamma = 0 case with a bonus row.

    logits [rows, V], uniforms [rows] -> int32[rows].
    """
    lg = np.asarray(logits, dtype=np.float64)
    rows, V = lg.shape
    _, tok, _ = spec_accept(lg.reshape(rows, 1, V), np.empty((rows, 0, V)),
                            np.empty((rows, 0), np.int32),
                            np.asarray(uniforms, np.float64).reshape(rows, 1), temperature)
    return tok


def greedy_accept(p_logits, draft_tokens):
    """Greedy verification: p_logits [rows, n_p_rows, V], draft_tokens int [rows, gamma] with
    n_p_rows in {gamma, gamma+1} -> (accept_len int32[rows], token int32[rows])."""
    lp = np.ascontiguousarray(p_logits, dtype=np.float64)
    x = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    rows, n_p_rows, V = lp.shape
    gamma = x.shape[1]
    if x.shape[0] != rows:
        raise ValueError("p and draft_tokens disagree on rows")
    out_n = np.empty(rows, np.int32)
    out_tok = np.empty(rows, np.int32)
    rc = _load().oracle_greedy_accept(lp.ctypes.data, x.ctypes.data, rows, gamma, n_p_rows, V,
                                      out_n.ctypes.data, out_tok.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_greedy_accept rejected its arguments")
    return out_n, out_tok
