"""ctypes loader and numpy marshalling for the C oracle.  Test infrastructure only."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lotts_oracle.c")
_LIB = os.path.join(_HERE, "liblotts_oracle.so")
_lib = None

F32, BF16 = 0, 1


def build(force: bool = True) -> str:
    """Compile lotts_oracle.c with gcc (OpenMP only spreads independent outputs over threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _bind(lib):
    """Declare the C signatures on a loaded oracle library (also used by the tests that load
    deliberately broken copies of it)."""
    c_int, c_dbl, vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
    lib.oracle_verify_attention.restype = c_int
    lib.oracle_verify_attention.argtypes = [c_int] * 8 + [c_dbl] + [vp] * 8
    lib.oracle_spec_accept.restype = c_int
    lib.oracle_spec_accept.argtypes = [c_int] * 3 + [vp] * 6
    lib.oracle_majority_vote.restype = c_int
    lib.oracle_majority_vote.argtypes = [c_int] * 2 + [vp] * 3
    lib.oracle_logit_weights.restype = ctypes.c_uint64
    lib.oracle_logit_weights.argtypes = [c_int, vp, c_int, ctypes.c_float, vp]
    lib.oracle_spec_accept_logits.restype = c_int
    lib.oracle_spec_accept_logits.argtypes = [c_int] * 3 + [vp, vp, c_int, ctypes.c_float] + [vp] * 5
    lib.oracle_skinny_gemm.restype = c_int
    lib.oracle_skinny_gemm.argtypes = [c_int] * 4 + [vp] * 3
    lib.oracle_kv_append.restype = c_int
    lib.oracle_kv_append.argtypes = [c_int] * 6 + [vp] * 5
    lib.oracle_confidence_vote.restype = c_int
    lib.oracle_confidence_vote.argtypes = [c_int] * 3 + [vp] * 3 + [c_int] * 2 + [vp] * 2
    return lib


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def set_threads(n: int) -> None:
    """Limit the OpenMP team (libgomp) of later oracle calls."""
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def n_threads() -> int:
    return int(ctypes.CDLL("libgomp.so.1").omp_get_max_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _kv(a: np.ndarray) -> Tuple[np.ndarray, int]:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError("Q/K/V must be float32 or uint16 (bf16 bit patterns), got %s" % a.dtype)


def verify_attention(Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, scale: float = 0.0, want_lse: bool = True):
    """fp64 attention of the k+1 new rows of each branch.  Shapes as in lotts_oracle.c.
    Returns (O [B][R][Hq][D] float64, lse [B][R][Hq] float64 or None)."""
    Q, dt = _kv(Q)
    B, R, Hq, D = Q.shape
    Kpriv, dt2 = _kv(Kpriv)
    Vpriv, _ = _kv(Vpriv)
    _, Hkv, Lmax, _ = Kpriv.shape
    if Kpre is None or Kpre.shape[1] == 0:
        P, Kpre, Vpre = 0, None, None
    else:
        Kpre, _ = _kv(Kpre)
        Vpre, _ = _kv(Vpre)
        P = Kpre.shape[1]
    assert dt == dt2
    priv_len = np.ascontiguousarray(priv_len, dtype=np.int32)
    O = np.empty((B, R, Hq, D), dtype=np.float64)
    lse = np.empty((B, R, Hq), dtype=np.float64) if want_lse else None
    rc = _load().oracle_verify_attention(B, R - 1, Hq, Hkv, D, P, Lmax, dt, float(scale), _ptr(Q), _ptr(Kpre),
                                         _ptr(Vpre), _ptr(Kpriv), _ptr(Vpriv), _ptr(priv_len), _ptr(O), _ptr(lse))
    if rc != 0:
        raise ValueError("oracle_verify_attention rejected the call (rc=%d)" % rc)
    return O, lse


def spec_accept(p, q, draft, u):
    """Returns (accept_len [B] int32, next_token [B] int32)."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    B, R, V = p.shape
    k = R - 1
    u = np.ascontiguousarray(u, dtype=np.float32)
    assert u.shape == (B, R)
    if k > 0:
        q = np.ascontiguousarray(q, dtype=np.float32)
        draft = np.ascontiguousarray(draft, dtype=np.int32)
        assert q.shape == (B, k, V) and draft.shape == (B, k)
    else:
        q, draft = None, None
    n = np.empty((B,), dtype=np.int32)
    t = np.empty((B,), dtype=np.int32)
    rc = _load().oracle_spec_accept(B, k, V, _ptr(p), _ptr(q), _ptr(draft), _ptr(u), _ptr(n), _ptr(t))
    if rc != 0:
        raise ValueError("oracle_spec_accept rejected the call (rc=%d)" % rc)
    return n, t


def majority_vote(answers):
    """answers [N][B] (or [B]) int32 -> (winner [N], count [N])."""
    a = np.ascontiguousarray(answers, dtype=np.int32)
    if a.ndim == 1:
        a = a[None, :]
    N, B = a.shape
    w = np.empty((N,), dtype=np.int32)
    c = np.empty((N,), dtype=np.int32)
    rc = _load().oracle_majority_vote(N, B, _ptr(a), _ptr(w), _ptr(c))
    if rc != 0:
        raise ValueError("oracle_majority_vote rejected the call (rc=%d)" % rc)
    return w, c


def logit_weights(z_row, inv_temp: float = 1.0):
    """Integer softmax weights of one row of logits: (E [V] uint64, S)."""
    z, dt = _kv(np.ascontiguousarray(z_row))
    E = np.empty((z.shape[0],), dtype=np.uint64)
    S = _load().oracle_logit_weights(z.shape[0], _ptr(z), dt, float(inv_temp), _ptr(E))
    return E, int(S)


def spec_accept_logits(zt, zd, draft, u, inv_temp: float = 1.0, priv_len=None):
    """Acceptance from target logits zt [B][k+1][V] and draft logits zd [B][k][V] (float32 or uint16 = bf16
    bit patterns).  Returns (accept_len [B], next_token [B]); priv_len (contiguous int32 [B], optional) is
    updated in place: the rejected drafts are dropped from each branch's private length."""
    zt, dt = _kv(zt)
    B, R, V = zt.shape
    k = R - 1
    u = np.ascontiguousarray(u, dtype=np.float32)
    if k > 0:
        zd, dt2 = _kv(zd)
        assert dt2 == dt and zd.shape == (B, k, V)
        draft = np.ascontiguousarray(draft, dtype=np.int32)
    else:
        zd, draft = None, None
    n = np.empty((B,), dtype=np.int32)
    t = np.empty((B,), dtype=np.int32)
    if priv_len is not None:
        assert priv_len.dtype == np.int32 and priv_len.shape == (B,) and priv_len.flags.c_contiguous
    rc = _load().oracle_spec_accept_logits(B, k, V, _ptr(zt), _ptr(zd), dt, float(inv_temp), _ptr(draft), _ptr(u),
                                           _ptr(n), _ptr(t), _ptr(priv_len))
    if rc != 0:
        raise ValueError("oracle_spec_accept_logits rejected the call (rc=%d)" % rc)
    return n, t


def confidence_vote(answers, conf, conf_len=None, weight_mode: str = "avg", select_mode: str = "vote"):
    """answers [N][B] int32, conf [N][B][T] float32 -> (winner [N] int32, score [N] float32)."""
    a = np.ascontiguousarray(answers, dtype=np.int32)
    c = np.ascontiguousarray(conf, dtype=np.float32)
    N, B, T = c.shape
    assert a.shape == (N, B)
    cl = None if conf_len is None else np.ascontiguousarray(conf_len, dtype=np.int32)
    w = np.empty((N,), dtype=np.int32)
    s = np.empty((N,), dtype=np.float32)
    rc = _load().oracle_confidence_vote(N, B, T, _ptr(a), _ptr(c), _ptr(cl), {"min": 0, "avg": 1}[weight_mode],
                                        {"max": 0, "vote": 1}[select_mode], _ptr(w), _ptr(s))
    if rc != 0:
        raise ValueError("oracle_confidence_vote rejected the call (rc=%d)" % rc)
    return w, s


def skinny_gemm(X, W):
    """Y = X @ W.T in fp64.  X [M][K], W [N][K], float32 or uint16 (bf16 bit patterns)."""
    X, dt = _kv(X)
    W, dt2 = _kv(W)
    assert dt == dt2 and X.shape[1] == W.shape[1]
    M, K = X.shape
    N = W.shape[0]
    Y = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_skinny_gemm(M, N, K, dt, _ptr(X), _ptr(W), _ptr(Y))
    if rc != 0:
        raise ValueError("oracle_skinny_gemm rejected the call (rc=%d)" % rc)
    return Y


def kv_append(Knew, Vnew, Kpriv, Vpriv, priv_len):
    """Returns copies of Kpriv, Vpriv [B][Hkv][Lmax][D] with the rows Knew, Vnew [B][k+1][Hkv][D] of the new tokens
    written at positions priv_len[b] - (k+1) .. priv_len[b] - 1 (float32, or uint16 bf16 bit patterns)."""
    Knew, Vnew = np.ascontiguousarray(Knew), np.ascontiguousarray(Vnew)
    Kout, Vout = np.array(Kpriv, copy=True, order="C"), np.array(Vpriv, copy=True, order="C")
    B, R, Hkv, D = Knew.shape
    assert Vnew.shape == Knew.shape and Kout.shape == Vout.shape and Kout.shape[:2] == (B, Hkv) and Kout.shape[3] == D
    assert Knew.dtype == Vnew.dtype == Kout.dtype == Vout.dtype and Knew.dtype in (np.float32, np.uint16)
    priv_len = np.ascontiguousarray(priv_len, dtype=np.int32)
    rc = _load().oracle_kv_append(B, R - 1, Hkv, D, Kout.shape[2], Knew.dtype.itemsize, _ptr(Knew), _ptr(Vnew),
                                  _ptr(Kout), _ptr(Vout), _ptr(priv_len))
    if rc != 0:
        raise ValueError("oracle_kv_append rejected the call (rc=%d)" % rc)
    return Kout, Vout
