"""Thin Python binding of liblotts.so: argument marshalling only.

torch supplies device memory and the current stream; every step of the verify path runs in
the library's HIP kernels.  There is no fallback: if the library is missing the import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblotts.so")

LOTTS_F32, LOTTS_BF16 = 0, 1

EXPORTS = ("lotts_strerror", "verify_attention_workspace_bytes", "verify_attention", "verify_attention_noalloc",
           "spec_accept_workspace_bytes", "spec_accept", "spec_accept_logits_workspace_bytes", "spec_accept_logits",
           "majority_vote", "confidence_vote", "skinny_gemm_workspace_bytes", "skinny_gemm", "kv_append", "greedy_search",
           "lotts_timer_start", "lotts_timer_pause", "lotts_timer_stop")


class AttnDesc(ctypes.Structure):
    """Mirror of lotts_attn_desc."""
    _fields_ = [("B", ctypes.c_int32), ("k", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("P", ctypes.c_int32), ("Lmax", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float),
                ("q_stride_b", ctypes.c_int64), ("q_stride_r", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("kpre_stride_h", ctypes.c_int64), ("kpre_stride_t", ctypes.c_int64),
                ("kpriv_stride_b", ctypes.c_int64), ("kpriv_stride_h", ctypes.c_int64),
                ("kpriv_stride_t", ctypes.c_int64),
                ("o_stride_b", ctypes.c_int64), ("o_stride_r", ctypes.c_int64), ("o_stride_h", ctypes.c_int64)]


TTS_TASK_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p)


class LottsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, strerror(status), status))


_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("liblotts.so is not built: run paper_2505_19634_amd/build.py "
                              "(or __graft_entry__.build())")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.lotts_strerror.restype = ctypes.c_char_p
        lib.lotts_strerror.argtypes = [ctypes.c_int]
        lib.verify_attention_workspace_bytes.restype = sz
        lib.verify_attention_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
        lib.verify_attention.restype = ctypes.c_int
        lib.verify_attention.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 8 + [vp, sz, vp]
        lib.verify_attention_noalloc.restype = ctypes.c_int
        lib.verify_attention_noalloc.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 8 + [vp]
        lib.spec_accept_workspace_bytes.restype = sz
        lib.spec_accept_workspace_bytes.argtypes = [i32, i32, i32]
        lib.spec_accept.restype = ctypes.c_int
        lib.spec_accept.argtypes = [i32, i32, i32] + [vp] * 6 + [vp, sz, vp]
        lib.majority_vote.restype = ctypes.c_int
        lib.majority_vote.argtypes = [i32, i32, vp, vp, vp, vp]
        lib.spec_accept_logits_workspace_bytes.restype = sz
        lib.spec_accept_logits_workspace_bytes.argtypes = [i32, i32, i32]
        lib.spec_accept_logits.restype = ctypes.c_int
        lib.spec_accept_logits.argtypes = [i32, i32, i32, vp, vp, i32, ctypes.c_float] + [vp] * 5 + [vp, sz, vp]
        lib.skinny_gemm_workspace_bytes.restype = sz
        lib.skinny_gemm_workspace_bytes.argtypes = [i32, i32, i32]
        lib.skinny_gemm.restype = ctypes.c_int
        lib.skinny_gemm.argtypes = [i32, i32, i32, vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, vp, sz, vp]
        lib.kv_append.restype = ctypes.c_int
        lib.kv_append.argtypes = [i32, i32, i32, i32, i32, vp, vp] + [ctypes.c_int64] * 3 + [vp, vp] + [ctypes.c_int64] * 3 + [i32, vp, vp]
        lib.greedy_search.restype = ctypes.c_int
        lib.greedy_search.argtypes = [TTS_TASK_FN, vp, ctypes.c_double, i32, i32, ctypes.POINTER(ctypes.c_int32),
                                      ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.lotts_timer_start.restype = ctypes.c_int
        lib.lotts_timer_start.argtypes = [i32]
        lib.lotts_timer_pause.restype = ctypes.c_int
        lib.lotts_timer_pause.argtypes = [i32]
        lib.lotts_timer_stop.restype = ctypes.c_int
        lib.lotts_timer_stop.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)]
        lib.confidence_vote.restype = ctypes.c_int
        lib.confidence_vote.argtypes = [i32, i32, i32, vp, vp, vp, i32, i32, vp, vp, vp]
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load().lotts_strerror(int(status)).decode()


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


_workspaces: Dict[Tuple[str, int, int], torch.Tensor] = {}
_retired = []   # grown-out workspaces: kept alive, a kernel enqueued earlier may still be using them


def _workspace(kind: str, device: torch.device, nbytes: int, stream: Optional[torch.cuda.Stream]) -> torch.Tensor:
    """One cached scratch tensor per entry point, device and stream, grown on demand.  Calls on different streams
    may overlap in time, so they never share one.  The tensor is allocated and zero-filled on the stream that will
    use it (verify_attention wants its arrival cells zero at first use), so the fill is ordered before the kernel."""
    s = torch.cuda.current_stream(device) if stream is None else stream
    key = (kind, device.index if device.index is not None else torch.cuda.current_device(), int(s.cuda_stream))
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            _retired.append(ws)
        with torch.cuda.stream(s):
            ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def make_attn_desc(Q: torch.Tensor, Kpre: Optional[torch.Tensor], Kpriv: torch.Tensor, O: torch.Tensor,
                   scale: float = 0.0) -> AttnDesc:
    B, R, Hq, D = Q.shape
    Bk, Hkv, Lmax, Dk = Kpriv.shape
    if Bk != B or Dk != D:
        raise ValueError("Q %s and Kpriv %s disagree" % (tuple(Q.shape), tuple(Kpriv.shape)))
    if Q.dtype == torch.bfloat16:
        dt = LOTTS_BF16
    elif Q.dtype == torch.float32:
        dt = LOTTS_F32
    else:
        raise TypeError("Q/K/V must be bfloat16 or float32")
    for t in (Q, Kpriv, O) + ((Kpre,) if Kpre is not None else ()):
        if t.stride(-1) != 1:
            raise ValueError("the head dimension must be contiguous")
    d = AttnDesc()
    d.B, d.k, d.Hq, d.Hkv, d.D, d.Lmax, d.dtype, d.scale = B, R - 1, Hq, Hkv, D, Lmax, dt, float(scale)
    d.P = 0 if Kpre is None else Kpre.shape[1]
    d.q_stride_b, d.q_stride_r, d.q_stride_h = Q.stride(0), Q.stride(1), Q.stride(2)
    d.o_stride_b, d.o_stride_r, d.o_stride_h = O.stride(0), O.stride(1), O.stride(2)
    d.kpriv_stride_b, d.kpriv_stride_h, d.kpriv_stride_t = Kpriv.stride(0), Kpriv.stride(1), Kpriv.stride(2)
    if Kpre is not None and d.P > 0:
        d.kpre_stride_h, d.kpre_stride_t = Kpre.stride(0), Kpre.stride(1)
    return d


def verify_attention(Q: torch.Tensor, Kpre: Optional[torch.Tensor], Vpre: Optional[torch.Tensor],
                     Kpriv: torch.Tensor, Vpriv: torch.Tensor, priv_len: torch.Tensor, *, scale: float = 0.0,
                     out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                     return_lse: bool = False, workspace: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None):
    """Q [B][k+1][Hq][D], Kpre/Vpre [Hkv][P][D] or None, Kpriv/Vpriv [B][Hkv][Lmax][D], priv_len [B] int32;
    all on one GPU.  Returns O [B][k+1][Hq][D] (same dtype), and LSE [B][k+1][Hq] fp32 if asked."""
    lib = load()
    if not Q.is_cuda:
        raise ValueError("verify_attention runs on the GPU only")
    if Kpre is not None and Kpre.shape[1] == 0:
        Kpre, Vpre = None, None
    if Vpriv.stride() != Kpriv.stride() or (Kpre is not None and Vpre.stride() != Kpre.stride()):
        raise ValueError("K and V of a segment must share strides")
    if priv_len.dtype != torch.int32:
        raise TypeError("priv_len must be int32")
    if out is None:
        out = torch.empty(Q.shape, dtype=Q.dtype, device=Q.device)
    if return_lse and lse is None:
        lse = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    desc = make_attn_desc(Q, Kpre, Kpriv, out, scale)
    need = lib.verify_attention_workspace_bytes(ctypes.byref(desc))
    if need == 0:
        raise LottsError(-2, "verify_attention_workspace_bytes")
    ws = _workspace("attn", Q.device, need, stream) if workspace is None else workspace
    rc = lib.verify_attention(ctypes.byref(desc), _ptr(Q), _ptr(Kpre), _ptr(Vpre), _ptr(Kpriv), _ptr(Vpriv),
                              _ptr(priv_len), _ptr(out), _ptr(lse), _ptr(ws), ws.numel() * ws.element_size(),
                              _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "verify_attention")
    return (out, lse) if return_lse else out


def verify_attention_noalloc(Q: torch.Tensor, Kpre: Optional[torch.Tensor], Vpre: Optional[torch.Tensor],
                             Kpriv: torch.Tensor, Vpriv: torch.Tensor, priv_len: torch.Tensor, out: torch.Tensor, *,
                             scale: float = 0.0, lse: Optional[torch.Tensor] = None,
                             stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """verify_attention through the entry point that allocates nothing: the caller brings `out` (and `lse`), the
    library's built-in scratch replaces the workspace.  Geometries beyond that scratch raise LottsError(-4)."""
    lib = load()
    if not Q.is_cuda:
        raise ValueError("verify_attention_noalloc runs on the GPU only")
    if Kpre is not None and Kpre.shape[1] == 0:
        Kpre, Vpre = None, None
    if Vpriv.stride() != Kpriv.stride() or (Kpre is not None and Vpre.stride() != Kpre.stride()):
        raise ValueError("K and V of a segment must share strides")
    if priv_len.dtype != torch.int32:
        raise TypeError("priv_len must be int32")
    desc = make_attn_desc(Q, Kpre, Kpriv, out, scale)
    rc = lib.verify_attention_noalloc(ctypes.byref(desc), _ptr(Q), _ptr(Kpre), _ptr(Vpre), _ptr(Kpriv), _ptr(Vpriv),
                                      _ptr(priv_len), _ptr(out), _ptr(lse), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "verify_attention_noalloc")
    return out


def spec_accept(p: torch.Tensor, q: Optional[torch.Tensor], draft: Optional[torch.Tensor], u: torch.Tensor, *,
                accept_len: Optional[torch.Tensor] = None, next_token: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """p [B][k+1][V] fp32, q [B][k][V] fp32, draft [B][k] int32, u [B][k+1] fp32 (contiguous, on the GPU).
    Returns (accept_len [B] int32, next_token [B] int32)."""
    lib = load()
    if not p.is_cuda:
        raise ValueError("spec_accept runs on the GPU only")
    B, R, V = p.shape
    k = R - 1
    if p.dtype != torch.float32 or u.dtype != torch.float32 or not p.is_contiguous() or not u.is_contiguous():
        raise TypeError("p and u must be contiguous float32")
    if tuple(u.shape) != (B, R):
        raise ValueError("u must be [B][k+1]")
    if k > 0:
        if q is None or draft is None or tuple(q.shape) != (B, k, V) or tuple(draft.shape) != (B, k):
            raise ValueError("q must be [B][k][V] and draft [B][k]")
        if q.dtype != torch.float32 or draft.dtype != torch.int32 or not q.is_contiguous() or not draft.is_contiguous():
            raise TypeError("q must be contiguous float32 and draft contiguous int32")
    else:
        q, draft = None, None
    if accept_len is None:
        accept_len = torch.empty((B,), dtype=torch.int32, device=p.device)
    if next_token is None:
        next_token = torch.empty((B,), dtype=torch.int32, device=p.device)
    need = lib.spec_accept_workspace_bytes(B, k, V)
    if need == 0:
        raise LottsError(-2, "spec_accept_workspace_bytes")
    ws = _workspace("accept", p.device, need, stream) if workspace is None else workspace
    rc = lib.spec_accept(B, k, V, _ptr(p), _ptr(q), _ptr(draft), _ptr(u), _ptr(accept_len), _ptr(next_token),
                         _ptr(ws), ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "spec_accept")
    return accept_len, next_token


def majority_vote(answers: torch.Tensor, *, winner: Optional[torch.Tensor] = None,
                  winner_count: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """answers [N][B] (or [B]) int32 on the GPU -> (winner [N], winner_count [N]) int32."""
    lib = load()
    if not answers.is_cuda:
        raise ValueError("majority_vote runs on the GPU only")
    if answers.dim() == 1:
        answers = answers[None, :]
    if answers.dtype != torch.int32 or not answers.is_contiguous():
        raise TypeError("answers must be contiguous int32")
    N, B = answers.shape
    if winner is None:
        winner = torch.empty((N,), dtype=torch.int32, device=answers.device)
    if winner_count is None:
        winner_count = torch.empty((N,), dtype=torch.int32, device=answers.device)
    rc = lib.majority_vote(N, B, _ptr(answers), _ptr(winner), _ptr(winner_count), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "majority_vote")
    return winner, winner_count


def spec_accept_logits(target_logits: torch.Tensor, draft_logits: Optional[torch.Tensor], draft: Optional[torch.Tensor],
                       u: torch.Tensor, *, inv_temperature: float = 1.0, accept_len: Optional[torch.Tensor] = None,
                       next_token: Optional[torch.Tensor] = None, priv_len: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """target_logits [B][k+1][V], draft_logits [B][k][V] (both bfloat16 or both float32, contiguous), draft [B][k]
    int32, u [B][k+1] fp32, on the GPU.  Returns (accept_len [B] int32, next_token [B] int32).  priv_len (int32 [B],
    optional) is updated in place: priv_len[b] -= k - accept_len[b]."""
    lib = load()
    if not target_logits.is_cuda:
        raise ValueError("spec_accept_logits runs on the GPU only")
    B, R, V = target_logits.shape
    k = R - 1
    if target_logits.dtype == torch.bfloat16:
        dt = LOTTS_BF16
    elif target_logits.dtype == torch.float32:
        dt = LOTTS_F32
    else:
        raise TypeError("logits must be bfloat16 or float32")
    if not target_logits.is_contiguous() or u.dtype != torch.float32 or not u.is_contiguous() or tuple(u.shape) != (B, R):
        raise TypeError("target_logits must be contiguous and u contiguous float32 [B][k+1]")
    if k > 0:
        if (draft_logits is None or draft is None or draft_logits.dtype != target_logits.dtype or
                tuple(draft_logits.shape) != (B, k, V) or not draft_logits.is_contiguous() or
                draft.dtype != torch.int32 or tuple(draft.shape) != (B, k) or not draft.is_contiguous()):
            raise TypeError("draft_logits must be [B][k][V] of the same dtype, draft [B][k] int32, both contiguous")
    else:
        draft_logits, draft = None, None
    if accept_len is None:
        accept_len = torch.empty((B,), dtype=torch.int32, device=u.device)
    if next_token is None:
        next_token = torch.empty((B,), dtype=torch.int32, device=u.device)
    if priv_len is not None and (priv_len.dtype != torch.int32 or tuple(priv_len.shape) != (B,) or
                                 not priv_len.is_contiguous() or priv_len.device != u.device):
        raise TypeError("priv_len must be a contiguous int32 [B] tensor on the same GPU")
    need = lib.spec_accept_logits_workspace_bytes(B, k, V)
    if need == 0:
        raise LottsError(-2, "spec_accept_logits_workspace_bytes")
    ws = _workspace("accept_logits", u.device, need, stream) if workspace is None else workspace
    rc = lib.spec_accept_logits(B, k, V, _ptr(target_logits), _ptr(draft_logits), dt, float(inv_temperature), _ptr(draft),
                                _ptr(u), _ptr(accept_len), _ptr(next_token), _ptr(priv_len), _ptr(ws),
                                ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "spec_accept_logits")
    return accept_len, next_token


def confidence_vote(answers: torch.Tensor, conf: torch.Tensor, conf_len: Optional[torch.Tensor] = None, *,
                    weight_mode: str = "avg", select_mode: str = "vote", stream: Optional[torch.cuda.Stream] = None):
    """answers [N][B] int32, conf [N][B][T] fp32, conf_len [N][B] int32 or None, on the GPU.
    Returns (winner [N] int32, winner_score [N] fp32)."""
    lib = load()
    if not answers.is_cuda:
        raise ValueError("confidence_vote runs on the GPU only")
    N, B, T = conf.shape
    if (answers.dtype != torch.int32 or tuple(answers.shape) != (N, B) or not answers.is_contiguous() or
            conf.dtype != torch.float32 or not conf.is_contiguous()):
        raise TypeError("answers must be contiguous int32 [N][B], conf contiguous float32 [N][B][T]")
    if conf_len is not None and (conf_len.dtype != torch.int32 or tuple(conf_len.shape) != (N, B) or
                                 not conf_len.is_contiguous()):
        raise TypeError("conf_len must be contiguous int32 [N][B]")
    winner = torch.empty((N,), dtype=torch.int32, device=answers.device)
    score = torch.empty((N,), dtype=torch.float32, device=answers.device)
    rc = lib.confidence_vote(N, B, T, _ptr(answers), _ptr(conf), _ptr(conf_len), {"min": 0, "avg": 1}[weight_mode],
                             {"max": 0, "vote": 1}[select_mode], _ptr(winner), _ptr(score), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "confidence_vote")
    return winner, score


def greedy_search(tts_task, T: float, B_max: int = 64, gamma_max: int = 7):
    """Algorithm 1 on the host: tts_task(B, gamma, T) -> accuracy.  Returns (B, gamma, acc, rounds, evaluations)."""
    lib = load()
    cb = TTS_TASK_FN(lambda B, g, t, _user: float(tts_task(int(B), int(g), float(t))))
    B = ctypes.c_int32()
    g = ctypes.c_int32()
    acc = ctypes.c_double()
    rounds = ctypes.c_int32()
    evals = ctypes.c_int32()
    rc = lib.greedy_search(cb, None, float(T), int(B_max), int(gamma_max), ctypes.byref(B), ctypes.byref(g),
                           ctypes.byref(acc), ctypes.byref(rounds), ctypes.byref(evals))
    if rc != 0:
        raise LottsError(rc, "greedy_search")
    return B.value, g.value, acc.value, rounds.value, evals.value


def skinny_gemm(X: torch.Tensor, W: torch.Tensor, *, out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Y = X @ W.T for bf16 X [M][K] (M <= 256) and W [N][K] on the GPU; rows may be strided."""
    lib = load()
    if not X.is_cuda or X.dtype != torch.bfloat16 or W.dtype != torch.bfloat16:
        raise TypeError("skinny_gemm takes bfloat16 tensors on the GPU")
    M, K = X.shape
    N, K2 = W.shape
    if K2 != K or X.stride(1) != 1 or W.stride(1) != 1:
        raise ValueError("X [M][K] and W [N][K] must share K and have contiguous rows")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    need = lib.skinny_gemm_workspace_bytes(M, N, K)
    if need == 0:
        raise LottsError(-2, "skinny_gemm_workspace_bytes")
    ws = _workspace("gemm", X.device, need, stream) if workspace is None else workspace
    rc = lib.skinny_gemm(M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(out), out.stride(0), _ptr(ws),
                         ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "skinny_gemm")
    return out


def kv_append(Knew: torch.Tensor, Vnew: torch.Tensor, Kpriv: torch.Tensor, Vpriv: torch.Tensor, priv_len: torch.Tensor, *,
              stream: Optional[torch.cuda.Stream] = None) -> None:
    """Knew/Vnew [B][k+1][Hkv][D] (views are fine: only D has to be contiguous, V with K's strides) go to positions
    priv_len[b] - (k+1) .. priv_len[b] - 1 of Kpriv/Vpriv [B][Hkv][Lmax][D] (in place)."""
    lib = load()
    if not Kpriv.is_cuda:
        raise ValueError("kv_append runs on the GPU only")
    if Knew.dtype == torch.bfloat16:
        dt = LOTTS_BF16
    elif Knew.dtype == torch.float32:
        dt = LOTTS_F32
    else:
        raise TypeError("K and V must be bfloat16 or float32")
    if not (Vnew.dtype == Kpriv.dtype == Vpriv.dtype == Knew.dtype):
        raise TypeError("all four buffers share one dtype")
    B, R, Hkv, D = Knew.shape
    if (tuple(Vnew.shape) != (B, R, Hkv, D) or Kpriv.shape[0] != B or Kpriv.shape[1] != Hkv or Kpriv.shape[3] != D or
            Vpriv.shape != Kpriv.shape or Vnew.stride() != Knew.stride() or Vpriv.stride() != Kpriv.stride() or
            Knew.stride(3) != 1 or Kpriv.stride(3) != 1):
        raise ValueError("Knew/Vnew [B][k+1][Hkv][D] and Kpriv/Vpriv [B][Hkv][Lmax][D] with shared strides, D contiguous")
    if priv_len.dtype != torch.int32 or tuple(priv_len.shape) != (B,):
        raise TypeError("priv_len must be int32 [B]")
    rc = lib.kv_append(B, R - 1, Hkv, D, dt, _ptr(Knew), _ptr(Vnew), Knew.stride(0), Knew.stride(1), Knew.stride(2),
                       _ptr(Kpriv), _ptr(Vpriv), Kpriv.stride(0), Kpriv.stride(1), Kpriv.stride(2), Kpriv.shape[2],
                       _ptr(priv_len), _stream_handle(stream))
    if rc != 0:
        raise LottsError(rc, "kv_append")


class kernel_timer:
    """Context manager around lotts_timer_start / lotts_timer_stop: `with kernel_timer(n) as t: ...` leaves the
    device milliseconds of up to n kernel launches made inside, in launch order, in t.ms."""

    def __init__(self, max_launches: int):
        self.max_launches = int(max_launches)
        self.ms = []

    def __enter__(self):
        rc = load().lotts_timer_start(self.max_launches)
        if rc != 0:
            raise LottsError(rc, "lotts_timer_start")
        return self

    def pause(self, paused: bool = True):
        """Launches made while paused are not timed (and cost nothing extra)."""
        load().lotts_timer_pause(1 if paused else 0)

    def __exit__(self, *exc):
        n = ctypes.c_int32()
        buf = (ctypes.c_float * self.max_launches)()
        rc = load().lotts_timer_stop(ctypes.byref(n), buf)
        if rc != 0 and exc[0] is None:
            raise LottsError(rc, "lotts_timer_stop")
        self.ms = list(buf[:n.value])
        return False
