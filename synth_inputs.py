"""Seeded synthetic inputs for the speculative verification step across B branches.

This module only *draws inputs*; it holds none of the method's arithmetic (no attention,
no acceptance rule, no voting) and imports neither the CPU oracle nor the HIP binding.
Both sides are fed the arrays made here, so a disagreement can never come from the data.

Workload shapes stand in for the paper's models (Section 4.1: s1.1-3B / s1.1-32B, i.e.
Qwen2.5-3B/32B attention geometry), its prompt lengths (Appendix, prefill discussion:
88% of prompts under 360 tokens, 99% under 800), its generation lengths (up to 8192
tokens) and its measured acceptance rates (Appendix, 0.70 - 0.90).  None of the paper's
datasets or weights is used or needed.

Random numbers: numpy's counter-based Philox generator, key = 1000 * config_number +
tensor_id (tensor ids below), so every tensor of every config can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np
from scipy.special import softmax as _softmax

# tensor ids (the "+ tensor_id" of the seed)
T_Q, T_KPRE, T_VPRE, T_KPRIV, T_VPRIV, T_TLOGIT, T_NOISE, T_DRAFT, T_UNIF, T_ANSWER, T_CONF = range(1, 12)


@dataclass(frozen=True)
class VerifyConfig:
    """One verify-step workload.  R = k + 1 query rows per branch; L counts the private
    tokens of a branch *including* its k + 1 new tokens, so the context is P + L."""
    name: str
    number: int          # 1..5, enters the seed
    B: int               # concurrent branches (Section 3.2, branch-wise parallelism)
    k: int               # draft length gamma (Section 3.3)
    Hq: int
    Hkv: int
    D: int
    P: int               # shared prompt-prefix tokens
    L: int               # private tokens per branch
    V: int               # vocabulary
    dtype: str           # "f32" or "bf16": storage type of Q, K, V
    qkv_std: float       # Q, K, V ~ qkv_std * N(0, 1)
    logit_std: float     # target logits ~ N(0, logit_std)
    noise_std: Optional[float]  # draft logits = target + N(0, noise_std); None = independent N(0, logit_std)
    n_answer_classes: int = 50
    zipf_a: float = 1.5

    @property
    def R(self) -> int:
        return self.k + 1

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def with_(self, **kw) -> "VerifyConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, VerifyConfig] = {
    # tiny fp32 case the CPU oracle finishes at once
    "C1": VerifyConfig("C1-tiny-f32", 1, B=2, k=3, Hq=4, Hkv=4, D=64, P=32, L=64, V=1000,
                       dtype="f32", qkv_std=1.0, logit_std=2.0, noise_std=None),
    # 3B-shaped
    "C2": VerifyConfig("C2-3B", 2, B=8, k=4, Hq=16, Hkv=2, D=128, P=512, L=2048, V=151936,
                       dtype="bf16", qkv_std=0.5, logit_std=2.0, noise_std=0.5),
    # 32B-shaped, the configuration the headline metric is quoted on
    "C3": VerifyConfig("C3-32B", 3, B=16, k=3, Hq=40, Hkv=8, D=128, P=256, L=3840, V=152064,
                       dtype="bf16", qkv_std=0.5, logit_std=2.0, noise_std=0.5),
    # branch-scaling sweep on 3B shapes; B is overridden to 1, 4, 16, 64
    "C4": VerifyConfig("C4-3B-sweep", 4, B=16, k=2, Hq=16, Hkv=2, D=128, P=1024, L=7168, V=151936,
                       dtype="bf16", qkv_std=0.5, logit_std=2.0, noise_std=0.5),
    # long context, long draft, frequent rejection
    "C5": VerifyConfig("C5-32B-long", 5, B=4, k=8, Hq=40, Hkv=8, D=128, P=512, L=15872, V=152064,
                       dtype="bf16", qkv_std=0.5, logit_std=2.0, noise_std=1.0),
}


def rng_for(cfg_number: int, tensor_id: int, salt: int = 0) -> np.random.Generator:
    """Philox stream for one tensor.  `salt` selects further independent copies of the same
    tensor (the bench rotates several KV sets so that the memory-side cache cannot serve them)."""
    return np.random.Generator(np.random.Philox(key=1000 * cfg_number + tensor_id + 1_000_000 * salt))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> 16) & 1) + np.uint32(0x7FFF)
    return ((b + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32)


def _normal(cfg: VerifyConfig, tid: int, shape, std: float, salt: int = 0) -> np.ndarray:
    g = rng_for(cfg.number, tid, salt)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def _store(cfg: VerifyConfig, x: np.ndarray) -> np.ndarray:
    return f32_to_bf16_bits(x) if cfg.dtype == "bf16" else x


def attention_inputs(cfg: VerifyConfig, priv_len: Optional[np.ndarray] = None, salt: int = 0,
                     Lmax: Optional[int] = None) -> dict:
    """Q [B][R][Hq][D], Kpre/Vpre [Hkv][P][D] (one copy for all branches), Kpriv/Vpriv
    [B][Hkv][Lmax][D], priv_len [B] (defaults to L for every branch).  bf16 configs return
    uint16 bit patterns; the values both sides see are the *stored* (rounded) ones."""
    Lmax = cfg.L if Lmax is None else Lmax
    out = {
        "Q": _store(cfg, _normal(cfg, T_Q, (cfg.B, cfg.R, cfg.Hq, cfg.D), cfg.qkv_std, salt)),
        "Kpre": _store(cfg, _normal(cfg, T_KPRE, (cfg.Hkv, cfg.P, cfg.D), cfg.qkv_std, salt)),
        "Vpre": _store(cfg, _normal(cfg, T_VPRE, (cfg.Hkv, cfg.P, cfg.D), cfg.qkv_std, salt)),
        "Kpriv": _store(cfg, _normal(cfg, T_KPRIV, (cfg.B, cfg.Hkv, Lmax, cfg.D), cfg.qkv_std, salt)),
        "Vpriv": _store(cfg, _normal(cfg, T_VPRIV, (cfg.B, cfg.Hkv, Lmax, cfg.D), cfg.qkv_std, salt)),
    }
    if priv_len is None:
        priv_len = np.full((cfg.B,), cfg.L, dtype=np.int32)
    out["priv_len"] = np.ascontiguousarray(priv_len, dtype=np.int32)
    return out


def accept_inputs(cfg: VerifyConfig, salt: int = 0) -> dict:
    """p [B][k+1][V] target probabilities, q [B][k][V] draft probabilities (fp32, each row the
    fp64 softmax of its logits rounded to fp32), draft [B][k] tokens drawn from q by inverse
    CDF, u [B][k+1] uniforms m / 2^24 (exact in fp32)."""
    B, k, V = cfg.B, cfg.k, cfg.V
    z = _normal(cfg, T_TLOGIT, (B, k + 1, V), cfg.logit_std, salt).astype(np.float64)
    if cfg.noise_std is None:
        zq = _normal(cfg, T_NOISE, (B, k, V), cfg.logit_std, salt).astype(np.float64)
    else:
        zq = z[:, :k, :] + _normal(cfg, T_NOISE, (B, k, V), cfg.noise_std, salt).astype(np.float64)
    p = _softmax(z, axis=-1).astype(np.float32)
    q = _softmax(zq, axis=-1).astype(np.float32) if k > 0 else np.zeros((B, 0, V), np.float32)
    g = rng_for(cfg.number, T_DRAFT, salt)
    draft = np.zeros((B, k), dtype=np.int32)
    ud = g.random(size=(B, k))
    for b in range(B):
        for j in range(k):
            c = np.cumsum(q[b, j].astype(np.float64))
            draft[b, j] = min(int(np.searchsorted(c, ud[b, j] * c[-1], side="right")), V - 1)
    gu = rng_for(cfg.number, T_UNIF, salt)
    m = gu.integers(0, 1 << 24, size=(B, k + 1), dtype=np.int64)
    u = (m.astype(np.float64) / float(1 << 24)).astype(np.float32)
    return {"p": p, "q": q, "draft": draft, "u": u}


def zipf_pmf(n_classes: int, a: float) -> np.ndarray:
    w = np.arange(1, n_classes + 1, dtype=np.float64) ** (-a)
    return w / w.sum()


def vote_inputs(cfg: VerifyConfig, N: int = 1, salt: int = 0) -> np.ndarray:
    """answers [N][B]: ids 0..n_classes-1 from the truncated Zipf(a) pmf (proportional to
    c^-a, c = 1..n_classes) -- a stand-in for the final answers the branches extract."""
    g = rng_for(cfg.number, T_ANSWER, salt)
    pmf = zipf_pmf(cfg.n_answer_classes, cfg.zipf_a)
    return g.choice(cfg.n_answer_classes, size=(N, cfg.B), p=pmf).astype(np.int32)


def expected_acceptance(noise_std: float) -> float:
    """Large-vocabulary acceptance rate of the correlated-logit draft: 2 * Phi(-noise_std / 2)."""
    from math import erf, sqrt
    return 2.0 * 0.5 * (1.0 + erf((-noise_std / 2.0) / sqrt(2.0)))
