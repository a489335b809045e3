"""Pins for the attention oracle: none of these re-uses the oracle's own loops.

Each check is a definition written independently with numpy/scipy library routines on tiny
shapes, a closed form, or an invariant of causal attention behind a shared prefix.
"""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import synth_inputs as S

TINY = S.CONFIGS["C1"]


def brute_force(Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, k, scale=None):
    """softmax(Q K^T / sqrt d) V per row with explicitly concatenated key lists (fp64)."""
    B, R, Hq, D = Q.shape
    Hkv = Kpriv.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    O = np.zeros((B, R, Hq, D))
    LSE = np.zeros((B, R, Hq))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(R):
                n_priv = int(priv_len[b]) - k + i
                K = np.concatenate([Kpre[g], Kpriv[b, g, :n_priv]], axis=0).astype(np.float64)
                Vv = np.concatenate([Vpre[g], Vpriv[b, g, :n_priv]], axis=0).astype(np.float64)
                s = (K @ Q[b, i, h].astype(np.float64)) * scale
                O[b, i, h] = softmax(s) @ Vv
                LSE[b, i, h] = logsumexp(s)
    return O, LSE


def as_f(cfg, a):
    return S.bf16_bits_to_f32(a) if cfg.dtype == "bf16" else a


@pytest.mark.parametrize("cfg", [
    TINY,
    TINY.with_(Hq=6, Hkv=2, D=16, P=5, L=11, k=2, B=3),          # GQA 3:1, odd sizes
    TINY.with_(Hq=4, Hkv=1, D=8, P=0, L=9, k=4, B=2),            # no prefix at all
    TINY.with_(Hq=8, Hkv=4, D=32, P=7, L=13, k=1, B=2, dtype="bf16", qkv_std=0.5),
])
def test_matches_brute_force(oracle, cfg):
    a = S.attention_inputs(cfg)
    O, lse = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    f = {n: as_f(cfg, a[n]) for n in ("Q", "Kpre", "Vpre", "Kpriv", "Vpriv")}
    Ob, Lb = brute_force(f["Q"], f["Kpre"], f["Vpre"], f["Kpriv"], f["Vpriv"], a["priv_len"], cfg.k)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, Lb, rtol=0, atol=1e-12)


def test_ragged_private_lengths_and_scale(oracle):
    cfg = TINY.with_(B=3, Hq=4, Hkv=2, D=16, P=6, L=20, k=3)
    pl = np.array([20, 4, 11], dtype=np.int32)       # 4 = k + 1: only the new tokens are private
    a = S.attention_inputs(cfg, priv_len=pl)
    O, lse = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], pl, scale=0.37)
    Ob, Lb = brute_force(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], pl, cfg.k, scale=0.37)
    np.testing.assert_allclose(O, Ob, atol=1e-12)
    np.testing.assert_allclose(lse, Lb, atol=1e-12)


def test_k0_is_decode_attention(oracle):
    """k = 0: one row per branch over the whole context -- ordinary decode attention."""
    cfg = TINY.with_(k=0)
    a = S.attention_inputs(cfg)
    O, lse = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    assert O.shape == (cfg.B, 1, cfg.Hq, cfg.D)
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            K = np.concatenate([a["Kpre"][h], a["Kpriv"][b, h]]).astype(np.float64)   # Hq == Hkv here
            V = np.concatenate([a["Vpre"][h], a["Vpriv"][b, h]]).astype(np.float64)
            w = softmax(K @ a["Q"][b, 0, h].astype(np.float64) / 8.0)                  # sqrt(64) = 8
            np.testing.assert_allclose(O[b, 0, h], w @ V, atol=1e-12)
            assert abs(w.sum() - 1) < 1e-12


def test_prefix_boundary_can_move(oracle):
    """Moving tokens from the shared prefix to the head of every branch's private cache must not
    change anything: the identity that lets the prefix KV be kept (and read) once."""
    cfg = TINY.with_(B=3, Hq=4, Hkv=2, D=16, P=12, L=10, k=2)
    a = S.attention_inputs(cfg)
    O0, l0 = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    for move in (1, 5, 12):
        P2 = cfg.P - move
        kp = np.concatenate([np.broadcast_to(a["Kpre"][None, :, P2:], (cfg.B, cfg.Hkv, move, cfg.D)), a["Kpriv"]], 2)
        vp = np.concatenate([np.broadcast_to(a["Vpre"][None, :, P2:], (cfg.B, cfg.Hkv, move, cfg.D)), a["Vpriv"]], 2)
        O1, l1 = oracle.verify_attention(a["Q"], a["Kpre"][:, :P2], a["Vpre"][:, :P2], kp, vp, a["priv_len"] + move)
        np.testing.assert_allclose(O1, O0, atol=1e-12)
        np.testing.assert_allclose(l1, l0, atol=1e-12)


def test_causality_row_i_equals_decode_on_truncated_cache(oracle):
    cfg = TINY.with_(B=2, Hq=4, Hkv=2, D=16, P=6, L=15, k=3)
    a = S.attention_inputs(cfg)
    O, lse = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    for i in range(cfg.R):
        Lt = cfg.L - cfg.k + i                       # cache cut right after new token i
        Oi, li = oracle.verify_attention(a["Q"][:, i:i + 1], a["Kpre"], a["Vpre"], a["Kpriv"][:, :, :Lt],
                                         a["Vpriv"][:, :, :Lt], np.full(cfg.B, Lt, np.int32))
        np.testing.assert_allclose(O[:, i], Oi[:, 0], atol=1e-12)
        np.testing.assert_allclose(lse[:, i], li[:, 0], atol=1e-12)
    # and what a row cannot see cannot matter: garbage in the later drafts' K/V rows
    a2 = {n: v.copy() for n, v in a.items()}
    a2["Kpriv"][:, :, cfg.L - 1] = 1e6
    a2["Vpriv"][:, :, cfg.L - 1] = -1e6
    O2, _ = oracle.verify_attention(a2["Q"], a2["Kpre"], a2["Vpre"], a2["Kpriv"], a2["Vpriv"], a2["priv_len"])
    np.testing.assert_allclose(O2[:, :cfg.k], O[:, :cfg.k], atol=1e-12)
    assert not np.allclose(O2[:, cfg.k], O[:, cfg.k])


def test_uniform_limit_closed_form(oracle):
    """Q = 0: every visible key weighs the same, so O is the mean of the visible V rows and
    LSE = log(number of visible keys)."""
    cfg = TINY.with_(B=2, Hq=4, Hkv=2, D=16, P=5, L=9, k=2)
    a = S.attention_inputs(cfg)
    Q0 = np.zeros_like(a["Q"])
    O, lse = oracle.verify_attention(Q0, a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            for i in range(cfg.R):
                n_priv = cfg.L - cfg.k + i
                mean = (a["Vpre"][h // 2].astype(np.float64).sum(0) +
                        a["Vpriv"][b, h // 2, :n_priv].astype(np.float64).sum(0)) / (cfg.P + n_priv)
                np.testing.assert_allclose(O[b, i, h], mean, atol=1e-13)
                assert abs(lse[b, i, h] - np.log(cfg.P + n_priv)) < 1e-13


def test_one_hot_limit(oracle):
    """A huge scale turns softmax into arg-max: O is the V row of the best-scoring visible key."""
    cfg = TINY.with_(B=2, Hq=2, Hkv=2, D=8, P=4, L=7, k=1)
    a = S.attention_inputs(cfg)
    O, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"], scale=1e4)
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            for i in range(cfg.R):
                n_priv = cfg.L - cfg.k + i
                K = np.concatenate([a["Kpre"][h], a["Kpriv"][b, h, :n_priv]]).astype(np.float64)
                V = np.concatenate([a["Vpre"][h], a["Vpriv"][b, h, :n_priv]]).astype(np.float64)
                s = K @ a["Q"][b, i, h].astype(np.float64)
                top = np.sort(s)[-2:]
                assert top[1] - top[0] > 1e-2           # gap * 1e4 > 100: the rest is < e^-100
                np.testing.assert_allclose(O[b, i, h], V[int(np.argmax(s))], atol=1e-12)


def test_bf16_bits_are_read_exactly(oracle):
    """A bf16 bit pattern means the fp32 with those upper 16 bits; nothing is rounded again."""
    cfg = TINY.with_(B=1, Hq=1, Hkv=1, D=4, P=0, L=2, k=0, dtype="bf16")
    q = S.f32_to_bf16_bits(np.array([[[[1.0, 0.0, 0.0, 0.0]]]], np.float32))
    K = S.f32_to_bf16_bits(np.array([[[[0.0, 0, 0, 0], [2.0, 0, 0, 0]]]], np.float32))
    Vv = S.f32_to_bf16_bits(np.array([[[[1.0, 2.0, 3.0, 4.0], [-0.5, 0.25, 1.5, 3.0e-3]]]], np.float32))
    O, lse = oracle.verify_attention(q, None, None, K, Vv, np.array([2], np.int32))
    w1 = 1.0 / (1.0 + np.exp(-1.0))                  # scores 0 and 2 / sqrt(4) = 1
    v = S.bf16_bits_to_f32(Vv)[0, 0].astype(np.float64)
    np.testing.assert_allclose(O[0, 0, 0], (1 - w1) * v[0] + w1 * v[1], atol=1e-15)
    assert abs(lse[0, 0, 0] - np.log(1 + np.e)) < 1e-15


def test_rejects_malformed(oracle):
    cfg = TINY
    a = S.attention_inputs(cfg)
    with pytest.raises(ValueError):
        oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"],
                                np.array([cfg.L, cfg.k], np.int32))      # shorter than the new tokens
