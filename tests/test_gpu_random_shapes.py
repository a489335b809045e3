"""GPU parity on shapes drawn at random (fixed seeds) inside the documented limits of each entry point:
the hand-picked cases of test_gpu_parity.py aim at known plan boundaries, these look for the ones nobody
thought of (fold / stacked prefix, one or two row tiles, one or two launches, ragged lengths, odd sizes)."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from gpu_util import DEV, TOL, attn_errors, attn_to_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lotts():
    import paper_2505_19634_amd as m
    assert torch.cuda.is_available()
    return m


def random_attention_case(seed):
    g = np.random.default_rng(1000 + seed)
    Hkv = int(g.choice([1, 2, 3, 4, 5, 7, 8]))
    G = int(g.choice([1, 2, 3, 4, 5, 7, 8]))
    k = int(g.integers(0, 17))
    while G * (k + 1) > 128:                                  # keep the fp64 oracle quick
        k -= 1
    D = int(g.choice([64, 128]))
    B = int(g.integers(1, 20)) if g.random() < 0.8 else int(g.integers(64, 320))   # sometimes far more items than CUs
    P = int(g.choice([0, int(g.integers(1, 40)), int(g.integers(40, 700))]))
    L = int(g.integers(k + 1, 900))
    dtype = "bf16" if g.random() < 0.8 else "f32"
    if dtype == "f32":                                        # the fp32 path is a plain VALU kernel: small cases
        B, L, P = min(B, 4), min(L, 150), min(P, 80)
        L = max(L, k + 1)
    if B > 20:                                                # many branches: keep the total work in bounds
        L, P = max(k + 1, min(L, 120)), min(P, 300)
    cfg = S.CONFIGS["C3"].with_(B=B, k=k, Hq=Hkv * G, Hkv=Hkv, D=D, P=P, L=L, dtype=dtype)
    ragged = g.random() < 0.5
    pl = g.integers(k + 1, L + 1, B).astype(np.int32) if ragged else None
    return cfg, pl


@pytest.mark.parametrize("seed", range(48))
def test_attention_random_shape(lotts, oracle, seed):
    cfg, pl = random_attention_case(seed)
    print("random attention case", seed, cfg, None if pl is None else pl.tolist(), flush=True)
    a = S.attention_inputs(cfg, priv_len=pl, salt=seed)
    d = attn_to_dev(cfg, a)
    O, lse = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], return_lse=True)
    torch.cuda.synchronize()
    Oref, lref = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    e_abs, e_fro, _ = attn_errors(O, Oref)
    tol = TOL[cfg.dtype]
    assert e_abs <= tol["abs"] and e_fro <= tol["fro"], (e_abs, e_fro)
    assert np.abs(lse.cpu().numpy().astype(np.float64) - lref).max() <= tol["lse"]


@pytest.mark.parametrize("seed", range(16))
def test_accept_random_shape(lotts, oracle, seed):
    g = np.random.default_rng(2000 + seed)
    B, k = int(g.integers(1, 40)), int(g.integers(0, 9))
    V = int(g.choice([int(g.integers(1, 300)), int(g.integers(300, 9000)), 4 * int(g.integers(500, 9000))]))
    cfg = S.CONFIGS["C2"].with_(B=B, k=k, V=V, noise_std=float(g.choice([0.3, 1.0, 3.0])))
    print("random accept case", seed, B, k, V, flush=True)
    s = S.accept_inputs(cfg, salt=seed)
    n, t = lotts.spec_accept(to_dev(s["p"]), to_dev(s["q"]) if k else None, to_dev(s["draft"]) if k else None,
                             to_dev(s["u"]))
    n_ref, t_ref = oracle.spec_accept(s["p"], s["q"], s["draft"], s["u"])
    assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)


@pytest.mark.parametrize("seed", range(16))
def test_accept_logits_random_shape(lotts, oracle, seed):
    g = np.random.default_rng(3000 + seed)
    B, k = int(g.integers(1, 24)), int(g.integers(0, 7))
    V = int(g.choice([int(g.integers(1, 300)), int(g.integers(300, 9000)), 8 * int(g.integers(300, 6000))]))
    bf16 = bool(g.random() < 0.5)
    inv_temp = float(g.choice([0.5, 1.0, 1.7]))
    print("random accept-from-logits case", seed, B, k, V, bf16, inv_temp, flush=True)
    zt = (g.standard_normal((B, k + 1, V)) * 2.0).astype(np.float32)
    zd = (zt[:, :k] + g.standard_normal((B, k, V)) * float(g.choice([0.3, 1.0]))).astype(np.float32)
    if bf16:
        zt, zd = S.f32_to_bf16_bits(zt), S.f32_to_bf16_bits(zd)
    draft = g.integers(0, V, (B, k)).astype(np.int32)
    if k and V > 1:                                           # mostly plausible drafts: the draft row's arg-max
        zd_f = S.bf16_bits_to_f32(zd) if bf16 else zd
        likely = zd_f.argmax(-1).astype(np.int32)
        draft = np.where(g.random((B, k)) < 0.7, likely, draft).astype(np.int32)
    u = (g.integers(0, 1 << 24, (B, k + 1)) / float(1 << 24)).astype(np.float32)
    pl = g.integers(k + 1, 5000, B).astype(np.int32)
    pl_dev = to_dev(pl)
    n, t = lotts.spec_accept_logits(to_dev(zt, bf16), to_dev(zd, bf16) if k else None, to_dev(draft) if k else None,
                                    to_dev(u), inv_temperature=inv_temp, priv_len=pl_dev)
    pl_ref = pl.copy()
    n_ref, t_ref = oracle.spec_accept_logits(zt, zd if k else None, draft if k else None, u, inv_temp, priv_len=pl_ref)
    assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)
    assert np.array_equal(pl_dev.cpu().numpy(), pl_ref)


@pytest.mark.parametrize("seed", range(12))
def test_skinny_gemm_random_shape(lotts, oracle, seed):
    g = np.random.default_rng(4000 + seed)
    M = int(g.integers(1, 257))
    N = 8 * int(g.integers(1, 400))
    K = 128 * int(g.integers(1, 40))
    print("random gemm case", seed, M, N, K, flush=True)
    X = S.f32_to_bf16_bits((g.standard_normal((M, K)) * 1.0).astype(np.float32))
    W = S.f32_to_bf16_bits((g.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    Y = lotts.skinny_gemm(to_dev(X, True), to_dev(W, True))
    ref = oracle.skinny_gemm(X, W)
    y = Y.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(y - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-3)
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) <= 3e-3


@pytest.mark.parametrize("seed", range(8))
def test_votes_random_shape(lotts, oracle, seed):
    g = np.random.default_rng(5000 + seed)
    N, B, T = int(g.integers(1, 9)), int(g.integers(1, 300)), int(g.integers(1, 200))
    ans = g.integers(-1, int(g.integers(1, 12)), (N, B)).astype(np.int32)
    conf = g.random((N, B, T)).astype(np.float32)
    clen = g.integers(0, T + 1, (N, B)).astype(np.int32)
    w, c = lotts.majority_vote(to_dev(ans))
    w_ref, c_ref = oracle.majority_vote(ans)
    assert np.array_equal(w.cpu().numpy(), w_ref) and np.array_equal(c.cpu().numpy(), c_ref)
    for wm in ("min", "avg"):
        for sm in ("max", "vote"):
            w, s = lotts.confidence_vote(to_dev(ans), to_dev(conf), conf_len=to_dev(clen), weight_mode=wm, select_mode=sm)
            w_ref, s_ref = oracle.confidence_vote(ans, conf, clen, wm, sm)
            assert np.array_equal(w.cpu().numpy(), w_ref), (wm, sm)
            assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), (wm, sm)
