"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the CPU
oracle on the same seeded inputs.  Indices must match bit for bit; attention must stay within
2e-2 max-abs and 1e-2 Frobenius-relative of the fp64 oracle for bf16 (1e-4 / 1e-4 for fp32)."""
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


def run_attention(lotts, oracle, cfg, priv_len=None, Lmax=None, scale=0.0):
    a = S.attention_inputs(cfg, priv_len=priv_len, Lmax=Lmax)
    d = attn_to_dev(cfg, a)
    print("attention case", cfg, "priv_len", None if priv_len is None else list(priv_len), flush=True)
    O, lse = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"],
                                    scale=scale, return_lse=True)
    torch.cuda.synchronize()
    Oref, lref = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"],
                                         scale=scale)
    e_abs, e_fro, e_rel = attn_errors(O, Oref)
    tol = TOL[cfg.dtype]
    print("  max-abs %.3g  fro-rel %.3g  max-rel(not small) %.3g" % (e_abs, e_fro, e_rel), flush=True)
    assert e_abs <= tol["abs"] and e_fro <= tol["fro"]
    assert e_fro <= tol["fro_band"], "accuracy regression: Frobenius-relative error %g" % e_fro
    assert tol["rel_band"] is None or e_rel <= tol["rel_band"], "accuracy regression: element-wise relative error %g" % e_rel
    assert np.abs(lse.cpu().numpy().astype(np.float64) - lref).max() <= tol["lse"]
    return O


BF = S.CONFIGS["C3"]
SMALL_ATTN = [
    S.CONFIGS["C1"],                                                 # tiny fp32, the configs[0] case
    S.CONFIGS["C1"].with_(B=3, Hq=8, Hkv=2, D=128, P=50, L=77, k=2),  # fp32, GQA, D=128, ragged tiles
    BF.with_(B=3, P=96, L=200),                                      # several tiles + ragged tail, G*R = 20
    BF.with_(B=2, P=0, L=131),                                       # no prefix
    BF.with_(B=5, P=33, L=4, k=3),                                   # private cache = the new tokens only
    BF.with_(B=2, P=70, L=300, k=0),                                 # k = 0: decode attention
    BF.with_(B=3, Hq=16, Hkv=2, k=4, P=64, L=257),                   # G*R = 40: two row tiles
    BF.with_(B=2, Hq=40, Hkv=8, k=8, P=40, L=190),                   # G*R = 45
    BF.with_(B=64, Hq=16, Hkv=2, k=4, P=64, L=600),                  # G*R = 40 on 128 (head, branch) pairs: eight wavefronts per item, merge in the launch
    BF.with_(B=2, Hq=32, Hkv=2, k=4, P=64, L=140),                   # G*R = 80: more than one row group
    BF.with_(B=4, Hq=8, Hkv=4, D=64, P=100, L=333, k=3),             # head_dim 64
    BF.with_(B=2, Hq=12, Hkv=2, D=64, k=6, P=31, L=95),              # head_dim 64, two row tiles
    BF.with_(B=37, Hq=4, Hkv=4, k=1, P=300, L=65),                   # many branches stacked on the prefix
    BF.with_(B=8, P=2048, L=512),                                    # long prefix: stacked plan, several prefix splits
    BF.with_(B=5, Hq=16, Hkv=2, k=4, P=1500, L=300),                 # stacked plan with two row tiles per item
    BF.with_(B=2, Hq=16, Hkv=2, k=2, P=64, L=4000),                  # few (head, branch) pairs: 16 key splits, separate merge launch
    BF.with_(B=3, Hq=8, Hkv=8, k=0, P=16, L=1000),                   # k = 0 with folded prefix shorter than a tile
]


@pytest.mark.parametrize("cfg", SMALL_ATTN, ids=lambda c: "B%d_k%d_H%d-%d_D%d_P%d_L%d_%s" % (
    c.B, c.k, c.Hq, c.Hkv, c.D, c.P, c.L, c.dtype))
def test_attention_small(lotts, oracle, cfg):
    run_attention(lotts, oracle, cfg)


def test_attention_ragged_private_lengths(lotts, oracle):
    cfg = BF.with_(B=6, P=128, L=700)
    pl = np.array([700, 4, 5, 333, 32, 699], dtype=np.int32)
    run_attention(lotts, oracle, cfg, priv_len=pl)
    run_attention(lotts, oracle, cfg.with_(dtype="f32", Hq=8, Hkv=8, D=64, L=90, P=20),
                  priv_len=np.array([90, 4, 5, 33, 32, 89], dtype=np.int32))


def test_attention_explicit_scale(lotts, oracle):
    run_attention(lotts, oracle, BF.with_(B=2, P=64, L=100), scale=0.2)


def test_attention_token_major_layout(lotts, oracle):
    """K/V stored [B][L][Hkv][D] (token-major) reach the kernel through the strides."""
    cfg = BF.with_(B=3, P=96, L=200)
    a = S.attention_inputs(cfg)
    d = attn_to_dev(cfg, a)
    kp = d["Kpriv"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    vp = d["Vpriv"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    kpre = d["Kpre"].permute(1, 0, 2).contiguous().permute(1, 0, 2)
    vpre = d["Vpre"].permute(1, 0, 2).contiguous().permute(1, 0, 2)
    assert not kp.is_contiguous()
    O = lotts.verify_attention(d["Q"], kpre, vpre, kp, vp, d["priv_len"])
    O2 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    assert torch.equal(O, O2)            # same arithmetic, only the addresses differ
    Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    e_abs, e_fro, _ = attn_errors(O, Oref)
    assert e_abs <= 2e-2 and e_fro <= 1e-2


def test_attention_workspace_survives_geometry_changes(lotts, oracle):
    """One caller-owned workspace, zero-filled once, serves calls of different geometry in any order:
    every call leaves the arrival counters zero."""
    import ctypes
    from paper_2505_19634_amd import binding
    lib = binding.load()
    ws = torch.zeros(32 << 20, dtype=torch.uint8, device=DEV)
    cases = [BF.with_(B=3, P=96, L=200), BF.with_(B=37, Hq=4, Hkv=4, k=1, P=300, L=65), BF.with_(B=2, P=0, L=131),
             BF.with_(B=2, Hq=16, Hkv=2, k=2, P=64, L=4000), BF.with_(B=3, P=96, L=200)]
    for cfg in cases:
        a = S.attention_inputs(cfg)
        d = attn_to_dev(cfg, a)
        O = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], workspace=ws)
        torch.cuda.synchronize()
        Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
        e_abs, e_fro, _ = attn_errors(O, Oref)
        assert e_abs <= 2e-2 and e_fro <= 1e-2, cfg
        assert int(ws[:131072].view(torch.int64).abs().sum()) == 0     # completed calls leave their arrival cells zero


def test_attention_is_deterministic(lotts):
    cfg = BF.with_(B=4, P=128, L=900)
    d = attn_to_dev(cfg, S.attention_inputs(cfg))
    O1 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"]).clone()
    O2 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    assert torch.equal(O1, O2)


def test_attention_ignores_what_rows_cannot_see(lotts):
    """NaNs in later drafts' K/V rows and beyond priv_len must not reach earlier rows."""
    cfg = BF.with_(B=2, P=64, L=150)
    a = S.attention_inputs(cfg, priv_len=np.array([150, 100], np.int32))
    d = attn_to_dev(cfg, a)
    O1 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"]).clone()
    d["Kpriv"][1, :, 100:] = float("nan")          # beyond the branch's length
    d["Vpriv"][1, :, 100:] = float("nan")
    d["Kpriv"][0, :, 149] = float("inf")           # the last draft's own K/V: only row k may see it
    O2 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    assert torch.equal(O1[1], O2[1])
    assert torch.equal(O1[0, :cfg.k], O2[0, :cfg.k])


@pytest.mark.parametrize("name", ["C2", "C3", "C5"])
def test_attention_full_size(lotts, oracle, name):
    """The paper-shaped workloads at full size, in the launch configuration bench.py times."""
    run_attention(lotts, oracle, S.CONFIGS[name])


@pytest.mark.parametrize("B", [1, 4, 16, 64])
def test_attention_branch_sweep(lotts, oracle, B):
    """The branch-scaling workload (Section 3.2, branch-wise parallelism) at every point of its sweep."""
    run_attention(lotts, oracle, S.CONFIGS["C4"].with_(B=B))


# ---------------------------------------------------------------------------- acceptance
def run_accept(lotts, oracle, s):
    p, q, draft, u = s["p"], s["q"], s["draft"], s["u"]
    k = p.shape[1] - 1
    n, t = lotts.spec_accept(to_dev(p), to_dev(q) if k else None, to_dev(draft) if k else None, to_dev(u))
    torch.cuda.synchronize()
    n_ref, t_ref = oracle.spec_accept(p, q, draft, u)
    assert np.array_equal(n.cpu().numpy(), n_ref), (n.cpu().numpy(), n_ref)
    assert np.array_equal(t.cpu().numpy(), t_ref), (t.cpu().numpy(), t_ref)
    return n_ref, t_ref


@pytest.mark.parametrize("cfg", [
    S.CONFIGS["C1"],
    S.CONFIGS["C1"].with_(B=7, V=999, k=2),            # V not a multiple of 4: scalar loads
    S.CONFIGS["C1"].with_(B=5, V=2048 * 3 + 1, k=5),   # one element into a fourth chunk
    S.CONFIGS["C1"].with_(B=9, V=4, k=1),
    S.CONFIGS["C1"].with_(B=3, V=1, k=2),
    S.CONFIGS["C1"].with_(B=6, V=5000, k=0),           # k = 0: plain sampling from p_0
    S.CONFIGS["C2"].with_(B=33, V=20000, k=8),
    S.CONFIGS["C5"].with_(B=64, V=40000),              # frequent rejection
    S.CONFIGS["C2"].with_(B=3, V=262144, k=2),         # the largest vocabulary the one-launch path takes
    S.CONFIGS["C2"].with_(B=3, V=262148, k=2),         # just beyond it: two launches
    S.CONFIGS["C2"].with_(B=5, V=16384 + 4, k=3),      # a last sub-chunk of one group of 4
    S.CONFIGS["C2"].with_(B=300, V=1024, k=1),         # many branches, one workgroup each
    S.CONFIGS["C2"].with_(B=2000, V=8192, k=2),        # more workgroups than the chip holds at once: collectors wait for earlier ones
    S.CONFIGS["C2"].with_(B=65535, V=256, k=1),        # the largest branch count
], ids=lambda c: "B%d_k%d_V%d" % (c.B, c.k, c.V))
def test_accept_small(lotts, oracle, cfg):
    print("accept case", cfg, flush=True)
    run_accept(lotts, oracle, S.accept_inputs(cfg))


def full_size(name):
    return S.CONFIGS["C4"].with_(B=int(name[3:])) if name.startswith("C4x") else S.CONFIGS[name]


@pytest.mark.parametrize("name", ["C2", "C3", "C5", "C4x16", "C4x64"])
def test_accept_full_size(lotts, oracle, name):
    cfg = full_size(name)
    print("accept case", cfg, flush=True)
    n, _ = run_accept(lotts, oracle, S.accept_inputs(cfg))
    assert n.min() < cfg.k or cfg.B < 4                # rejections do occur


def test_accept_many_uniforms_on_one_row(lotts, oracle):
    """Sweep the sampling uniform densely over fixed rows: every crossing the oracle finds, the GPU finds."""
    cfg = S.CONFIGS["C2"].with_(B=1, V=30000, k=2)
    s = S.accept_inputs(cfg)
    N = 4096
    g = np.random.default_rng(5)
    p = np.ascontiguousarray(np.broadcast_to(s["p"], (N, 3, cfg.V)))
    q = np.ascontiguousarray(np.broadcast_to(s["q"], (N, 2, cfg.V)))
    draft = g.integers(0, cfg.V, size=(N, 2)).astype(np.int32)
    u = (g.integers(0, 1 << 24, size=(N, 3)) / float(1 << 24)).astype(np.float32)
    u[::5, 2] = 0.0
    u[1::5, 2] = np.nextafter(np.float32(1), np.float32(0))
    n, t = run_accept(lotts, oracle, dict(p=p, q=q, draft=draft, u=u))
    assert len(np.unique(t)) > 1000


def test_accept_degenerate_rows(lotts, oracle):
    V, k = 4096, 2
    g = np.random.default_rng(9)
    x = g.random((4, k + 1, V)).astype(np.float32)
    p = (x / x.sum(-1, keepdims=True)).astype(np.float32)
    q = p[:, :k].copy()                         # identical: everything is accepted unless p(x) = 0
    draft = np.array([[5, 6], [7, 8], [9, 10], [11, 12]], np.int32)
    p[1, 0, 7] = 0.0
    q[1, 0, 7] = 0.0                            # branch 1: rejected at 0 with an empty residual -> sample p_0
    p[2] = 0.0
    q[2] = 0.0                                  # branch 2: no mass anywhere -> -1
    p[3, 1, :] = 0.0
    p[3, 1, 100] = 1.0                          # branch 3: one-hot target at position 1, draft 12 rejected
    u = np.array([[0.3, 0.4, 0.5]] * 4, np.float32)
    n, t = run_accept(lotts, oracle, dict(p=p, q=q, draft=draft, u=u))
    assert list(n) == [2, 0, 0, 1] and t[2] == -1 and t[3] == 100


def test_accept_with_a_workspace_full_of_garbage(lotts, oracle):
    """The words the workgroups of a branch exchange carry a per-call tag, so whatever the workspace holds -- random
    bytes, or the words of earlier calls -- is not mistaken for this call's sums."""
    cfg = S.CONFIGS["C3"].with_(B=8, V=50000)
    s = S.accept_inputs(cfg)
    d = [to_dev(s[x]) for x in ("p", "q", "draft", "u")]
    n_ref, t_ref = oracle.spec_accept(s["p"], s["q"], s["draft"], s["u"])
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    ws = torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device=DEV, generator=g)
    for _ in range(3):                                   # the second and third call find the first one's leftovers
        n, t = lotts.spec_accept(*d, workspace=ws)
        assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)


def test_accept_is_deterministic(lotts):
    cfg = S.CONFIGS["C3"].with_(B=8, V=50000)
    s = S.accept_inputs(cfg)
    d = [to_dev(s[x]) for x in ("p", "q", "draft", "u")]
    n1, t1 = lotts.spec_accept(*d)
    n1, t1 = n1.clone(), t1.clone()
    n2, t2 = lotts.spec_accept(*d)
    assert torch.equal(n1, n2) and torch.equal(t1, t2)


# ---------------------------------------------------------------------------- vote
@pytest.mark.parametrize("N,B", [(1, 16), (1, 1), (7, 64), (5, 65), (4, 63), (3, 4096), (50, 33)])
def test_vote(lotts, oracle, N, B):
    cfg = S.CONFIGS["C3"].with_(B=B)
    a = S.vote_inputs(cfg, N=N, salt=B)
    if N > 1:
        a[1, ::3] = -1
        a[2, :] = -1
    w, c = lotts.majority_vote(to_dev(a))
    w_ref, c_ref = oracle.majority_vote(a)
    assert np.array_equal(w.cpu().numpy(), w_ref) and np.array_equal(c.cpu().numpy(), c_ref)


def test_vote_ties_go_to_first_occurrence(lotts, oracle):
    a = np.array([[4, 9, 9, 4, 2], [9, 4, 4, 9, 2], [1, 2, 3, 4, 5], [-1, 3, -1, 3, 7]], np.int32)
    w, c = lotts.majority_vote(to_dev(a))
    assert w.cpu().tolist() == [4, 9, 1, 3] and c.cpu().tolist() == [2, 2, 1, 2]
    w_ref, c_ref = oracle.majority_vote(a)
    assert w.cpu().tolist() == list(w_ref) and c.cpu().tolist() == list(c_ref)


# ---------------------------------------------------------------------------- acceptance from logits
def logit_inputs(cfg, noise_std, salt=0, bf16=False):
    g = S.rng_for(cfg.number, 20, salt)
    zt = (g.standard_normal((cfg.B, cfg.k + 1, cfg.V), dtype=np.float32) * np.float32(2.0))
    zd = zt[:, :cfg.k] + g.standard_normal((cfg.B, cfg.k, cfg.V), dtype=np.float32) * np.float32(noise_std)
    if bf16:
        zt, zd = S.f32_to_bf16_bits(zt), S.f32_to_bf16_bits(zd)
        zd_f = S.bf16_bits_to_f32(zd)
    else:
        zd_f = zd
    from scipy.special import softmax
    draft = np.zeros((cfg.B, cfg.k), np.int32)
    for b in range(cfg.B):
        for j in range(cfg.k):
            c = np.cumsum(softmax(zd_f[b, j].astype(np.float64)))
            draft[b, j] = min(int(np.searchsorted(c, g.random() * c[-1], side="right")), cfg.V - 1)
    u = (g.integers(0, 1 << 24, (cfg.B, cfg.k + 1)) / float(1 << 24)).astype(np.float32)
    return np.ascontiguousarray(zt), np.ascontiguousarray(zd), draft, u


@pytest.mark.parametrize("cfg,bf16,inv_temp", [
    (S.CONFIGS["C1"], False, 1.0),
    (S.CONFIGS["C1"].with_(B=7, V=999, k=2), False, 0.8),          # scalar loads
    (S.CONFIGS["C1"].with_(B=5, V=2048 * 3 + 8, k=5), True, 1.0),
    (S.CONFIGS["C1"].with_(B=6, V=5000, k=0), True, 1.3),
    (S.CONFIGS["C1"].with_(B=3, V=1, k=2), False, 1.0),
    (S.CONFIGS["C2"].with_(B=33, V=20000, k=8), True, 1.0),
    (S.CONFIGS["C5"].with_(B=16, V=40000), False, 1.0),
    (S.CONFIGS["C3"], True, 1.0),                                  # full 32B-shaped size, bf16 logits
    (S.CONFIGS["C3"], False, 0.7),
    (S.CONFIGS["C4"].with_(B=64), True, 1.0),                      # the branch sweep's largest point, bf16 logits
    (S.CONFIGS["C2"].with_(B=1500, V=4096, k=2), True, 1.0),       # more workgroups than the chip holds at once
    # many token decisions at a temperature other than 1
    (S.CONFIGS["C1"].with_(B=2, V=1 << 20, k=1), True, 1.0),       # the largest vocabulary: 64 pieces per row, 512 chunks
    (S.CONFIGS["C1"].with_(B=600, V=999, k=2), False, 0.8),
    (S.CONFIGS["C1"].with_(B=300, V=4096, k=2), True, 1.3),
], ids=lambda x: str(x) if not hasattr(x, "B") else "B%d_k%d_V%d" % (x.B, x.k, x.V))
def test_accept_logits(lotts, oracle, cfg, bf16, inv_temp):
    print("accept-from-logits case", cfg, bf16, inv_temp, flush=True)
    zt, zd, draft, u = logit_inputs(cfg, cfg.noise_std or 1.0, bf16=bf16)
    n, t = lotts.spec_accept_logits(to_dev(zt, bf16), to_dev(zd, bf16) if cfg.k else None,
                                    to_dev(draft) if cfg.k else None, to_dev(u), inv_temperature=inv_temp)
    torch.cuda.synchronize()
    n_ref, t_ref = oracle.spec_accept_logits(zt, zd, draft, u, inv_temp)
    assert np.array_equal(n.cpu().numpy(), n_ref), (n.cpu().numpy(), n_ref)
    assert np.array_equal(t.cpu().numpy(), t_ref), (t.cpu().numpy(), t_ref)


def test_accept_logits_degenerate(lotts, oracle):
    V, k = 4096, 2
    g = np.random.default_rng(9)
    zt = g.normal(0, 2, (6, k + 1, V)).astype(np.float32)
    zd = zt[:, :k].copy()                          # identical rows: accepted unless the token has no weight
    zt[1, 0, 7] = zd[1, 0, 7] = -1e5               # branch 1: draft 7 weighs 0 on both sides -> rejected, empty residual
    zt[2, 1, :] = -1e5
    zt[2, 1, 100] = 0.0                            # branch 2: one-hot target at position 1
    zd[3, 0, :] = -np.inf
    zd[3, 0, 11] = 0.0                             # branch 3: -inf logits in the draft row
    zt[4, 1, :] = -np.inf                          # branch 4: a target row without any weight -> rejected there, token -1
    zt[5, 2, :] = -np.inf                          # branch 5: everything accepted, then a bonus row without weight -> -1
    draft = np.array([[5, 6], [7, 8], [9, 10], [11, 12], [13, 14], [15, 16]], np.int32)
    u = np.array([[0.3, 0.4, 0.5]] * 6, np.float32)
    nt = torch.full((6,), -7, dtype=torch.int32, device=DEV)
    n, t = lotts.spec_accept_logits(to_dev(zt), to_dev(zd), to_dev(draft), to_dev(u), next_token=nt)
    n_ref, t_ref = oracle.spec_accept_logits(zt, zd, draft, u)
    assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)
    assert n_ref[0] == 2 and n_ref[1] == 0 and n_ref[2] == 1 and t_ref[2] == 100
    assert n_ref[4] == 1 and t_ref[4] == -1 and n_ref[5] == 2 and t_ref[5] == -1


@pytest.mark.parametrize("bf16,inv_temp", [(False, 0.8), (True, 1.3), (True, 1.0)])
def test_accept_logits_row_sums_are_the_definitions(lotts, oracle, bf16, inv_temp):
    """White box: the integer weight sum S and the maximum of every row, as the launches leave them in the
    workspace, against the oracle's bit for bit.  The outputs alone hardly see a weight that is off by one (a
    token changes only if the threshold falls into that sliver of the CDF), and that is what a scaling and a
    subtraction merged into one fused operation -- one rounding instead of the definition's two -- produces."""
    cfg = S.CONFIGS["C1"].with_(B=5, V=40000, k=2)
    zt, zd, draft, u = logit_inputs(cfg, 1.0, salt=77, bf16=bf16)
    rows = cfg.B * (2 * cfg.k + 1)
    up = lambda x: (x + 255) & ~255
    npieces = (cfg.V + 16383) // 16384
    off_rmax = up(rows * npieces * 4)                      # piece maxima come first
    off_rsum = off_rmax + up(rows * 4)
    ws = torch.zeros((lotts.load().spec_accept_logits_workspace_bytes(cfg.B, cfg.k, cfg.V),), dtype=torch.uint8, device=DEV)
    lotts.spec_accept_logits(to_dev(zt, bf16), to_dev(zd, bf16), to_dev(draft), to_dev(u), inv_temperature=inv_temp,
                             workspace=ws)
    torch.cuda.synchronize()
    rmax = ws[off_rmax:off_rmax + rows * 4].view(torch.float32).cpu().numpy()
    rsum = ws[off_rsum:off_rsum + rows * 8].view(torch.int64).cpu().numpy()
    all_rows = [zt[b, j] for b in range(cfg.B) for j in range(cfg.k + 1)] + \
               [zd[b, j] for b in range(cfg.B) for j in range(cfg.k)]
    for r, z in enumerate(all_rows):
        E, S_ref = oracle.logit_weights(z, inv_temp)
        zf = S.bf16_bits_to_f32(z) if bf16 else z
        assert int(rsum[r]) == S_ref, (r, int(rsum[r]), S_ref)
        assert rmax[r] == (zf.astype(np.float32) * np.float32(inv_temp)).max(), r


def test_accept_logits_with_a_workspace_full_of_garbage(lotts, oracle):
    """Every word the workgroups of the one launch hand to each other carries the call's tag: random bytes, or
    the words of earlier calls on other sizes, are not taken for this call's."""
    g = torch.Generator(device=DEV)
    g.manual_seed(12)
    ws = torch.randint(0, 256, (8 << 20,), dtype=torch.uint8, device=DEV, generator=g)
    for cfg in (S.CONFIGS["C2"].with_(B=6, V=40000, k=3), S.CONFIGS["C2"].with_(B=9, V=20000, k=2),
                S.CONFIGS["C2"].with_(B=6, V=40000, k=3)):
        print("garbage workspace, logits", cfg, flush=True)
        zt, zd, draft, u = logit_inputs(cfg, 1.0, salt=cfg.B, bf16=True)
        n_ref, t_ref = oracle.spec_accept_logits(zt, zd, draft, u)
        for _ in range(2):
            n, t = lotts.spec_accept_logits(to_dev(zt, True), to_dev(zd, True), to_dev(draft), to_dev(u), workspace=ws)
            assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)


def test_accept_and_accept_logits_can_share_one_workspace(lotts, oracle):
    """Both exchange tagged words through the workspace; the tags come from one counter, so calls of the two
    entry points that alternate on one buffer never take each other's leftovers for their own."""
    cfg = S.CONFIGS["C2"].with_(B=8, V=50000, k=3)
    s = S.accept_inputs(cfg)
    d = [to_dev(s[x]) for x in ("p", "q", "draft", "u")]
    n_ref, t_ref = oracle.spec_accept(s["p"], s["q"], s["draft"], s["u"])
    zt, zd, draft, u = logit_inputs(cfg, 1.0, salt=5, bf16=True)
    z = [to_dev(zt, True), to_dev(zd, True), to_dev(draft), to_dev(u)]
    ln_ref, lt_ref = oracle.spec_accept_logits(zt, zd, draft, u)
    ws = torch.zeros((8 << 20,), dtype=torch.uint8, device=DEV)
    for _ in range(4):
        n, t = lotts.spec_accept(*d, workspace=ws)
        ln, lt = lotts.spec_accept_logits(*z, workspace=ws)
        assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref)
        assert np.array_equal(ln.cpu().numpy(), ln_ref) and np.array_equal(lt.cpu().numpy(), lt_ref)


def test_accept_logits_can_be_captured_and_replayed_on_new_logits(lotts, oracle):
    """A captured launch keeps its tag, so the launch itself clears every word it exchanged: replays on new
    logits in the same buffers must equal eager calls, with eager calls on the same workspace in between."""
    cfg = S.CONFIGS["C2"].with_(B=8, V=50000, k=3)
    sets = [logit_inputs(cfg, 1.0, salt=40 + i, bf16=True) for i in range(3)]
    refs = [oracle.spec_accept_logits(*x) for x in sets]
    zt, zd = to_dev(sets[0][0], True), to_dev(sets[0][1], True)
    draft, u = to_dev(sets[0][2]), to_dev(sets[0][3])
    n = torch.empty((cfg.B,), dtype=torch.int32, device=DEV)
    t = torch.empty((cfg.B,), dtype=torch.int32, device=DEV)
    ws = torch.zeros((lotts.load().spec_accept_logits_workspace_bytes(cfg.B, cfg.k, cfg.V),), dtype=torch.uint8, device=DEV)
    call = lambda stream=None: lotts.spec_accept_logits(zt, zd, draft, u, accept_len=n, next_token=t, workspace=ws,
                                                        stream=stream)
    call()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream())
    for rep in range(6):
        i = rep % 3
        zt.copy_(to_dev(sets[i][0], True)); zd.copy_(to_dev(sets[i][1], True))
        draft.copy_(to_dev(sets[i][2])); u.copy_(to_dev(sets[i][3]))
        if rep % 2:                                        # an eager call (new tag) on the same workspace in between
            call()
        n.fill_(-7); t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(n.cpu().numpy(), refs[i][0]) and np.array_equal(t.cpu().numpy(), refs[i][1]), rep


def test_accept_logits_against_the_probability_oracle(lotts, oracle):
    """A check of spec_accept_logits that shares nothing with its integer softmax: the same logits go through an
    fp64 softmax (scipy) into the probability-path ORACLE.  The two paths quantise differently (2^-30 integer
    weights against fp32 probabilities), so single decisions that sit on a boundary may differ, but on nearly
    every branch accepted length and token must be the same."""
    from scipy.special import softmax
    cfg = S.CONFIGS["C2"].with_(B=768, V=6000, k=3)
    zt, zd, draft, u = logit_inputs(cfg, 0.7, salt=3, bf16=True)
    print("logits against the probability oracle", cfg, flush=True)
    n, t = lotts.spec_accept_logits(to_dev(zt, True), to_dev(zd, True), to_dev(draft), to_dev(u))
    torch.cuda.synchronize()
    p = softmax(S.bf16_bits_to_f32(zt).astype(np.float64), axis=-1).astype(np.float32)
    q = softmax(S.bf16_bits_to_f32(zd).astype(np.float64), axis=-1).astype(np.float32)
    n_ref, t_ref = oracle.spec_accept(p, q, draft, u)
    same = (n.cpu().numpy() == n_ref) & (t.cpu().numpy() == t_ref)
    print("  agreement %.4f, mean accepted %.2f" % (same.mean(), n_ref.mean()), flush=True)
    assert same.mean() >= 0.995
    assert 0 < n_ref.mean() < cfg.k                 # both outcomes occur


def test_multi_step_decode_loop_stays_on_the_device(lotts, oracle):
    """Several verify steps enqueued back to back with no host round trip: the step's new K and V rows appended at
    each branch's tail, attention over each branch's current cache, acceptance from logits, and the rollback that
    tells the next step where each branch's cache ends (its append then overwrites the rejected drafts' rows).
    Branches drift apart in length as they accept different numbers of drafts; every step is checked."""
    cfg = BF.with_(B=6, P=96, L=640, k=3, V=5000)
    steps = 5
    a = S.attention_inputs(cfg)
    d = attn_to_dev(cfg, a)
    cache0 = np.array([10, 100, 200, 37, 0, 300], dtype=np.int32)   # valid private tokens before the first step
    logits = [logit_inputs(cfg, 0.8, salt=s, bf16=True) for s in range(steps)]
    g = S.rng_for(3, 41)
    new_rows = [tuple(S.f32_to_bf16_bits((0.5 * g.standard_normal((cfg.B, cfg.k + 1, cfg.Hkv, cfg.D))).astype(np.float32))
                      for _ in range(2)) for _ in range(steps)]
    print("multi-step loop", cfg, flush=True)
    pl_dev = to_dev(cache0 + cfg.k + 1)
    got = []
    for s in range(steps):
        zt, zd, draft, u = logits[s]
        lotts.kv_append(to_dev(new_rows[s][0], True), to_dev(new_rows[s][1], True), d["Kpriv"], d["Vpriv"], pl_dev)
        O = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], pl_dev)
        n, t = lotts.spec_accept_logits(to_dev(zt, True), to_dev(zd, True), to_dev(draft), to_dev(u), priv_len=pl_dev)
        got.append((O.clone(), n.clone(), t.clone(), pl_dev.clone()))
        pl_dev += cfg.k + 1                                          # the next step appends its k + 1 new tokens
    torch.cuda.synchronize()
    pl = (cache0 + cfg.k + 1).astype(np.int32)
    Kc, Vc = a["Kpriv"], a["Vpriv"]
    for s in range(steps):
        zt, zd, draft, u = logits[s]
        Kc, Vc = oracle.kv_append(new_rows[s][0], new_rows[s][1], Kc, Vc, pl)
        Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], Kc, Vc, pl)
        n_ref, t_ref = oracle.spec_accept_logits(zt, zd, draft, u, priv_len=pl)
        O, n, t, pl_after = got[s]
        e_abs, e_fro, _ = attn_errors(O, Oref)
        assert e_abs <= 2e-2 and e_fro <= 1e-2, (s, e_abs, e_fro)
        assert np.array_equal(n.cpu().numpy(), n_ref) and np.array_equal(t.cpu().numpy(), t_ref), s
        assert np.array_equal(pl_after.cpu().numpy(), pl), s
        pl = (pl + cfg.k + 1).astype(np.int32)
    assert len(set((pl - cache0).tolist())) > 1                      # the branches did drift apart
    assert np.array_equal(d["Kpriv"].view(torch.uint16).cpu().numpy(), Kc)   # the caches went through the same history


# ---------------------------------------------------------------------------- confidence-weighted vote
@pytest.mark.parametrize("N,B,T", [(1, 16, 64), (5, 16, 1000), (3, 64, 37), (2, 1, 5), (2, 1024, 3)])
def test_confidence_vote(lotts, oracle, N, B, T):
    cfg = S.CONFIGS["C3"].with_(B=B)
    g = S.rng_for(3, S.T_CONF, salt=B + T)
    answers = S.vote_inputs(cfg, N=N, salt=T)
    answers[g.random((N, B)) < 0.1] = -1
    conf = (0.3 + 0.7 * g.random((N, B, T))).astype(np.float32)
    lens = g.integers(0, T + 1, (N, B)).astype(np.int32)
    for wm in ("min", "avg"):
        for sm in ("max", "vote"):
            for cl in (None, lens):
                w, s = lotts.confidence_vote(to_dev(answers), to_dev(conf), None if cl is None else to_dev(cl),
                                             weight_mode=wm, select_mode=sm)
                w_ref, s_ref = oracle.confidence_vote(answers, conf, cl, wm, sm)
                assert np.array_equal(w.cpu().numpy(), w_ref), (wm, sm)
                assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), (wm, sm)


# ---------------------------------------------------------------------------- cache append
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_kv_append_matches_the_oracle_bit_for_bit(lotts, oracle, dtype):
    """The new tokens' K and V, taken as strided views out of a projection-shaped matrix, land at the tail of every
    branch's private cache (ragged lengths, one branch shorter than k + 1 and one beyond the cache: skipped rows);
    every other element of the caches keeps its bits."""
    g = S.rng_for(7, 40, salt=len(dtype))
    B, k, Hq, Hkv, D, Lmax = 5, 3, 6, 2, 128 if dtype == "bf16" else 64, 300
    R = k + 1
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    qkv = (torch.from_numpy(g.standard_normal((B * R, (Hq + 2 * Hkv) * D), dtype=np.float32)).to(DEV)).to(tdt)
    v5 = qkv.view(B, R, Hq + 2 * Hkv, D)
    Knew, Vnew = v5[:, :, Hq:Hq + Hkv], v5[:, :, Hq + Hkv:]
    Kpriv = torch.from_numpy(g.standard_normal((B, Hkv, Lmax, D), dtype=np.float32)).to(DEV).to(tdt)
    Vpriv = torch.from_numpy(g.standard_normal((B, Hkv, Lmax, D), dtype=np.float32)).to(DEV).to(tdt)
    priv_len = np.array([Lmax, R, 77, 2, Lmax + 2], dtype=np.int32)
    host = (lambda t: t.contiguous().view(torch.uint16).cpu().numpy()) if dtype == "bf16" else (lambda t: t.contiguous().cpu().numpy())
    Kref, Vref = oracle.kv_append(host(Knew), host(Vnew), host(Kpriv), host(Vpriv), priv_len)
    lotts.kv_append(Knew, Vnew, Kpriv, Vpriv, to_dev(priv_len))
    torch.cuda.synchronize()
    assert np.array_equal(host(Kpriv), Kref) and np.array_equal(host(Vpriv), Vref)


def test_append_then_attention_equals_attention_on_a_cache_built_in_place(lotts):
    """kv_append followed by verify_attention gives the same bits as verify_attention on caches that already held
    the new rows: the append writes exactly where the attention reads."""
    cfg = BF.with_(B=4, Hq=8, Hkv=2, k=2, P=40, L=333)
    d = attn_to_dev(cfg, S.attention_inputs(cfg))
    want = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    R = cfg.k + 1
    Knew = d["Kpriv"][:, :, cfg.L - R:cfg.L].permute(0, 2, 1, 3).contiguous()   # [B][R][Hkv][D]
    Vnew = d["Vpriv"][:, :, cfg.L - R:cfg.L].permute(0, 2, 1, 3).contiguous()
    K2, V2 = d["Kpriv"].clone(), d["Vpriv"].clone()
    K2[:, :, cfg.L - R:cfg.L] = 0
    V2[:, :, cfg.L - R:cfg.L] = 0
    lotts.kv_append(Knew, Vnew, K2, V2, d["priv_len"])
    got = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], K2, V2, d["priv_len"])
    assert torch.equal(K2, d["Kpriv"]) and torch.equal(V2, d["Vpriv"]) and torch.equal(got, want)


# ---------------------------------------------------------------------------- weight GEMM of the verify forward
@pytest.mark.parametrize("M,N,K", [
    (64, 512, 1024), (40, 136, 256), (5, 8, 128), (1, 1000, 384), (128, 256, 512), (97, 264, 640),
    (129, 520, 384), (192, 2048, 2048), (256, 640, 1280), (231, 136, 128),   # 5, 6 and 8 token tiles
    (80, 1032, 768),        # three token tiles on the four-wavefront form, the last one ragged
    (170, 1032, 768),       # pairs of wavefronts with three token tiles each, the last one ragged; 8 weight rows in the last block
    (192, 11008, 2048),     # 3B-shaped MLP up projection for B = 64 branches, k = 2
    (64, 7168, 5120),       # 32B-shaped QKV projection for B * (k + 1) = 64 tokens (K split over workgroups)
    (64, 5120, 27648),      # 32B-shaped MLP down projection
    (36, 27648, 5120),      # 32B-shaped MLP up projection, M of the long-draft config
    (64, 5120, 5120),       # 32B-shaped O projection
    (33, 40, 2176),         # a second token tile of one row, weight rows past the end, an odd number of chunks
    (64, 64, 32768),        # very long K on few rows: the deepest K split
    (256, 55296, 5120),     # 32B-shaped gate+up projection at the largest token count (B = 64, k = 3)
    (256, 5120, 27648),     # 32B-shaped down projection at the largest token count
    (224, 296, 896),        # seven token tiles on eight wavefronts, weight rows past the end, 7 chunks
    (199, 1288, 1152),      # a ragged seventh token tile: X pieces past the tile are fetched and not staged
    (160, 55296, 5120),     # 32B-shaped gate+up projection with five token tiles (no pairs)
    (199, 27656, 5120),     # a ragged seventh token tile, 8 weight rows in the last block, K split in two
    (130, 55432, 4224),     # five token tiles, 33 chunks per workgroup, no K split
])
def test_skinny_gemm(lotts, oracle, M, N, K):
    print("gemm case", M, N, K, flush=True)
    g = S.rng_for(7, 30, salt=M + N + K)
    X = S.f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))
    W = S.f32_to_bf16_bits(g.standard_normal((N, K), dtype=np.float32) * np.float32(K ** -0.5))
    Y = lotts.skinny_gemm(to_dev(X, True), to_dev(W, True))
    torch.cuda.synchronize()
    ref = oracle.skinny_gemm(X, W)
    y = Y.float().cpu().numpy().astype(np.float64)
    # bf16 output rounding (2^-9 relative) dominates; fp32 accumulation over K adds ~1e-6
    err = np.abs(y - ref)
    assert (err <= 2.0 ** -8 * np.abs(ref) + 1e-3).all(), err.max()
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) <= 3e-3


@pytest.mark.parametrize("M", [48, 256])    # one row tile per wavefront; pairs of wavefronts
def test_skinny_gemm_strided_rows_and_determinism(lotts, oracle, M):
    g = S.rng_for(7, 31, salt=M)
    N, K = 640, 768
    Xf = torch.from_numpy(S.f32_to_bf16_bits(g.standard_normal((M, K + 64), dtype=np.float32))).to(DEV).view(torch.bfloat16)
    Wf = torch.from_numpy(S.f32_to_bf16_bits(g.standard_normal((N, K + 8), dtype=np.float32) * 0.03)).to(DEV).view(torch.bfloat16)
    X, W = Xf[:, :K], Wf[:, :K]
    out = torch.zeros((M, N + 12), dtype=torch.bfloat16, device=DEV)
    Y1 = lotts.skinny_gemm(X, W, out=out[:, :N]).clone()
    Y2 = lotts.skinny_gemm(X.contiguous(), W.contiguous())
    assert torch.equal(Y1, Y2) and float(out[:, N:].abs().sum()) == 0.0
    ref = oracle.skinny_gemm(X.contiguous().view(torch.uint16).cpu().numpy(), W.contiguous().view(torch.uint16).cpu().numpy())
    assert np.linalg.norm(Y1.float().cpu().numpy() - ref) / np.linalg.norm(ref) <= 3e-3


def test_skinny_gemm_weights_beyond_4_gib(lotts, oracle):
    """A weight matrix of 4.56 GB: the rows past the 4 GiB mark are reached through 64-bit addresses.  The oracle
    checks the first and the last 256 weight rows (the whole product would take it minutes); the rows around the
    2 GiB and 4 GiB marks are compared with a plain matrix product."""
    M, N, K = 40, 278528, 8192
    g = torch.Generator(device=DEV)
    g.manual_seed(41)
    W = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, N, 32768):                        # generated in pieces: no fp32 copy of the whole matrix
        r1 = min(N, r0 + 32768)
        W[r0:r1] = (torch.randn((r1 - r0, K), generator=g, device=DEV) * K ** -0.5).to(torch.bfloat16)
    assert W.numel() * 2 > (1 << 32)
    X = torch.randn((M, K), generator=g, device=DEV).to(torch.bfloat16)
    Y = lotts.skinny_gemm(X, W)
    torch.cuda.synchronize()
    xb = X.view(torch.uint16).cpu().numpy()
    for lo, hi in ((0, 256), (N - 256, N)):
        ref = oracle.skinny_gemm(xb, W[lo:hi].contiguous().view(torch.uint16).cpu().numpy())
        y = Y[:, lo:hi].float().cpu().numpy().astype(np.float64)
        assert (np.abs(y - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-3).all(), (lo, np.abs(y - ref).max())
    # rows around the 2 GiB mark (where a signed 32-bit byte offset would wrap), around the 4 GiB mark and at the end,
    # against a plain matrix product of the same rows
    for lo in ((1 << 31) // (2 * K) - 1024, (1 << 32) // (2 * K) - 1024, N - 2048):
        want = X.float() @ W[lo:lo + 2048].float().t()
        assert torch.allclose(Y[:, lo:lo + 2048].float(), want, rtol=2 ** -7, atol=1e-2), lo


# ---------------------------------------------------------------------------- kernel timer
def test_kernel_timer_counts_launches_and_changes_no_result(lotts, oracle):
    """Launches made while the timer runs carry their own events: the count per entry point is the documented
    one, every duration is positive and shorter than the host-side bracket around it, outputs are untouched,
    and launches after the timer is full or stopped run untimed."""
    import time
    cfg = BF.with_(B=16, P=128, L=500)                   # 128 (head, branch) pairs: two partials per row, merged in the launch
    d = attn_to_dev(cfg, S.attention_inputs(cfg))
    s = S.accept_inputs(S.CONFIGS["C2"].with_(B=4, V=30000))
    sd = {n: to_dev(s[n]) for n in ("p", "q", "draft", "u")}
    votes = to_dev(S.vote_inputs(cfg))
    attn = lambda: lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    O0 = attn().clone()
    n0, t0 = [x.clone() for x in lotts.spec_accept(sd["p"], sd["q"], sd["draft"], sd["u"])]
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    with lotts.kernel_timer(16) as t:
        O1 = attn().clone()
        n1, t1 = lotts.spec_accept(sd["p"], sd["q"], sd["draft"], sd["u"])
        lotts.majority_vote(votes)
    wall_ms = (time.perf_counter() - c0) * 1e3        # the exit waited for the kernels
    assert len(t.ms) == 1 + 1 + 1, t.ms                  # this attention plan merges inside its one launch; one-launch acceptance
    assert all(0.0 < v < wall_ms for v in t.ms), (t.ms, wall_ms)
    assert torch.equal(O0, O1) and torch.equal(n0, n1) and torch.equal(t0, t1)
    with lotts.kernel_timer(1) as t:                     # full after one launch: the rest is simply not timed
        O2 = attn()
        lotts.majority_vote(votes)
    assert len(t.ms) == 1 and torch.equal(O0, O2)
    with lotts.kernel_timer(4) as t:
        pass
    assert t.ms == []
    few = BF.with_(B=2, Hq=16, Hkv=2, k=2, P=64, L=4000)   # few pairs: many partials per row, a second launch merges
    d2 = attn_to_dev(few, S.attention_inputs(few))
    with lotts.kernel_timer(4) as t:
        lotts.verify_attention(d2["Q"], d2["Kpre"], d2["Vpre"], d2["Kpriv"], d2["Vpriv"], d2["priv_len"])
    assert len(t.ms) == 2 and min(t.ms) > 0.0
    assert torch.equal(O0, attn())                       # timer off again


# ---------------------------------------------------------------------------- HIP graph capture
def test_step_can_be_captured_in_a_hip_graph_and_replayed(lotts, oracle):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no host
    synchronisation), so a whole step can be captured.  The graph is replayed several times with eager work
    and synchronisations in between, on changing inputs, and every replay must equal the eager result."""
    cfg = BF.with_(B=16, P=128, L=600, V=30000)
    a = S.attention_inputs(cfg)
    d = attn_to_dev(cfg, a)
    s = S.accept_inputs(cfg)
    sd = {n: to_dev(s[n]) for n in ("p", "q", "draft", "u")}
    votes = to_dev(S.vote_inputs(cfg))
    O = torch.empty_like(d["Q"])
    n = torch.empty((cfg.B,), dtype=torch.int32, device=DEV)
    t = torch.empty((cfg.B,), dtype=torch.int32, device=DEV)

    def step(stream=None):
        lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], out=O, stream=stream)
        lotts.spec_accept(sd["p"], sd["q"], sd["draft"], sd["u"], accept_len=n, next_token=t, stream=stream)
        return lotts.majority_vote(votes, stream=stream)

    w_eager, c_eager = step()                              # also creates the cached workspaces outside the capture
    torch.cuda.synchronize()
    Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    e_abs, e_fro, _ = attn_errors(O, Oref)
    assert e_abs <= 2e-2 and e_fro <= 1e-2
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                          # the binding caches one workspace per stream: create the
        step(side)                                         # capture stream's outside the capture (no allocation inside)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        w_g, c_g = step(torch.cuda.current_stream())
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for rep in range(4):
        if rep > 0:                                        # new inputs in the same buffers
            d["Q"].copy_((torch.randn(d["Q"].shape, generator=gen, device=DEV) * 0.5).to(torch.bfloat16))
            sd["u"].copy_(torch.randint(0, 1 << 24, sd["u"].shape, generator=gen, device=DEV).float() / float(1 << 24))
        step()
        torch.cuda.synchronize()
        want = (O.clone(), n.clone(), t.clone())
        O.zero_(); n.fill_(-7); t.fill_(-7); w_g.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want[0]) and torch.equal(n, want[1]) and torch.equal(t, want[2]), rep
        assert torch.equal(w_g, w_eager) and torch.equal(c_g, c_eager)


# ---------------------------------------------------------------------------- search on measured latencies
def test_greedy_search_on_measured_step_latencies(lotts):
    """Algorithm 1 driven by kernel times measured on this GPU (tiny decoder shape) and a synthetic accuracy surface:
    the latency side is real, the bookkeeping of the search must hold, and every evaluated point carries a measured
    step time."""
    from paper_2505_19634_amd import latency_model as lm
    shape = lm.ModelShape("tiny decoder", 2, 512, 8, 2, 64, 1024, 4096)
    out = lm.search(shape, 0.5, prefix=64, context=512, B_max=8, gamma_max=3)
    print("greedy on measured latencies:", {k: out[k] for k in ("B", "gamma", "accuracy", "rounds", "evaluations")}, flush=True)
    assert out["B"] in (1, 2, 4, 8) and 0 <= out["gamma"] <= 3
    assert out["evaluations"] <= 2 * out["rounds"] + 1 and out["evaluations"] <= out["grid_evaluations"]
    assert len(out["evaluated"]) == out["evaluations"]
    assert all(v["step_ms"] > 0.0 and 0.0 <= v["accuracy"] <= 1.0 for v in out["evaluated"].values())
    assert out["accuracy"] == max(v["accuracy"] for k, v in out["evaluated"].items()
                                  if k == "B%d_g%d" % (out["B"], out["gamma"]))
    assert lm.expected_tokens_per_step(0.8, 3) == pytest.approx(1 + 0.8 + 0.64 + 0.512)
    assert lm.expected_tokens_per_step(1.0, 3) == 4.0 and lm.expected_tokens_per_step(0.5, 0) == 1.0


def test_whole_stack_verify_step_replays_what_it_ran_eagerly(lotts):
    """Every layer of a tiny decoder shape resident, one verify step of the whole stack (projections, attention on
    the strided Q columns, LM head, acceptance from logits) enqueued eagerly and then replayed from a captured
    graph: the replay reproduces the eager results bit for bit and reports a device time."""
    from paper_2505_19634_amd import latency_model as lm
    shape = lm.ModelShape("tiny decoder", 2, 512, 8, 2, 64, 1024, 4096)
    fm = lm.FullModel(shape, prefix=64, private=200, B=4, gamma=2)
    fm.enqueue()
    torch.cuda.synchronize()
    want = [t.clone() for t in (fm.o, fm.zt, fm.accept_len, fm.next_token)]
    # layer 0's QKV projection and the LM head against plain matrix products of the same bf16 inputs
    ref = fm.h.float() @ fm.layers[0]["qkv"].float().t()
    lotts.skinny_gemm(fm.h, fm.layers[0]["qkv"], out=fm.qkv, workspace=fm.ws_gemm)
    assert torch.allclose(fm.qkv.float(), ref, rtol=2 ** -7, atol=1e-2)
    assert torch.allclose(fm.zt.view(-1, shape.V).float(), fm.o.float() @ fm.lm_head.float().t(), rtol=2 ** -7, atol=1e-2)
    for t in (fm.o, fm.zt):
        t.zero_()
    ms = fm.step_ms(reps=3)
    got = (fm.o, fm.zt, fm.accept_len, fm.next_token)
    assert all(torch.equal(a, b) for a, b in zip(got, want))
    assert ms > 0.0 and bool(((fm.next_token >= 0) & (fm.next_token < shape.V)).all())
    assert bool(((fm.accept_len >= 0) & (fm.accept_len <= 2)).all())


def test_attention_private_caches_beyond_4_gib(lotts, oracle):
    """Private K and V of 5.7 GB each (20 branches of 139264 tokens, ragged lengths): the branches whose caches lie
    around the 2 GiB and 4 GiB marks and the last one are checked against the oracle, one branch at a time."""
    B, Hq, Hkv, D, k, L = 20, 8, 8, 128, 1, 139264
    g = torch.Generator(device=DEV)
    g.manual_seed(43)
    mk = lambda *sh: (torch.randn(*sh, generator=g, device=DEV) * 0.5).to(torch.bfloat16)
    Kpriv = torch.empty((B, Hkv, L, D), dtype=torch.bfloat16, device=DEV)
    Vpriv = torch.empty((B, Hkv, L, D), dtype=torch.bfloat16, device=DEV)
    for b in range(B):                                   # in pieces: no fp32 copy of a whole cache
        Kpriv[b] = mk(Hkv, L, D)
        Vpriv[b] = mk(Hkv, L, D)
    assert Kpriv.numel() * 2 > (1 << 32)
    Q = mk(B, k + 1, Hq, D)
    priv_len = torch.tensor([L - 37 * b for b in range(B)], dtype=torch.int32, device=DEV)
    O, lse = lotts.verify_attention(Q, None, None, Kpriv, Vpriv, priv_len, return_lse=True)
    torch.cuda.synchronize()
    bits = lambda t: t.contiguous().view(torch.uint16).cpu().numpy()
    tol = TOL["bf16"]
    for b in (0, 7, 15, B - 1):                          # 285 MB per branch: 7 holds the 2 GiB mark, 15 the 4 GiB mark
        Oref, lref = oracle.verify_attention(bits(Q[b:b + 1]), None, None, bits(Kpriv[b:b + 1]), bits(Vpriv[b:b + 1]),
                                             priv_len[b:b + 1].cpu().numpy())
        e_abs, e_fro, _ = attn_errors(O[b:b + 1], Oref)
        print("  branch %d: max-abs %.3g  fro-rel %.3g" % (b, e_abs, e_fro), flush=True)
        assert e_abs <= tol["abs"] and e_fro <= tol["fro_band"], b
        assert np.abs(lse[b:b + 1].cpu().numpy().astype(np.float64) - lref).max() <= tol["lse"], b


def test_attention_strided_q_and_o(lotts, oracle):
    """Q and O handed over as views into larger tensors (extra heads and extra positions around them): only the
    strides change, the padding is never touched."""
    cfg = BF.with_(B=3, P=96, L=200)
    a = S.attention_inputs(cfg)
    d = attn_to_dev(cfg, a)
    big_q = torch.zeros((cfg.B, cfg.R + 2, cfg.Hq + 3, cfg.D), dtype=torch.bfloat16, device=DEV)
    q_view = big_q[:, 1:1 + cfg.R, 2:2 + cfg.Hq]
    q_view.copy_(d["Q"])
    big_o = torch.full((cfg.B, cfg.R + 1, cfg.Hq + 5, cfg.D), 7.0, dtype=torch.bfloat16, device=DEV)
    o_view = big_o[:, :cfg.R, 4:4 + cfg.Hq]
    assert not q_view.is_contiguous() and not o_view.is_contiguous()
    lotts.verify_attention(q_view, d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], out=o_view)
    O2 = lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"])
    assert torch.equal(o_view, O2)
    untouched = big_o.clone()
    untouched[:, :cfg.R, 4:4 + cfg.Hq] = 7.0
    assert bool((untouched == 7.0).all())                 # nothing outside the view was written
    Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    e_abs, e_fro, _ = attn_errors(o_view, Oref)
    assert e_abs <= 2e-2 and e_fro <= 1e-2


def test_attention_on_two_streams_with_separate_workspaces(lotts):
    """Calls that overlap in time need workspaces of their own (the arrival counters live there); given that, two
    streams can run verify_attention side by side and get exactly the results of running alone."""
    cfg = BF.with_(B=16, P=128, L=1500)
    d1 = attn_to_dev(cfg, S.attention_inputs(cfg, salt=1))
    d2 = attn_to_dev(cfg, S.attention_inputs(cfg, salt=2))
    call = lambda d, **kw: lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], **kw)
    ref1, ref2 = call(d1).clone(), call(d2).clone()
    torch.cuda.synchronize()
    ws1 = torch.zeros(16 << 20, dtype=torch.uint8, device=DEV)
    ws2 = torch.zeros(16 << 20, dtype=torch.uint8, device=DEV)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o1 = [torch.empty_like(d1["Q"]) for _ in range(6)]
    o2 = [torch.empty_like(d2["Q"]) for _ in range(6)]
    for i in range(6):
        call(d1, out=o1[i], workspace=ws1, stream=s1)
        call(d2, out=o2[i], workspace=ws2, stream=s2)
    torch.cuda.synchronize()
    assert all(torch.equal(o, ref1) for o in o1) and all(torch.equal(o, ref2) for o in o2)
    assert int(ws1[:131072].view(torch.int64).abs().sum()) == 0 and int(ws2[:131072].view(torch.int64).abs().sum()) == 0


def test_attention_default_workspace_follows_the_stream(lotts, oracle):
    """With no workspace given, the binding keeps one per stream, created and zero-filled on that stream: calls on a
    stream that is not the current one, and calls on two streams side by side, give the results of running alone."""
    cfg = BF.with_(B=16, P=128, L=1500)
    a1, a2 = S.attention_inputs(cfg, salt=3), S.attention_inputs(cfg, salt=4)
    d1, d2 = attn_to_dev(cfg, a1), attn_to_dev(cfg, a2)
    call = lambda d, **kw: lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], **kw)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o1 = [torch.empty_like(d1["Q"]) for _ in range(4)]
    o2 = [torch.empty_like(d2["Q"]) for _ in range(4)]
    for i in range(4):                                     # the first call on each stream creates that stream's workspace
        call(d1, out=o1[i], stream=s1)
        call(d2, out=o2[i], stream=s2)
    torch.cuda.synchronize()
    for a, outs in ((a1, o1), (a2, o2)):
        Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
        for o in outs:
            e_abs, e_fro, _ = attn_errors(o, Oref)
            assert e_abs <= 2e-2 and e_fro <= 1e-2
        assert all(torch.equal(o, outs[0]) for o in outs)
    # a bigger geometry on the same stream grows that stream's workspace; the old one is not freed under a running kernel
    big = BF.with_(B=4, k=8, P=128, L=6000)
    ab = S.attention_inputs(big)
    db = attn_to_dev(big, ab)
    ob = call(db, stream=s1)
    o_again = call(d1, stream=s1)
    torch.cuda.synchronize()
    Oref, _ = oracle.verify_attention(ab["Q"], ab["Kpre"], ab["Vpre"], ab["Kpriv"], ab["Vpriv"], ab["priv_len"])
    e_abs, e_fro, _ = attn_errors(ob, Oref)
    assert e_abs <= 2e-2 and e_fro <= 1e-2
    assert torch.equal(o_again, o1[0])


def test_attention_workspace_recovers_from_a_call_that_never_completed(lotts, oracle):
    """Arrival cells carry the tag of the call that wrote them.  What a call that never completed would leave behind
    is planted from the host -- cells with an old tag and some arrivals already counted -- and the next call must
    start from zero arrivals all the same.  (The cells of a fresh buffer are zero; tag 0 is never used.)"""
    cfg = BF.with_(B=16, P=128, L=900)                     # two partials per row, merged inside the launch
    a = S.attention_inputs(cfg)
    d = attn_to_dev(cfg, a)
    ws = torch.zeros(16 << 20, dtype=torch.uint8, device=DEV)
    call = lambda: lotts.verify_attention(d["Q"], d["Kpre"], d["Vpre"], d["Kpriv"], d["Vpriv"], d["priv_len"], workspace=ws)
    ref = call().clone()                                   # this call's tag is larger than 1
    torch.cuda.synchronize()
    cells = ws[:131072].view(torch.int64)
    assert int(cells.abs().sum()) == 0
    cells[:cfg.B * cfg.Hkv] = (1 << 16) | 1                # tag 1 (the oldest possible), one arrival counted, then "aborted"
    torch.cuda.synchronize()
    again = call()
    torch.cuda.synchronize()
    assert torch.equal(again, ref)
    assert int(cells.abs().sum()) == 0
    Oref, _ = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
    e_abs, e_fro, _ = attn_errors(again, Oref)
    assert e_abs <= 2e-2 and e_fro <= 1e-2
