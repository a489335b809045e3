"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects malformed calls before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(os.path.join(ROOT, "paper_2505_19634_amd", "liblotts.so")):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2505_19634_amd import binding
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lotts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"typedef[^;]*\(\s*\*[^;]*;", "", text)          # function-pointer typedefs declare no symbol
    return sorted(set(re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*\([^;{]*\)\s*;", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2505_19634_amd import binding
    syms = declared_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None


def test_strerror(lib):
    from paper_2505_19634_amd import binding
    assert binding.strerror(0) == "ok"
    for code in range(-5, 0):
        assert binding.strerror(code) not in ("ok", "unknown lotts status")
    assert binding.strerror(-99) == "unknown lotts status"


def make_desc(**kw):
    from paper_2505_19634_amd.binding import AttnDesc
    d = AttnDesc()
    base = dict(B=16, k=3, Hq=40, Hkv=8, D=128, P=256, Lmax=3840, dtype=1, scale=0.0)
    base.update(kw)
    for n, v in base.items():
        setattr(d, n, v)
    return d


def test_workspace_queries(lib):
    d = make_desc()
    need = lib.verify_attention_workspace_bytes(ctypes.byref(d))
    assert 0 < need < 64 << 20 and need % 256 == 0
    for bad in (dict(Hq=41), dict(D=96), dict(k=-1), dict(B=0), dict(Lmax=3), dict(dtype=7), dict(P=-1),
                dict(q_stride_h=12), dict(B=4096, Hkv=8, Hq=8)):
        assert lib.verify_attention_workspace_bytes(ctypes.byref(make_desc(**bad))) == 0, bad
    assert lib.verify_attention_workspace_bytes(None) == 0
    assert lib.spec_accept_workspace_bytes(16, 3, 152064) > 0
    assert lib.spec_accept_workspace_bytes(0, 3, 100) == 0
    assert lib.spec_accept_workspace_bytes(4, -1, 100) == 0
    assert lib.spec_accept_workspace_bytes(4, 3, 0) == 0


def test_calls_are_rejected_before_any_launch(lib):
    """Only error paths: each returns on the host, so this is safe without a GPU."""
    d = make_desc()
    one = ctypes.c_void_p(4096)        # never dereferenced: a different check fails first
    assert lib.verify_attention(None, one, one, one, one, one, one, one, None, one, 1 << 30, None) == -1
    assert lib.verify_attention(ctypes.byref(d), None, one, one, one, one, one, one, None, one, 1 << 30, None) == -1
    assert lib.verify_attention(ctypes.byref(d), one, None, one, one, one, one, one, None, one, 1 << 30, None) == -1
    assert lib.verify_attention(ctypes.byref(d), one, one, one, one, one, one, one, None, one, 16, None) == -4
    assert lib.verify_attention(ctypes.byref(make_desc(Hq=41)), one, one, one, one, one, one, one, None, one,
                                1 << 30, None) == -2
    assert lib.verify_attention(ctypes.byref(make_desc(dtype=5)), one, one, one, one, one, one, one, None, one,
                                1 << 30, None) == -3
    # a geometry whose partials would pass 2 GiB: the workspace query answers 0 and the call is refused, not launched
    huge = make_desc(B=16384, Hkv=1, Hq=64, k=8, P=0, Lmax=4096)
    assert lib.verify_attention_workspace_bytes(ctypes.byref(huge)) == 0
    assert lib.verify_attention(ctypes.byref(huge), one, None, None, one, one, one, one, None, one, 1 << 40, None) == -2
    odd = ctypes.c_void_p(4096 + 2)    # bf16 rows must be 16-byte aligned
    assert lib.verify_attention(ctypes.byref(d), odd, one, one, one, one, one, one, None, one, 1 << 30, None) == -2
    assert lib.spec_accept(4, 2, 100, None, one, one, one, one, one, one, 1 << 20, None) == -1
    assert lib.spec_accept(4, 2, 100, one, None, one, one, one, one, one, 1 << 20, None) == -1
    assert lib.spec_accept(4, 2, 100, one, one, one, one, one, one, one, 8, None) == -4
    assert lib.spec_accept(4, 300, 100, one, one, one, one, one, one, one, 1 << 20, None) == -2
    assert lib.spec_accept(0, 2, 100, one, one, one, one, one, one, one, 1 << 20, None) == -2
    assert lib.majority_vote(1, 16, None, one, one, None) == -1
    assert lib.majority_vote(1, 0, one, one, one, None) == -2
    assert lib.majority_vote(1, 5000, one, one, one, None) == -2


def test_widenings_are_rejected_before_any_launch(lib):
    """Error paths of the later entry points; nothing here reaches a launch."""
    one = ctypes.c_void_p(4096)
    f1 = ctypes.c_float(1.0)
    big = 1 << 30
    lg = lambda B, k, V, zt, zd, dt, it, dr, u, n, t, ws, wsb: lib.spec_accept_logits(B, k, V, zt, zd, dt, it, dr, u, n, t,
                                                                                   None, ws, wsb, None)
    assert lib.spec_accept_logits_workspace_bytes(16, 3, 152064) > 0
    assert lib.spec_accept_logits_workspace_bytes(16, 3, (1 << 20) + 1) == 0
    assert lib.spec_accept_logits_workspace_bytes(16, 257, 100) == 0
    assert lib.spec_accept_logits_workspace_bytes(65535, 256, 1 << 20) == 0       # more (piece, row) pairs than one grid holds
    assert lg(65535, 256, 1 << 20, one, one, 1, f1, one, one, one, one, one, 1 << 60) == -2
    assert lg(4, 2, 100, None, one, 1, f1, one, one, one, one, one, big) == -1
    assert lg(4, 2, 100, one, None, 1, f1, one, one, one, one, one, big) == -1
    assert lg(4, 2, 100, one, one, 1, f1, None, one, one, one, one, big) == -1
    assert lg(4, 0, 100, one, None, 1, f1, None, one, one, one, one, 8) == -4           # k = 0 needs no draft side: the workspace check is reached
    assert lg(4, 2, 100, one, one, 7, f1, one, one, one, one, one, big) == -3
    assert lg(4, 2, 100, one, one, 1, ctypes.c_float(0.0), one, one, one, one, one, big) == -2
    assert lg(4, 2, 100, one, one, 1, ctypes.c_float(float("nan")), one, one, one, one, one, big) == -2
    assert lg(4, 2, 100, one, one, 1, f1, one, one, one, one, one, 8) == -4
    assert lg(4, 2, 100, one, one, 1, f1, one, one, one, one, ctypes.c_void_p(4096 + 4), big) == -2
    assert lg(0, 2, 100, one, one, 1, f1, one, one, one, one, one, big) == -2
    cv = lib.confidence_vote
    assert cv(1, 16, 8, None, one, None, 1, 1, one, one, None) == -1
    assert cv(1, 16, 8, one, one, None, 2, 1, one, one, None) == -2
    assert cv(1, 16, 8, one, one, None, 1, -1, one, one, None) == -2
    assert cv(1, 2000, 8, one, one, None, 1, 1, one, one, None) == -2
    assert cv(1, 16, 0, one, one, None, 1, 1, one, one, None) == -2
    assert lib.skinny_gemm_workspace_bytes(64, 5120, 5120) > 0
    assert lib.skinny_gemm_workspace_bytes(257, 5120, 5120) == 0
    assert lib.skinny_gemm_workspace_bytes(64, 5124, 5120) == 0
    assert lib.skinny_gemm_workspace_bytes(64, 5120, 5100) == 0
    gm = lib.skinny_gemm
    assert gm(64, 512, 512, None, 512, one, 512, one, 512, one, big, None) == -1
    assert gm(64, 512, 512, one, 512, one, 512, one, 512, None, big, None) == -1
    assert gm(64, 512, 512, one, 500, one, 512, one, 512, one, big, None) == -2          # row pitch shorter than K
    assert gm(64, 512, 512, one, 512, one, 516, one, 512, one, big, None) == -2          # pitch not a multiple of 8
    assert gm(64, 512, 512, ctypes.c_void_p(4096 + 8), 512, one, 512, one, 512, one, big, None) == -2
    assert gm(64, 512, 512, one, 512, one, 512, one, 512, one, 16, None) == -4
    assert gm(0, 512, 512, one, 512, one, 512, one, 512, one, big, None) == -2
    ka = lambda B, k, H, D, dt, kn, vn, sb, sr, sh, kp, vp_, pb, ph, pt, Lmax, pl: lib.kv_append(
        B, k, H, D, dt, kn, vn, sb, sr, sh, kp, vp_, pb, ph, pt, Lmax, pl, None)
    ok = (4, 3, 8, 128, 1, one, one, 4 * 8 * 128, 8 * 128, 128, one, one, 8 * 4096 * 128, 4096 * 128, 128, 4096, one)
    bad = lambda **kw: ka(*[kw.get(n, v) for n, v in zip(
        ("B", "k", "H", "D", "dt", "kn", "vn", "sb", "sr", "sh", "kp", "vp", "pb", "ph", "pt", "Lmax", "pl"), ok)])
    assert bad(kn=None) == -1 and bad(vp=None) == -1 and bad(pl=None) == -1
    assert bad(dt=7) == -3
    assert bad(B=0) == -2 and bad(k=-1) == -2 and bad(H=0) == -2
    assert bad(D=4) == -2                                  # a bf16 row of 8 bytes: not a multiple of 16
    assert bad(Lmax=3) == -2                               # shorter than the k + 1 new tokens
    assert bad(sh=120) == -2 and bad(pt=100) == -2         # strides that are not multiples of 16 bytes, or shorter than a row
    assert bad(kp=ctypes.c_void_p(4096 + 8)) == -2         # misaligned cache


def test_kernel_timer_host_side(lib):
    n = ctypes.c_int32(-1)
    assert lib.lotts_timer_start(0) == -2 and lib.lotts_timer_start((1 << 20) + 1) == -2
    assert lib.lotts_timer_stop(None, None) == -1
    assert lib.lotts_timer_stop(ctypes.byref(n), None) == 0 and n.value == 0          # never started: nothing timed
    assert lib.lotts_timer_pause(1) == 0 and lib.lotts_timer_pause(0) == 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    import paper_2505_19634_amd as lotts
    with pytest.raises(ValueError):
        lotts.majority_vote(torch.zeros(4, dtype=torch.int32))
    with pytest.raises(ValueError):
        lotts.spec_accept(torch.zeros(1, 1, 8), None, None, torch.zeros(1, 1))
