"""verify_attention_noalloc -- the entry point that allocates nothing (arrival cells and partials live in a scratch
array built into the library) -- called through the C ABI and compared with verify_attention: the same kernels on the
same inputs must give the same bits, and both must sit within the attention tolerance of the CPU oracle.  Two calls
in a row, the second on a smaller input, so that whatever the first call left in the shared scratch is still there
when the second one runs."""
import ctypes

import numpy as np
import pytest
import torch

import synth_inputs as S
from gpu_util import DEV, TOL, attn_errors, attn_to_dev

pytestmark = pytest.mark.gpu


def c_call(lib, fn, desc, d, O, lse, extra):
    P = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(int(torch.cuda.current_stream().cuda_stream))
    return fn(ctypes.byref(desc), P(d["Q"]), P(d["Kpre"]), P(d["Vpre"]), P(d["Kpriv"]), P(d["Vpriv"]), P(d["priv_len"]),
              P(O), P(lse), *extra, stream)


def test_noalloc_entry_point_matches_the_workspace_one(oracle):
    from paper_2505_19634_amd import binding
    lib = binding.load()
    big = S.CONFIGS["C3"].with_(B=16, P=256, L=1200)                  # 2 partials per row, merged inside the launch
    small = S.CONFIGS["C3"].with_(B=3, Hq=16, Hkv=2, k=2, P=64, L=700)  # fewer, longer rows of partials; separate merge launch
    for cfg, priv_len in ((big, None), (small, np.array([700, 3, 333], np.int32))):
        print("noalloc case", cfg, flush=True)
        a = S.attention_inputs(cfg, priv_len=priv_len)
        d = attn_to_dev(cfg, a)
        O_ws, O_na = torch.zeros_like(d["Q"]), torch.zeros_like(d["Q"])
        lse_ws = torch.zeros(d["Q"].shape[:3], dtype=torch.float32, device=DEV)
        lse_na = torch.zeros_like(lse_ws)
        desc = binding.make_attn_desc(d["Q"], d["Kpre"], d["Kpriv"], O_ws)
        need = lib.verify_attention_workspace_bytes(ctypes.byref(desc))
        assert 0 < need <= 16 << 20
        ws = torch.zeros(need, dtype=torch.uint8, device=DEV)
        torch.cuda.synchronize()
        rc = c_call(lib, lib.verify_attention, desc, d, O_ws, lse_ws, (ctypes.c_void_p(ws.data_ptr()), need))
        assert rc == 0
        rc = c_call(lib, lib.verify_attention_noalloc, desc, d, O_na, lse_na, ())
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.equal(O_na, O_ws) and torch.equal(lse_na, lse_ws)
        Oref, lref = oracle.verify_attention(a["Q"], a["Kpre"], a["Vpre"], a["Kpriv"], a["Vpriv"], a["priv_len"])
        e_abs, e_fro, _ = attn_errors(O_na, Oref)
        tol = TOL[cfg.dtype]
        assert e_abs <= tol["abs"] and e_fro <= tol["fro"]
        assert np.abs(lse_na.cpu().numpy().astype(np.float64) - lref).max() <= tol["lse"]


def test_noalloc_entry_point_rejects_what_its_scratch_cannot_hold():
    """Host-side checks only: nothing is launched."""
    from paper_2505_19634_amd import binding
    lib = binding.load()
    one = ctypes.c_void_p(4096)
    d = binding.AttnDesc()
    d.B, d.k, d.Hq, d.Hkv, d.D, d.P, d.Lmax, d.dtype = 512, 7, 32, 8, 128, 0, 64, 1   # 131072 output rows: 64 MiB of partials
    assert lib.verify_attention_workspace_bytes(ctypes.byref(d)) > 16 << 20
    assert lib.verify_attention_noalloc(ctypes.byref(d), one, None, None, one, one, one, one, None, None) == -4
    assert lib.verify_attention_noalloc(ctypes.byref(d), None, None, None, one, one, one, one, None, None) == -1
