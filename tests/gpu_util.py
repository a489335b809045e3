"""Helpers of the GPU parity tests: move seeded numpy inputs to the GPU, compare with the oracle."""
import numpy as np
import torch

DEV = "cuda:0"


def to_dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.view(torch.bfloat16) if bf16 else t


def attn_to_dev(cfg, a):
    bf = cfg.dtype == "bf16"
    out = {n: to_dev(a[n], bf) for n in ("Q", "Kpre", "Vpre", "Kpriv", "Vpriv")}
    out["priv_len"] = to_dev(a["priv_len"])
    return out


def attn_errors(O_gpu: torch.Tensor, O_ref: np.ndarray):
    """max-abs error, Frobenius relative error, max element-wise relative error over elements
    that are not small (|ref| > 10% of max |ref|)."""
    o = O_gpu.float().cpu().numpy().astype(np.float64)
    diff = np.abs(o - O_ref)
    big = np.abs(O_ref) > 1e-1 * np.abs(O_ref).max()
    return diff.max(), np.linalg.norm(o - O_ref) / np.linalg.norm(O_ref), (diff[big] / np.abs(O_ref[big])).max()


# Tolerances of the attention comparison against the fp64 oracle: "abs" and "fro" are the stated bar (max-abs and
# Frobenius-relative).  "fro_band" and "rel_band" are a regression band on top of it, a small multiple of what the
# arithmetic gives: bf16 rounding of the softmax weights and of the output, 2^-9 relative each, is expected to leave
# about 1.5e-3 Frobenius-relative (measured 2.2e-3 to 2.4e-3 over all cases) -- a kernel that got several times less
# accurate would still pass the stated bar, but not the band.
TOL = {"bf16": dict(abs=2e-2, fro=1e-2, lse=2e-3, fro_band=4e-3, rel_band=None),
       "f32": dict(abs=1e-4, fro=1e-4, lse=1e-4, fro_band=2e-6, rel_band=None)}
