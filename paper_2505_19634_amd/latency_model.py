"""Latency-aware configuration search on measured kernel times (paper Section 3.3, Algorithm 1).

The paper picks the number of branches B and the draft length gamma that maximise accuracy under a
latency budget T.  Its accuracy side needs the paper's models and datasets; its latency side is what
this library computes.  This module measures the latency side on the GPU -- the device time of the
kernels of one verify step of a decoder of a given shape, taken with the library's kernel timer --
and runs the library's greedy_search over it with a SYNTHETIC accuracy surface (stated below), so the
search is exercised end to end on real MI355X latencies.  Nothing here is one of the paper's
experiments.

Verify step of the target model for B branches and gamma drafts (M = B * (gamma + 1) new tokens):
per layer QKV projection, append of the new K and V rows to the caches, attention, O projection, gate+up
and down projections (skinny_gemm, kv_append and verify_attention, one layer's buffers timed and
multiplied by the layer count), then the LM head and the acceptance from logits.  Norms, rotary
embedding and activation are not modelled (they are outside this library); the draft model's gamma sequential steps cost `draft_ratio` times a
one-token step of the target each (an assumption: a draft model a tenth of the target's size).

    python -m paper_2505_19634_amd.latency_model --shape 3B --budget-s 4
    python -m paper_2505_19634_amd.latency_model --shape 32B --budget-s 20 --full-model 16,3
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
from dataclasses import dataclass

import numpy as np
import torch

from . import binding


@dataclass(frozen=True)
class ModelShape:
    name: str
    layers: int
    hidden: int
    Hq: int
    Hkv: int
    D: int
    mlp: int
    V: int


SHAPES = {
    "3B": ModelShape("3B-shaped decoder", 36, 2048, 16, 2, 128, 11008, 151936),
    "32B": ModelShape("32B-shaped decoder", 64, 5120, 40, 8, 128, 27648, 152064),
}


class StepTimer:
    """Holds one layer's worth of synthetic weights and caches for a shape and times verify steps on them."""

    def __init__(self, shape: ModelShape, prefix: int, max_private: int, max_B: int, max_gamma: int, device="cuda:0"):
        self.s, self.P, self.Lmax, self.dev = shape, prefix, max_private, torch.device(device)
        g = torch.Generator(device=self.dev)
        g.manual_seed(7)
        bf = lambda *sh: (torch.randn(*sh, generator=g, device=self.dev) * 0.5).to(torch.bfloat16)
        w = lambda n, k: (torch.randn(n, k, generator=g, device=self.dev) * k ** -0.5).to(torch.bfloat16)
        s = shape
        self.W = {"qkv": w((s.Hq + 2 * s.Hkv) * s.D, s.hidden), "o": w(s.hidden, s.Hq * s.D),
                  "gate_up": w(2 * s.mlp, s.hidden), "down": w(s.hidden, s.mlp), "lm_head": w(s.V, s.hidden)}
        self.Kpre, self.Vpre = bf(s.Hkv, prefix, s.D), bf(s.Hkv, prefix, s.D)
        self.Kpriv, self.Vpriv = bf(max_B, s.Hkv, max_private, s.D), bf(max_B, s.Hkv, max_private, s.D)
        self.max_B, self.max_gamma = max_B, max_gamma
        self._cache = {}

    def _gemm_ms(self, M: int, W: torch.Tensor) -> float:
        """Kernel time of Y = X W^T for M tokens (pieces of at most 256 tokens, the library's limit)."""
        total = 0.0
        for m0 in range(0, M, 256):
            m = min(256, M - m0)
            X = torch.zeros((m, W.shape[1]), dtype=torch.bfloat16, device=self.dev)
            total += self._timed(lambda: binding.skinny_gemm(X, W))
        return total

    @staticmethod
    def _timed(call, reps: int = 3) -> float:
        """Smallest of `reps` sums of the kernel times of one call (after one untimed call)."""
        call()
        best = float("inf")
        for _ in range(reps):
            with binding.kernel_timer(8) as t:
                call()
            best = min(best, sum(t.ms))
        return best

    def verify_step_ms(self, B: int, gamma: int, private: int) -> dict:
        """Device milliseconds of the kernels of one verify step: {"layer": per layer, "head": LM head + acceptance,
        "total": layers * layer + head}.  `private` = private tokens per branch before the step."""
        key = (B, gamma, private)
        if key in self._cache:
            return self._cache[key]
        s, R = self.s, gamma + 1
        assert 1 <= B <= self.max_B and 0 <= gamma <= self.max_gamma and private + R <= self.Lmax
        M = B * R
        layer = sum(self._gemm_ms(M, self.W[n]) for n in ("qkv", "o", "gate_up", "down"))
        Q = torch.zeros((B, R, s.Hq, s.D), dtype=torch.bfloat16, device=self.dev)
        pl = torch.full((B,), private + R, dtype=torch.int32, device=self.dev)
        args = (Q, self.Kpre, self.Vpre, self.Kpriv[:B], self.Vpriv[:B], pl)
        layer += self._timed(lambda: binding.verify_attention(*args))
        heads = torch.zeros((B, R, s.Hq + 2 * s.Hkv, s.D), dtype=torch.bfloat16, device=self.dev)
        layer += self._timed(lambda: binding.kv_append(heads[:, :, s.Hq:s.Hq + s.Hkv], heads[:, :, s.Hq + s.Hkv:],
                                                       self.Kpriv[:B], self.Vpriv[:B], pl))
        head = self._gemm_ms(M, self.W["lm_head"])
        zt = torch.zeros((B, R, s.V), dtype=torch.bfloat16, device=self.dev)
        zd = torch.zeros((B, gamma, s.V), dtype=torch.bfloat16, device=self.dev) if gamma else None
        dr = torch.zeros((B, gamma), dtype=torch.int32, device=self.dev) if gamma else None
        u = torch.full((B, R), 0.5, dtype=torch.float32, device=self.dev)
        head += self._timed(lambda: binding.spec_accept_logits(zt, zd, dr, u))
        out = {"layer": layer, "head": head, "total": s.layers * layer + head}
        self._cache[key] = out
        return out


class FullModel:
    """Every layer of a decoder shape resident on one GPU -- its bf16 weights (62 GB for the 32B shape) and the KV
    caches of B branches, each layer its own memory -- and one verify step of the whole stack as one captured graph:
    per layer the QKV projection, kv_append of its K and V columns to the caches, verify_attention on its Q columns, the
    O projection, gate+up, and
    down on the first half of gate+up's output (norms, rotary embedding and activation are outside this
    library, so the values that flow are not a language model's; the shapes, the memory traffic and the launch
    sequence are), then the LM head and the acceptance from logits.  Replaying the graph gives the step's device
    time with the gaps between launches and with nothing left in a cache by an earlier use of the same weights:
    the check on StepTimer's sum of isolated kernel times."""

    def __init__(self, shape: ModelShape, prefix: int, private: int, B: int, gamma: int, device="cuda:0"):
        s, R = shape, gamma + 1
        M = B * R
        if M > 256:
            raise ValueError("one GEMM call takes at most 256 tokens")
        self.s, self.B, self.R, self.dev = s, B, R, torch.device(device)
        g = torch.Generator(device=self.dev)
        g.manual_seed(11)
        bf = lambda *sh: (torch.randn(*sh, generator=g, device=self.dev) * 0.5).to(torch.bfloat16)
        w = lambda n, k: (torch.randn(n, k, generator=g, device=self.dev) * k ** -0.5).to(torch.bfloat16)
        qkv_n = (s.Hq + 2 * s.Hkv) * s.D
        first = {"qkv": w(qkv_n, s.hidden), "o": w(s.hidden, s.Hq * s.D), "gate_up": w(2 * s.mlp, s.hidden),
                 "down": w(s.hidden, s.mlp), "Kpre": bf(s.Hkv, prefix, s.D), "Vpre": bf(s.Hkv, prefix, s.D),
                 "Kpriv": bf(B, s.Hkv, private + R, s.D), "Vpriv": bf(B, s.Hkv, private + R, s.D)}
        # the other layers hold copies: the values do not matter to the time, that each layer is its own memory does
        self.layers = [first] + [{k: v.clone() for k, v in first.items()} for _ in range(s.layers - 1)]
        self.lm_head = w(s.V, s.hidden)
        self.priv_len = torch.full((B,), private + R, dtype=torch.int32, device=self.dev)
        z = lambda *sh: torch.zeros(sh, dtype=torch.bfloat16, device=self.dev)
        self.h = bf(M, s.hidden)
        self.qkv, self.attn, self.o, self.gu = z(M, qkv_n), z(B, R, s.Hq, s.D), z(M, s.hidden), z(M, 2 * s.mlp)
        heads = self.qkv.view(B, R, s.Hq + 2 * s.Hkv, s.D)
        self.q_view, self.k_view, self.v_view = heads[:, :, :s.Hq], heads[:, :, s.Hq:s.Hq + s.Hkv], heads[:, :, s.Hq + s.Hkv:]
        self.zt = z(B, R, s.V)
        self.zd = bf(B, gamma, s.V) if gamma else None
        self.draft = torch.zeros((B, gamma), dtype=torch.int32, device=self.dev) if gamma else None
        self.u = torch.full((B, R), 0.5, dtype=torch.float32, device=self.dev)
        self.accept_len = torch.zeros((B,), dtype=torch.int32, device=self.dev)
        self.next_token = torch.zeros((B,), dtype=torch.int32, device=self.dev)
        lib = binding.load()
        gemm_ws = max(lib.skinny_gemm_workspace_bytes(M, n, k) for n, k in
                      ((qkv_n, s.hidden), (s.hidden, s.Hq * s.D), (2 * s.mlp, s.hidden), (s.hidden, s.mlp), (s.V, s.hidden)))
        ws = lambda n: torch.zeros(max(int(n), 256), dtype=torch.uint8, device=self.dev)
        desc = binding.make_attn_desc(self.q_view, first["Kpre"], first["Kpriv"], self.attn)
        self.ws_gemm = ws(gemm_ws)
        self.ws_attn = ws(lib.verify_attention_workspace_bytes(ctypes.byref(desc)))
        self.ws_accept = ws(lib.spec_accept_logits_workspace_bytes(B, gamma, s.V))
        self.graph = None

    def enqueue(self) -> None:
        """One verify step of the whole stack on the current stream; allocates nothing."""
        s, M = self.s, self.B * self.R
        h = self.h
        for L in self.layers:
            binding.skinny_gemm(h, L["qkv"], out=self.qkv, workspace=self.ws_gemm)
            binding.kv_append(self.k_view, self.v_view, L["Kpriv"], L["Vpriv"], self.priv_len)
            binding.verify_attention(self.q_view, L["Kpre"], L["Vpre"], L["Kpriv"], L["Vpriv"], self.priv_len,
                                     out=self.attn, workspace=self.ws_attn)
            binding.skinny_gemm(self.attn.view(M, s.Hq * s.D), L["o"], out=self.o, workspace=self.ws_gemm)
            binding.skinny_gemm(self.o, L["gate_up"], out=self.gu, workspace=self.ws_gemm)
            binding.skinny_gemm(self.gu[:, :s.mlp], L["down"], out=self.o, workspace=self.ws_gemm)
            h = self.o
        binding.skinny_gemm(h, self.lm_head, out=self.zt.view(M, s.V), workspace=self.ws_gemm)
        binding.spec_accept_logits(self.zt, self.zd, self.draft, self.u, accept_len=self.accept_len,
                                   next_token=self.next_token, workspace=self.ws_accept)

    def step_ms(self, reps: int = 5) -> float:
        """Device milliseconds of one verify step: mean over `reps` replays of the captured step."""
        if self.graph is None:
            self.enqueue()  # once outside the capture: whatever is created lazily exists before it
            torch.cuda.synchronize()
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph):
                self.enqueue()
        for _ in range(2):
            self.graph.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            self.graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps


def expected_tokens_per_step(alpha: float, gamma: int) -> float:
    """Tokens a branch emits per verify step when each draft is accepted with probability alpha:
    1 + alpha + ... + alpha^gamma (the accepted drafts plus the resampled or bonus token)."""
    return float(gamma + 1) if alpha >= 1.0 else (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def synthetic_accuracy(B: int, tokens: float, *, p_inf: float = 0.62, half_tokens: float = 2500.0,
                       wrong_classes: int = 12, trials: int = 4000, seed: int = 11) -> float:
    """A stand-in for the paper's accuracy measurements, NOT data: a branch that may generate `tokens` tokens answers
    correctly with probability p = p_inf * (1 - 2^(-tokens / half_tokens)); wrong answers spread evenly over
    `wrong_classes` ids; the question counts as solved when the correct id wins the plurality vote, a tie for the
    first place counting as one share among the tied ids.  Seeded Monte Carlo, so the surface is a fixed function
    of (B, tokens)."""
    p = p_inf * (1.0 - 2.0 ** (-tokens / half_tokens))
    g = np.random.default_rng(seed)
    right = g.random((trials, B)) < p
    wrong_id = g.integers(0, wrong_classes, (trials, B))
    n_right = right.sum(1)
    wrong_counts = np.zeros((trials, wrong_classes), dtype=np.int64)
    for c in range(wrong_classes):
        wrong_counts[:, c] = ((wrong_id == c) & ~right).sum(1)
    top = wrong_counts.max(1)
    tied = (wrong_counts == top[:, None]).sum(1)
    credit = np.where(n_right > top, 1.0, np.where((n_right == top) & (n_right > 0), 1.0 / (1.0 + tied), 0.0))
    return float(credit.mean())


def search(shape, budget_s: float, *, prefix: int = 512, context: int = 4096, alpha: float = 0.8,
           draft_ratio: float = 0.1, B_max: int = 64, gamma_max: int = 7, verbose: bool = False) -> dict:
    """Greedy (B, gamma) search under the latency budget on measured step times.  Returns the chosen configuration,
    the table of evaluated points and the search's own counters."""
    shape = SHAPES[shape] if isinstance(shape, str) else shape
    timer = StepTimer(shape, prefix, context, B_max, gamma_max)
    evaluated = {}

    def tts_task(B: int, gamma: int, T: float) -> float:
        # mid-generation cache length: half the context is a fair average over a generation
        private = max(gamma + 1, context // 2) - (gamma + 1)
        verify = timer.verify_step_ms(B, gamma, private)["total"]
        draft = gamma * draft_ratio * timer.verify_step_ms(B, 0, private)["total"]
        step_ms = verify + draft
        per_token_ms = step_ms / expected_tokens_per_step(alpha, gamma)
        tokens = min(float(context - prefix), T * 1e3 / per_token_ms)
        acc = synthetic_accuracy(B, tokens)
        evaluated[(B, gamma)] = {"step_ms": step_ms, "ms_per_token": per_token_ms, "tokens_in_budget": tokens, "accuracy": acc}
        if verbose:
            print("  B=%-3d gamma=%d  step %.3f ms  %.3f ms/token  %6.0f tokens in %.0f s  accuracy %.3f" % (
                B, gamma, step_ms, per_token_ms, tokens, T, acc), flush=True)
        return acc

    B, gamma, acc, rounds, evals = binding.greedy_search(tts_task, budget_s, B_max, gamma_max)
    return {"shape": shape.name, "budget_s": budget_s, "B": B, "gamma": gamma, "accuracy": acc, "rounds": rounds,
            "evaluations": evals, "grid_evaluations": (int(math.log2(B_max)) + 1) * (gamma_max + 1),
            "evaluated": {"B%d_g%d" % k: v for k, v in evaluated.items()},
            "assumptions": {"alpha": alpha, "draft_ratio": draft_ratio, "prefix": prefix, "context": context,
                            "accuracy": "synthetic surface, see synthetic_accuracy"}}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--shape", choices=sorted(SHAPES), default="3B")
    ap.add_argument("--budget-s", type=float, default=4.0, help="latency budget of the search; 0 = no search")
    ap.add_argument("--alpha", type=float, default=0.8)
    ap.add_argument("--draft-ratio", type=float, default=0.1)
    ap.add_argument("--B-max", type=int, default=64)
    ap.add_argument("--gamma-max", type=int, default=7)
    ap.add_argument("--full-model", metavar="B,GAMMA", action="append", default=[],
                    help="also hold every layer of the shape on the GPU and time one verify step of the whole stack "
                         "for this (B, gamma), against the sum of isolated kernel times the search uses")
    a = ap.parse_args()
    for spec in a.full_model:
        B, gamma = (int(x) for x in spec.split(","))
        prefix, context = 512, 4096
        private = max(gamma + 1, context // 2) - (gamma + 1)
        fm = FullModel(SHAPES[a.shape], prefix, private, B, gamma)
        measured = fm.step_ms()
        del fm
        torch.cuda.empty_cache()
        modelled = StepTimer(SHAPES[a.shape], prefix, context, B, gamma).verify_step_ms(B, gamma, private)
        print(json.dumps({"full_model": SHAPES[a.shape].name, "B": B, "gamma": gamma, "private_tokens": private,
                          "step_ms_whole_stack_graph_replay": measured, "step_ms_sum_of_kernel_times": modelled["total"],
                          "per_layer_ms_sum_of_kernel_times": modelled["layer"]}), flush=True)
    if a.budget_s <= 0.0:  # only the whole-stack measurements were asked for
        return 0
    out = search(a.shape, a.budget_s, alpha=a.alpha, draft_ratio=a.draft_ratio, B_max=a.B_max, gamma_max=a.gamma_max,
                 verbose=True)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
