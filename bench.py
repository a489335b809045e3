#!/usr/bin/env python3
"""Throughput of the speculative verification step across B branches on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input, all launched on one
stream: verify_attention (one layer) -> spec_accept -> majority_vote.  Inputs are resident in
HBM before the timed region; several independent input sets are rotated so that the 256 MB
memory-side cache cannot serve the KV stream.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--sets 4]

Beside the contract's fields the line carries: `roofline` (the attention kernel against the HBM peak, timed by
event pairs attached to its launches, with the statistics of the sample and a read-only streaming probe over
the same buffers as the ceiling of this machine), `layers_back_to_back` (the amortised per-layer figure: one
verify_attention call per decoder layer, launched back to back over rotated inputs), and `cpu_baseline`
(the CPU oracle on the same inputs on this machine's host cores).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def attn_algorithmic_bytes(cfg, priv_len_sum=None) -> int:
    """What the method must move per layer: every prefix token once (whatever B is), every private
    token once, Q in and O out.  2 (K and V) * Hkv * D * element size per token."""
    es = 2 if cfg.dtype == "bf16" else 4
    per_token = 2 * cfg.Hkv * cfg.D * es
    priv = cfg.B * cfg.L if priv_len_sum is None else priv_len_sum
    return per_token * (cfg.P + priv) + 2 * cfg.B * cfg.R * cfg.Hq * cfg.D * es


def accept_algorithmic_bytes(cfg, accept_len) -> int:
    """One read of the row(s) that are sampled: p_n and q_n after a rejection, p_k otherwise."""
    return int(sum((2 if n < cfg.k else 1) * cfg.V * 4 for n in accept_len))


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", "attn_kernel_%s_traffic.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="C3", help="C2, C3, C5 or C4xB (e.g. C4x16)")
    ap.add_argument("--sets", type=int, default=4, help="independent input sets rotated per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gemm-tokens", type=int, default=0,
                    help="token count M of the weight-GEMM legs (default: the workload's B * (k + 1), at most 256)")
    ap.add_argument("--min-timed-launches", type=int, default=64,
                    help="attention launches timed in all (timed region plus a labelled leg after it)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (the path shards by branch with no "
              "exchange inside attention or acceptance: N GPUs would run N independent copies of these kernels)"
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2505_19634_amd as lotts
    from paper_2505_19634_amd import binding
    import synth_inputs as S

    if args.workload.startswith("C4x"):
        cfg = S.CONFIGS["C4"].with_(B=int(args.workload[3:]))
    else:
        cfg = S.CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = binding.load()
    bf = cfg.dtype == "bf16"
    nsets = max(1, args.sets)

    # ---- inputs: set 0 from the host generator (also fed to the oracle), the others drawn on the
    # GPU from the same distributions (they only have to occupy distinct memory)
    a0 = S.attention_inputs(cfg)
    s0 = S.accept_inputs(cfg)
    answers0 = S.vote_inputs(cfg, N=1)

    def dev_kv(x):
        t = torch.from_numpy(x).to(dev)
        return t.view(torch.bfloat16) if bf else t

    gen = torch.Generator(device=dev)
    gen.manual_seed(1000 * cfg.number)
    sets = []
    for i in range(nsets):
        if i == 0:
            d = {n: dev_kv(a0[n]) for n in ("Q", "Kpre", "Vpre", "Kpriv", "Vpriv")}
            d.update({n: torch.from_numpy(s0[n]).to(dev) for n in ("p", "q", "draft", "u")})
        else:
            d = {}
            for n in ("Q", "Kpre", "Vpre", "Kpriv", "Vpriv"):
                t = torch.randn(a0[n].shape, generator=gen, device=dev, dtype=torch.float32) * cfg.qkv_std
                d[n] = t.to(torch.bfloat16) if bf else t
            z = torch.randn(s0["p"].shape, generator=gen, device=dev) * cfg.logit_std
            zq = z[:, :cfg.k] + torch.randn(s0["q"].shape, generator=gen, device=dev) * (cfg.noise_std or cfg.logit_std)
            d["p"] = torch.softmax(z.double(), -1).float().contiguous()
            d["q"] = torch.softmax(zq.double(), -1).float().contiguous()
            d["draft"] = torch.multinomial(d["q"].view(-1, cfg.V), 1, generator=gen).view(cfg.B, cfg.k).int()
            d["u"] = (torch.randint(0, 1 << 24, (cfg.B, cfg.R), generator=gen, device=dev).float() / float(1 << 24))
            del z, zq
        d["priv_len"] = torch.from_numpy(a0["priv_len"]).to(dev)
        d["answers"] = torch.from_numpy(answers0).to(dev)
        d["O"] = torch.empty_like(d["Q"])
        d["accept_len"] = torch.empty((cfg.B,), dtype=torch.int32, device=dev)
        d["next_token"] = torch.empty((cfg.B,), dtype=torch.int32, device=dev)
        d["winner"] = torch.empty((1,), dtype=torch.int32, device=dev)
        d["winner_count"] = torch.empty((1,), dtype=torch.int32, device=dev)
        sets.append(d)

    # ---- marshal every call once; the timed loop only issues C-ABI calls
    stream = torch.cuda.current_stream()
    sh = ctypes.c_void_p(int(stream.cuda_stream))
    desc = binding.make_attn_desc(sets[0]["Q"], sets[0]["Kpre"], sets[0]["Kpriv"], sets[0]["O"])
    ws_attn_bytes = lib.verify_attention_workspace_bytes(ctypes.byref(desc))
    ws_acc_bytes = lib.spec_accept_workspace_bytes(cfg.B, cfg.k, cfg.V)
    ws_attn = torch.zeros(ws_attn_bytes, dtype=torch.uint8, device=dev)   # arrival counters start at zero
    ws_acc = torch.zeros(ws_acc_bytes, dtype=torch.uint8, device=dev)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    calls = []
    for d in sets:
        attn_args = (ctypes.byref(desc), P(d["Q"]), P(d["Kpre"]), P(d["Vpre"]), P(d["Kpriv"]), P(d["Vpriv"]),
                     P(d["priv_len"]), P(d["O"]), None, P(ws_attn), ws_attn_bytes, sh)
        acc_args = (cfg.B, cfg.k, cfg.V, P(d["p"]), P(d["q"]) if cfg.k else None, P(d["draft"]) if cfg.k else None,
                    P(d["u"]), P(d["accept_len"]), P(d["next_token"]), P(ws_acc), ws_acc_bytes, sh)
        vote_args = (1, cfg.B, P(d["answers"]), P(d["winner"]), P(d["winner_count"]), sh)
        calls.append((attn_args, acc_args, vote_args))

    def step(i, ev=None, split=False):
        attn_args, acc_args, vote_args = calls[i % nsets]
        if ev is not None:
            ev[0].record(stream)
        rc = lib.verify_attention(*attn_args)
        if ev is not None:
            ev[1].record(stream)
        rc |= lib.spec_accept(*acc_args)
        if split:
            ev[2].record(stream)
        rc |= lib.majority_vote(*vote_args)
        if split:
            ev[3].record(stream)
        if rc != 0:
            raise RuntimeError("a lotts call failed (status %d)" % rc)

    # The first launches of a process run on a GPU that is still at idle clocks (measured: up to 63 us for the
    # attention kernel instead of 46).  SETTLE untimed steps bring it to its running state whatever --warmup is;
    # the W warm-up steps of the contract follow.
    SETTLE = 200
    for i in range(SETTLE + args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps, sync on both sides.  The library's kernel timer picks out the
    # verify_attention call of every 8th step: its launch carries its own HIP event pair on the launch
    # stream, which reads the kernel's start and end on the device (the dominant kernel's launch
    # duration, without the gaps that event records around a call would add).  A timed launch costs the
    # queue about 7 us more than a plain one, hence not every step.  After the region the same pattern of
    # steps (one timed, seven plain) goes on until --min-timed-launches launches have been timed in all, so
    # that the roofline figure rests on a sample of that size whatever K is.
    K = args.steps
    EVERY = 8
    n_launch = ctypes.c_int32()
    assert lib.lotts_timer_start(8) == 0
    lib.verify_attention(*calls[0][0])
    assert lib.lotts_timer_stop(ctypes.byref(n_launch), None) == 0
    attn_launches = n_launch.value                     # 1, or 2 when a second launch merges the partials

    def steps_with_sampling(first, count):
        """`count` steps starting at step number `first`; every EVERYth carries the timer.  Returns (kernel ms of
        the timed launches in launch order, host clock before the first step, host clock after the device has
        finished the last)."""
        n_t = (count + EVERY - 1) // EVERY
        buf = (ctypes.c_float * (n_t * attn_launches))()
        assert lib.lotts_timer_start(n_t * attn_launches) == 0     # creates its events on first use: before the clock starts
        lib.lotts_timer_pause(1)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(first, first + count):
            if (i - first) % EVERY == 0:
                attn_args, acc_args, vote_args = calls[i % nsets]
                lib.lotts_timer_pause(0)
                rc = lib.verify_attention(*attn_args)
                lib.lotts_timer_pause(1)
                rc |= lib.spec_accept(*acc_args)
                rc |= lib.majority_vote(*vote_args)
                if rc != 0:
                    raise RuntimeError("a lotts call failed (status %d)" % rc)
            else:
                step(i)
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        got = ctypes.c_int32()
        assert lib.lotts_timer_stop(ctypes.byref(got), buf) == 0 and got.value == n_t * attn_launches
        return list(buf), t_begin, t_end

    kernel_ms, t0, t1 = steps_with_sampling(0, K)
    ms_per_step = (t1 - t0) * 1e3 / K
    n_in_region = len(kernel_ms) // attn_launches
    extra_steps = max(0, args.min_timed_launches - n_in_region) * EVERY
    if extra_steps:
        more, _, _ = steps_with_sampling(K, extra_steps)
        kernel_ms += more
    attn_samples = sorted(kernel_ms[0::attn_launches])   # attn_kernel: the launch that streams K and V
    n_timed = len(attn_samples)
    attn_ms = sum(attn_samples) / n_timed
    merge_ms = sum(kernel_ms[1::attn_launches]) / n_timed if attn_launches == 2 else 0.0
    in_region = kernel_ms[0:n_in_region * attn_launches:attn_launches]

    # ---- outside the timed region: the same K steps with the timer off (what the event pairs cost the step),
    # and verify_attention calls bracketed by event records on the stream (gaps around the call included)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    ms_per_step_timer_off = (time.perf_counter() - t2) * 1e3 / K
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(min(K, 100))]
    for i, e in enumerate(evs):
        step(4 * i, e)
        for j in range(1, 4):
            step(4 * i + j)
    torch.cuda.synchronize()
    attn_ms_bracket = sum(e[0].elapsed_time(e[1]) for e in evs) / len(evs)

    # ---- outside the timed region: per-entry-point split, and verify_attention launched back to back
    K2 = min(K, 200)
    ev4 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K2)]
    for i in range(K2):
        step(i, ev4[i], split=True)
    torch.cuda.synchronize()
    acc_ms = sum(e[1].elapsed_time(e[2]) for e in ev4) / K2
    vote_ms = sum(e[2].elapsed_time(e[3]) for e in ev4) / K2
    # spec_accept back to back (the amortised figure of a launch-bound pass)
    eb = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    eb[0].record(stream)
    for i in range(64):
        lib.spec_accept(*calls[i % nsets][1])
    eb[1].record(stream)
    torch.cuda.synchronize()
    acc_ms_b2b = eb[0].elapsed_time(eb[1]) / 64

    # the whole step replayed from a HIP graph (one graph holds one step per input set; the entry points only enqueue
    # kernels, so they can be captured): what is left of the step when the host-side launch cost is gone
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        gsh = ctypes.c_void_p(int(side.cuda_stream))
        gcalls = [tuple(a[:-1] + (gsh,) for a in c) for c in calls]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for c in gcalls:
                rc = lib.verify_attention(*c[0]) | lib.spec_accept(*c[1]) | lib.majority_vote(*c[2])
                if rc != 0:
                    raise RuntimeError("capture failed")
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        reps = max(1, min(K, 200) // nsets)
        g0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / (reps * nsets)
        del graph
    except Exception as exc:  # a graph leg that fails must not take the bench line with it
        graph_ms = "failed: %s" % exc

    # the amortised figure: one verify_attention call per decoder layer of the model the shape stands for,
    # launched back to back over the rotated inputs, between two event records
    n_layers = 64 if cfg.Hkv == 8 else 36
    layer_ms = []
    for rep in range(3):
        eb = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        eb[0].record(stream)
        for i in range(n_layers):
            lib.verify_attention(*calls[i % nsets][0])
        eb[1].record(stream)
        torch.cuda.synchronize()
        layer_ms.append(eb[0].elapsed_time(eb[1]) / n_layers)
    attn_ms_b2b = sorted(layer_ms)[1]

    # cache-resident variant for comparison: one input set only
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(min(K, 50))]
    for e in ev2:
        e[0].record(stream)
        lib.verify_attention(*calls[0][0])
        e[1].record(stream)
    torch.cuda.synchronize()
    attn_ms_resident = sum(e[0].elapsed_time(e[1]) for e in ev2) / len(ev2)

    # the ceiling of this machine: a kernel that only reads the same K and V buffers (rotated in the same way), launched in
    # the attention kernel's shape and timed in the same way (event pair attached to the dispatch)
    probe_path = os.path.join(ROOT, "paper_2505_19634_amd", "libread_probe.so")
    read_ceiling = None
    if bf and os.path.exists(probe_path):
        probe = ctypes.CDLL(probe_path)
        probe.read_probe.restype = ctypes.c_int
        probe.read_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.POINTER(ctypes.c_float)]
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        kv_bytes = sets[0]["Kpriv"].numel() * sets[0]["Kpriv"].element_size()
        pm = ctypes.c_float()
        probe_ms = []
        for i in range(8 + 64):
            d = sets[i % nsets]
            rc = probe.read_probe(d["Kpriv"].data_ptr(), d["Vpriv"].data_ptr(), kv_bytes, sink.data_ptr(), sh, ctypes.byref(pm))
            if rc != 0:
                raise RuntimeError("read_probe failed")
            if i >= 8:
                probe_ms.append(pm.value)
        probe_ms.sort()
        probe_bytes = 2 * (kv_bytes // 8192) * 8192
        read_ceiling = {"bytes_per_launch": probe_bytes, "launches": len(probe_ms),
                        "avg_launch_ms": sum(probe_ms) / len(probe_ms), "median_launch_ms": probe_ms[len(probe_ms) // 2],
                        "min_launch_ms": probe_ms[0], "max_launch_ms": probe_ms[-1],
                        "GB/s": probe_bytes / (sum(probe_ms) / len(probe_ms) * 1e-3) / 1e9}

    tokens = cfg.B * cfg.R
    n0 = sets[0]["accept_len"].cpu().numpy()
    bytes_attn = attn_algorithmic_bytes(cfg)
    bytes_acc = accept_algorithmic_bytes(cfg, n0)
    achieved = bytes_attn / (attn_ms * 1e-3) / 1e9

    out = {
        "metric": "verified branch-tokens/sec per verify step",
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "untimed_settle_steps_before_warmup": SETTLE,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d k=%d Hq=%d Hkv=%d D=%d prefix=%d private=%d V=%d, 1 layer; step = "
                               "verify_attention + spec_accept + majority_vote" % (
                                   cfg.name, cfg.B, cfg.k, cfg.Hq, cfg.Hkv, cfg.D, cfg.P, cfg.L, cfg.V),
                   "input_sets_rotated": nsets},
        "ms_per_step_timer_off": ms_per_step_timer_off,
        "ms_per_step_hip_graph_replay": graph_ms,
        "roofline": {"bound": "hbm",
                     "kernel": "attn_kernel (%s)" % ("all of verify_attention: one launch" if attn_launches == 1 else
                                                     "streams K and V; attn_merge_kernel follows"),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(args.workload),
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary committed under profiles/ (counters "
                                       "cannot be read from inside this process)",
                     "algorithmic_bytes_per_launch": bytes_attn, "avg_launch_ms": attn_ms, "launches_timed": n_timed,
                     "launch_ms": {"min": attn_samples[0], "median": attn_samples[n_timed // 2], "mean": attn_ms,
                                   "max": attn_samples[-1]},
                     "launches_timed_inside_timed_region": n_in_region,
                     "avg_launch_ms_inside_timed_region": sum(in_region) / len(in_region),
                     "frac_at_median": bytes_attn / (attn_samples[n_timed // 2] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "timing": "HIP event pair attached to the dispatch; the verify_attention launch of every %dth step, in the "
                               "timed region and in the same pattern of steps after it" % EVERY,
                     "read_ceiling_GBs": None if read_ceiling is None else read_ceiling["GB/s"],
                     "frac_of_read_ceiling": None if read_ceiling is None else achieved / read_ceiling["GB/s"],
                     "read_ceiling": read_ceiling,
                     "avg_merge_launch_ms": merge_ms,
                     "avg_call_ms_event_records_around_call": attn_ms_bracket,
                     "avg_call_ms_single_set_cache_resident": attn_ms_resident,
                     "avg_call_ms_back_to_back": attn_ms_b2b},
        "layers_back_to_back": {"layers": n_layers, "ms_per_layer": attn_ms_b2b,
                                "GB/s": bytes_attn / (attn_ms_b2b * 1e-3) / 1e9,
                                "frac_of_hbm_peak": bytes_attn / (attn_ms_b2b * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "note": "verify_attention only, one call per layer back to back over rotated inputs, median of "
                                        "3 runs; launch gaps included"},
        "breakdown_ms": {"verify_attention": attn_ms_bracket, "spec_accept": acc_ms, "majority_vote": vote_ms},
        "spec_accept": {"algorithmic_bytes": bytes_acc, "GB/s": bytes_acc / (acc_ms * 1e-3) / 1e9,
                        "frac_of_hbm_peak": bytes_acc / (acc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "ms_back_to_back": acc_ms_b2b,
                        "mean_accepted": float(n0.mean()),
                        "acceptance_rate_sum_min_p_q": (None if cfg.k == 0 else
                                                        float(np.minimum(s0["p"][:, :cfg.k], s0["q"]).sum(-1).mean())),
                        "acceptance_rate_closed_form": (None if (cfg.k == 0 or not cfg.noise_std) else
                                                        float(math.erfc(cfg.noise_std / 2.0 / math.sqrt(2.0)))),
                        "emitted_tokens_per_s": float((n0 + 1).sum()) / (ms_per_step * 1e-3)},
    }

    def time_op(call, reps, launches_per_call):
        """(average ms of the call between event records on the stream, [average kernel ms per launch of the call])."""
        evs_ = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
        for i, e in enumerate(evs_):
            e[0].record(stream)
            if call(i) != 0:
                raise RuntimeError("a lotts call failed")
            e[1].record(stream)
        torch.cuda.synchronize()
        nl = ctypes.c_int32()
        buf = (ctypes.c_float * (reps * launches_per_call))()
        assert lib.lotts_timer_start(reps * launches_per_call) == 0
        for i in range(reps):
            call(i)
        assert lib.lotts_timer_stop(ctypes.byref(nl), buf) == 0 and nl.value == reps * launches_per_call
        kern = [sum(buf[j::launches_per_call]) / reps for j in range(launches_per_call)]
        return sum(e[0].elapsed_time(e[1]) for e in evs_) / reps, kern

    # ---- the widenings, outside the timed region: acceptance straight from bf16 logits (reads every
    # logit row once instead of reading logits, writing p and q and reading them back), and the
    # confidence-weighted aggregation
    zsets = []
    for i in range(nsets):
        z = (torch.randn((cfg.B, cfg.R, cfg.V), generator=gen, device=dev) * cfg.logit_std)
        zq = z[:, :cfg.k] + torch.randn((cfg.B, cfg.k, cfg.V), generator=gen, device=dev) * (cfg.noise_std or cfg.logit_std)
        zsets.append((z.to(torch.bfloat16).contiguous(), zq.to(torch.bfloat16).contiguous()))
        del z, zq
    ws_lg_bytes = lib.spec_accept_logits_workspace_bytes(cfg.B, cfg.k, cfg.V)
    ws_lg = torch.empty(ws_lg_bytes, dtype=torch.uint8, device=dev)
    d0 = sets[0]

    def lg_call(i):
        zt, zd = zsets[i % nsets]
        return lib.spec_accept_logits(cfg.B, cfg.k, cfg.V, P(zt), P(zd) if cfg.k else None, binding.LOTTS_BF16,
                                      ctypes.c_float(1.0), P(d0["draft"]) if cfg.k else None, P(d0["u"]),
                                      P(d0["accept_len"]), P(d0["next_token"]), None, P(ws_lg), ws_lg_bytes, sh)
    for i in range(8):
        assert lg_call(i) == 0
    lg_ms, lg_kern = time_op(lg_call, 100, 3)
    lg_bytes = cfg.B * (2 * cfg.k + 1) * cfg.V * 2
    out["spec_accept_logits"] = {"ms": lg_ms, "kernel_ms": dict(zip(("lg_max", "lg_sum", "lg_scan_pick"), lg_kern)),
                                 "algorithmic_bytes": lg_bytes, "logit_dtype": "bf16",
                                 "GB/s": lg_bytes / (lg_ms * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": lg_bytes / (lg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    Tc = 1024
    conf = 0.3 + 0.7 * torch.rand((1, cfg.B, Tc), generator=gen, device=dev)
    cw = torch.empty((1,), dtype=torch.int32, device=dev)
    cs = torch.empty((1,), dtype=torch.float32, device=dev)
    cv_ms, cv_kern = time_op(lambda i: lib.confidence_vote(1, cfg.B, Tc, P(d0["answers"]), P(conf), None, 1, 1, P(cw),
                                                           P(cs), sh), 50, 1)
    out["confidence_vote"] = {"ms": cv_ms, "kernel_ms": cv_kern[0], "scores_per_branch": Tc, "mode": "avg-vote"}

    # cache append of the step's new tokens: K and V columns of a QKV-projection-shaped matrix to the tails of the
    # private caches of input set 0
    heads = torch.randn((cfg.B, cfg.R, cfg.Hq + 2 * cfg.Hkv, cfg.D), generator=gen, device=dev).to(sets[0]["Kpriv"].dtype)
    kn, vn = heads[:, :, cfg.Hq:cfg.Hq + cfg.Hkv], heads[:, :, cfg.Hq + cfg.Hkv:]
    kp, vp_ = sets[0]["Kpriv"].clone(), sets[0]["Vpriv"].clone()
    ka_dt = binding.LOTTS_BF16 if kp.dtype == torch.bfloat16 else binding.LOTTS_F32
    ka_ms, ka_kern = time_op(lambda i: lib.kv_append(cfg.B, cfg.k, cfg.Hkv, cfg.D, ka_dt, P(kn), P(vn), kn.stride(0),
                                                     kn.stride(1), kn.stride(2), P(kp), P(vp_), kp.stride(0), kp.stride(1),
                                                     kp.stride(2), kp.shape[2], P(sets[0]["priv_len"]), sh), 50, 1)
    out["kv_append"] = {"ms": ka_ms, "kernel_ms": ka_kern[0], "bytes_moved": 2 * 2 * cfg.B * cfg.R * cfg.Hkv * cfg.D * kp.element_size()}
    del heads, kp, vp_

    # weight GEMMs of one 32B-shaped decoder layer for the step's M = B * (k + 1) tokens (hidden 5120,
    # 40/8 heads of 128, MLP 27648): QKV, O, gate+up, down.  Weight copies are rotated like the KV sets.
    Mg = args.gemm_tokens if 1 <= args.gemm_tokens <= 256 else min(cfg.B * cfg.R, 256)
    gemms = {}
    for name_, (Ng, Kg) in {"qkv_proj": (7168, 5120), "o_proj": (5120, 5120), "gate_up_proj": (55296, 5120),
                            "down_proj": (5120, 27648)}.items():
        ncopies = 3
        Ws = [(torch.randn((Ng, Kg), generator=gen, device=dev) * Kg ** -0.5).to(torch.bfloat16) for _ in range(ncopies)]
        Xg = torch.randn((Mg, Kg), generator=gen, device=dev).to(torch.bfloat16)
        Yg = torch.empty((Mg, Ng), dtype=torch.bfloat16, device=dev)
        wsb = lib.skinny_gemm_workspace_bytes(Mg, Ng, Kg)
        wsg = torch.empty(wsb, dtype=torch.uint8, device=dev)
        call = lambda i: lib.skinny_gemm(Mg, Ng, Kg, P(Xg), Kg, P(Ws[i % ncopies]), Kg, P(Yg), Ng, P(wsg), wsb, sh)
        for i in range(6):
            assert call(i) == 0
        assert lib.lotts_timer_start(4) == 0
        call(0)
        nl = ctypes.c_int32()
        assert lib.lotts_timer_stop(ctypes.byref(nl), None) == 0   # 2 launches when K is split
        ms, kern = time_op(call, 40, nl.value)
        nbytes = 2 * (Ng * Kg + Mg * Kg + Mg * Ng)
        gemms[name_] = {"M": Mg, "N": Ng, "K": Kg, "ms": ms, "kernel_ms": kern, "algorithmic_bytes": nbytes,
                        "GB/s": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "TFLOP/s": 2.0 * Mg * Ng * Kg / (ms * 1e-3) / 1e12}
        del Ws, Xg, Yg, wsg
    out["skinny_gemm"] = gemms

    # ---- the CPU oracle on the same inputs (set 0), on this machine's host cores: a baseline, not the target
    if not args.no_cpu_baseline:
        import oracle
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 50:
            c0 = time.perf_counter()
            oracle.verify_attention(a0["Q"], a0["Kpre"], a0["Vpre"], a0["Kpriv"], a0["Vpriv"], a0["priv_len"],
                                    want_lse=False)
            oracle.spec_accept(s0["p"], s0["q"], s0["draft"], s0["u"])
            oracle.majority_vote(answers0)
            t_cpu += time.perf_counter() - c0
            reps += 1
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        out["cpu_baseline"] = {"value": tokens * reps / t_cpu, "unit": "tokens/s", "cores": oracle.n_threads(),
                               "kind": "oracle", "cpu_model": cpu_model,
                               "sample": "%d full steps of the same workload (input set 0), fp64, OpenMP over "
                                         "(branch, head)" % reps}
        # the same on one thread (a shorter sample: about 5 s)
        all_threads = oracle.n_threads()
        oracle.set_threads(1)
        reps1, t1cpu = 0, 0.0
        while t1cpu < 5.0 and reps1 < 10:
            c0 = time.perf_counter()
            oracle.verify_attention(a0["Q"], a0["Kpre"], a0["Vpre"], a0["Kpriv"], a0["Vpriv"], a0["priv_len"],
                                    want_lse=False)
            oracle.spec_accept(s0["p"], s0["q"], s0["draft"], s0["u"])
            oracle.majority_vote(answers0)
            t1cpu += time.perf_counter() - c0
            reps1 += 1
        oracle.set_threads(all_threads)
        out["cpu_baseline"]["value_one_thread"] = tokens * reps1 / t1cpu
        out["cpu_baseline"]["sample_one_thread"] = "%d full steps" % reps1
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
