"""The byte accounting behind the roofline figure, pinned to what the paper prints."""
import os
import re

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_values.txt")):
        m = re.match(r"\s*([a-z_0-9]+)\s*=\s*([0-9.e+-]+)", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out


def test_kv_bytes_per_token_match_the_papers_memory_figure():
    import bench
    g = golden()
    cfg = S.CONFIGS["C3"]
    # private KV of ONE branch of 1024 tokens, no prefix, Q/O excluded, times the layers
    one = cfg.with_(B=1, P=0, L=1024)
    kv = bench.attn_algorithmic_bytes(one) - 2 * one.B * one.R * one.Hq * one.D * 2
    assert kv == 4096 * 1024
    total = kv * g["layers_32b"]
    assert total == 2 ** 28                                   # 0.25 GiB
    assert abs(total - g["kv_cache_bytes_per_branch_32b_1024_tokens"]) / total < 0.08   # "0.25 GB" as printed


def test_prefix_is_counted_once_whatever_b_is():
    import bench
    cfg = S.CONFIGS["C3"]
    b1 = bench.attn_algorithmic_bytes(cfg.with_(B=1))
    b16 = bench.attn_algorithmic_bytes(cfg)
    per_token = 2 * cfg.Hkv * cfg.D * 2
    qo = 2 * cfg.R * cfg.Hq * cfg.D * 2
    assert b16 - b1 == 15 * (cfg.L * per_token + qo)          # only private tokens and Q/O scale with B
    assert b16 == per_token * (cfg.P + 16 * cfg.L) + 16 * qo == 254017536


def test_accept_bytes():
    import bench
    cfg = S.CONFIGS["C3"]
    assert bench.accept_algorithmic_bytes(cfg, [cfg.k] * 16) == 16 * cfg.V * 4          # all accepted: p_k only
    assert bench.accept_algorithmic_bytes(cfg, [0] * 16) == 2 * 16 * cfg.V * 4          # all rejected: p_n and q_n


def test_recipe_acceptance_inside_the_papers_band():
    g = golden()
    assert g["acceptance_rate_min"] - 0.1 < S.expected_acceptance(1.0) < S.expected_acceptance(0.5) < g["acceptance_rate_max"]
