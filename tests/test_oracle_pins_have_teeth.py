"""The pins must be able to fail: plant one plausible mistake at a time into a COPY of the oracle's source
(CPU only), compile it, run the pins of that area against the broken copy and require that at least one
of them objects.  The real oracle is never touched."""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

import synth_inputs as S
import test_oracle_accept as TA
import test_oracle_attention as TT
import test_oracle_confidence as TC
import test_oracle_gemm as TG
import test_oracle_kv_append as TK
import test_oracle_logits as TL
import test_oracle_vote as TV

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lotts_oracle.c")

BATTERY = {
    "attention": [lambda o: [TT.test_matches_brute_force(o, c) for c in (
                      TT.TINY.with_(Hq=6, Hkv=2, D=16, P=5, L=11, k=2, B=3),
                      TT.TINY.with_(Hq=8, Hkv=4, D=32, P=7, L=13, k=1, B=2, dtype="bf16", qkv_std=0.5))],
                  TT.test_ragged_private_lengths_and_scale, TT.test_uniform_limit_closed_form,
                  TT.test_causality_row_i_equals_decode_on_truncated_cache, TT.test_prefix_boundary_can_move,
                  TT.test_bf16_bits_are_read_exactly],
    "accept": [TA.test_greedy_accepts_exactly_the_longest_matching_prefix, TA.test_accept_boundary_is_strict,
               TA.test_resample_matches_python_integer_sampler, TA.test_weight_rounding_edges, TA.test_u_extremes,
               TA.test_degenerate_rows, TA.test_k0_is_plain_inverse_cdf, lambda o: TA.test_lossless_monte_carlo(o, 2)],
    "vote": [TV.test_hand_cases, TV.test_against_counting_dictionary_on_zipf_answers],
    "logits": [TL.test_integer_weights_follow_two_to_the_t, lambda o: TL.test_normalised_weights_are_softmax(o, 0.7),
               TL.test_greedy_limit, TL.test_decisions_recomputed_with_python_integers,
               TL.test_agrees_with_the_probability_path, TL.test_power_of_two_rescaling_changes_nothing,
               TL.test_rollback_keeps_exactly_the_verified_tokens],
    "confidence": [TC.test_hand_cases, TC.test_against_dictionary, TC.test_equal_confidences_reduce_to_majority_voting],
    "gemm": [TG.test_matches_numpy_matmul, TG.test_identity_and_orientation],
    "append": [TK.test_rows_land_at_the_tail_and_nothing_else_moves, TK.test_positions_outside_the_cache_are_skipped,
               TK.test_the_appended_keys_are_the_ones_each_new_row_sees_last],
}

# (area, what is planted, text to find, replacement)
MUTATIONS = [
    ("append", "new tokens one position late", "const int64_t t = (int64_t)priv_len[b] - R + r;",
     "const int64_t t = (int64_t)priv_len[b] - R + r + 1;"),
    ("append", "values written where keys go", "memcpy((char *)Vpriv + dst, (const char *)Vnew + src, row);",
     "memcpy((char *)Kpriv + dst, (const char *)Vnew + src, row);"),
    ("append", "heads and rows of the new tokens swapped", "const size_t src = (((size_t)b * R + r) * Hkv + h) * row;",
     "const size_t src = (((size_t)b * Hkv + h) * R + r) * row;"),
    ("attention", "causal window one key too long", "const int n_priv = Lb - k + i;", "const int n_priv = Lb - k + i + 1;"),
    ("attention", "causal window ignores the row index", "const int n_priv = Lb - k + i;", "const int n_priv = Lb - k;"),
    ("attention", "interleaved instead of contiguous GQA grouping", "const int g = h / G;", "const int g = h % Hkv;"),
    ("attention", "scale dropped", "s[j] = acc * scale;", "s[j] = acc;"),
    ("attention", "head dimension of V reversed", "acc += s[j] * load_elem(Vb, dtype, voff + d);",
     "acc += s[j] * load_elem(Vb, dtype, voff + (D - 1 - d));"),
    ("attention", "prefix values taken from the private cache", "Vb = Vpre;\n                            voff = ((int64_t)g * P + j) * D;",
     "Vb = Vpriv;\n                            voff = (((int64_t)b * Hkv + g) * Lmax + j) * D;"),
    ("attention", "LSE without the maximum", "lse[((int64_t)b * R + i) * Hq + h] = mx + log(denom);",
     "lse[((int64_t)b * R + i) * Hq + h] = log(denom);"),
    ("attention", "bf16 read as the low half of an fp32", "<< 16;\n    float f;", "<< 0;\n    float f;"),
    ("accept", "accept test not strict", "if (uv * qv < pv)", "if (uv * qv <= pv)"),
    ("accept", "accept test inverted ratio", "if (uv * qv < pv)", "if (uv * pv < qv)"),
    ("accept", "residual with the wrong sign", "float r = prow[v] - qrow[v];", "float r = qrow[v] - prow[v];"),
    ("accept", "residual without the clamp at zero", "return r > 0.0f ? r : 0.0f;", "return r > 0.0f ? r : -r;"),
    ("accept", "fixed point one bit short", "float scaled = r * 1099511627776.0f;", "float scaled = r * 549755813888.0f;"),
    ("accept", "threshold shifted by one bit", "(unsigned __int128)Z) >> 24);", "(unsigned __int128)Z) >> 23);"),
    ("accept", "CDF crossing inclusive", "if (run > T) {\n                tok = v;", "if (run >= T) {\n                tok = v;"),
    ("accept", "empty-residual fallback missing", "if (Z == 0 && qrow) {", "if (0) {"),
    ("accept", "bonus row sampled from the residual of the last draft", "const float *qrow = (n < k) ? qb + (int64_t)n * V : NULL;",
     "const float *qrow = qb + (int64_t)(n < k ? n : k - 1) * V;"),
    ("vote", "tie goes to the later answer", "if (c > best_count) {", "if (c >= best_count) {"),
    ("vote", "missing answers counted", "if (a[i] < 0)\n                continue;", ""),
    ("logits", "accept test with p and q swapped", "if (U * Eq[x] * Sp < ((u128)1 << 24) * Ep[x] * Sq)",
     "if (U * Ep[x] * Sq < ((u128)1 << 24) * Eq[x] * Sp)"),
    ("logits", "normalisers swapped in the residual", "const u128 a = (u128)Ep[v] * Sq, c = (u128)Eq[v] * Sp;\n                Z += a > c ? a - c : 0;",
     "const u128 a = (u128)Ep[v] * Sp, c = (u128)Eq[v] * Sq;\n                Z += a > c ? a - c : 0;"),
    ("logits", "a polynomial coefficient with the wrong sign", "g = fmaf(g, f, 0x1.ebfbaap-3f);", "g = fmaf(g, f, -0x1.ebfbaap-3f);"),
    ("logits", "natural exponent instead of base 2", "float t = (y - m) * 0x1.715476p+0f;", "float t = (y - m);"),
    ("logits", "temperature ignored", "return (float)load_elem(z, dtype, idx) * inv_temp;", "return (float)load_elem(z, dtype, idx);"),
    ("logits", "rollback also drops the last accepted draft", "priv_len[b] -= k - n;", "priv_len[b] -= k - n + 1;"),
    ("logits", "rollback drops every draft", "priv_len[b] -= k - n;", "priv_len[b] -= k;"),
    ("confidence", "min and avg exchanged", "w[b] = weight_mode == 0 ?", "w[b] = weight_mode == 1 ?"),
    ("confidence", "vote adds every branch's weight", "if (ok[j] && a[j] == a[i])\n                        score = score + w[j];",
     "if (ok[j])\n                        score = score + w[j];"),
    ("confidence", "tie goes to the later answer", "if (!have || score > best_score) {", "if (!have || score >= best_score) {"),
    ("gemm", "weight not transposed", "load_elem(W, dtype, (int64_t)n * K + k);", "load_elem(W, dtype, (int64_t)(k % N) * K + (n % K));"),
]


class BrokenOracle:
    """Looks like the `oracle` package, but its calls go to a library built from a mutated source."""

    def __init__(self, lib):
        import oracle.oracle as real
        self._real, self._lib = real, lib
        for name in ("verify_attention", "spec_accept", "majority_vote", "spec_accept_logits", "logit_weights",
                     "confidence_vote", "skinny_gemm", "kv_append"):
            setattr(self, name, self._wrap(getattr(real, name)))

    def _wrap(self, fn):
        def call(*a, **kw):
            saved = self._real._lib
            self._real._lib = self._lib
            try:
                return fn(*a, **kw)
            finally:
                self._real._lib = saved
        return call


def run_battery(area, lib_path):
    """Runs the pins of one area against the library at lib_path; returns the names of the exceptions raised."""
    import oracle.oracle as real
    real._load()
    broken = BrokenOracle(real._bind(ctypes.CDLL(lib_path)))
    caught = []
    for pin in BATTERY[area]:
        try:
            pin(broken)
        except (AssertionError, ValueError) as e:
            caught.append(type(e).__name__)
    return caught


@pytest.mark.parametrize("area,what,old,new", MUTATIONS, ids=[m[1].replace(" ", "-") for m in MUTATIONS])
def test_a_planted_mistake_is_caught(tmp_path, area, what, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, "mutation target not found: %r" % old
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new, 1))
    lib_path = tmp_path / "libmut.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-w", "-o",
                    str(lib_path), str(mutated), "-lm"], check=True)
    # a broken oracle may also corrupt memory: the battery runs in a process of its own, and dying counts as noticed
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([ROOT, os.path.join(ROOT, "tests")]))
    res = subprocess.run([sys.executable, os.path.abspath(__file__), area, str(lib_path)], env=env,
                         stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, timeout=300)
    crashed = res.returncode != 0
    caught = [l for l in res.stdout.splitlines() if l.startswith("CAUGHT ")]
    assert crashed or caught, "no pin of the %s battery noticed: %s" % (area, what)


def test_the_real_oracle_passes_every_battery():
    import oracle.oracle as real
    real._load()
    for area in BATTERY:
        assert run_battery(area, real._LIB) == [], area


if __name__ == "__main__":
    for name in run_battery(sys.argv[1], sys.argv[2]):
        print("CAUGHT", name)
