"""Pins for the cache-append oracle.  It is a copy, so the pins are about WHERE the rows go: numpy slice assignment
written from the definition, nothing else touched, out-of-range positions skipped -- and the position convention tied
to the attention oracle: the appended keys are exactly the ones the causal window of each new row ends with."""
import numpy as np

import synth_inputs as S


def _case(g, B, k, Hkv, D, Lmax, dtype):
    R = k + 1
    mk = (lambda *sh: g.normal(0, 1, sh).astype(np.float32)) if dtype == np.float32 else \
         (lambda *sh: S.f32_to_bf16_bits(g.normal(0, 1, sh).astype(np.float32)))
    return mk(B, R, Hkv, D), mk(B, R, Hkv, D), mk(B, Hkv, Lmax, D), mk(B, Hkv, Lmax, D)


def test_rows_land_at_the_tail_and_nothing_else_moves(oracle):
    g = np.random.default_rng(5)
    for B, k, Hkv, D, Lmax, dtype in [(3, 2, 2, 8, 11, np.float32), (2, 0, 3, 16, 5, np.uint16), (4, 3, 1, 8, 9, np.uint16)]:
        Kn, Vn, K, V = _case(g, B, k, Hkv, D, Lmax, dtype)
        R = k + 1
        priv_len = g.integers(R, Lmax + 1, B).astype(np.int32)
        K2, V2 = oracle.kv_append(Kn, Vn, K, V, priv_len)
        Kw, Vw = K.copy(), V.copy()
        for b in range(B):
            L = int(priv_len[b])
            Kw[b, :, L - R:L] = Kn[b].transpose(1, 0, 2)   # [R][Hkv][D] -> [Hkv][R][D]
            Vw[b, :, L - R:L] = Vn[b].transpose(1, 0, 2)
        assert np.array_equal(K2, Kw) and np.array_equal(V2, Vw)
        assert K2.dtype == K.dtype and (K2 != K).sum() <= B * R * Hkv * D   # only the tails can differ


def test_positions_outside_the_cache_are_skipped(oracle):
    g = np.random.default_rng(6)
    Kn, Vn, K, V = _case(g, 3, 2, 2, 8, 6, np.float32)
    K2, V2 = oracle.kv_append(Kn, Vn, K, V, [1, 7, 6])     # too short, too long, exactly full
    assert np.array_equal(K2[0, :, 0], Kn[0, 2]) and np.array_equal(K2[0, :, 1:], K[0, :, 1:])   # rows 0, 1 fall before 0
    assert np.array_equal(K2[1, :, 4:6], Kn[1, :2].transpose(1, 0, 2)) and np.array_equal(K2[1, :, :4], K[1, :, :4])
    assert np.array_equal(V2[2, :, 3:6], Vn[2].transpose(1, 0, 2))


def test_the_appended_keys_are_the_ones_each_new_row_sees_last(oracle):
    """Position convention shared with the attention oracle: with a huge scale and Q = the new key of the same
    position, row i of the verify attention returns exactly the value appended for new token i (one-hot limit), for
    every branch and ragged length -- which only holds if token i sits at priv_len - (k+1) + i, the last key row i sees."""
    g = np.random.default_rng(7)
    B, k, H, D, Lmax = 3, 2, 2, 16, 12
    R = k + 1
    Kn = g.normal(0, 1, (B, R, H, D)).astype(np.float32)
    Kn /= np.linalg.norm(Kn, axis=-1, keepdims=True)       # unit keys: a key matches itself best
    Vn = g.normal(0, 1, (B, R, H, D)).astype(np.float32)
    K = (0.1 * g.normal(0, 1, (B, H, Lmax, D))).astype(np.float32)   # old keys: short, never the best match
    V = g.normal(0, 1, (B, H, Lmax, D)).astype(np.float32)
    priv_len = np.array([Lmax, R, 7], np.int32)
    K2, V2 = oracle.kv_append(Kn, Vn, K, V, priv_len)
    O, _ = oracle.verify_attention(Kn.copy(), None, None, K2, V2, priv_len, scale=1e4)   # Hq = Hkv: Q[b][i][h] = Knew[b][i][h]
    np.testing.assert_allclose(O, Vn.astype(np.float64), rtol=0, atol=1e-9)
