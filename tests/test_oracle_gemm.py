"""Pins for the weight-GEMM oracle: it is a plain matrix product, so numpy's matmul on the exactly
converted inputs is the reference; plus identity weights and the transposition being the right one."""
import numpy as np

import synth_inputs as S


def test_matches_numpy_matmul(oracle):
    g = np.random.default_rng(0)
    for M, N, K, bf in [(3, 5, 7, False), (64, 96, 256, True), (40, 33, 128, True), (1, 1, 1, False)]:
        X = g.normal(0, 1, (M, K)).astype(np.float32)
        W = g.normal(0, 0.05, (N, K)).astype(np.float32)
        if bf:
            Xb, Wb = S.f32_to_bf16_bits(X), S.f32_to_bf16_bits(W)
            Y = oracle.skinny_gemm(Xb, Wb)
            ref = S.bf16_bits_to_f32(Xb).astype(np.float64) @ S.bf16_bits_to_f32(Wb).astype(np.float64).T
        else:
            Y = oracle.skinny_gemm(X, W)
            ref = X.astype(np.float64) @ W.astype(np.float64).T
        np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)


def test_identity_and_orientation(oracle):
    g = np.random.default_rng(1)
    X = g.normal(0, 1, (4, 6)).astype(np.float32)
    assert np.array_equal(oracle.skinny_gemm(X, np.eye(6, dtype=np.float32)), X.astype(np.float64))
    W = np.zeros((3, 6), np.float32)
    W[2, 4] = 2.0                                      # output feature 2 reads input feature 4
    Y = oracle.skinny_gemm(X, W)
    assert np.array_equal(Y[:, 2], 2.0 * X[:, 4].astype(np.float64)) and not Y[:, :2].any()
