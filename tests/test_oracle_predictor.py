"""Pins of the oracle's Importance Predictor MLP (Sec. 4.1; App. A "Predictor Overhead") against library
matrix products, the collapsed linear map, special cases and symmetries."""
import numpy as np
import pytest
from scipy.special import expit

from oracle import dynts_oracle as orc


def _weights(rng, d, m1, m2, Nb=3):
    return (rng.standard_normal((Nb, d)), rng.standard_normal((m1, d)) / np.sqrt(d), rng.standard_normal(m1) * 0.1,
            rng.standard_normal((m2, m1)) / np.sqrt(m1), rng.standard_normal(m2) * 0.1,
            rng.standard_normal(m2) / np.sqrt(m2), rng.standard_normal(1))


def test_equals_library_matrix_products():
    rng = np.random.default_rng(61)
    h, W1, b1, W2, b2, w3, b3 = _weights(rng, 24, 48, 12)
    acts = {orc.ACT_NONE: lambda x: x, orc.ACT_RELU: lambda x: np.maximum(x, 0), orc.ACT_SILU: lambda x: x * expit(x)}
    for code, f in acts.items():
        want = f(f(h @ W1.T + b1) @ W2.T + b2) @ w3 + b3[0]
        np.testing.assert_allclose(orc.predictor(h, W1, b1, W2, b2, w3, b3, code), want, rtol=1e-12, atol=1e-14)
        want0 = f(f(h @ W1.T) @ W2.T) @ w3
        np.testing.assert_allclose(orc.predictor(h, W1, None, W2, None, w3, None, code), want0, rtol=1e-12, atol=1e-14)


def test_without_activation_it_is_one_linear_map():
    """A "linear" three-layer MLP collapses to h . (W1^T W2^T w3) + const: a different association order."""
    rng = np.random.default_rng(62)
    h, W1, b1, W2, b2, w3, b3 = _weights(rng, 16, 32, 8, Nb=5)
    v = W1.T @ (W2.T @ w3)
    const = b1 @ (W2.T @ w3) + b2 @ w3 + b3[0]
    np.testing.assert_allclose(orc.predictor(h, W1, b1, W2, b2, w3, b3, orc.ACT_NONE), h @ v + const, rtol=1e-11)


def test_relu_special_cases_and_symmetries():
    rng = np.random.default_rng(63)
    h, W1, b1, W2, b2, w3, b3 = _weights(rng, 16, 32, 8)
    # all pre-activations positive: ReLU does nothing
    hp, W1p, W2p = np.abs(h), np.abs(W1), np.abs(W2)
    np.testing.assert_allclose(orc.predictor(hp, W1p, np.abs(b1), W2p, np.abs(b2), w3, b3, orc.ACT_RELU),
                               orc.predictor(hp, W1p, np.abs(b1), W2p, np.abs(b2), w3, b3, orc.ACT_NONE), rtol=1e-13)
    # all first-layer pre-activations negative: only the biases of the later layers survive
    s = orc.predictor(hp, -W1p, -np.abs(b1), W2, b2, w3, b3, orc.ACT_RELU)
    np.testing.assert_allclose(s, np.maximum(b2, 0) @ w3 + b3[0], rtol=1e-13)
    # hidden units may be renumbered; each token is scored on its own
    p1, p2 = rng.permutation(32), rng.permutation(8)
    base = orc.predictor(h, W1, b1, W2, b2, w3, b3, orc.ACT_SILU)
    np.testing.assert_allclose(orc.predictor(h, W1[p1], b1[p1], np.ascontiguousarray(W2[:, p1][p2]), b2[p2], w3[p2], b3,
                                             orc.ACT_SILU), base, rtol=1e-12)
    np.testing.assert_allclose(orc.predictor(np.ascontiguousarray(h[::-1]), W1, b1, W2, b2, w3, b3, orc.ACT_SILU),
                               base[::-1], rtol=1e-13)
    # transposed weights are a different function
    W1t = np.ascontiguousarray(W1[:16, :].T)
    W1x = W1.copy(); W1x[:16, :] = W1t
    assert not np.allclose(orc.predictor(h, W1x, b1, W2, b2, w3, b3, orc.ACT_SILU), base)
    with pytest.raises(Exception):
        orc.predictor(h, W1, b1, W2, b2, w3, b3, 7)


def test_cost_matches_the_papers_count():
    """App. A: 2 (d m1 + m1 m2 + m2) = 6 d^2 + d multiply-adds-as-flops for m1 = 2d, m2 = d/2."""
    for d in (3584, 4096):
        assert orc.mlp_flops(d, 2 * d, d // 2, 1) == 6 * d * d + d
