"""Pins for the bf16-operand variant of the oracle (CPU only)."""
import numpy as np
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL


def test_round_bf16_against_torch_and_ties():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-20, 20, 4000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38]]).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_bf16(v), ref)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_bf16(np.float32(1.00390625)) == 1.0
    assert O.round_bf16(np.float32(1.01171875)) == 1.015625
    assert np.isnan(O.round_bf16(np.float32(np.nan)))


def test_bf16_variant_equals_exact_oracle_on_representable_inputs():
    """Small integers everywhere and gamma = 1/2: no operand is changed by the bf16
    rounding and every sum is exact, so the contract must reproduce Definition 2."""
    rng = np.random.default_rng(1)
    dims, has_bias = [6, 5, 4, 3], True
    d = O.num_params(dims, has_bias)
    x = rng.integers(-1, 2, d).astype(np.float32)
    G = (2 * rng.integers(-1, 2, (5, d))).astype(np.float32)
    feats = rng.integers(-1, 3, (7, 6)).astype(np.float32)
    labels = rng.integers(0, 3, 7)
    a = O.scores(x, G, 0.5, 0.125, dims, has_bias, O.LOSS_SOFTMAX_CE, feats, labels)
    b = O.scores_bf16(x, G, 0.5, 0.125, dims, has_bias, O.LOSS_SOFTMAX_CE, feats, labels)
    np.testing.assert_allclose(b, a, rtol=1e-13, atol=1e-13)
    assert np.any(a != a[0])
    # squared loss, no bias
    dims2 = [5, 4, 1]
    d2 = O.num_params(dims2, False)
    x2 = rng.integers(-1, 2, d2).astype(np.float32)
    G2 = (2 * rng.integers(-1, 2, (4, d2))).astype(np.float32)
    f2 = rng.integers(-2, 3, (6, 5)).astype(np.float32)
    y2 = rng.integers(-3, 4, 6).astype(np.float32)
    a2 = O.scores(x2, G2, 0.5, 0.25, dims2, False, O.LOSS_SQUARED, f2, targets=y2)
    b2 = O.scores_bf16(x2, G2, 0.5, 0.25, dims2, False, O.LOSS_SQUARED, f2, targets=y2)
    np.testing.assert_allclose(b2, a2, rtol=1e-13, atol=1e-13)


def test_bf16_variant_is_close_to_exact_on_random_inputs():
    """Forward error of bf16 operands: a few units of 2^-8 per layer, relative to
    |f_r(x) - f_r(x - gamma u)| + rho ||u||^2."""
    w = WL.make_mlp_workload("t", 80, [256, 128, 10], 8, 2, 32, 0.05, 1e-3, "bf16", n_flip=2, n_noise=1,
                             noise_std=10.0)
    npy = lambda t: None if t is None else t.numpy()
    args = (npy(w.x), npy(w.G), w.gamma, w.rho, w.dims, w.has_bias, w.loss, npy(w.features), npy(w.labels))
    a, b = O.scores(*args), O.scores_bf16(*args)
    assert np.max(np.abs(a - b) / np.abs(a)) < 8 * 2.0 ** -8
    assert np.max(np.abs(a - b) / np.abs(a)) > 1e-6      # the rounding is really applied


def test_bf16_variant_counts_m_plus_one_forwards():
    w = WL.make_mlp_workload("t", 81, [12, 8, 3], 5, 1, 4, 0.1, 1e-3, "bf16")
    O.forward_evaluations = 0
    O.scores_bf16(w.x.numpy(), w.G.numpy(), w.gamma, w.rho, w.dims, True, w.loss, w.features.numpy(), w.labels.numpy())
    assert O.forward_evaluations == w.m + 1
