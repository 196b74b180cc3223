"""Pins for the bf16-operand variant of the oracle (CPU only)."""
import numpy as np
import pytest
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


# ---------------------------------------------------------------------------
# A pin for scores_bf16 that owes nothing to the HIP kernels: Definition 2 written as two forward
# passes per candidate in the paper's order, with every matrix operand rounded to bf16 and W and U
# rounded separately (z = rb(h) rb(W)^T - gamma rb(h) rb(U)^T + (b - gamma ub), h = relu(z)).
# No change propagation, no stored differences, no float32 intermediate roundings.  It is not
# bit-equal to scores_bf16 (the two round the candidate's activations at different points), but
# both are the same function up to operand rounding, so they must agree to a few units of 2^-8 of
# the score scale once the perturbation moves the loss by as much as the loss itself; a wrong
# sign, a transposed operand or a missing term moves the result by the scale itself.
# ---------------------------------------------------------------------------
def _plain_split_scores(x, G, gamma, rho, dims, has_bias, loss, features, labels=None, targets=None, *,
                        sign=-1.0, second_term=True, bias_term=True):
    rb = O.round_bf16
    L = len(dims) - 1
    layers_x = O.unflatten(x, dims, has_bias)
    batch = np.asarray(features, dtype=np.float64)

    def losses(z):
        return O.sample_losses(z, loss, labels, targets)

    h = batch
    for l, (W, bias) in enumerate(layers_x):
        z = rb(h) @ rb(W).T + bias
        h = np.maximum(z, 0.0) if l + 1 < L else z
    f0 = float(np.mean(losses(h)))
    out = []
    for i in range(G.shape[0]):
        u = np.asarray(G[i], dtype=np.float64)
        h = batch
        for l, ((W, bias), (U, ub)) in enumerate(zip(layers_x, O.unflatten(u, dims, has_bias))):
            z = rb(h) @ rb(W).T + bias
            if second_term:
                z = z + sign * gamma * (rb(h) @ rb(U).T)
            if bias_term:
                z = z + sign * gamma * ub
            h = np.maximum(z, 0.0) if l + 1 < L else z
        out.append(f0 - float(np.mean(losses(h))) - rho * float(u @ u))
    return np.array(out)


def _pin_case(seed, dims, loss, has_bias):
    rng = np.random.default_rng(seed)
    d = O.num_params(dims, has_bias)
    x = np.concatenate([rng.normal(size=d)]) * 0.2
    x = x.astype(np.float32)
    G = rng.normal(size=(6, d)).astype(np.float32)          # dense rows: every layer and every bias moves
    n_r = 24
    feats = rng.normal(size=(n_r, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], n_r) if loss == O.LOSS_SOFTMAX_CE else None
    targets = rng.normal(size=n_r).astype(np.float32) if loss == O.LOSS_SQUARED else None
    return x, G, feats, labels, targets


@pytest.mark.parametrize("seed,dims,loss,has_bias", [(0, [96, 64, 48, 5], O.LOSS_SOFTMAX_CE, True),
                                                      (1, [80, 40, 1], O.LOSS_SQUARED, True),
                                                      (2, [64, 7], O.LOSS_SOFTMAX_CE, False)])
def test_bf16_variant_against_the_plain_two_pass_split_form(seed, dims, loss, has_bias):
    x, G, feats, labels, targets = _pin_case(seed, dims, loss, has_bias)
    gamma, rho = 0.2, 1e-5           # the step moves the loss by about the loss itself; the penalty is small
    args = (x, G, gamma, rho, dims, has_bias, loss, feats, labels, targets)
    ref = _plain_split_scores(*args)
    got = O.scores_bf16(*args)
    exact = O.scores(*args)
    pen = rho * np.sum(G.astype(np.float64) ** 2, axis=1)
    f0 = O.f_r(x.astype(np.float64), dims, has_bias, loss, feats, labels, targets)
    fi = f0 - exact - pen
    assert np.all(np.abs(f0 - fi) > 0.05 * f0)               # the perturbation really moves the loss
    # The plain form evaluates two losses separately, so its operand-rounding error is relative
    # to the losses themselves, |f_r(x)| + |f_r(x - gamma u)|, not to their difference.
    mag = np.abs(f0) + np.abs(fi)
    bound = 2.0 ** -8
    assert np.max(np.abs(got - ref) / mag) < bound
    assert np.max(np.abs(ref - exact) / mag) < bound         # and the plain form is Definition 2 up to operand rounding
    # what the bound is worth: each planted slip in the plain form lands far outside it
    for slip in (dict(sign=+1.0), dict(second_term=False)) + ((dict(bias_term=False),) if has_bias else ()):
        wrong = _plain_split_scores(*args, **slip)
        assert np.max(np.abs(got - wrong) / mag) > 4 * bound, slip
    if len(dims) > 2:
        # candidates that perturb only the layers after the first: the first-layer terms vanish and
        # the whole score rides on the products with the changed activations of later layers
        Gz = G.copy()
        off = dims[1] * dims[0] + (dims[1] if has_bias else 0)
        Gz[:, :off] = 0.0
        a2 = (x, Gz, gamma, rho, dims, has_bias, loss, feats, labels, targets)
        assert np.max(np.abs(O.scores_bf16(*a2) - _plain_split_scores(*a2)) / mag) < bound
        Gz = G.copy()
        Gz[:, off:] = 0.0                                    # and only the first layer: everything later is D W^T
        a3 = (x, Gz, gamma, rho, dims, has_bias, loss, feats, labels, targets)
        s3, r3 = O.scores_bf16(*a3), _plain_split_scores(*a3)
        assert np.max(np.abs(s3 - r3) / mag) < bound
        assert np.max(np.abs(r3) / mag) > 10 * bound         # (a missing D W^T term would leave these scores at ~0)
