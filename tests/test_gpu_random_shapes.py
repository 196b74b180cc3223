"""Seeded random sweep over the shapes the C-ABI accepts: depth, widths (multiples of the tile sizes and
not), number of candidates, server batch size, loss, bias, operand precision, row pitch and the alignment
of a densely packed matrix inside its allocation are drawn together, so that combinations no hand-written
case lists still get run.  Every case compares ALL scores with the float64 oracle (bf16 forward: with the
oracle's bf16-operand variant) under the stated tolerances, and selection + average, Median and Krum on the
same matrix with the oracle bit for bit (Krum: within its Gram tolerance, chosen row bit for bit).

The candidates are N(0, 0.02^2) rows with one row scaled by 50: shapes and value ranges of gradients, no
training behind them; what is checked here is arithmetic, not which rows get trimmed."""
import random

import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL
from tests._util import SCORE_TOL, exact_terms, npy, oracle_terms, rows_to_gpu, score_error

pytestmark = pytest.mark.gpu

ORACLE_FLOPS = 3e10      # bound on 2 m n_r d per case: the oracle scores a case in about a second
MAX_ELEMENTS = 2e8       # bound on m d (0.8 GB of candidates; the oracle's median sorts them all)
MAX_KRUM_WORK = 1e10     # bound on m m d for the oracle's pairwise distances
N_CASES = 36


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


def _draw(case):
    rng = random.Random(4242 + case)
    depth = rng.choice([1, 2, 2, 3, 3, 4])
    d_in = rng.choice([64, 200, 785, 1000, 1024, 2048, 3072])
    hidden = [rng.choice([40, 100, 256, 500, 512, 1000, 1024, 1536, 2048]) for _ in range(depth - 1)]
    loss, d_out = "softmax_ce", rng.choice([2, 10, 12, 100, 257, 1000])
    if rng.random() < 0.15:
        loss, d_out = "squared", 1
    dims = [d_in] + hidden + [d_out]
    fwd = rng.choice(["fp32", "bf16"])
    n_r = rng.choice([1, 4, 5, 16, 31, 32, 33, 64, 96, 128, 129, 160])
    m = rng.choice([1, 3, 17, 20, 33, 60, 64, 65, 96, 100, 127, 128])
    has_bias = rng.random() < 0.8
    d = WL.num_params(dims, has_bias)
    while m > 1 and (2.0 * m * n_r * d > ORACLE_FLOPS or m * d > MAX_ELEMENTS):
        m //= 2
    b = rng.randrange(0, m)
    row_align = rng.choice([1, 1, 32])
    offset = rng.choice([0, 1, 2, 4]) if row_align == 1 else 0
    gamma, rho = rng.choice([0.05, 0.1]), rng.choice([1e-3, 5e-4])
    krum_b = rng.randrange(0, (m - 3) // 2 + 1) if m >= 5 and m * m * d <= MAX_KRUM_WORK else None
    big_row = rng.randrange(m) if m > 2 else None
    return dims, has_bias, loss, fwd, n_r, m, b, row_align, offset, gamma, rho, krum_b, big_row


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_shape(B, case):
    dims, has_bias, loss, fwd, n_r, m, b, row_align, offset, gamma, rho, krum_b, big_row = _draw(case)
    d = WL.num_params(dims, has_bias)
    print(f"\n  dims={dims} bias={has_bias} {loss} {fwd} n_r={n_r} m={m} b={b} row_align={row_align} offset={offset}",
          flush=True)
    g = torch.Generator().manual_seed(977 * case + 5)
    x = WL.init_params(dims, has_bias, g, "cpu")
    features = torch.randn(n_r, dims[0], generator=g)
    labels = targets = None
    if loss == "softmax_ce":
        labels = torch.randint(0, dims[-1], (n_r,), generator=g).to(torch.int32)
    else:
        targets = torch.randn(n_r, generator=g)
    G = torch.randn(m, d, generator=g) * 0.02
    if big_row is not None:
        G[big_row] *= 50.0
    w = WL.Workload(f"random{case}", dims, has_bias, loss, fwd, m, b, n_r, gamma, rho, x, G, features, labels, targets)
    dev = torch.device("cuda", 0)
    if offset:
        buf = torch.empty(m * d + offset, dtype=torch.float32, device=dev)
        Gd = buf[offset:].view(m, d)
        Gd.copy_(G)
    else:
        Gd = rows_to_gpu(B, G, row_align, dev)
    mdl = B.ZenoModel(dims, has_bias, loss, fwd)
    s = B.zeno_score(mdl, x.to(dev), Gd, features.to(dev), gamma, rho,
                     labels=None if labels is None else labels.to(dev),
                     targets=None if targets is None else targets.to(dev))
    torch.cuda.synchronize()
    s_ref, scale = oracle_terms(w)
    err = score_error(npy(s), s_ref, scale)
    ok = err <= SCORE_TOL[fwd]
    if fwd == "fp32" and n_r <= 5 and not np.all(ok):
        # a handful of samples whose loss hardly moves although the logits do: the difference of the two
        # losses cancels, and the row is held to 1e-6 of the magnitudes that enter the score instead
        s_exact, sc, mag = exact_terms(w, with_losses=True)
        mixed = np.abs(npy(s).astype(np.float64) - s_exact) / (mag + sc)
        ok = ok | ((sc <= 2e-3 * mag) & (mixed <= 1e-6) & (err <= 1e-4))
    assert np.all(ok), (float(err.max()), int(err.argmax()))

    out, sel = B.zeno_aggregate(Gd, s, b)
    torch.cuda.synchronize()
    ref_out, ref_sel = O.zeno_aggregate(G.numpy(), npy(s), b)
    assert np.array_equal(npy(sel).astype(np.int64), ref_sel)
    assert np.array_equal(npy(out), ref_out.astype(np.float32))
    assert np.array_equal(npy(B.zeno_mean(Gd)), O.mean(G.numpy()).astype(np.float32))
    assert np.array_equal(npy(B.zeno_median(Gd)), O.median(G.numpy()).astype(np.float32))
    if krum_b is not None:
        ref = O.krum_scores(G.numpy(), krum_b)
        k_out, k_idx, k_scores = B.zeno_krum(Gd, krum_b)
        torch.cuda.synchronize()
        sq = (G.numpy().astype(np.float64) ** 2).sum(1)
        tol = 2e-5 * (m - krum_b - 2) * 4.0 * sq.max()
        idx = int(k_idx.item())
        assert np.all(np.abs(npy(k_scores).astype(np.float64) - ref) <= tol + 1e-6 * np.abs(ref))
        assert ref[idx] <= ref.min() + 2 * tol
        assert np.array_equal(npy(k_out), G.numpy()[idx])
