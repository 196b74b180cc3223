"""GPU parity of zeno_krum (Definition 5, the paper's main baseline) against the CPU oracle."""
import os

import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL
from tests._util import npy, rows_to_gpu

pytestmark = pytest.mark.gpu

# The squared distances come from a Gram matrix accumulated in fp32 on the matrix cores (operands split
# into three bf16 pieces each, six piece products: fp32-level products) and summed in float64 over
# workgroups: exact to about sqrt(columns per wave) * 2^-24 of ||G_i||^2 + ||G_j||^2.
# Gate: 2e-5 of that scale per distance, times the number of distances in a score.
DIST_TOL = 2e-5


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


def _check(B, G, b, row_align=1):
    m, d = G.shape
    ref = O.krum_scores(npy(G), b)
    out, chosen, ks = B.zeno_krum(rows_to_gpu(B, G, row_align), b)
    torch.cuda.synchronize()
    idx = int(chosen.item())
    sq = (npy(G).astype(np.float64) ** 2).sum(1)
    tol = DIST_TOL * (m - b - 2) * 4.0 * sq.max()
    assert np.all(np.abs(npy(ks).astype(np.float64) - ref) <= tol + 1e-6 * np.abs(ref)), (np.abs(npy(ks) - ref).max(), tol)
    # the chosen row is the oracle's whenever the oracle's margin over the runner-up exceeds the tolerance;
    # in any case it is a minimiser up to the tolerance, and the output is that row bit for bit
    order = np.argsort(ref, kind="stable")
    if ref[order[1]] - ref[order[0]] > 2 * tol:
        assert idx == O.krum(npy(G), b)[1]
    assert ref[idx] <= ref.min() + 2 * tol
    assert np.array_equal(npy(out), npy(G[idx]))
    return idx


@pytest.mark.parametrize("m,d,b,row_align", [(5, 7, 1, 1), (20, 7850, 8, 32), (33, 1000, 10, 1), (64, 40003, 16, 32),
                                             (100, 5003, 40, 1), (128, 300, 60, 32), (32, 64, 3, 1), (65, 129, 20, 1)])
def test_krum_against_oracle(B, m, d, b, row_align):
    """An honest cluster (common direction + noise) and b far-away rows at random positions."""
    g = torch.Generator().manual_seed(17 * m + b)
    G = torch.randn(1, d, generator=g) + 0.5 * torch.randn(m, d, generator=g)
    bad = torch.randperm(m, generator=g)[:b]
    G[bad] = -4.0 * G[bad] + 3.0 * torch.randn(b, d, generator=g)
    idx = _check(B, G, b, row_align)
    assert idx not in set(bad.tolist())


def test_krum_row_counts_around_the_block_sizes(B):
    """Row counts on both sides of every 32-row block boundary and in between (one to four row
    blocks, the last one from one live row to full), d with a ragged last chunk."""
    d = 333
    for m in (3, 4, 7, 12, 13, 20, 21, 31, 32, 33, 40, 63, 64, 65, 72, 90, 95, 96, 97, 100, 111, 127, 128):
        g = torch.Generator().manual_seed(900 + m)
        G = torch.randn(1, d, generator=g) + 0.5 * torch.randn(m, d, generator=g)
        b = min(m // 4, m - 3)
        bad = torch.randperm(m, generator=g)[:b]
        G[bad] = -3.0 * G[bad]
        _check(B, G, b, row_align=1 if m % 2 else 32)


def test_krum_full_mantissas_and_wide_exponents(B):
    """Entries whose 24 mantissa bits are all in use (random, and the all-ones pattern) over 40 binades
    and both signs: every one of the three bf16 pieces of a value carries weight, and the piece
    products that the Gram kernel leaves out must stay below the stated tolerance."""
    g = torch.Generator().manual_seed(77)
    m, d = 40, 4099
    mant = torch.randint(0, 1 << 23, (m, d), generator=g, dtype=torch.int32)
    mant[:, ::5] = (1 << 23) - 1
    expo = torch.randint(127 - 20, 127 + 20, (m, d), generator=g, dtype=torch.int32)
    sign = torch.randint(0, 2, (m, d), generator=g, dtype=torch.int32)
    G = ((sign << 31) | (expo << 23) | mant).view(torch.float32)
    assert torch.isfinite(G).all()
    _check(B, G, 9, row_align=32)


def test_krum_discussion_example(B):
    """The one-dimensional example of the Discussion section: four honest gradients with mean 1,
    two colluding ones at -1, b = 2: Krum returns the faulty value."""
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "discussion_1d_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or ":" not in line:
                continue
            k, v = line.split(":")
            vals[k.strip()] = [float(t) for t in v.split()]
    G = torch.tensor(vals["candidates"], dtype=torch.float32)[:, None]
    out, chosen, _ = B.zeno_krum(G.cuda(), int(vals["b"][0]))
    assert float(out[0]) == vals["krum"][0] and int(chosen.item()) in (0, 1)


def test_krum_on_workload_3(B):
    """Workload 3 (sign-flipped colluders, q = b = 8 of 20): identical colluding rows are each
    other's nearest neighbours at distance 0, the failure the paper's Discussion describes."""
    w = WL.make_config(3)
    idx = _check(B, w.G, w.b)
    print("Krum on workload 3 chose row", idx, "(faulty rows:", w.faulty, ")")


def test_krum_error_codes(B):
    G = torch.zeros(6, 8, device="cuda")
    with pytest.raises(B.ZenoError) as e:
        B.zeno_krum(G, 4)                       # m - b - 2 < 1
    assert e.value.status == 1
    with pytest.raises(B.ZenoError) as e:
        B.zeno_krum(torch.zeros(129, 8, device="cuda"), 3, workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 2
    with pytest.raises(B.ZenoError) as e:
        B.zeno_krum(G, 1, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3


def test_krum_non_finite_rows(B):
    """'Arbitrary values' (Section 3, Eq. 1): a row that holds NaN or Inf is infinitely far from every
    row.  It is nobody's near neighbour, its own score is +inf, and the scores of the other rows are
    those of the matrix without it (with one neighbour more to sum)."""
    g = torch.Generator().manual_seed(5)
    m, d, b = 12, 515, 3
    G = torch.randn(1, d, generator=g) + 0.5 * torch.randn(m, d, generator=g)
    G[4, 100] = float("nan")
    G[9, 7] = float("inf")
    ref = O.krum_scores(npy(G), b)
    assert ref[4] == np.inf and ref[9] == np.inf
    out, chosen, ks = B.zeno_krum(G.cuda(), b)
    torch.cuda.synchronize()
    ks = npy(ks).astype(np.float64)
    assert ks[4] == np.inf and ks[9] == np.inf
    ok = [i for i in range(m) if i not in (4, 9)]
    sq = (npy(G[ok]).astype(np.float64) ** 2).sum(1)
    assert np.all(np.abs(ks[ok] - ref[ok]) <= DIST_TOL * (m - b - 2) * 4.0 * sq.max())
    idx = int(chosen.item())
    assert idx not in (4, 9) and np.array_equal(npy(out), npy(G[idx]))


@pytest.mark.parametrize("m,d,b,spread", [(24, 50003, 6, 1e-4), (70, 9000, 20, 1e-5), (100, 4099, 30, 1e-3)])
def test_krum_tight_honest_cluster(B, m, d, b, spread):
    """The late-training case of the Discussion section: honest gradients that agree to `spread` of
    their norm, plus b rows far away.  Squared distances inside the cluster are `spread`^2 of the
    squared norms, far below the 1e-7 that S_ii + S_jj - 2 S_ij can resolve, so the scores of the
    honest rows must come from the second pass (rows minus the first pass's choice): they are held
    to 1e-3 of THEMSELVES against the float64 oracle, and the chosen row must be a minimiser."""
    g = torch.Generator().manual_seed(31 * m + b)
    centre = torch.randn(1, d, generator=g)
    G = centre + spread * torch.randn(m, d, generator=g)
    bad = torch.randperm(m, generator=g)[:b]
    G[bad] = -2.0 * centre + 0.5 * torch.randn(b, d, generator=g)
    ref = O.krum_scores(npy(G), b)
    out, chosen, ks = B.zeno_krum(rows_to_gpu(B, G, 32), b)
    torch.cuda.synchronize()
    ks = npy(ks).astype(np.float64)
    honest = np.array([i for i in range(m) if i not in set(bad.tolist())])
    sq_min = float((npy(G).astype(np.float64) ** 2).sum(1).min())
    assert ref[honest].max() / (m - b - 2) < 1e-5 * sq_min      # every distance inside the cluster is a cancelling one
    rel = np.abs(ks[honest] - ref[honest]) / ref[honest]
    assert rel.max() <= 1e-3, rel.max()
    idx = int(chosen.item())
    assert idx in set(honest.tolist()) and ref[idx] <= ref.min() * (1.0 + 2e-3)
    assert np.array_equal(npy(out), npy(G[idx]))
