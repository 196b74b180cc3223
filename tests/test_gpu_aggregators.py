"""GPU parity of zeno_aggregate / zeno_mean / zeno_median against the CPU oracle.

Integer work (the selected index set) and the three aggregators must match
bit for bit: the kernels sum the selected rows in ascending index order in fp64
and round once, exactly as the oracle does."""
import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


def _rand_G(m, d, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(m, d, generator=g, dtype=torch.float32) * scale


SHAPES = [(1, 1), (1, 5), (2, 3), (3, 4), (5, 1023), (8, 64), (20, 7850), (7, 4099), (64, 10001),
          (100, 5002), (33, 65537), (128, 777), (1024, 130)]


@pytest.mark.parametrize("m,d", SHAPES)
def test_aggregate_bit_exact(B, m, d):
    G = _rand_G(m, d, 100 * m + d)
    rng = np.random.default_rng(m * 7 + d)
    scores = rng.normal(size=m).astype(np.float32)
    Gd = G.cuda()
    for b in sorted({0, m // 3, m - 1}):
        out, sel = B.zeno_aggregate(Gd, torch.from_numpy(scores).cuda(), b)
        torch.cuda.synchronize()
        ref, ref_sel = O.zeno_aggregate(G.numpy(), scores, b)
        assert np.array_equal(sel.cpu().numpy().astype(np.int64), ref_sel), (m, d, b)
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32)), (m, d, b)


def test_aggregate_b0_equals_mean_kernel(B):
    G = _rand_G(20, 7850, 5).cuda()
    s = torch.randn(20).cuda()
    out, _ = B.zeno_aggregate(G, s, 0)
    assert torch.equal(out, B.zeno_mean(G))


def test_selection_ties_nan_and_infinities(B):
    scores = np.array([1.0, 2.0, 2.0, np.nan, 2.0, -np.inf, np.inf, -0.0, 0.0, np.nan], dtype=np.float32)
    m = len(scores)
    G = _rand_G(m, 37, 1)
    for b in range(m):
        out, sel = B.zeno_aggregate(G.cuda(), torch.from_numpy(scores).cuda(), b)
        ref, ref_sel = O.zeno_aggregate(G.numpy(), scores, b)
        assert sel.cpu().numpy().tolist() == ref_sel.tolist(), b
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))


def test_identical_colluding_rows_and_selected_null(B):
    """All faulty rows equal (Section 6.4): ties between them are broken by index."""
    G = _rand_G(10, 515, 2)
    G[3] = G[7] = G[8] = G[1]
    scores = torch.randn(10)
    scores[3] = scores[7] = scores[8] = scores[1]
    for b in (1, 2, 3, 8):
        out, sel = B.zeno_aggregate(G.cuda(), scores.cuda(), b, want_selected=False)
        assert sel is None
        ref, _ = O.zeno_aggregate(G.numpy(), scores.numpy(), b)
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))


def test_rows_only_four_byte_aligned(B):
    """d mod 4 != 0 and a base pointer that is only 4-byte aligned."""
    m, d = 9, 1001
    flat = torch.randn(m * d + 3, generator=torch.Generator().manual_seed(3)).cuda()
    for shift in (1, 2, 3):
        G = flat[shift:shift + m * d].view(m, d)
        assert G.data_ptr() % 16 != 0
        scores = torch.randn(m, generator=torch.Generator().manual_seed(4))
        out_buf = torch.empty(d + 1, device="cuda")[1:]
        out, sel = B.zeno_aggregate(G, scores.cuda(), 3, out=out_buf)
        ref, ref_sel = O.zeno_aggregate(G.cpu().numpy(), scores.numpy(), 3)
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))
        assert np.array_equal(B.zeno_mean(G).cpu().numpy(), O.mean(G.cpu().numpy()).astype(np.float32))
        assert np.array_equal(B.zeno_median(G).cpu().numpy(), O.median(G.cpu().numpy()).astype(np.float32))


@pytest.mark.parametrize("m,d", [(1, 7), (2, 9), (3, 100), (4, 5), (7, 4099), (8, 64), (20, 7850), (21, 1000),
                                 (33, 2049), (64, 3001), (100, 5002), (127, 300), (128, 515),
                                 # more than 128 rows: the median by rank selection in LDS
                                 (129, 300), (130, 31), (200, 1000), (255, 64), (256, 4099), (513, 777), (1000, 2049),
                                 (1023, 33), (1024, 130)])
def test_mean_and_median_bit_exact(B, m, d):
    G = _rand_G(m, d, 31 * m + d, scale=3.0)
    Gd = G.cuda()
    assert np.array_equal(B.zeno_mean(Gd).cpu().numpy(), O.mean(G.numpy()).astype(np.float32))
    med = B.zeno_median(Gd).cpu().numpy()
    assert np.array_equal(med, O.median(G.numpy()).astype(np.float32))


@pytest.mark.parametrize("row_align", [1, 32])
def test_median_every_m(B, row_align):
    """Every number of candidates the median accepts: each has its own count of compile-time and
    run-time padding keys (and the small ones the four-column lanes when the rows are aligned);
    d = 263 leaves a ragged tail behind the four-column part.  NaN and infinite entries included."""
    from tests._util import rows_to_gpu
    d = 263
    for m in range(1, 129):
        G = _rand_G(m, d, 5000 + m, scale=2.0)
        G[m // 2, ::17] = float("inf")
        G[0, 5::29] = float("nan")
        G[m - 1, 3::31] = float("-inf")
        med = B.zeno_median(rows_to_gpu(B, G, row_align)).cpu().numpy()
        ref = O.median(G.numpy()).astype(np.float32)
        assert np.array_equal(np.isnan(med), np.isnan(ref)), m
        ok = ~np.isnan(ref)
        assert np.array_equal(med[ok], ref[ok]), m


@pytest.mark.parametrize("row_align", [1, 32])
@pytest.mark.parametrize("m", [129, 192, 500, 1024])
def test_median_by_selection_with_ties_and_nonfinite_entries(B, m, row_align):
    """m > 128: ties (few distinct values, so the two middle keys are often equal), columns of one value,
    NaN, +inf and -inf entries, a column that is NaN in more than half of its rows; dense and line-aligned rows."""
    from tests._util import rows_to_gpu
    d = 333
    g = torch.Generator().manual_seed(7000 + m)
    G = torch.randint(-3, 4, (m, d), generator=g).to(torch.float32) * 0.5
    G[:, 1::4] = _rand_G(m, d, 7100 + m)[:, 1::4]
    G[:, 2] = 1.25
    G[m // 3, ::13] = float("inf")
    G[m // 2, 4::17] = float("-inf")
    G[1, 6::19] = float("nan")
    G[: m // 2 + 2, 8] = float("nan")
    G[: m // 2 + 2, 9] = float("inf")
    G[: m // 2, 10] = float("-inf")
    G[m // 2:, 10] = float("inf")
    med = B.zeno_median(rows_to_gpu(B, G, row_align)).cpu().numpy()
    ref = O.median(G.numpy()).astype(np.float32)
    assert np.array_equal(np.isnan(med), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(med[ok], ref[ok])


def test_median_with_nonfinite_entries(B):
    m, d = 6, 200
    G = _rand_G(m, d, 9)
    G[0, ::3] = float("nan")
    G[1, ::5] = float("inf")
    G[2, ::7] = float("-inf")
    G[3, ::2] = float("nan")
    G[4, 1::2] = -0.0
    med = B.zeno_median(G.cuda()).cpu().numpy()
    ref = O.median(G.numpy()).astype(np.float32)
    assert np.array_equal(np.isnan(med), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(med[ok], ref[ok])


def test_error_codes(B):
    G = torch.zeros(4, 8, device="cuda")
    s = torch.zeros(4, device="cuda")
    for bad_b in (-1, 4, 9):
        with pytest.raises(B.ZenoError) as e:
            B.zeno_aggregate(G, s, bad_b, want_selected=False)
        assert e.value.status == 1
    big = torch.zeros(1025, 8, device="cuda")     # more candidates than any call accepts
    with pytest.raises(B.ZenoError) as e:
        B.zeno_median(big)
    assert e.value.status == 1
    with pytest.raises(ValueError):
        B.zeno_mean(torch.zeros(4, 8))          # host tensor: no silent CPU path
