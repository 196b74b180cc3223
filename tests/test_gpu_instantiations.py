"""Every instantiation of the streaming layer kernel that a caller can reach at scale is executed
here at sizes the float64 oracle scores in seconds, ALL rows compared: four- and eight-wave
workgroups in fp32 and bf16, with and without the second matrix product, one, two and four
32-sample row blocks, densely packed rows (plain loads, or the shifted column grid where rows are
16-byte aligned) and rows on 128-byte lines (streaming loads), ragged widths, and the pass at x riding in an eight-wave candidate launch.  Which launch
shapes really ran is read back from the library's per-launch records and asserted, so the
coverage cannot silently move when the dispatch heuristics change."""
import numpy as np
import pytest
import torch

from paper_1805_10032_amd import workloads as WL
from tests._util import SCORE_TOL, check_selection, exact_terms, npy, oracle_terms, rows_to_gpu, score_error

pytestmark = pytest.mark.gpu

SEEN = set()     # (fwd, second product, waves, k_split, streaming, row_blocks, merged) of every layer launch
TAILS = set()    # (fwd, second product, streaming, row_blocks) of every launch with a sliced tail


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


_CACHE = {}


def _workload(key, dims, m, b, n_r, fwd, n_flip, n_noise):
    """Workloads and their oracle scores are shared by the row-pitch variants of a case."""
    if key not in _CACHE:
        _CACHE.clear()           # one big case at a time in host memory
        w = WL.make_mlp_workload(f"inst{key}", 60, dims, m, b, n_r, 0.05, 1e-3, fwd, seed=len(dims) + n_r,
                                 n_flip=n_flip, n_noise=n_noise, noise_std=5.0, worker_batch=16)
        s_ref, scale = oracle_terms(w)
        s_exact = exact_terms(w)[0] if fwd == "bf16" else s_ref
        _CACHE[key] = (w, s_ref, s_exact, scale)
    return _CACHE[key]


def _run(B, w, s_ref, s_exact, scale, row_align, offset_floats=0):
    dev = torch.device("cuda", 0)
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    if offset_floats:
        # densely packed rows that start offset_floats past the start of an allocation
        m, d = w.G.shape
        buf = torch.empty(m * d + offset_floats, dtype=torch.float32, device=dev)
        G = buf[offset_floats:].view(m, d)
        G.copy_(w.G)
    else:
        G = rows_to_gpu(B, w.G, row_align, dev)
    B.profile_enable(True)
    try:
        s = B.zeno_score(mdl, w.x.to(dev), G, w.features.to(dev), w.gamma, w.rho, labels=w.labels.to(dev))
        torch.cuda.synchronize()
        recs = B.profile_collect(detail=True)
    finally:
        B.profile_enable(False)
    shapes = []
    for r in recs:
        if r["kernel"] in ("layer_base", "layer_cand"):
            shape = (w.fwd, r["second"], r["waves"], r["k_split"], r["streaming"], r["row_blocks"], r["merged"])
            SEEN.add(shape)
            if r["tail_candidates"] > 0:
                TAILS.add((w.fwd, r["second"], r["streaming"], r["row_blocks"]))
            shapes.append((r["kernel"], r["layer"]) + shape[1:] + (r["candidates"], r["tail_candidates"], r["k_slices"]))
    tol = SCORE_TOL[w.fwd]
    err = score_error(npy(s), s_ref, scale)
    assert np.all(err <= tol), (w.name, row_align, float(err.max()), int(err.argmax()), shapes)
    if w.fwd == "bf16":   # every layer is at least 512 wide on its input side: the float64 definition at 2e-2
        err_exact = score_error(npy(s), s_exact, scale)
        print(f"  {w.name}: vs contract {err.max():.2e}, vs float64 definition {err_exact.max():.2e}")
        assert np.all(err_exact <= 2e-2), (w.name, row_align, float(err_exact.max()), shapes)
    out, sel = B.zeno_aggregate(G, s, w.b)
    torch.cuda.synchronize()
    check_selection(npy(sel), s_exact, w.b, tol, scale)
    return shapes


# dims, m, b, n_r: wide layers so that (feature tiles x candidates) reaches 256 workgroups
WIDE = [1024, 2048, 1024, 10]


@pytest.mark.parametrize("row_align", [1, 32])
@pytest.mark.parametrize("n_r", [32, 64, 128])
@pytest.mark.parametrize("fwd", ["fp32", "bf16"])
def test_wide_layers_all_rows(B, fwd, n_r, row_align):
    """2048- and 1024-wide layers with 64 candidates: eight- (or four-) wave workgroups in the first
    layer and in the layer with the second product, a ten-class layer behind them; one, two and
    four row blocks; d mod 4 = 2, so densely packed odd rows are only 8-byte aligned."""
    w, s_ref, s_exact, scale = _workload(("wide", fwd, n_r), WIDE, 64, 20, n_r, fwd, 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, row_align)
    print(f"\n  wide {fwd} n_r={n_r} align={row_align}: {shapes}")
    cand = [s for s in shapes if s[0] == "layer_cand"]
    # streaming loads on line-aligned rows; dense rows (8-byte aligned here) take the shifted column grid in the
    # wide bf16 workgroups and plain loads elsewhere
    for s in cand:
        assert s[5] == (1 if row_align == 32 else 3 if (fwd == "bf16" and s[3] >= 4) else 0), cand
    assert all(s[6] == {32: 1, 64: 2, 128: 4}[n_r] for s in cand)
    assert all(s[3] >= 4 for s in cand if s[1] < 2), cand                       # the wide layers run in wide workgroups


# d mod 4 = 0 and widths that are multiples of 64: densely packed rows are 16-byte aligned and start
# 0, 48, 96, 16, ... bytes past a 128-byte line, the case of the shifted column grid
SHIFTED = [1024, 2048, 1024, 12]


@pytest.mark.parametrize("offset_floats", [0, 4])
@pytest.mark.parametrize("n_r", [32, 64, 128])
def test_dense_rows_on_the_shifted_grid(B, n_r, offset_floats):
    """bf16 forward on a dense G[m x d] whose rows are 16-byte aligned but not line-aligned: the wide layers
    load their weight tiles on a column grid shifted to the lines of each candidate's rows (launch
    records say streaming = 2), all rows compared.  With the whole matrix 16 bytes past the start of
    its allocation the first candidate's rows are shifted too, and the columns in front of its first
    row, which lie before the matrix, must not be read."""
    assert WL.num_params(SHIFTED, True) % 4 == 0 and (4 * WL.num_params(SHIFTED, True)) % 128 not in (0, 64)
    w, s_ref, s_exact, scale = _workload(("shifted", n_r), SHIFTED, 64, 20, n_r, "bf16", 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, 1, offset_floats)
    print(f"\n  shifted grid n_r={n_r} offset={offset_floats}: {shapes}")
    cand = [s for s in shapes if s[0] == "layer_cand" and s[3] >= 4]
    assert cand and all(s[5] == 2 for s in cand), shapes


@pytest.mark.parametrize("offset_floats", [0, 2])
@pytest.mark.parametrize("n_r", [32, 64, 128])
def test_dense_rows_eight_byte_aligned_on_the_shifted_grid(B, n_r, offset_floats):
    """d mod 4 = 2: every other row of a dense G[m x d] is only 8-byte aligned.  The shifted column grid then
    stages a lane's four columns as two pairs, and the tiles at the ends of a row are loaded and masked in
    halves.  With the matrix 8 bytes past the start of its allocation it is the even rows, the first
    candidate's included, that are 8-byte aligned."""
    assert WL.num_params(WIDE, True) % 4 == 2
    w, s_ref, s_exact, scale = _workload(("wide", "bf16", n_r), WIDE, 64, 20, n_r, "bf16", 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, 1, offset_floats)
    print(f"\n  shifted grid, 8-byte rows, n_r={n_r} offset={offset_floats}: {shapes}")
    cand = [s for s in shapes if s[0] == "layer_cand" and s[3] >= 4]
    assert cand and all(s[5] == 3 for s in cand), shapes


ODD_D = [1024, 2048, 1024, 11]


@pytest.mark.parametrize("n_r", [32, 64, 128])
def test_dense_rows_four_byte_aligned(B, n_r):
    """d odd: the rows of a dense G[m x d] are only 4-byte aligned, no column grid lines up with the memory
    lines and the wide bf16 workgroups read them with plain 128-bit loads."""
    assert WL.num_params(ODD_D, True) % 2 == 1
    w, s_ref, s_exact, scale = _workload(("odd", n_r), ODD_D, 64, 20, n_r, "bf16", 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, 1)
    print(f"\n  four-byte aligned rows n_r={n_r}: {shapes}")
    cand = [s for s in shapes if s[0] == "layer_cand" and s[3] >= 4]
    assert cand and all(s[5] == 0 for s in cand), shapes


def test_pass_at_x_rides_in_a_launch_on_the_shifted_grid(B):
    """The merged launch of the test below with dense, 16-byte aligned rows: the pass at x (its own
    parameter vector is line-aligned, shift 0) and the candidates (shifted) share a launch."""
    w, s_ref, s_exact, scale = _workload(("merge8s",), [1024, 2048, 2048, 12], 60, 20, 64, "bf16", 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, 1)
    print(f"\n  merge8 on the shifted grid: {shapes}")
    merged = [s for s in shapes if s[0] == "layer_cand" and s[7] == 1]
    assert any(s[3] == 8 and s[5] == 2 for s in merged), shapes


@pytest.mark.parametrize("row_align", [1, 32])
@pytest.mark.parametrize("fwd", ["fp32", "bf16"])
def test_ragged_widths_in_wide_workgroups(B, fwd, row_align):
    """Input widths that are not multiples of 64 (element-wise guards in the last chunk) and output
    widths that leave the last feature tile of a four- or eight-wave workgroup partly empty."""
    w, s_ref, s_exact, scale = _workload(("ragged", fwd), [1000, 1100, 520, 10], 64, 20, 48, fwd, 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, row_align)
    print(f"\n  ragged {fwd} align={row_align}: {shapes}")
    cand = [s for s in shapes if s[0] == "layer_cand"]
    assert all(s[3] >= 4 for s in cand if s[1] < 2), cand


@pytest.mark.parametrize("fwd", ["bf16", "fp32"])
def test_pass_at_x_rides_in_an_eight_wave_launch(B, fwd):
    """A ten-class output layer behind a 2048-wide hidden layer with m = 60: the candidates' launch of
    the hidden layer has 480 eight-wave workgroups, so the pass at x through the output layer rides in
    it, and all eight waves of its one workgroup store their (mostly empty) tile of W in operand order.
    Those stores must stay inside the slot of that copy: the candidates' D operand lies behind it."""
    w, s_ref, s_exact, scale = _workload(("merge8", fwd), [1024, 2048, 2048, 10], 60, 20, 64, fwd, 12, 8)
    shapes = _run(B, w, s_ref, s_exact, scale, 32)
    print(f"\n  merge8 {fwd}: {shapes}")
    merged = [s for s in shapes if s[0] == "layer_cand" and s[7] == 1]
    assert any(s[3] == 8 for s in merged), shapes


TAIL_DIMS = {10: [1024, 2048, 2048, 10], 12: [1024, 2048, 2048, 12]}


@pytest.mark.parametrize("fwd,n_r,row_align,classes", [
    ("bf16", 64, 32, 10), ("bf16", 128, 32, 10), ("bf16", 32, 32, 10), ("fp32", 32, 32, 10), ("fp32", 32, 1, 10),
    ("fp32", 64, 32, 10), ("fp32", 64, 1, 10),
    ("bf16", 160, 32, 10),     # two passes over G (128 + 32 samples): the second finds the arrival counters at zero
    # dense bf16 rows: the sliced tail on the shifted column grid, 8-byte (d mod 4 = 2) and 16-byte aligned rows
    ("bf16", 32, 1, 10), ("bf16", 64, 1, 10), ("bf16", 128, 1, 10), ("bf16", 32, 1, 12), ("bf16", 64, 1, 12), ("bf16", 128, 1, 12),
    # fp32 with four row blocks: the layer with the second product is single-buffered and keeps its whole tiles
    ("fp32", 128, 32, 10)])
def test_last_round_of_a_launch_in_k_slices(B, fwd, n_r, row_align, classes):
    """36 candidates on 2048-wide layers are 288 eight-wave workgroups: one full round of 256 and a round that
    would be one-eighth full.  The tiles of candidates 32..35 and of the pass at x through the next layer run
    as K slices at the end of the launch (partial accumulators handed over through memory, partial norms in a
    range of slots of their own).  All rows compared; the launch records must name the sliced tail."""
    w, s_ref, s_exact, scale = _workload(("tail", fwd, n_r, classes), TAIL_DIMS[classes], 36, 10, n_r, fwd, 6, 4)
    shapes = _run(B, w, s_ref, s_exact, scale, row_align)
    print(f"\n  sliced tail {fwd} n_r={n_r} align={row_align}: {shapes}")
    passes = (n_r + 127) // 128
    for layer in (0, 1):
        launches = [s for s in shapes if s[0] == "layer_cand" and s[1] == layer]
        assert len(launches) == passes, shapes
        if fwd == "fp32" and n_r > 64 and layer == 1:
            assert all(one[9] == 0 for one in launches), shapes                                    # no tail there
            continue
        for one in launches:
            assert one[3] == 8 and one[7] == 1, shapes                                             # eight waves, merged
            assert one[8:10] == (36, 4) and one[10] >= 2, shapes                                   # tail of 4, sliced
            if fwd == "bf16" and row_align == 1:
                assert one[5] == (3 if classes == 10 else 2), shapes                               # shifted grid
    assert [s[8:10] for s in shapes if s[0] == "layer_cand" and s[1] == 2] == [(36, 0)] * passes, shapes
    # same scores from run to run: the slices are added in slice order whoever arrives last
    dev = torch.device("cuda", 0)
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    G = rows_to_gpu(B, w.G, row_align, dev)
    a = B.zeno_score(mdl, w.x.to(dev), G, w.features.to(dev), w.gamma, w.rho, labels=w.labels.to(dev))
    b = B.zeno_score(mdl, w.x.to(dev), G, w.features.to(dev), w.gamma, w.rho, labels=w.labels.to(dev))
    assert torch.equal(a, b)


@pytest.mark.parametrize("fwd,n_r,row_align", [("bf16", 64, 32), ("bf16", 64, 1), ("fp32", 32, 32)])
def test_sliced_tail_on_a_wide_output_layer(B, fwd, n_r, row_align):
    """A 2048-class output layer with 36 candidates: its launch has a sliced tail but carries no pass at x, and the
    slices' last workgroups write the change of the logits instead of activations.  1100 inputs: the first layer's
    K is ragged (no shifted grid there), the output layer's is not."""
    w, s_ref, s_exact, scale = _workload(("tailout", fwd, n_r), [1100, 2048, 2048], 36, 10, n_r, fwd, 6, 4)
    shapes = _run(B, w, s_ref, s_exact, scale, row_align)
    print(f"\n  sliced tail, wide output layer {fwd} n_r={n_r} align={row_align}: {shapes}")
    out = [s for s in shapes if s[0] == "layer_cand" and s[1] == 1]
    assert len(out) == 1 and out[0][3] == 8 and out[0][7] == 0 and out[0][8:10] == (36, 4) and out[0][10] >= 2, shapes


def test_zz_which_instantiations_ran(B):
    """The cases above, between them, executed every (operand type, second product, workgroup width,
    loads, row blocks) combination that the dispatch can pick for a large model."""
    if not SEEN:
        pytest.skip("runs after the cases of this file")
    missing = []
    for fwd in ("fp32", "bf16"):
        for second in (0, 1):
            for streaming in (0, 1):
                for mb in (1, 2, 4):
                    if not any(s[0] == fwd and s[1] == second and s[2] in (4, 8) and s[4] == streaming and s[5] == mb
                               for s in SEEN):
                        missing.append((fwd, second, "4|8 waves", streaming, mb))
        for waves in (4, 8):
            for second in (0, 1):
                if not any(s[0] == fwd and s[1] == second and s[2] == waves for s in SEEN):
                    missing.append((fwd, second, waves))
        if not any(s[0] == fwd and s[3] > 1 for s in SEEN):
            missing.append((fwd, "k_split"))
    for second in (0, 1):      # the shifted column grid (bf16 only): 16-byte aligned rows (2), 8-byte aligned rows (3)
        for mb in (1, 2, 4):
            for kind in (2, 3):
                if not any(s[0] == "bf16" and s[1] == second and s[2] in (4, 8) and s[4] == kind and s[5] == mb for s in SEEN):
                    missing.append(("bf16", second, "4|8 waves", "shifted grid", kind, mb))
    # sliced tails: every kind of row access, with and without the second product, every number of row blocks that
    # has the instantiation (fp32 with the second product and four row blocks is single-buffered: no tail)
    for fwd, kinds in (("bf16", (0, 1, 2, 3)), ("fp32", (0, 1))):
        for second in (0, 1):
            for kind in kinds:
                if kind == 0 and fwd == "bf16":
                    want = [(fwd, 0, 0, 2)]       # plain loads in bf16: ragged K (first layer of the wide-output case)
                    if second:
                        continue
                else:
                    want = [(fwd, second, kind, mb) for mb in ((1, 2, 4) if fwd == "bf16" else (1, 2))]
                missing += [("tail",) + t for t in want if t not in TAILS]
    if ("fp32", 0, 1, 4) not in TAILS:
        missing.append(("tail", "fp32", 0, 1, 4))
    print("\n  launch shapes seen:", sorted(SEEN))
    print("  sliced tails seen:", sorted(TAILS))
    assert not missing, missing


@pytest.mark.parametrize("fwd,n_r", [("fp32", 200), ("bf16", 300), ("bf16", 64)])
def test_pass_at_x_split_over_workgroups(B, fwd, n_r):
    """A pass at x on its own whose feature tiles are too few to fill the chip splits K over workgroups as well
    as over waves: partial accumulators go through memory and the last workgroup of a tile to arrive adds them.
    Batches of more than 128 samples run it once per pass over G (the arrival counters are cleared every pass);
    scores are compared on all rows and must not change from run to run."""
    w, s_ref, s_exact, scale = _workload(("slices", fwd, n_r), [2048, 320, 1024, 10], 12, 3, n_r, fwd, 2, 1)
    shapes = _run(B, w, s_ref, s_exact, scale, 32)
    print(f"\n  slices {fwd} n_r={n_r}: {shapes}")
    assert any(s[0] == "layer_base" for s in shapes)
    dev = torch.device("cuda", 0)
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    G = rows_to_gpu(B, w.G, 32, dev)
    B.profile_enable(True)
    try:
        a = B.zeno_score(mdl, w.x.to(dev), G, w.features.to(dev), w.gamma, w.rho, labels=w.labels.to(dev))
        torch.cuda.synchronize()
        recs = B.profile_collect(detail=True)
    finally:
        B.profile_enable(False)
    assert max(r["k_slices"] for r in recs if r["kernel"] == "layer_base") > 1, recs
    b = B.zeno_score(mdl, w.x.to(dev), G, w.features.to(dev), w.gamma, w.rho, labels=w.labels.to(dev))
    assert torch.equal(a, b)
