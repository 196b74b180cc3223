"""Parity at the full sizes of the two bandwidth-bound workloads (4 and 5), in the launch
configuration bench.py times, on both row layouts: rows padded to 128-byte lines (streaming loads)
and densely packed G[m x d] (plain loads; workload 4's odd rows are then only 8-byte aligned).
The inputs are generated on the GPU with the seeded recipe; the CPU oracle gets copies of exactly
those tensors.  EVERY candidate is scored by the float64 oracle (Definition 2 as written, x - gamma u
materialised) and the HIP scores are held to the bf16-forward tolerance against it; the selection
(Definition 3) is checked against the ORACLE's scores; a few rows are also compared with the
oracle's bf16-operand variant as a tighter diagnostic; the aggregators are compared bit for bit on
sampled coordinates, which the oracle computes one by one from the same rows."""
import time

import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL
from tests._util import SCORE_TOL, check_selection, npy, score_error

pytestmark = pytest.mark.gpu


def _say(capsys, msg):
    with capsys.disabled():
        print(f"\n  [full-size] {msg}", end="", flush=True)


def _sample_rows(w):
    faulty = set(w.faulty)
    honest = [i for i in range(w.m) if i not in faulty]
    rows = [honest[0], honest[len(honest) // 2], honest[-1]]
    # one faulty row of each kind (identical flipped rows share a value; noise rows differ)
    seen = []
    for i in w.faulty:
        kind = float(w.G[i, 0])
        if all(abs(kind - k) > 0 for k in seen):
            seen.append(kind)
            rows.append(i)
        if len(seen) >= 2:
            break
    return sorted(set(rows))


@pytest.mark.timeout(2400)
@pytest.mark.parametrize("cfg", [4, 5])
def test_full_size_parity(cfg, capsys):
    from paper_1805_10032_amd import binding as B
    B.load_library()
    dev = torch.device("cuda", 0)
    t0 = time.time()
    w = WL.make_config(cfg, device=dev, row_align=32)     # the row pitch bench.py times
    torch.cuda.synchronize()
    _say(capsys, f"config {cfg}: d={w.d} m={w.m} generated in {time.time() - t0:.1f}s")
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    tol = SCORE_TOL["bf16"]

    # ---- the float64 oracle on all m candidates, row by row from the device tensor
    x, feats, labels = npy(w.x), npy(w.features), npy(w.labels)
    x64 = x.astype(np.float64)
    t0 = time.time()
    f0 = O.f_r(x64, w.dims, w.has_bias, w.loss, feats, labels)
    s_exact, scale = np.empty(w.m), np.empty(w.m)
    for i in range(w.m):
        u = npy(w.G[i]).astype(np.float64)
        fi = O.f_r(x64 - w.gamma * u, w.dims, w.has_bias, w.loss, feats, labels)
        pen = w.rho * float(u @ u)
        s_exact[i], scale[i] = f0 - fi - pen, abs(f0 - fi) + pen
        if i % 16 == 15:
            _say(capsys, f"oracle (float64 definition): {i + 1} of {w.m} rows, {time.time() - t0:.0f}s")
    ref_sel = O.select(s_exact, w.b)
    assert set(ref_sel.tolist()).isdisjoint(set(w.faulty))          # the oracle itself trims every faulty row

    # ---- contract variant on sampled rows (diagnostic: same rounding points as the bf16 mode states)
    rows = _sample_rows(w)
    Gs = np.stack([npy(w.G[i]) for i in rows])
    t0 = time.time()
    s_contract = O.scores_bf16(x, Gs, w.gamma, w.rho, w.dims, w.has_bias, w.loss, feats, labels)
    _say(capsys, f"oracle (bf16 contract) on rows {rows}: {time.time() - t0:.1f}s")
    del Gs

    g = torch.Generator().manual_seed(cfg)
    idx = torch.cat([torch.arange(0, 64), torch.arange(w.d - 64, w.d),
                     torch.randint(0, w.d, (20000,), generator=g)]).to(dev)
    cols = npy(w.G[:, idx])                       # [m, n_idx]

    for layout in ("padded", "dense"):
        if layout == "padded":
            G = w.G
        else:
            G = w.G.contiguous()                  # G[m x d], ld = d
            assert G.stride(0) == w.d
        s_gpu = B.zeno_score(mdl, w.x, G, w.features, w.gamma, w.rho, labels=w.labels)
        out, sel = B.zeno_aggregate(G, s_gpu, w.b)
        mean = B.zeno_mean(G)
        med = B.zeno_median(G)
        torch.cuda.synchronize()
        s = npy(s_gpu).astype(np.float64)
        err_e = score_error(s, s_exact, scale)
        err_c = score_error(s[rows], s_contract, scale[rows])
        _say(capsys, f"{layout} rows (pitch {G.stride(0)}): score error vs float64 definition on {w.m} of {w.m} rows "
                     f"max {err_e.max():.2e} (row {int(err_e.argmax())}), median {np.median(err_e):.2e}; "
                     f"vs contract on {len(rows)} rows {err_c.max():.2e}")
        assert np.all(err_e <= tol), (layout, err_e)
        assert np.all(err_c <= tol), (layout, err_c)

        # ---- selection against the oracle's scores (Definition 3), tolerance from the rows at the cut
        sel_np = npy(sel).astype(np.int64)
        how = check_selection(sel_np, s_exact, w.b, tol, scale)
        assert set(sel_np.tolist()).isdisjoint(set(w.faulty))
        # and, as integer work, bit for bit from the GPU's own fp32 scores
        assert np.array_equal(sel_np, O.select(npy(s_gpu), w.b))
        _say(capsys, f"{layout}: selection vs oracle scores: {how}; {len(w.faulty)} of {len(w.faulty)} faulty rows trimmed")

        # ---- aggregators on sampled coordinates
        ref_sel_avg = np.zeros(cols.shape[1])
        for i in sel_np:
            ref_sel_avg += cols[int(i)].astype(np.float64)
        ref_sel_avg /= len(sel_np)
        assert np.array_equal(npy(out[idx]), ref_sel_avg.astype(np.float32))
        # the same pass with the server's SGD step (Algorithm 1): x_next = x - gamma * average
        x_next, _, _ = B.zeno_aggregate_update(G, s_gpu, w.b, w.gamma, w.x, want_out=False, want_selected=False)
        ref_next = O.sgd_update(npy(w.x[idx]), ref_sel_avg, float(np.float32(w.gamma)))
        assert np.array_equal(npy(x_next[idx]), ref_next.astype(np.float32))
        assert np.array_equal(npy(mean[idx]), O.mean(cols).astype(np.float32))
        assert np.array_equal(npy(med[idx]), O.median(cols).astype(np.float32))
        _say(capsys, f"{layout}: aggregate / update / mean / median bit-exact on 20128 sampled coordinates")
        del G, s_gpu, out, sel, mean, med, x_next
    _say(capsys, "done\n")
