"""Parity at the full sizes of the two bandwidth-bound workloads (4 and 5), in the
launch configuration bench.py times.  The inputs are generated on the GPU with the
same seeded recipe; the CPU oracle gets copies of exactly those tensors.  Scores are
checked on sampled candidates (one of each kind), the selection on all m scores,
and the three aggregators on sampled coordinates, which the oracle computes one
by one from the same rows."""
import sys
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


@pytest.mark.timeout(1500)
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
    s_gpu = B.zeno_score(mdl, w.x, w.G, w.features, w.gamma, w.rho, labels=w.labels)
    out, sel = B.zeno_aggregate(w.G, s_gpu, w.b)
    mean = B.zeno_mean(w.G)
    med = B.zeno_median(w.G)
    torch.cuda.synchronize()
    s = npy(s_gpu).astype(np.float64)
    _say(capsys, "HIP path done")

    # ---- scores of sampled candidates against the oracle (contract variant and float64 definition)
    rows = _sample_rows(w)
    x, feats, labels = npy(w.x), npy(w.features), npy(w.labels)
    Gs = np.stack([npy(w.G[i]) for i in rows])
    args = (w.gamma, w.rho, w.dims, w.has_bias, w.loss, feats, labels)
    t0 = time.time()
    s_contract = O.scores_bf16(x, Gs, *args)
    _say(capsys, f"oracle (bf16 contract) on rows {rows}: {time.time() - t0:.1f}s")
    t0 = time.time()
    f0 = O.f_r(x.astype(np.float64), w.dims, w.has_bias, w.loss, feats, labels)
    s_exact, scale = np.empty(len(rows)), np.empty(len(rows))
    for n in range(len(rows)):
        u = Gs[n].astype(np.float64)
        fi = O.f_r(x.astype(np.float64) - w.gamma * u, w.dims, w.has_bias, w.loss, feats, labels)
        pen = w.rho * float(u @ u)
        s_exact[n], scale[n] = f0 - fi - pen, abs(f0 - fi) + pen
    _say(capsys, f"oracle (float64 definition): {time.time() - t0:.1f}s")
    err_c = score_error(s[rows], s_contract, scale)
    err_e = score_error(s[rows], s_exact, scale)
    _say(capsys, f"score error vs contract {err_c.max():.2e}, vs float64 definition {err_e.max():.2e}")
    assert np.all(err_c <= SCORE_TOL["bf16"]), err_c
    assert np.all(err_e <= SCORE_TOL["bf16"]), err_e     # large layers: rounding errors average out

    # ---- selection: integer work on the GPU's own fp32 scores must match the oracle bit for bit,
    #      and agree with the sampled oracle scores where those decide
    sel_np = npy(sel).astype(np.int64)
    assert np.array_equal(sel_np, O.select(npy(s_gpu), w.b))
    check_selection(sel_np, s, w.b, 0.0)
    noise_or_flip_excluded = [i for i in w.faulty if i not in set(sel_np.tolist())]
    _say(capsys, f"{len(noise_or_flip_excluded)} of {len(w.faulty)} faulty rows trimmed (reported, not asserted)")

    # ---- aggregators on sampled coordinates
    g = torch.Generator().manual_seed(cfg)
    idx = torch.cat([torch.arange(0, 64), torch.arange(w.d - 64, w.d),
                     torch.randint(0, w.d, (20000,), generator=g)]).to(dev)
    cols = npy(w.G[:, idx])                       # [m, n_idx]
    ref_sel = np.zeros(cols.shape[1])
    for i in sel_np:
        ref_sel += cols[int(i)].astype(np.float64)
    ref_sel /= len(sel_np)
    assert np.array_equal(npy(out[idx]), ref_sel.astype(np.float32))
    # the same pass with the server's SGD step (Algorithm 1): x_next = x - gamma * average
    x_next, _, _ = B.zeno_aggregate_update(w.G, s_gpu, w.b, w.gamma, w.x, want_out=False, want_selected=False)
    ref_next = O.sgd_update(npy(w.x[idx]), ref_sel, float(np.float32(w.gamma)))
    assert np.array_equal(npy(x_next[idx]), ref_next.astype(np.float32))
    assert np.array_equal(npy(mean[idx]), O.mean(cols).astype(np.float32))
    assert np.array_equal(npy(med[idx]), O.median(cols).astype(np.float32))
    _say(capsys, "aggregate / update / mean / median bit-exact on 20128 sampled coordinates\n")
