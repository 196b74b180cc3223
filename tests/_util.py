"""Helpers shared by the GPU parity tests: run the HIP path on a workload and
compare it with the CPU oracle under the stated tolerances."""
import numpy as np
import torch

from oracle import zeno_oracle as O

# Score tolerance (relative): fp32 forward 1e-5, bf16 forward 1e-2.  The error is
# measured against the two quantities the score is the difference of once f_r(x)
# is shared: |f_r(x) - f_r(x - gamma u)| + rho ||u||^2.  This scale is never
# larger than |f_r(x)| + |f_r(x - gamma u)| + rho ||u||^2 and equals |score|
# whenever the descent and the penalty have the same sign.
SCORE_TOL = {"fp32": 1e-5, "bf16": 1e-2}
AGG_TOL = 1e-6


def npy(t):
    return None if t is None else t.detach().cpu().numpy()


def oracle_terms(w, rows=None):
    """(reference scores, scale) for all rows or the listed ones.  The reference is
    the float64 oracle for fp32-forward workloads and the oracle's bf16-operand
    variant (same definition, operands rounded as the bf16 mode states) for
    bf16-forward workloads; the scale always comes from the float64 oracle."""
    s_exact, scale = exact_terms(w, rows)
    if w.fwd == "bf16":
        s_ref = O.scores_bf16(npy(w.x), npy(w.G), w.gamma, w.rho, w.dims, w.has_bias, w.loss,
                              npy(w.features), npy(w.labels), npy(w.targets), rows=rows)
        return s_ref, scale
    return s_exact, scale


def exact_terms(w, rows=None, with_losses=False):
    """(scores, scale) from the float64 oracle; with_losses: also |f_r(x)| + |f_r(x - gamma u)| per row."""
    x = npy(w.x).astype(np.float64)
    args = (w.dims, w.has_bias, w.loss, npy(w.features), npy(w.labels), npy(w.targets))
    f0 = O.f_r(x, *args)
    idx = list(range(w.m)) if rows is None else list(rows)
    s, scale, mag = np.empty(len(idx)), np.empty(len(idx)), np.empty(len(idx))
    for n, i in enumerate(idx):
        u = npy(w.G[i]).astype(np.float64)
        with np.errstate(invalid="ignore", over="ignore"):
            fi = O.f_r(x - w.gamma * u, *args)
            pen = w.rho * float(u @ u)
            s[n] = f0 - fi - pen
            scale[n] = abs(f0 - fi) + pen
            mag[n] = abs(f0) + abs(fi)
    if with_losses:
        return s, scale, mag
    return s, scale


def rows_to_gpu(B, G, row_align=1, device="cuda"):
    """Copy of the candidate matrix on the GPU whose rows are row_align floats aligned
    (1: densely packed, whatever alignment that gives)."""
    if row_align <= 1:
        return G.contiguous().to(device)
    out = B.alloc_candidates(G.shape[0], G.shape[1], torch.device(device), row_align)
    out.copy_(G)
    return out


def gpu_scores(B, w, device="cuda", row_align=1):
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    dev = torch.device(device)
    lab = None if w.labels is None else w.labels.to(dev)
    tgt = None if w.targets is None else w.targets.to(dev)
    s = B.zeno_score(mdl, w.x.to(dev), rows_to_gpu(B, w.G, row_align, dev), w.features.to(dev), w.gamma, w.rho,
                     labels=lab, targets=tgt)
    torch.cuda.synchronize()
    return s


def score_error(s_gpu, s_ref, scale):
    s_gpu = np.asarray(s_gpu, dtype=np.float64)
    with np.errstate(invalid="ignore", divide="ignore"):
        err = np.abs(s_gpu - s_ref) / scale
    both_nan = np.isnan(s_gpu) & np.isnan(s_ref)
    same_inf = np.isinf(s_ref) & (s_gpu == s_ref)
    err[both_nan | same_inf] = 0.0
    err[(scale == 0) & (s_gpu == s_ref)] = 0.0
    return err


def check_selection(sel_gpu, s_ref, b, tol, scale=None):
    """Definition 3 against reference scores s_ref: exact set equality when the reference's gap at
    the cut exceeds the tolerance; otherwise every chosen row must lie within the tolerance of the
    cut.  The tolerance is relative (tol x scale[i], the error scale of each row's score) when
    `scale` is given, so that one huge-penalty row elsewhere cannot slacken the rule at a cut between
    two small-scale rows; without `scale`, tol is absolute."""
    m = len(s_ref)
    ref_sel = O.select(s_ref, b)
    sel_gpu = np.asarray(sel_gpu, dtype=np.int64)
    assert len(sel_gpu) == m - b and np.all(np.diff(sel_gpu) > 0)
    if b == 0:
        assert np.array_equal(sel_gpu, ref_sel)
        return "exact"
    key = np.where(np.isnan(s_ref), -np.inf, np.asarray(s_ref, dtype=np.float64))
    order = sorted(range(m), key=lambda i: (-key[i], i))
    i_in, i_out = order[m - b - 1], order[m - b]          # last row kept, first row trimmed
    lo_in, hi_out = key[i_in], key[i_out]
    if scale is None:
        tol_abs = np.full(m, float(tol))
    else:
        sc = np.asarray(scale, dtype=np.float64)
        tol_abs = np.where(np.isfinite(sc), tol * sc, 0.0)
    # both scores may be off by their own tolerance
    if lo_in - hi_out > tol_abs[i_in] + tol_abs[i_out]:
        assert np.array_equal(sel_gpu, ref_sel), (sel_gpu, ref_sel)
        return "exact"
    chosen = np.zeros(m, dtype=bool)
    chosen[sel_gpu] = True
    slack = tol_abs + max(tol_abs[i_in], tol_abs[i_out])
    assert np.all(key[chosen] >= hi_out - slack[chosen]) and np.all(key[~chosen] <= lo_in + slack[~chosen])
    return "near-tie"
