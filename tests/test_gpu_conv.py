"""GPU parity of zeno_score with a convolutional f_r (Section 6.1's model class on synthetic shapes)
against the float64 CPU oracle, through the C ABI: every candidate's score at the fp32 tolerance,
the selection against the oracle's scores, the aggregate."""
import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL
from tests._util import AGG_TOL, SCORE_TOL, check_selection, npy, score_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


def _gpu_scores(B, w, static=False):
    dev = torch.device("cuda", 0)
    mdl = B.ZenoCnnModel(w.desc, w.loss)
    assert mdl.num_params == w.d == O.cnn_num_params(w.desc)
    lab = None if w.labels is None else w.labels.to(dev)
    tgt = None if w.targets is None else w.targets.to(dev)
    fn = B.zeno_score_static if static else B.zeno_score
    s = fn(mdl, w.x.to(dev), w.G.contiguous().to(dev), w.features.to(dev), w.gamma, w.rho, labels=lab, targets=tgt)
    torch.cuda.synchronize()
    return s


def _check(B, w, tol=SCORE_TOL["fp32"]):
    s_gpu = _gpu_scores(B, w)
    s_ref, scale = O.cnn_scores(npy(w.x), npy(w.G), w.gamma, w.rho, w.desc, w.loss, npy(w.features), npy(w.labels),
                                npy(w.targets))
    err = score_error(npy(s_gpu), s_ref, scale)
    assert np.all(err <= tol), (w.name, float(np.nanmax(err)), int(np.nanargmax(err)))
    G = w.G.contiguous().cuda()
    out, sel = B.zeno_aggregate(G, s_gpu, w.b)
    torch.cuda.synchronize()
    check_selection(npy(sel), s_ref, w.b, tol, scale)
    ref, _ = O.zeno_aggregate(npy(w.G), npy(s_gpu), w.b)
    assert np.linalg.norm(npy(out).astype(np.float64) - ref) <= AGG_TOL * np.linalg.norm(ref)
    return err


CASES = [
    # desc, m, b, n_r
    (dict(in_h=6, in_w=5, in_c=2, conv_c=[4, 3], conv_stride=[1, 2], fc_out=3, has_bias=True), 5, 1, 6),
    (dict(in_h=8, in_w=8, in_c=3, conv_c=[8, 8, 16, 16], conv_stride=[1, 2, 1, 2], fc_out=10, has_bias=True), 9, 3, 4),
    (dict(in_h=7, in_w=9, in_c=1, conv_c=[33], conv_stride=[1], fc_out=5, has_bias=False), 4, 1, 3),          # one convolution, 33 channels
    (dict(in_h=5, in_w=5, in_c=3, conv_c=[5, 7, 9], conv_stride=[2, 1, 2], fc_out=4, has_bias=True), 6, 2, 1),   # one sample, odd widths
    (dict(in_h=12, in_w=12, in_c=3, conv_c=[16, 40], conv_stride=[1, 1], fc_out=10, has_bias=True), 8, 2, 33),  # two sample blocks, two channel tiles
    (dict(in_h=4, in_w=4, in_c=8, conv_c=[8], conv_stride=[1], fc_out=1, has_bias=True), 5, 1, 7),              # squared loss
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_cnn_small_shapes(B, case):
    desc, m, b, n_r = CASES[case]
    loss = "squared" if desc["fc_out"] == 1 else "softmax_ce"
    q = min(2, m - 1)
    w = WL.make_cnn_workload(f"cnn{case}", 30 + case, desc, m, b, n_r, 0.1, 1e-3, seed=case, loss=loss,
                             n_flip=min(1, q), n_noise=q - min(1, q), noise_std=0.5)
    _check(B, w)


def test_cnn_paper_shaped(B):
    """The shape of the paper's experiments (Section 6: 32 x 32 x 3 images, four convolutions and one fully
    connected layer, 10 classes, m = 20 workers of which q = 8 fail, n_r = 4, gamma = 0.1, rho = 5e-4); the
    widths 32-32-64-64 and the strides are this test's choice.  Sign-flipped rows (-4 x the honest mean)."""
    desc = dict(in_h=32, in_w=32, in_c=3, conv_c=[32, 32, 64, 64], conv_stride=[1, 2, 1, 2], fc_out=10, has_bias=True)
    w = WL.make_cnn_workload("cnn_paper", 37, desc, 20, 8, 4, 0.1, 5e-4, n_flip=8, worker_batch=16)
    _check(B, w)


def test_cnn_on_the_static_scratch_array(B):
    """zeno_score_static serves convolutional models as well (same kernels, bit for bit) while their scratch fits."""
    desc, m, b, n_r = CASES[1]
    w = WL.make_cnn_workload("cnn_static", 39, desc, m, b, n_r, 0.1, 1e-3, n_flip=1)
    assert torch.equal(_gpu_scores(B, w, static=True), _gpu_scores(B, w))


def test_cnn_nonfinite_rows_and_workspace_contents(B):
    desc = dict(in_h=6, in_w=6, in_c=2, conv_c=[6, 6], conv_stride=[1, 2], fc_out=3, has_bias=True)
    w = WL.make_cnn_workload("cnn_nf", 38, desc, 7, 2, 5, 0.1, 1e-3)
    w.G[1, 3] = float("nan")            # a kernel entry of the first convolution
    w.G[4, -1] = float("inf")           # the last bias of the fully connected layer
    dev = torch.device("cuda", 0)
    mdl = B.ZenoCnnModel(w.desc, w.loss)
    args = (mdl, w.x.to(dev), w.G.contiguous().to(dev), w.features.to(dev), w.gamma, w.rho)
    out = []
    for fill in (0.0, float("nan")):    # the scratch memory is written before it is read
        ws = B.alloc_workspace(mdl, w.m, w.n_r, dev)
        ws.view(torch.float32).fill_(fill)
        out.append(npy(B.zeno_score(*args, labels=w.labels.to(dev), workspace=ws)))
    assert np.array_equal(out[0], out[1], equal_nan=True)
    s = out[0].astype(np.float64)
    for i in (1, 4):
        assert np.isnan(s[i]) or s[i] == -np.inf
    ok = [i for i in range(w.m) if i not in (1, 4)]
    s_ref, scale = O.cnn_scores(npy(w.x), npy(w.G), w.gamma, w.rho, w.desc, w.loss, npy(w.features), npy(w.labels), rows=ok)
    assert np.all(score_error(s[ok], s_ref, scale) <= SCORE_TOL["fp32"])


def test_cnn_error_codes(B):
    with pytest.raises(B.ZenoError):
        B.ZenoCnnModel(dict(in_h=4, in_w=4, in_c=1, conv_c=[4], conv_stride=[3], fc_out=2, has_bias=True))
    with pytest.raises(B.ZenoError):
        B.ZenoCnnModel(dict(in_h=4, in_w=4, in_c=1, conv_c=[4], conv_stride=[1], fc_out=2, has_bias=True), "squared")
    mdl = B.ZenoCnnModel(dict(in_h=4, in_w=4, in_c=1, conv_c=[4], conv_stride=[1], fc_out=2, has_bias=True))
    assert mdl.workspace_bytes(4, 129) == 0 and mdl.workspace_bytes(4, 128) > 0
    assert mdl.plan_check(4, 4) == 2
