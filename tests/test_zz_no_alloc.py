"""zeno_score_static (the entry point that allocates nothing: scratch in a static device array)
against zeno_score, through the C ABI, on two calls in a row, the second with a smaller input; the
array keeps the first call's contents, which the second must not depend on."""
import numpy as np
import pytest
import torch

from paper_1805_10032_amd import workloads as WL
from tests._util import SCORE_TOL, npy, oracle_terms, score_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


def _both(B, w):
    dev = torch.device("cuda", 0)
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    assert 0 < mdl.workspace_bytes(w.m, w.n_r) <= B.STATIC_SCRATCH_BYTES
    x, G, F = w.x.to(dev), w.G.contiguous().to(dev), w.features.to(dev)
    lab = None if w.labels is None else w.labels.to(dev)
    tgt = None if w.targets is None else w.targets.to(dev)
    out = torch.full((w.m,), float("nan"), device=dev)
    n_alloc = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    B.zeno_score_static(mdl, x, G, F, w.gamma, w.rho, labels=lab, targets=tgt, scores=out)
    torch.cuda.synchronize()
    # nothing was requested from torch's allocator either (the library itself contains no call that
    # allocates device memory: tests/test_library_cpu.py scans its sources for them)
    assert torch.cuda.memory_stats(dev)["allocation.all.allocated"] == n_alloc
    ref = B.zeno_score(mdl, x, G, F, w.gamma, w.rho, labels=lab, targets=tgt)
    torch.cuda.synchronize()
    return npy(out), npy(ref)


def test_static_scratch_matches_workspace_entry_point_twice(B):
    big = WL.make_config(3)                                    # 3072 -> 512 -> 10, m = 20, fp32 (about 4 MB of scratch)
    small = WL.make_mlp_workload("small", 71, [130, 67, 5], 5, 1, 9, 0.1, 1e-3, "bf16", n_flip=1, n_noise=1, noise_std=3.0)
    for w in (big, small, WL.make_config(1)):                  # large first, then smaller inputs on the same array
        got, ref = _both(B, w)
        assert np.array_equal(got, ref), w.name                # same kernels, same order: bit for bit
        s_ref, scale = oracle_terms(w)
        assert np.all(score_error(got, s_ref, scale) <= SCORE_TOL[w.fwd]), w.name


def test_static_scratch_rejects_what_does_not_fit(B):
    mdl = B.ZenoModel([3072, 2048, 2048, 2048, 10], True, "softmax_ce", "bf16")
    assert mdl.workspace_bytes(100, 64) > B.STATIC_SCRATCH_BYTES
    lib = B.load_library()
    import ctypes
    batch = B._Batch()
    batch.n_r = 64
    one = torch.zeros(64, device="cuda")
    batch.features = one.data_ptr()
    batch.labels = torch.zeros(64, dtype=torch.int32, device="cuda").data_ptr()
    # sizes are checked on the host before anything is read: the pointers only have to be non-NULL and aligned
    st = lib.zeno_score_static(mdl._h, one.data_ptr(), one.data_ptr(), mdl.num_params, 100, ctypes.byref(batch),
                               0.05, 1e-3, one.data_ptr(), None)
    assert st == 2
    small = WL.make_config(1)
    m1 = B.ZenoModel(small.dims, small.has_bias, small.loss, small.fwd)
    with pytest.raises(B.ZenoError) as e:
        B.zeno_score_static(m1, small.x.cuda(), small.G.cuda(), small.features.cuda(), float("nan"), 1e-3,
                            targets=small.targets.cuda())
    assert e.value.status == 1
