"""GPU parity and behaviour of zeno_aggregate_update: Definition 3 plus the server's SGD
step of Algorithm 1 in one pass (x_next = x - gamma * Zeno_b(G))."""
import numpy as np
import pytest
import torch

from oracle import zeno_oracle as O
from paper_1805_10032_amd import workloads as WL
from tests._util import npy, rows_to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("m,d,b,row_align", [(1, 7, 0, 1), (5, 4, 2, 1), (8, 1001, 3, 1), (20, 7850, 8, 32),
                                             (33, 40000, 11, 32), (64, 300007, 16, 1)])
def test_update_bit_exact(B, m, d, b, row_align):
    """x_next and the aggregate against the oracle, bit for bit (the kernel sums the chosen rows
    in ascending order in float64 and takes the step from the unrounded average, as the oracle does);
    both outputs, x_next only, and in place."""
    g = torch.Generator().manual_seed(1000 * m + b)
    G = torch.randn(m, d, generator=g) * torch.rand(m, 1, generator=g) * 10
    x = torch.randn(d, generator=g)
    scores = torch.randn(m, generator=g)
    gamma = float(np.float32(0.0371))
    ref_x, ref_sel = O.zeno_update(npy(x), npy(G), npy(scores), b, gamma)
    ref_out, _ = O.zeno_aggregate(npy(G), npy(scores), b)
    Gd, xd, sd = rows_to_gpu(B, G, row_align), x.cuda(), scores.cuda()
    x_next, out, sel = B.zeno_aggregate_update(Gd, sd, b, gamma, xd)
    assert np.array_equal(npy(sel), ref_sel)
    assert np.array_equal(npy(x_next), ref_x.astype(np.float32))
    assert np.array_equal(npy(out), ref_out.astype(np.float32))
    assert np.array_equal(npy(xd), npy(x))                                   # x itself untouched
    x_only, none_out, _ = B.zeno_aggregate_update(Gd, sd, b, gamma, xd, want_out=False, want_selected=False)
    assert none_out is None and np.array_equal(npy(x_only), ref_x.astype(np.float32))
    x_inplace = xd.clone()
    B.zeno_aggregate_update(Gd, sd, b, gamma, x_inplace, x_next=x_inplace, want_out=False)
    assert np.array_equal(npy(x_inplace), ref_x.astype(np.float32))


def test_update_error_codes(B):
    G, s, x = torch.zeros(4, 8, device="cuda"), torch.zeros(4, device="cuda"), torch.zeros(8, device="cuda")
    for bad in (float("nan"), -0.1, float("inf")):
        with pytest.raises(B.ZenoError) as e:
            B.zeno_aggregate_update(G, s, 1, bad, x)
        assert e.value.status == 1
    with pytest.raises(ValueError):
        B.zeno_aggregate_update(G, s, 1, 0.1, torch.zeros(9, device="cuda"))


def _teacher_task(seed, dims, n, dev):
    g = torch.Generator().manual_seed(seed)
    teacher = WL.init_params(dims, True, g, torch.device("cpu"), "he")
    feats = torch.randn(n, dims[0], generator=g)
    layers = WL._views(teacher, dims, True)
    h = feats
    for l, (W, bias) in enumerate(layers):
        h = torch.nn.functional.linear(h, W, bias)
        if l + 1 < len(layers):
            h = torch.relu(h)
    return feats.to(dev), h.argmax(1).to(torch.int32).to(dev)


@pytest.mark.timeout(600)
def test_training_loop_zeno_descends_where_mean_and_median_ascend(B):
    """Algorithm 1 end to end on one GPU with every server-side step in the HIP library:
    m = 20 workers, q = 12 of them (a majority) send -4 x their gradient (sign-flipping,
    Section 6.4), the server scores with n_r = 32 fresh samples, keeps m-b = 8 and steps.
    Zeno's training loss falls (3.14 -> 1.49 in the oracle's run of this recipe); the same loop with the Mean or the Median rule rises
    (Section 6.4: Zeno tolerates q > m/2, majority-based rules cannot).  The workers' gradients are
    input generation (autograd); teacher-labelled synthetic data stands in for CIFAR-10."""
    dev = torch.device("cuda")
    dims, m, q, b, n_r, gamma, rho, T = [48, 64, 10], 20, 12, 12, 32, 0.1, 5e-4, 80
    feats, labels = _teacher_task(7, dims, 8192, dev)
    mdl = B.ZenoModel(dims, True, "softmax_ce", "fp32")
    d = mdl.num_params
    gen = torch.Generator(device=dev).manual_seed(3)

    def full_loss(x):
        return float(torch.nn.functional.cross_entropy(
            _forward(x), labels.long()))

    def _forward(x):
        h = feats
        layers = WL._views(x, dims, True)
        for l, (W, bias) in enumerate(layers):
            h = torch.nn.functional.linear(h, W, bias)
            if l + 1 < len(layers):
                h = torch.relu(h)
        return h

    def candidates(x, G):
        faulty = set(torch.randperm(m, generator=gen, device=dev)[:q].tolist())
        for i in range(m):
            idx = torch.randint(0, feats.shape[0], (32,), generator=gen, device=dev)
            gi = WL.minibatch_gradient(x, dims, True, "softmax_ce", feats[idx], labels[idx])
            G[i] = -4.0 * gi if i in faulty else gi
        return faulty

    x0 = WL.init_params(dims, True, torch.Generator().manual_seed(1), torch.device("cpu"), "he").to(dev)
    start = full_loss(x0)
    final = {}
    for rule in ("zeno", "mean", "median"):
        x = x0.clone()
        G = B.alloc_candidates(m, d, dev)
        ws = B.alloc_workspace(mdl, m, n_r, dev)
        kept_faulty = 0
        for t in range(T):
            faulty = candidates(x, G)
            if rule == "zeno":
                idx = torch.randint(0, feats.shape[0], (n_r,), generator=gen, device=dev)
                s = B.zeno_score(mdl, x, G, feats[idx].contiguous(), gamma, rho, labels=labels[idx].contiguous(),
                                 workspace=ws)
                _, _, sel = B.zeno_aggregate_update(G, s, b, gamma, x, x_next=x, want_out=False)
                kept_faulty += len(faulty & set(sel.tolist()))
            else:
                v = B.zeno_mean(G) if rule == "mean" else B.zeno_median(G)
                x = x - gamma * v
        final[rule] = full_loss(x)
        if rule == "zeno":
            # a sign-flipped row is only ever kept when it happens to beat a noisy honest one on the
            # server's batch (about 7 % of the kept rows in the oracle's run of this recipe)
            assert kept_faulty <= 0.15 * T * (m - b), kept_faulty
    print(f"training loss: start {start:.3f}  zeno {final['zeno']:.3f}  mean {final['mean']:.3f}  "
          f"median {final['median']:.3f}")
    assert final["zeno"] < 0.7 * start
    assert not (final["mean"] < start) and not (final["median"] < start)     # risen, or overflowed to inf/NaN


@pytest.mark.timeout(900)
@pytest.mark.parametrize("attack,disjoint", [("bit_flip", False), ("label_flip", False), ("label_flip", True)])
def test_training_loop_under_the_failures_of_section_6(B, attack, disjoint):
    """Algorithm 1 with q = 12 of m = 20 workers failing as Sections 6.3-6.5 describe, every
    server-side rule in the HIP library (Zeno with b = 12, Mean, Median, and Krum with b = 8, the
    largest value Definition 5's condition 2b + 2 < m admits at m = 20 and the paper's own choice).
    What is asserted is what those sections claim and what the oracle's run of this recipe
    shows over several seeds (start 3.14; Zeno 1.46-1.55 i.i.d. and 1.83-1.93 on disjoint data):
      bit flipping            Zeno descends, the three baselines end above where they started;
      label flipping          Zeno descends and ends below Mean and Median;
      label flipping on       Zeno descends and ends below Median and Krum (Mean is within
      disjoint data           noise of Zeno there and is only printed).
    Teacher-labelled synthetic data stands in for CIFAR-10."""
    dev = torch.device("cuda")
    dims, m, q, b, n_r, gamma, rho, T = [48, 64, 10], 20, 12, 12, 32, 0.1, 5e-4, 80
    b_krum = 8
    assert 2 * b_krum + 2 < m
    feats, labels = _teacher_task(7, dims, 8192, dev)
    shards = WL.class_sorted_shards(labels, m) if disjoint else None
    mdl = B.ZenoModel(dims, True, "softmax_ce", "fp32")
    d = mdl.num_params

    def full_loss(x):
        h = feats
        layers = WL._views(x, dims, True)
        for l, (W, bias) in enumerate(layers):
            h = torch.nn.functional.linear(h, W, bias)
            if l + 1 < len(layers):
                h = torch.relu(h)
        return float(torch.nn.functional.cross_entropy(h, labels.long()))

    x0 = WL.init_params(dims, True, torch.Generator().manual_seed(1), torch.device("cpu"), "he").to(dev)
    start = full_loss(x0)
    final = {}
    for rule in ("zeno", "mean", "median", "krum"):
        gen = torch.Generator(device=dev).manual_seed(3)
        x = x0.clone()
        G = B.alloc_candidates(m, d, dev)
        ws = B.alloc_workspace(mdl, m, n_r, dev)
        for t in range(T):
            faulty = torch.randperm(m, generator=gen, device=dev)[:q].tolist()
            WL.worker_gradients(G, x, dims, True, feats, labels, faulty, attack, gen, shards=shards)
            if rule == "zeno":
                idx = torch.randint(0, feats.shape[0], (n_r,), generator=gen, device=dev)
                s = B.zeno_score(mdl, x, G, feats[idx].contiguous(), gamma, rho, labels=labels[idx].contiguous(),
                                 workspace=ws)
                B.zeno_aggregate_update(G, s, b, gamma, x, x_next=x, want_out=False, want_selected=False)
            else:
                v = B.zeno_mean(G) if rule == "mean" else B.zeno_median(G) if rule == "median" else B.zeno_krum(G, b_krum)[0]
                x = x - gamma * v
        final[rule] = full_loss(x)
    print(f"{attack}{' disjoint' if disjoint else ''}: start {start:.3f}  " +
          "  ".join(f"{k} {v:.3f}" for k, v in final.items()))
    assert final["zeno"] < 0.7 * start
    if attack == "bit_flip":
        assert all(not (final[r] < start) for r in ("mean", "median", "krum"))
    elif not disjoint:
        assert final["zeno"] < final["mean"] - 0.1 and final["zeno"] < final["median"] - 0.1
    else:
        assert final["zeno"] < final["median"] - 0.1 and final["zeno"] < final["krum"] - 0.1
