"""Seeded synthetic inputs for the Zeno aggregation step.

This module only *makes inputs*: parameters x, the server's batch, and the m
candidate gradients (honest minibatch gradients plus injected faults).  It holds
none of the method's arithmetic (no score, no selection, no aggregation) and is
the one piece of code that both the CPU oracle's tests and the HIP path's tests
consume.  Honest gradients come from torch autograd, which is used here as a
library and nowhere on the hot path.

The five numbered workloads follow the shapes of the paper's experiments
(Section 6: m = 20 workers, q = 8 faulty, 32x32x3 inputs, 10 classes,
gamma in {0.1, 0.05}, rho = 5e-4) scaled up to models whose candidate matrix
no longer fits in cache.  They stand in for CIFAR-10, which is not used.

Fault injectors (Section 3, Definition 1; Section 6.4): a large negative multiple
of the honest mean copied over all faulty rows ("sign flip"), and independent
large-variance Gaussian rows ("noise").  worker_gradients() produces one
iteration's candidates of a training loop under the failures of Section 6:
label flipping (6.3), bit flipping (6.4), a scaled sign flip, and workers that
draw from disjoint shards of the data (6.5).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import torch


@dataclass
class Workload:
    name: str
    dims: list            # [d_in, ..., d_out]
    has_bias: bool
    loss: str             # "squared" | "softmax_ce"
    fwd: str              # "fp32" | "bf16" (operand precision of the forward passes)
    m: int
    b: int
    n_r: int
    gamma: float
    rho: float
    x: torch.Tensor                    # [d] fp32
    G: torch.Tensor                    # [m, d] fp32
    features: torch.Tensor             # [n_r, d_in] fp32
    labels: Optional[torch.Tensor]     # [n_r] int32 (softmax_ce)
    targets: Optional[torch.Tensor]    # [n_r] fp32 (squared)
    faulty: list = field(default_factory=list)   # indices of injected rows
    desc: Optional[dict] = None        # convolutional models: in_h, in_w, in_c, conv_c, conv_stride, fc_out, has_bias

    @property
    def d(self) -> int:
        return int(self.x.numel())


def num_params(dims, has_bias) -> int:
    return sum(dims[l] * dims[l - 1] + (dims[l] if has_bias else 0) for l in range(1, len(dims)))


def _gen(seed, cfg, stream, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + int(cfg) * 1009 + int(stream))
    return g


def _randn(shape, gen, device, std=1.0):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * std


def _rand(shape, gen, device):
    return torch.rand(shape, generator=gen, device=device, dtype=torch.float32)


def _views(p, dims, has_bias):
    out, off = [], 0
    for l in range(1, len(dims)):
        n_out, n_in = dims[l], dims[l - 1]
        W = p[off:off + n_out * n_in].view(n_out, n_in)
        off += n_out * n_in
        bias = None
        if has_bias:
            bias = p[off:off + n_out]
            off += n_out
        out.append((W, bias))
    return out


def init_params(dims, has_bias, gen, device, kind="he"):
    """He-normal weights (std sqrt(2/fan_in)) and zero biases, or N(0, 0.01^2)
    weights for kind="small", or N(0,1) for kind="unit"."""
    d = num_params(dims, has_bias)
    x = torch.zeros(d, dtype=torch.float32, device=device)
    for l, (W, bias) in enumerate(_views(x, dims, has_bias), start=1):
        if kind == "he":
            std = (2.0 / dims[l - 1]) ** 0.5
        elif kind == "small":
            std = 0.01
        else:
            std = 1.0
        W.copy_(_randn(W.shape, gen, device, std))
    return x


def minibatch_gradient(x, dims, has_bias, loss, features, labels=None, targets=None):
    """Gradient at x of the mean loss over the given batch, flattened in x's layout."""
    p = x.detach().clone().requires_grad_(True)
    h = features
    layers = _views(p, dims, has_bias)
    for l, (W, bias) in enumerate(layers):
        h = torch.nn.functional.linear(h, W, bias)
        if l + 1 < len(layers):
            h = torch.relu(h)
    if loss == "softmax_ce":
        val = torch.nn.functional.cross_entropy(h, labels.long())
    else:
        val = 0.5 * torch.mean((h[:, 0] - targets) ** 2)
    val.backward()
    return p.grad.detach()


def cnn_shapes(desc):
    """[(h, w, c)] of the input and of every map of a convolutional model (3 x 3 kernels, zero padding 1)."""
    shapes = [(desc["in_h"], desc["in_w"], desc["in_c"])]
    for c, st in zip(desc["conv_c"], desc["conv_stride"]):
        h, w, _ = shapes[-1]
        shapes.append(((h - 1) // st + 1, (w - 1) // st + 1, c))
    return shapes


def cnn_num_params(desc) -> int:
    shapes = cnn_shapes(desc)
    d = sum(co * 9 * ci + (co if desc["has_bias"] else 0) for (_, _, ci), (_, _, co) in zip(shapes[:-1], shapes[1:]))
    h, w, c = shapes[-1]
    return d + desc["fc_out"] * h * w * c + (desc["fc_out"] if desc["has_bias"] else 0)


def _cnn_views(p, desc):
    """([(kernel [c_out,3,3,c_in], bias)], (W_fc, b_fc)) as views of the flat vector p (the interface's layout)."""
    shapes = cnn_shapes(desc)
    off, convs = 0, []
    for (_, _, ci), (_, _, co) in zip(shapes[:-1], shapes[1:]):
        kern = p[off:off + co * 9 * ci].view(co, 3, 3, ci)
        off += co * 9 * ci
        bias = None
        if desc["has_bias"]:
            bias = p[off:off + co]
            off += co
        convs.append((kern, bias))
    h, w, c = shapes[-1]
    W = p[off:off + desc["fc_out"] * h * w * c].view(desc["fc_out"], h * w * c)
    off += desc["fc_out"] * h * w * c
    b = p[off:off + desc["fc_out"]] if desc["has_bias"] else None
    return convs, (W, b)


def init_cnn_params(desc, gen, device):
    """He-normal kernels and weights (std sqrt(2/fan_in)), zero biases."""
    x = torch.zeros(cnn_num_params(desc), dtype=torch.float32, device=device)
    convs, (W, _) = _cnn_views(x, desc)
    for kern, _ in convs:
        kern.copy_(_randn(kern.shape, gen, device, (2.0 / (9 * kern.shape[3])) ** 0.5))
    W.copy_(_randn(W.shape, gen, device, (2.0 / W.shape[1]) ** 0.5))
    return x


def cnn_minibatch_gradient(x, desc, loss, images, labels=None, targets=None):
    """Gradient at x of the mean loss of the convolutional model over the batch (torch's own convolution
    and autograd: input generation only), flattened in x's layout.  images: [n x in_h*in_w*in_c], NHWC."""
    p = x.detach().clone().requires_grad_(True)
    convs, (W, b) = _cnn_views(p, desc)
    h = images.view(-1, desc["in_h"], desc["in_w"], desc["in_c"]).permute(0, 3, 1, 2)
    for (kern, bias), st in zip(convs, desc["conv_stride"]):
        h = torch.relu(torch.nn.functional.conv2d(h, kern.permute(0, 3, 1, 2), bias, stride=st, padding=1))
    z = torch.nn.functional.linear(h.permute(0, 2, 3, 1).reshape(h.shape[0], -1), W, b)
    if loss == "softmax_ce":
        val = torch.nn.functional.cross_entropy(z, labels.long())
    else:
        val = 0.5 * torch.mean((z[:, 0] - targets) ** 2)
    val.backward()
    return p.grad.detach()


def make_cnn_workload(name, cfg, desc, m, b, n_r, gamma, rho, *, seed=0, device="cpu", loss="softmax_ce",
                      n_flip=0, flip_scale=-4.0, n_noise=0, noise_std=1.0, worker_batch=None, row_align=1):
    """m candidates for a convolutional model (Section 6.1's model class on synthetic images): honest rows are
    exact minibatch gradients at x on each worker's own i.i.d. batch of N(0,1) images with uniform labels;
    faults as in make_mlp_workload.  fp32 forward."""
    device = torch.device(device)
    d_in = desc["in_h"] * desc["in_w"] * desc["in_c"]
    dims = [d_in, desc["fc_out"]]
    x = init_cnn_params(desc, _gen(seed, cfg, 1, device), device)
    features, labels, targets = _draw_batch(dims, loss, n_r, _gen(seed, cfg, 2, device), device)
    d = x.numel()
    q = n_flip + n_noise
    assert q < m
    perm = torch.randperm(m, generator=_gen(seed, cfg, 3, "cpu")).tolist()
    flip_rows, noise_rows, faulty = sorted(perm[:n_flip]), sorted(perm[n_flip:q]), sorted(perm[:q])
    G = _alloc_rows(m, d, row_align, device)
    honest_sum = torch.zeros(d, dtype=torch.float64, device=device)
    n_honest = 0
    for i in range(m):
        if i in faulty:
            continue
        fi, li, ti = _draw_batch(dims, loss, worker_batch or n_r, _gen(seed, cfg, 100 + i, device), device)
        G[i] = cnn_minibatch_gradient(x, desc, loss, fi, li, ti)
        honest_sum += G[i].double()
        n_honest += 1
    if n_flip:
        flipped = (flip_scale * honest_sum / n_honest).float()
        for i in flip_rows:
            G[i] = flipped
    for i in noise_rows:
        G[i] = _randn((d,), _gen(seed, cfg, 100 + i, device), device, noise_std)
    return Workload(name, dims, bool(desc["has_bias"]), loss, "fp32", m, b, n_r, gamma, rho,
                    x, G, features, labels, targets, faulty, dict(desc))


ATTACKS = ("none", "sign_flip", "bit_flip", "label_flip")


def class_sorted_shards(labels, m):
    """Disjoint local datasets (Section 6.5): sample indices sorted by label and cut into m
    equal shards, so each worker sees only a few classes.  Returns an [m x shard] index tensor."""
    order = torch.argsort(labels.long(), stable=True)
    shard = order.numel() // m
    return order[: m * shard].view(m, shard)


def worker_gradients(G, x, dims, has_bias, features, labels, faulty, attack, gen, *, batch=32, scale=4.0,
                     shards=None):
    """Fill G[i] with worker i's candidate for one iteration of Algorithm 1 (worker side).

    Every worker takes the softmax-CE minibatch gradient at x on `batch` samples drawn with
    replacement from the whole data set, or from its own row of `shards` when given.  Workers
    listed in `faulty` fail as `attack` says:
      label_flip  labels replaced by C-1-label before the gradient is taken (Section 6.3);
      bit_flip    the negated gradient, and the first faulty worker's value overwrites the
                  other faulty rows, so all faulty rows are identical (Section 6.4);
      sign_flip   -scale times the worker's own gradient (the enlarged-magnitude case the
                  discussion in Section 6.7 points to);
      none        no failure.
    """
    if attack not in ATTACKS:
        raise ValueError(f"attack must be one of {ATTACKS}")
    faulty = list(faulty)
    bad = set(faulty)
    n, C, dev = features.shape[0], dims[-1], features.device
    for i in range(G.shape[0]):
        if shards is not None:
            idx = shards[i][torch.randint(0, shards.shape[1], (batch,), generator=gen, device=dev)]
        else:
            idx = torch.randint(0, n, (batch,), generator=gen, device=dev)
        lab = labels[idx]
        if i in bad and attack == "label_flip":
            lab = (C - 1 - lab).to(lab.dtype)
        gi = minibatch_gradient(x, dims, has_bias, "softmax_ce", features[idx], lab)
        if i in bad and attack == "sign_flip":
            gi = -scale * gi
        elif i in bad and attack == "bit_flip":
            gi = -gi
        G[i] = gi
    if attack == "bit_flip":
        for i in faulty[1:]:
            G[i] = G[faulty[0]]


def _draw_batch(dims, loss, n, gen, device, feat="normal"):
    if feat == "uniform":
        features = _rand((n, dims[0]), gen, device)
    else:
        features = _randn((n, dims[0]), gen, device)
    labels = targets = None
    if loss == "softmax_ce":
        labels = torch.randint(0, dims[-1], (n,), generator=gen, device=device).to(torch.int32)
    else:
        targets = _randn((n,), gen, device)
    return features, labels, targets


def _alloc_rows(m, d, row_align, device):
    """[m x d] float32 whose rows are row_align floats aligned (a view of a wider buffer).  Line-aligned
    layouts (row_align a multiple of 32 floats) take an odd number of 128-byte lines per row, the pitch
    the library's binding recommends (binding.candidate_pitch)."""
    ldg = (d + row_align - 1) // row_align * row_align
    if row_align % 32 == 0 and (ldg // 32) % 2 == 0:
        ldg += 32
    return torch.empty((m, ldg), dtype=torch.float32, device=device)[:, :d]


def make_mlp_workload(name, cfg, dims, m, b, n_r, gamma, rho, fwd, *, seed=0, device="cpu",
                      has_bias=True, loss="softmax_ce", n_flip=0, flip_scale=-4.0,
                      n_noise=0, noise_std=100.0, feat="normal", init="he",
                      worker_batch=None, faulty_first=False, row_align=1):
    """m candidates for an MLP/softmax model: honest rows are exact minibatch
    gradients at x on each worker's own i.i.d. batch; n_flip rows are identical
    copies of flip_scale x (mean of the honest rows); n_noise rows are
    independent N(0, noise_std^2) per coordinate.  Faulty rows sit at a seeded
    random subset of the m positions.  Rows of G are row_align-float aligned
    (1 = densely packed; the values do not depend on it)."""
    device = torch.device(device)
    x = init_params(dims, has_bias, _gen(seed, cfg, 1, device), device, init)
    features, labels, targets = _draw_batch(dims, loss, n_r, _gen(seed, cfg, 2, device), device, feat)
    d = x.numel()
    q = n_flip + n_noise
    assert q < m
    perm = torch.randperm(m, generator=_gen(seed, cfg, 3, "cpu")).tolist()
    if faulty_first:
        perm = list(range(m))
    flip_rows, noise_rows = sorted(perm[:n_flip]), sorted(perm[n_flip:q])
    faulty = sorted(perm[:q])
    G = _alloc_rows(m, d, row_align, device)
    honest_sum = torch.zeros(d, dtype=torch.float64, device=device)
    wb = worker_batch or n_r
    n_honest = 0
    for i in range(m):
        if i in faulty:
            continue
        fi, li, ti = _draw_batch(dims, loss, wb, _gen(seed, cfg, 100 + i, device), device, feat)
        G[i] = minibatch_gradient(x, dims, has_bias, loss, fi, li, ti)
        honest_sum += G[i].double()
        n_honest += 1
    if n_flip:
        flipped = (flip_scale * honest_sum / n_honest).float()
        for i in flip_rows:
            G[i] = flipped
    for i in noise_rows:
        G[i] = _randn((d,), _gen(seed, cfg, 100 + i, device), device, noise_std)
    return Workload(name, list(dims), has_bias, loss, fwd, m, b, n_r, gamma, rho,
                    x, G, features, labels, targets, faulty)


def make_least_squares(name="cfg1", cfg=1, d=64, n_r=16, m=8, b=2, q=2, gamma=0.1, rho=5e-4,
                       *, seed=0, device="cpu", noise=0.1, flip_scale=-4.0, row_align=1):
    """Linear model, squared loss, no bias: A ~ N(0,1), y = A w* + N(0, 0.01^2),
    x ~ N(0,1); honest rows = gradient of f_r itself plus N(0, noise^2); faulty
    rows = flip_scale x that gradient."""
    device = torch.device(device)
    g = _gen(seed, cfg, 1, device)
    A = _randn((n_r, d), g, device)
    w_star = _randn((d,), g, device)
    y = A @ w_star + _randn((n_r,), g, device, 0.01)
    x = _randn((d,), g, device)
    grad = (A.double().T @ (A.double() @ x.double() - y.double()) / n_r).float()
    perm = torch.randperm(m, generator=_gen(seed, cfg, 3, "cpu")).tolist()
    faulty = sorted(perm[:q])
    G = _alloc_rows(m, d, row_align, device)
    for i in range(m):
        if i in faulty:
            G[i] = flip_scale * grad
        else:
            G[i] = grad + _randn((d,), _gen(seed, cfg, 100 + i, device), device, noise)
    return Workload(name, [d, 1], False, "squared", "fp32", m, b, n_r, gamma, rho,
                    x, G, A, None, y, faulty)


def make_config(cfg: int, *, seed=0, device="cpu", row_align=1, n_r=None) -> Workload:
    """The five numbered workloads (1 = smallest ... 5 = 14 GB of candidates).  n_r
    overrides the size of the server's batch (the paper's own runs use n_r = 4,
    Section 6.1; the workers' batches keep the workload's size)."""
    if n_r is not None and cfg >= 2:
        base = {2: 32, 3: 32, 4: 64, 5: 128}[cfg]
        w = _make_config(cfg, seed=seed, device=device, row_align=row_align, n_r=int(n_r), worker_batch=base)
        return w
    return _make_config(cfg, seed=seed, device=device, row_align=row_align)


def _make_config(cfg, *, seed, device, row_align, n_r=None, worker_batch=None):
    if cfg == 1:
        return make_least_squares(seed=seed, device=device, row_align=row_align)
    if cfg == 2:
        return make_mlp_workload("cfg2", 2, [784, 10], 20, 8, n_r or 32, 0.1, 5e-4, "fp32",
                                 seed=seed, device=device, n_noise=8, noise_std=200.0,
                                 feat="uniform", init="small", worker_batch=32, row_align=row_align)
    if cfg == 3:
        return make_mlp_workload("cfg3", 3, [3072, 512, 10], 20, 8, n_r or 32, 0.05, 1e-3, "fp32",
                                 seed=seed, device=device, n_flip=8, flip_scale=-4.0, row_align=row_align,
                                 worker_batch=worker_batch)
    if cfg == 4:
        return make_mlp_workload("cfg4", 4, [3072, 2048, 2048, 2048, 10], 100, 40, n_r or 64, 0.05, 1e-3,
                                 "bf16", seed=seed, device=device, n_flip=20, flip_scale=-4.0,
                                 n_noise=20, noise_std=100.0, row_align=row_align, worker_batch=worker_batch)
    if cfg == 5:
        return make_mlp_workload("cfg5", 5, [4096, 4096, 4096, 4096, 1000], 64, 16, n_r or 128, 0.02, 1e-4,
                                 "bf16", seed=seed, device=device, n_flip=16, flip_scale=-10.0,
                                 row_align=row_align, worker_batch=worker_batch)
    raise ValueError(f"no such config: {cfg}")


CONFIG_IDS = (1, 2, 3, 4, 5)
