"""CPU oracle for the Zeno aggregation step (arXiv 1805.10032).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, float64 statement of
what the hot path computes.  Only the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may call it; the product path never does.
It shares no code with the HIP library and imports nothing from the package.

Everything is written one candidate at a time, in the order of the paper's
definitions, with the perturbed parameter vector ``x - gamma*u`` materialised.
No blocking, fusion or reordering.

Parameter layout (the interface convention, not part of the paper): a parameter
vector p of length d is, for l = 1..L, the weight matrix W_l stored row-major as
[dims[l] x dims[l-1]] (out x in) followed, if the model has biases, by the bias
b_l[dims[l]].  Candidate gradients use the same layout.

Pins (see tests/test_oracle_*.py): least-squares closed form, b=0 equals Mean,
b=m-1 equals the arg-max row, Lemma 1 (bounded score), the Assumption 2
sandwich for convex losses, ln C at zero parameters, library cross-checks for
logsumexp / mean / median / an MLP forward, brute-force subset enumeration,
the 1-D example in the Discussion section for Mean / Median / Krum, the
(m+1) forward-evaluation count of the Discussion section, and for the server's
update of Algorithm 1: the descent it achieves equals the score of the
aggregate (Definition 2 at rho = 0), and iterating it converges under a faulty
majority where the Mean diverges.
"""
from __future__ import annotations

import numpy as np

LOSS_SQUARED = "squared"
LOSS_SOFTMAX_CE = "softmax_ce"

# Number of calls of f_r since the last reset; the Discussion section prices
# Zeno at (m+1) loss evaluations of n_r samples each.
forward_evaluations = 0


def num_params(dims, has_bias):
    """d for a chain of linear layers dims[0] -> ... -> dims[L]."""
    d = 0
    for l in range(1, len(dims)):
        d += dims[l] * dims[l - 1]
        if has_bias:
            d += dims[l]
    return d


def unflatten(p, dims, has_bias):
    """Split a flat parameter vector into [(W_l, b_l)] following the layout above."""
    p = np.asarray(p, dtype=np.float64)
    assert p.ndim == 1 and p.shape[0] == num_params(dims, has_bias)
    layers = []
    off = 0
    for l in range(1, len(dims)):
        n_out, n_in = dims[l], dims[l - 1]
        W = p[off:off + n_out * n_in].reshape(n_out, n_in)
        off += n_out * n_in
        if has_bias:
            bias = p[off:off + n_out]
            off += n_out
        else:
            bias = np.zeros(n_out, dtype=np.float64)
        layers.append((W, bias))
    return layers


def forward(p, dims, has_bias, features):
    """Model output for every sample: linear layers with ReLU between them and
    none after the last (Section 3: f(x; z) for the model classes of the
    synthetic workloads)."""
    h = np.asarray(features, dtype=np.float64)
    layers = unflatten(p, dims, has_bias)
    for l, (W, bias) in enumerate(layers):
        z = h @ W.T + bias
        h = np.maximum(z, 0.0) if l + 1 < len(layers) else z
    return h


def sample_losses(z, loss, labels=None, targets=None):
    """Per-sample loss f(x; z_k) from the model output z [n_r x C]."""
    if loss == LOSS_SQUARED:
        y = np.asarray(targets, dtype=np.float64)
        return 0.5 * (z[:, 0] - y) ** 2
    if loss == LOSS_SOFTMAX_CE:
        lab = np.asarray(labels, dtype=np.int64)
        zmax = np.max(z, axis=1)
        lse = zmax + np.log(np.sum(np.exp(z - zmax[:, None]), axis=1))
        return lse - z[np.arange(z.shape[0]), lab]
    raise ValueError(loss)


def f_r(p, dims, has_bias, loss, features, labels=None, targets=None):
    """f_r(p) = (1/n_r) sum_k f(p; z_k)   (Definition 2)."""
    global forward_evaluations
    forward_evaluations += 1
    z = forward(p, dims, has_bias, features)
    with np.errstate(invalid="ignore", over="ignore"):
        return float(np.mean(sample_losses(z, loss, labels, targets)))


def score(x, u, gamma, rho, f0, dims, has_bias, loss, features, labels=None, targets=None):
    """Score_{gamma,rho}(u, x) = f_r(x) - f_r(x - gamma u) - rho ||u||^2
    (Definition 2); f0 = f_r(x) is evaluated once by the caller and shared."""
    x = np.asarray(x, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        xp = x - gamma * u
        fi = f_r(xp, dims, has_bias, loss, features, labels, targets)
        return f0 - fi - rho * float(np.dot(u, u))


def scores(x, G, gamma, rho, dims, has_bias, loss, features, labels=None, targets=None,
           rows=None):
    """Scores of the candidates G[i] (all rows, or only those listed in rows)."""
    f0 = f_r(np.asarray(x, dtype=np.float64), dims, has_bias, loss, features, labels, targets)
    idx = range(G.shape[0]) if rows is None else rows
    return np.array([score(x, G[i], gamma, rho, f0, dims, has_bias, loss, features,
                           labels, targets) for i in idx], dtype=np.float64)


def select(score_values, b):
    """Indices of the m-b highest scores (Definition 3), reported ascending.

    Reading where the paper is silent: ties go to the lower index, a NaN score
    ranks as minus infinity."""
    s = np.asarray(score_values, dtype=np.float64)
    m = s.shape[0]
    assert 0 <= b < m
    key = np.where(np.isnan(s), -np.inf, s)
    order = sorted(range(m), key=lambda i: (-key[i], i))
    return np.array(sorted(order[:m - b]), dtype=np.int64)


def zeno_aggregate(G, score_values, b):
    """Zeno_b: average of the m-b highest-scoring candidates (Definition 3)."""
    sel = select(score_values, b)
    acc = np.zeros(G.shape[1], dtype=np.float64)
    for i in sel:
        acc += np.asarray(G[i], dtype=np.float64)
    return acc / float(len(sel)), sel


def mean(G):
    """Mean aggregation rule (Section 6.1.1)."""
    acc = np.zeros(G.shape[1], dtype=np.float64)
    for i in range(G.shape[0]):
        acc += np.asarray(G[i], dtype=np.float64)
    return acc / float(G.shape[0])


def median(G):
    """Marginal median (Definition 4).  Reading for even m: the midpoint of the
    two middle values.  NaN sorts above +inf."""
    G = np.asarray(G, dtype=np.float64)
    m = G.shape[0]
    srt = np.sort(G, axis=0)  # NaN last
    if m % 2 == 1:
        return srt[m // 2].copy()
    with np.errstate(invalid="ignore", over="ignore"):
        return 0.5 * (srt[m // 2 - 1] + srt[m // 2])


def krum_scores(G, b):
    """Definition 5: for every candidate the sum of squared distances to its m-b-2
    nearest other candidates.  Reading where the paper is silent: a distance that is
    not finite (a row holding NaN or Inf, Section 3 Eq. 1 allows any value) counts as
    +infinity."""
    G = np.asarray(G, dtype=np.float64)
    m = G.shape[0]
    assert m - b - 2 >= 1
    out = np.empty(m)
    for i in range(m):
        with np.errstate(invalid="ignore", over="ignore"):
            dist = [float(np.sum((G[i] - G[j]) ** 2)) for j in range(m) if j != i]
        dist = sorted(v if np.isfinite(v) else np.inf for v in dist)
        out[i] = sum(dist[:m - b - 2])
    return out


def krum(G, b):
    """Krum_b (Definition 5): the candidate with the smallest sum of squared
    distances to its m-b-2 nearest neighbours; ties go to the lower index."""
    vals = krum_scores(G, b)
    best, best_val = -1, np.inf
    for i in range(len(vals)):
        if vals[i] < best_val:
            best, best_val = i, vals[i]
    return np.asarray(G, dtype=np.float64)[best].copy(), best


def sgd_update(x, v, gamma):
    """The server's update of Algorithm 1: x_next = x - gamma v, in float64."""
    return np.asarray(x, dtype=np.float64) - float(gamma) * np.asarray(v, dtype=np.float64)


def zeno_update(x, G, score_values, b, gamma):
    """Algorithm 1, server side after the scores: x_next = x - gamma Zeno_b(G).
    Returns (x_next float64, selected indices)."""
    v, sel = zeno_aggregate(G, score_values, b)
    return sgd_update(x, v, gamma), sel


def zeno_step(x, G, b, gamma, rho, dims, has_bias, loss, features, labels=None, targets=None):
    """One whole aggregation: scores, selection, average."""
    s = scores(x, G, gamma, rho, dims, has_bias, loss, features, labels, targets)
    out, sel = zeno_aggregate(G, s, b)
    return s, sel, out


# ---------------------------------------------------------------------------
# bf16-operand variant (workloads whose forward passes use bf16 operands with
# fp32 accumulation).  The paper fixes no precision; this is the rounding
# contract of the bf16 forward mode, stated in words and written out plainly:
#
#   * every operand of a matrix product is rounded to bfloat16 (round to
#     nearest, ties to even) first; products are accumulated exactly (float64
#     here stands for the fp32 accumulator); biases are added unrounded;
#   * the pass at x computes z0_l = rb(h0_{l-1}) rb(W_l)^T + b_l, h0_l = relu(z0_l),
#     h0_0 = the batch;
#   * candidate u is propagated as the CHANGE of the pre-activations relative to the pass at x,
#       dz_l = -gamma ( rb(h0_{l-1}) rb(U_l)^T + rb(D_{l-1}) rb(W'_l)^T + ub_l ),
#       W'_l = fl32( rb(W_l) - gamma rb(U_l) )   (one float32 rounding, a fused multiply-add),
#       D_l = (relu(z0_l + dz_l) - relu(z0_l)) (-1/gamma),  D_0 = 0,  h0_0 = the batch,
#     and only D_l is carried from layer to layer.  In exact arithmetic the candidate's
#     activations are h_l = h0_l - gamma D_l, so its own product h_{l-1} U_l^T + D_{l-1} W_l^T
#     equals h0_{l-1} U_l^T + D_{l-1} (W_l - gamma U_l)^T: the first product runs on the
#     activations of the pass at x, the second on the perturbed weights, and z0_l + dz_l equals
#     the pre-activation of the model at x - gamma u.  Without rounding this is Definition 2
#     unchanged;
#   * loss difference per sample and the final combine as in the exact oracle.
#
# Pinned by (tests/test_oracle_bf16.py): exact equality with the float64 oracle when
# every operand is bf16-representable; a forward-error bound against the float64
# oracle on random inputs; and agreement, within one unit of the bf16 rounding of
# the losses, with Definition 2 written as two plain forward passes per candidate
# whose operands are rounded to bf16 (no change propagation), a form in which a
# wrong sign, a dropped term or a missing product lands far outside that bound.
# Beyond that the contract has no external reference ("parity unpinned" applies to
# the choice of rounding points, not to the arithmetic).
# ---------------------------------------------------------------------------
def round_bf16(a):
    """Nearest bfloat16 (ties to even) of the fp32 rounding of a, as float64."""
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float32))
    bits = f.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    out = (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isnan(f), np.nan, out)


def _f32(a):
    with np.errstate(over="ignore", invalid="ignore"):
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def scores_bf16(x, G, gamma, rho, dims, has_bias, loss, features, labels=None, targets=None, rows=None):
    """Scores under the bf16 rounding contract above."""
    global forward_evaluations
    rb = round_bf16
    L = len(dims) - 1
    layers_x = unflatten(x, dims, has_bias)
    batch = np.asarray(features, dtype=np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        # pass at x
        forward_evaluations += 1
        h0, z0 = [batch], []
        for l, (W, bias) in enumerate(layers_x):
            z = _f32(rb(h0[-1]) @ rb(W).T + bias)
            z0.append(z)
            if l + 1 < L:
                h0.append(np.maximum(z, 0.0))
        base_losses = sample_losses(z0[-1], loss, labels, targets)
        idx = range(G.shape[0]) if rows is None else rows
        out = []
        neg_inv_gamma = _f32(-1.0 / np.float32(gamma)) if gamma > 0 else 0.0
        for i in idx:
            forward_evaluations += 1
            u = np.asarray(G[i], dtype=np.float64)
            layers_u = unflatten(u, dims, has_bias)
            dprime, dz = None, None
            g32 = np.float64(np.float32(gamma))
            for l, ((U, ub), (W, _)) in enumerate(zip(layers_u, layers_x)):
                acc = rb(h0[l]) @ rb(U).T + ub
                if dprime is not None:
                    w_perturbed = _f32(rb(W) - g32 * rb(U))
                    acc = acc + rb(dprime) @ rb(w_perturbed).T
                dz = _f32(-g32 * _f32(acc))
                if l + 1 < L:
                    zs = _f32(z0[l] + dz)
                    h_new = np.where(zs <= 0.0, 0.0, zs)
                    delta = np.where(z0[l] > 0.0, np.where(dz < -z0[l], -z0[l], dz), h_new)
                    dprime = _f32(delta * neg_inv_gamma)
            diff = sample_losses(z0[-1] + dz, loss, labels, targets) - base_losses
            out.append(-float(np.mean(diff)) - rho * float(np.dot(u, u)))
    return np.array(out, dtype=np.float64)


# ---------------------------------------------------------------------------
# Convolutional f_r (Section 6.1: "4 convolutional layers followed by 1 fully
# connected layer" on 32 x 32 x 3 images; the paper gives no widths, strides or
# pooling, so those are free choices of the model description, not of the paper).
#
# Model class: n_conv convolutions with 3 x 3 kernels, zero padding 1, stride 1 or 2,
# ReLU after each; then one fully connected layer on the flattened last map, no
# activation.  Images and maps are NHWC.  Parameter layout (interface convention): for
# every convolution the kernel W[c_out][ky][kx][c_in] row-major, then its bias[c_out]
# if the model has biases; then the fully connected W[fc_out][h * w * c] whose input is
# the last map flattened in (y, x, c) order, then its bias.
#
# Pinned by (tests/test_oracle_conv.py): a hand-computed 3 x 3 example, a six-loop
# brute force, torch.nn.functional.conv2d on the CPU, the reduction of a 1 x 1 image
# to a linear layer on the centre tap, and the same score pins as the linear models
# (zero candidate, rho shift, finite-difference limit against autograd).
# ---------------------------------------------------------------------------
def conv_out_size(n, stride):
    """Output width of a 3-wide kernel with zero padding 1 over n positions."""
    return (n - 1) // stride + 1


def cnn_shapes(desc):
    """[(h, w, c)] of the input and of every map, for desc = dict(in_h, in_w, in_c,
    conv_c=[...], conv_stride=[...], fc_out, has_bias)."""
    shapes = [(desc["in_h"], desc["in_w"], desc["in_c"])]
    for c, s in zip(desc["conv_c"], desc["conv_stride"]):
        h, w, _ = shapes[-1]
        shapes.append((conv_out_size(h, s), conv_out_size(w, s), c))
    return shapes


def cnn_num_params(desc):
    shapes = cnn_shapes(desc)
    d = 0
    for (h, w, c_in), (_, _, c_out) in zip(shapes[:-1], shapes[1:]):
        d += c_out * 9 * c_in + (c_out if desc["has_bias"] else 0)
    h, w, c = shapes[-1]
    d += desc["fc_out"] * h * w * c + (desc["fc_out"] if desc["has_bias"] else 0)
    return d


def cnn_unflatten(p, desc):
    """([(kernel[c_out,3,3,c_in], bias[c_out])], (W_fc, b_fc)) following the layout above."""
    p = np.asarray(p, dtype=np.float64)
    assert p.ndim == 1 and p.shape[0] == cnn_num_params(desc)
    shapes = cnn_shapes(desc)
    off, convs = 0, []
    for (h, w, c_in), (_, _, c_out) in zip(shapes[:-1], shapes[1:]):
        n = c_out * 9 * c_in
        kern = p[off:off + n].reshape(c_out, 3, 3, c_in)
        off += n
        if desc["has_bias"]:
            bias = p[off:off + c_out]
            off += c_out
        else:
            bias = np.zeros(c_out)
        convs.append((kern, bias))
    h, w, c = shapes[-1]
    n = desc["fc_out"] * h * w * c
    W = p[off:off + n].reshape(desc["fc_out"], h * w * c)
    off += n
    b = p[off:off + desc["fc_out"]] if desc["has_bias"] else np.zeros(desc["fc_out"])
    return convs, (W, b)


def conv3x3(h, kern, bias, stride):
    """z[n, y, x, co] = bias[co] + sum over ky, kx, ci of hpad[n, y*stride + ky, x*stride + kx, ci] * kern[co, ky, kx, ci],
    hpad = h with one ring of zeros around every image."""
    n, hh, ww, c_in = h.shape
    ho, wo = conv_out_size(hh, stride), conv_out_size(ww, stride)
    hpad = np.zeros((n, hh + 2, ww + 2, c_in))
    hpad[:, 1:hh + 1, 1:ww + 1, :] = h
    z = np.zeros((n, ho, wo, kern.shape[0]))
    for ky in range(3):
        for kx in range(3):
            patch = hpad[:, ky:ky + stride * (ho - 1) + 1:stride, kx:kx + stride * (wo - 1) + 1:stride, :]
            z += patch @ kern[:, ky, kx, :].T
    return z + bias


def cnn_forward(p, desc, images):
    """Model output [n x fc_out] for images [n x in_h x in_w x in_c]."""
    convs, (W, b) = cnn_unflatten(p, desc)
    h = np.asarray(images, dtype=np.float64).reshape(-1, desc["in_h"], desc["in_w"], desc["in_c"])
    for (kern, bias), s in zip(convs, desc["conv_stride"]):
        h = np.maximum(conv3x3(h, kern, bias, s), 0.0)
    return h.reshape(h.shape[0], -1) @ W.T + b


def cnn_f_r(p, desc, loss, images, labels=None, targets=None):
    """f_r(p) = (1/n_r) sum_k f(p; z_k) for the convolutional model (Definition 2)."""
    global forward_evaluations
    forward_evaluations += 1
    with np.errstate(invalid="ignore", over="ignore"):
        return float(np.mean(sample_losses(cnn_forward(p, desc, images), loss, labels, targets)))


def cnn_scores(x, G, gamma, rho, desc, loss, images, labels=None, targets=None, rows=None):
    """Definition 2 for the convolutional model: (scores, scale) with scale = |f_r(x) - f_r(x - gamma u)| + rho ||u||^2."""
    x = np.asarray(x, dtype=np.float64)
    f0 = cnn_f_r(x, desc, loss, images, labels, targets)
    idx = range(G.shape[0]) if rows is None else rows
    s, scale = [], []
    for i in idx:
        u = np.asarray(G[i], dtype=np.float64)
        with np.errstate(invalid="ignore", over="ignore"):
            fi = cnn_f_r(x - gamma * u, desc, loss, images, labels, targets)
            pen = rho * float(np.dot(u, u))
        s.append(f0 - fi - pen)
        scale.append(abs(f0 - fi) + pen)
    return np.array(s), np.array(scale)
