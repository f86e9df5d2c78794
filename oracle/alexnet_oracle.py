"""Float64 CPU oracle for one AlexNet SGD training step.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
HIP library is checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP
path and imports nothing from it.

What it computes (paper Section 2, "Methods"): the network the paper trains is
AlexNet -- 5 convolutional layers (3 followed by max pooling), 2 fully
connected layers and a softmax layer -- and one training iteration is forward,
backward and a momentum update on a minibatch.  Section 2.1 (footnote) names
the preprocessing: subtract the mean image, random crop, random flip.
Section 2.2 names the two-replica step: update each replica on its own
minibatch, exchange, then average weights, biases and momentum.

The paper defers every layer hyper-parameter to its citation of Krizhevsky et
al. 2012; the numbers used here are passed in through NetSpec.  Readings taken
where the paper is silent are listed beside each function.

Everything is float64, NCHW activations, OIHW convolution weights, [out, in]
fully connected weights.  Convolution is cross-correlation (no kernel flip),
zero padded, floor output size.

Pins (see tests/test_oracle_*.py): brute-force direct convolution, adjoint
identities, central finite differences, closed forms for LRN / update /
softmax, published splitmix64 vectors, torch-CPU float64 library routines.
Parity unpinned: nothing in this file (the paper's accuracy and Table 1 timings
are not reproduced by any function here).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

F64 = np.float64
U64 = np.uint64

# --------------------------------------------------------------------------
# Network description
# --------------------------------------------------------------------------


@dataclass
class ConvSpec:
    cout: int
    k: int
    stride: int
    pad: int
    groups: int
    lrn: bool
    pool: bool


@dataclass
class NetSpec:
    batch: int
    in_c: int
    crop_h: int
    crop_w: int
    raw_h: int
    raw_w: int
    conv: List[ConvSpec]
    fc: List[int]  # output widths of the three dense layers; fc[-1] = classes
    lrn_n: int = 5
    lrn_k: float = 2.0
    lrn_alpha: float = 1e-4
    lrn_beta: float = 0.75
    dropout_p: float = 0.5
    lr: float = 0.01
    momentum: float = 0.9
    weight_decay: float = 5e-4
    seed: int = 0
    pool_k: int = 3
    pool_s: int = 2


def conv_out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def pool_out_size(h: int, k: int = 3, s: int = 2) -> int:
    # floor convention; exact for 55->27->13->6
    return (h - k) // s + 1


def layer_shapes(spec: NetSpec):
    """Activation shape (C, H, W) after every stage, and the flatten size."""
    c, h, w = spec.in_c, spec.crop_h, spec.crop_w
    stages = []
    for i, cv in enumerate(spec.conv):
        ho = conv_out_size(h, cv.k, cv.stride, cv.pad)
        wo = conv_out_size(w, cv.k, cv.stride, cv.pad)
        entry = {"in": (c, h, w), "conv": (cv.cout, ho, wo)}
        c, h, w = cv.cout, ho, wo
        if cv.pool:
            h, w = pool_out_size(h, spec.pool_k, spec.pool_s), pool_out_size(w, spec.pool_k, spec.pool_s)
            entry["pool"] = (c, h, w)
        stages.append(entry)
    return stages, c * h * w


def param_shapes(spec: NetSpec) -> Dict[str, Tuple[int, ...]]:
    """Canonical parameter tensors.  Flat order: every weight tensor
    (conv1..conv5, fc6..fc8), then every bias in the same layer order."""
    stages, flat = layer_shapes(spec)
    shapes: Dict[str, Tuple[int, ...]] = {}
    names = []
    for i, cv in enumerate(spec.conv):
        cin = stages[i]["in"][0]
        names.append((f"conv{i+1}", (cv.cout, cin // cv.groups, cv.k, cv.k), cv.cout))
    fin = flat
    for j, fo in enumerate(spec.fc):
        names.append((f"fc{len(spec.conv)+1+j}", (fo, fin), fo))
        fin = fo
    for n, ws, _ in names:
        shapes[n + ".w"] = ws
    for n, _, bs in names:
        shapes[n + ".b"] = (bs,)
    return shapes


def flatten_params(spec: NetSpec, params: Dict[str, np.ndarray]) -> np.ndarray:
    return np.concatenate([np.asarray(params[k], F64).ravel() for k in param_shapes(spec)])


def unflatten_params(spec: NetSpec, flat: np.ndarray) -> Dict[str, np.ndarray]:
    out, o = {}, 0
    for k, s in param_shapes(spec).items():
        n = int(np.prod(s))
        out[k] = np.asarray(flat[o:o + n], F64).reshape(s).copy()
        o += n
    assert o == flat.size
    return out


def n_weight_elems(spec: NetSpec) -> int:
    return sum(int(np.prod(s)) for k, s in param_shapes(spec).items() if k.endswith(".w"))


# --------------------------------------------------------------------------
# Counter-based random numbers (crop offsets, flip bits, dropout masks).
# The paper gives no generator; "random" cropping / flipping (Section 2.1
# footnote) and dropout are made reproducible with a stateless hash of
# (seed, step, purpose, index) built on the public-domain splitmix64 output
# function.
# --------------------------------------------------------------------------

TAG_CROP_X, TAG_CROP_Y, TAG_FLIP, TAG_DROP6, TAG_DROP7 = 1, 2, 3, 6, 7
_GOLDEN = U64(0x9E3779B97F4A7C15)


def mix64(z):
    z = np.asarray(z, dtype=U64).copy()
    with np.errstate(over="ignore"):
        z ^= z >> U64(30)
        z *= U64(0xBF58476D1CE4E5B9)
        z ^= z >> U64(27)
        z *= U64(0x94D049BB133111EB)
        z ^= z >> U64(31)
    return z


def step_key(seed: int, step: int):
    with np.errstate(over="ignore"):
        k0 = mix64(U64(seed) + _GOLDEN)
    return mix64(k0 ^ U64(step))


def rand_u64(seed: int, step: int, tag: int, idx):
    k1 = step_key(seed, step)
    idx = np.asarray(idx, dtype=U64)
    return mix64(k1 ^ (U64(tag) << U64(56)) ^ idx)


def crop_flip_params(spec: NetSpec, step: int):
    """Per-image crop offsets (ox, oy) and flip bit for minibatch `step`."""
    n = np.arange(spec.batch, dtype=U64)
    rx = rand_u64(spec.seed, step, TAG_CROP_X, n)
    ry = rand_u64(spec.seed, step, TAG_CROP_Y, n)
    rf = rand_u64(spec.seed, step, TAG_FLIP, n)
    ox = ((rx >> U64(32)) % U64(spec.raw_w - spec.crop_w + 1)).astype(np.int32)
    oy = ((ry >> U64(32)) % U64(spec.raw_h - spec.crop_h + 1)).astype(np.int32)
    flip = (rf >> U64(63)).astype(np.int32)
    return ox, oy, flip


def dropout_mask(spec: NetSpec, step: int, tag: int, width: int) -> np.ndarray:
    """{0,1} keep mask of shape [batch, width]; element (n, f) uses index
    n*width + f; kept when the top 24 bits reach floor(p * 2^24)."""
    idx = np.arange(spec.batch * width, dtype=U64)
    r = rand_u64(spec.seed, step, tag, idx)
    thresh = U64(int(np.floor(spec.dropout_p * (1 << 24))))
    keep = (r >> U64(40)) >= thresh
    return keep.reshape(spec.batch, width).astype(F64)


# --------------------------------------------------------------------------
# Preprocessing (Section 2.1 footnote): mean subtract, crop, flip
# --------------------------------------------------------------------------


def preprocess(raw_u8: np.ndarray, mean: np.ndarray, ox, oy, flip, crop_h: int, crop_w: int) -> np.ndarray:
    """raw_u8 [B,C,H,W] uint8, mean [C,H,W].  The mean is subtracted at the
    source pixel, the window is then cut out and finally mirrored, so the mean
    image is mirrored together with the picture."""
    b = raw_u8.shape[0]
    out = np.empty((b, raw_u8.shape[1], crop_h, crop_w), F64)
    for n in range(b):
        t = raw_u8[n].astype(F64) - np.asarray(mean, F64)
        t = t[:, oy[n]:oy[n] + crop_h, ox[n]:ox[n] + crop_w]
        if flip[n]:
            t = t[:, :, ::-1]
        out[n] = t
    return out


# --------------------------------------------------------------------------
# Convolution: y[n,o,y,x] = b[o] + sum_{c,r,s} W[o,c,r,s] x[n, g(o)*Cg + c, y*st+r-p, x*st+s-p]
# --------------------------------------------------------------------------


def _im2col(xp: np.ndarray, k: int, stride: int, ho: int, wo: int) -> np.ndarray:
    """xp: padded [N,C,Hp,Wp] -> cols [N, C, k, k, ho, wo]."""
    n, c = xp.shape[:2]
    cols = np.empty((n, c, k, k, ho, wo), F64)
    for r in range(k):
        for s in range(k):
            cols[:, :, r, s] = xp[:, :, r:r + stride * ho:stride, s:s + stride * wo:stride]
    return cols


def _pad(x: np.ndarray, pad: int) -> np.ndarray:
    if pad == 0:
        return x
    return np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))


def conv_forward(x, w, b, stride: int, pad: int, groups: int, chunk: int = 8) -> np.ndarray:
    x = np.asarray(x, F64)
    w = np.asarray(w, F64)
    n, cin, h, wd = x.shape
    cout, cg, k, _ = w.shape
    assert cg * groups == cin and cout % groups == 0
    ho, wo = conv_out_size(h, k, stride, pad), conv_out_size(wd, k, stride, pad)
    og = cout // groups
    y = np.empty((n, cout, ho, wo), F64)
    for n0 in range(0, n, chunk):
        xp = _pad(x[n0:n0 + chunk], pad)
        nb = xp.shape[0]
        for g in range(groups):
            cols = _im2col(xp[:, g * cg:(g + 1) * cg], k, stride, ho, wo)
            wm = w[g * og:(g + 1) * og].reshape(og, cg * k * k)
            for i in range(nb):
                y[n0 + i, g * og:(g + 1) * og] = (wm @ cols[i].reshape(cg * k * k, ho * wo)).reshape(og, ho, wo)
    if b is not None:
        y += np.asarray(b, F64)[None, :, None, None]
    return y


def conv_backward_weight(x, dy, k: int, stride: int, pad: int, groups: int, chunk: int = 8):
    """dW[o,c,r,s] = sum_{n,y,x} dy[n,o,y,x] * x[n, g*Cg+c, y*st+r-p, x*st+s-p];  db[o] = sum dy."""
    x = np.asarray(x, F64)
    dy = np.asarray(dy, F64)
    n, cin, h, wd = x.shape
    _, cout, ho, wo = dy.shape
    cg, og = cin // groups, cout // groups
    dw = np.zeros((cout, cg, k, k), F64)
    for n0 in range(0, n, chunk):
        xp = _pad(x[n0:n0 + chunk], pad)
        nb = xp.shape[0]
        for g in range(groups):
            cols = _im2col(xp[:, g * cg:(g + 1) * cg], k, stride, ho, wo)
            for i in range(nb):
                dym = dy[n0 + i, g * og:(g + 1) * og].reshape(og, ho * wo)
                dw[g * og:(g + 1) * og] += (dym @ cols[i].reshape(cg * k * k, ho * wo).T).reshape(og, cg, k, k)
    db = dy.sum(axis=(0, 2, 3))
    return dw, db


def conv_backward_data(dy, w, in_hw: Tuple[int, int], stride: int, pad: int, groups: int, chunk: int = 8):
    """dx[n,c',i,j] = sum over (o,r,s,y,x) with y*st+r-p = i, x*st+s-p = j of dy[n,o,y,x] W[o,c,r,s]."""
    dy = np.asarray(dy, F64)
    w = np.asarray(w, F64)
    n, cout, ho, wo = dy.shape
    _, cg, k, _ = w.shape
    og = cout // groups
    h, wd = in_hw
    dx = np.empty((n, cg * groups, h, wd), F64)
    for n0 in range(0, n, chunk):
        nb = min(chunk, n - n0)
        dxp = np.zeros((nb, cg * groups, h + 2 * pad, wd + 2 * pad), F64)
        for g in range(groups):
            wm = w[g * og:(g + 1) * og].reshape(og, cg * k * k)
            for i in range(nb):
                dcols = (wm.T @ dy[n0 + i, g * og:(g + 1) * og].reshape(og, ho * wo)).reshape(cg, k, k, ho, wo)
                for r in range(k):
                    for s in range(k):
                        dxp[i, g * cg:(g + 1) * cg, r:r + stride * ho:stride, s:s + stride * wo:stride] += dcols[:, r, s]
        dx[n0:n0 + nb] = dxp[:, :, pad:pad + h, pad:pad + wd]
    return dx


# --------------------------------------------------------------------------
# ReLU, local response normalisation, max pooling
# --------------------------------------------------------------------------


def relu(x):
    return np.maximum(x, 0.0)


def lrn_forward(a, n: int, k: float, alpha: float, beta: float):
    """b_i = a_i * s_i^(-beta),  s_i = k + alpha * sum_{j=i-n//2}^{i+n//2} a_j^2  (channels clipped to
    [0, C-1]; alpha is NOT divided by n -- the formula of the 2012 AlexNet paper as printed)."""
    a = np.asarray(a, F64)
    c = a.shape[1]
    half = n // 2
    sq = a * a
    s = np.full_like(a, k)
    for d in range(-half, half + 1):
        lo, hi = max(0, -d), min(c, c - d)  # channels i with 0 <= i+d < c
        s[:, lo:hi] += alpha * sq[:, lo + d:hi + d]
    return a * s ** (-beta), s


def lrn_backward(dy, a, s, n: int, alpha: float, beta: float):
    """da_i = dy_i s_i^(-beta) - 2 alpha beta a_i sum_{j: i in win(j)} dy_j a_j s_j^(-beta-1)."""
    dy = np.asarray(dy, F64)
    c = a.shape[1]
    half = n // 2
    t = dy * a * s ** (-beta - 1.0)
    acc = np.zeros_like(a)
    for d in range(-half, half + 1):
        lo, hi = max(0, -d), min(c, c - d)
        acc[:, lo:hi] += t[:, lo + d:hi + d]
    return dy * s ** (-beta) - 2.0 * alpha * beta * a * acc


def maxpool_forward(x, k: int = 3, s: int = 2):
    """Window scanned row-major; a later tap replaces the running maximum only
    when strictly greater, so the first maximum wins ties.  argmax is the flat
    index y_in*W + x_in inside the input plane (int32)."""
    x = np.asarray(x)
    n, c, h, w = x.shape
    ho, wo = pool_out_size(h, k, s), pool_out_size(w, k, s)
    best = None
    arg = None
    yy = (np.arange(ho) * s)[:, None]
    xx = (np.arange(wo) * s)[None, :]
    for r in range(k):
        for q in range(k):
            tap = x[:, :, r:r + s * ho:s, q:q + s * wo:s]
            idx = ((yy + r) * w + (xx + q)).astype(np.int32)
            idx = np.broadcast_to(idx, tap.shape)
            if best is None:
                best, arg = tap.copy(), idx.copy()
            else:
                m = tap > best
                best = np.where(m, tap, best)
                arg = np.where(m, idx, arg)
    return best, arg.astype(np.int32)


def maxpool_backward(dy, arg, in_hw: Tuple[int, int]):
    dy = np.asarray(dy, F64)
    n, c, ho, wo = dy.shape
    h, w = in_hw
    dx = np.zeros((n, c, h * w), F64)
    flat_arg = arg.reshape(n, c, ho * wo)
    flat_dy = dy.reshape(n, c, ho * wo)
    for i in range(n):
        for j in range(c):
            np.add.at(dx[i, j], flat_arg[i, j], flat_dy[i, j])
    return dx.reshape(n, c, h, w)


# --------------------------------------------------------------------------
# Dense layers, softmax cross-entropy
# --------------------------------------------------------------------------


def fc_forward(x, w, b):
    return np.asarray(x, F64) @ np.asarray(w, F64).T + np.asarray(b, F64)


def fc_backward(x, w, dy):
    dy = np.asarray(dy, F64)
    return dy @ np.asarray(w, F64), dy.T @ np.asarray(x, F64), dy.sum(axis=0)  # dx, dW, db


def softmax_xent(z, labels):
    """p = softmax(z) row-wise; L = -(1/B) sum_n log p[n, label_n]; dz = (p - onehot)/B."""
    z = np.asarray(z, F64)
    b = z.shape[0]
    zm = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(zm).sum(axis=1, keepdims=True))
    logp = zm - lse
    p = np.exp(logp)
    rows = np.arange(b)
    loss = -logp[rows, labels].mean()
    dz = p.copy()
    dz[rows, labels] -= 1.0
    return loss, p, dz / b


# --------------------------------------------------------------------------
# Update (momentum + weight decay) and two-replica averaging (Section 2.2)
# --------------------------------------------------------------------------


def sgd_update(w, v, g, lr: float, mu: float, wd: float):
    """v <- mu v - lr (g + wd w);  w <- w + v."""
    v_new = mu * np.asarray(v, F64) - lr * (np.asarray(g, F64) + wd * np.asarray(w, F64))
    return np.asarray(w, F64) + v_new, v_new


def average_replicas(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Step 3 of Section 2.2: both replicas end up holding the mean."""
    return (np.asarray(a, F64) + np.asarray(b, F64)) / 2.0


def averaged_gradient_update(w_a, v_a, g_a, w_b, v_b, g_b, lr: float, mu: float, wd: float):
    """Exchange gradients instead of parameters (a variant of Section 2.2's exchange): both replicas
    apply the update rule to the mean of their two gradients.  The rule is affine in g, so for
    replicas that hold the same w and v this gives what updating separately and then averaging
    weights and momentum gives; replicas that differ keep their own w and v.
    Returns ((w_a', v_a'), (w_b', v_b'))."""
    g = (np.asarray(g_a, F64) + np.asarray(g_b, F64)) / 2.0
    return sgd_update(w_a, v_a, g, lr, mu, wd), sgd_update(w_b, v_b, g, lr, mu, wd)


def topk_correct(scores, labels, k: int) -> int:
    """Section 3's validation count: the number of rows whose label is among the k highest scores.
    A row counts when fewer than k classes score strictly higher than its label (so ties go to the
    label)."""
    scores = np.asarray(scores, F64)
    labels = np.asarray(labels)
    own = scores[np.arange(scores.shape[0]), labels][:, None]
    return int(np.sum(np.sum(scores > own, axis=1) < k))


def center_crop_params(spec: "NetSpec"):
    """Validation preprocessing: the central crop, no mirroring (offsets floor((raw - crop) / 2))."""
    n = spec.batch
    ox = np.full(n, (spec.raw_w - spec.crop_w) // 2, dtype=np.int32)
    oy = np.full(n, (spec.raw_h - spec.crop_h) // 2, dtype=np.int32)
    return ox, oy, np.zeros(n, dtype=np.int32)


# --------------------------------------------------------------------------
# Whole network
# --------------------------------------------------------------------------


def _forward_stack(spec: NetSpec, params, x, masks, train: bool):
    """Returns logits and a cache of every intermediate."""
    cache = {"x": np.asarray(x, F64)}
    h = cache["x"]
    for i, cv in enumerate(spec.conv):
        name = f"conv{i+1}"
        z = conv_forward(h, params[name + ".w"], params[name + ".b"], cv.stride, cv.pad, cv.groups)
        a = relu(z)
        cache[name + ".z"] = z
        cache[name + ".in"] = h
        cache[name + ".act"] = a
        h = a
        if cv.lrn:
            bnorm, s = lrn_forward(a, spec.lrn_n, spec.lrn_k, spec.lrn_alpha, spec.lrn_beta)
            cache[name + ".lrn_s"] = s
            cache[name + ".lrn"] = bnorm
            h = bnorm
        if cv.pool:
            cache[name + ".pool_in_hw"] = h.shape[2:]
            p, arg = maxpool_forward(h, spec.pool_k, spec.pool_s)
            cache[name + ".pool"] = p
            cache[name + ".argmax"] = arg
            h = p
    cache["flat_shape"] = h.shape
    h = h.reshape(h.shape[0], -1)  # (c, h, w) order
    nfc = len(spec.fc)
    for j in range(nfc):
        name = f"fc{len(spec.conv)+1+j}"
        cache[name + ".in"] = h
        z = fc_forward(h, params[name + ".w"], params[name + ".b"])
        cache[name + ".z"] = z
        if j < nfc - 1:
            a = relu(z)
            if train:
                a = a * masks[j]           # {0,1} mask, no rescale while training
            else:
                a = a * (1.0 - spec.dropout_p)  # expectation scaling at test time
            cache[name + ".act"] = a
            h = a
        else:
            h = z
    cache["logits"] = h
    return h, cache


def forward(spec: NetSpec, params, x) -> np.ndarray:
    """Inference pass on an already preprocessed batch: class probabilities."""
    z, _ = _forward_stack(spec, params, x, None, train=False)
    zm = z - z.max(axis=1, keepdims=True)
    e = np.exp(zm)
    return e / e.sum(axis=1, keepdims=True)


def loss_and_grads(spec: NetSpec, params, x, labels, masks, want_dx: bool = False, decisions=None):
    """Mean cross-entropy of the minibatch and its gradient w.r.t. every
    parameter, with the given dropout masks held fixed.

    The network is piecewise smooth: which side of a ReLU a unit is on and
    which tap wins a pooling window are discrete choices of the forward pass.
    `decisions` (optional) fixes them for the backward pass: keys
    "<layer>.gate" (bool, unit passes gradient) and "conv<i>.argmax" (int32,
    same convention as maxpool_forward).  Missing keys, or decisions=None, mean
    the choices this forward pass made itself.  A caller that passes choices
    made elsewhere is responsible for checking them against cache["<layer>.z"]
    and the pooled inputs (they may differ only where those are tied to within
    rounding)."""
    z, cache = _forward_stack(spec, params, x, masks, train=True)
    if callable(decisions):  # lets a caller inspect this forward pass before fixing the choices
        decisions = decisions(cache)
    decisions = decisions or {}
    loss, p, dz = softmax_xent(z, labels)
    cache["probs"] = p
    grads = {}
    d = dz
    nfc = len(spec.fc)
    for j in reversed(range(nfc)):
        name = f"fc{len(spec.conv)+1+j}"
        if j < nfc - 1:
            # ReLU and dropout: act>0 iff kept and positive
            d = d * decisions.get(name + ".gate", cache[name + ".act"] > 0)
        dx, dw, db = fc_backward(cache[name + ".in"], params[name + ".w"], d)
        grads[name + ".w"], grads[name + ".b"] = dw, db
        d = dx
    d = d.reshape(cache["flat_shape"])
    for i in reversed(range(len(spec.conv))):
        cv = spec.conv[i]
        name = f"conv{i+1}"
        if cv.pool:
            d = maxpool_backward(d, decisions.get(name + ".argmax", cache[name + ".argmax"]), cache[name + ".pool_in_hw"])
        if cv.lrn:
            d = lrn_backward(d, cache[name + ".act"], cache[name + ".lrn_s"], spec.lrn_n, spec.lrn_alpha, spec.lrn_beta)
        d = d * decisions.get(name + ".gate", cache[name + ".act"] > 0)
        cache[name + ".dact"] = d
        xin = cache[name + ".in"]
        dw, db = conv_backward_weight(xin, d, cv.k, cv.stride, cv.pad, cv.groups)
        grads[name + ".w"], grads[name + ".b"] = dw, db
        if i > 0 or want_dx:
            d = conv_backward_data(d, params[name + ".w"], xin.shape[2:], cv.stride, cv.pad, cv.groups)
    if want_dx:
        cache["dx"] = d
    return loss, grads, cache


def train_step(spec: NetSpec, params, momentum, x, labels, step: int, masks=None, decisions=None):
    """One SGD iteration.  Returns (loss, new_params, new_momentum, grads, cache).
    Weight decay applies to weight tensors only; biases decay with 0.
    `decisions`: see loss_and_grads."""
    if masks is None:
        widths = spec.fc[:-1]
        masks = [dropout_mask(spec, step, tag, wd_) for tag, wd_ in zip((TAG_DROP6, TAG_DROP7), widths)]
    loss, grads, cache = loss_and_grads(spec, params, x, labels, masks, decisions=decisions)
    new_p, new_v = {}, {}
    for kname in param_shapes(spec):
        wd = spec.weight_decay if kname.endswith(".w") else 0.0
        new_p[kname], new_v[kname] = sgd_update(params[kname], momentum[kname], grads[kname],
                                                 spec.lr, spec.momentum, wd)
    cache["masks"] = masks
    return loss, new_p, new_v, grads, cache
