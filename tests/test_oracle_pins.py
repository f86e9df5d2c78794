"""CPU-only pins for the float64 oracle: brute force, closed forms, adjoint
identities, finite differences, published vectors and torch-CPU float64
library routines.  None of these use the HIP path."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synthetic_inputs as S
from helpers import oracle_spec, to64
from oracle import alexnet_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


# ------------------------------------------------------------------ RNG ---

def test_mix64_matches_published_splitmix64_vectors():
    want = [int(l) for l in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) if l.strip() and l[0] != "#"]
    state = np.uint64(1234567)
    got = []
    with np.errstate(over="ignore"):
        for _ in want:
            state = state + np.uint64(0x9E3779B97F4A7C15)
            got.append(int(O.mix64(state)))
    assert got == want


def test_mix64_python_int_reimplementation():
    m = (1 << 64) - 1

    def ref(z):
        z ^= z >> 30
        z = (z * 0xBF58476D1CE4E5B9) & m
        z ^= z >> 27
        z = (z * 0x94D049BB133111EB) & m
        return z ^ (z >> 31)

    seed, step = 987654321, 17
    k0 = ref((seed + 0x9E3779B97F4A7C15) & m)
    k1 = ref(k0 ^ step)
    for tag, idx in [(1, 0), (3, 5), (6, 123456), (7, 4095 * 128 + 3)]:
        assert int(O.rand_u64(seed, step, tag, idx)) == ref(k1 ^ (tag << 56) ^ idx)


def test_crop_flip_ranges_and_dropout_rate():
    spec = oracle_spec(S.ALEXNET, 128, seed=99)
    seen_x, seen_f = set(), set()
    for step in range(20):
        ox, oy, fl = O.crop_flip_params(spec, step)
        assert ox.min() >= 0 and ox.max() <= 29 and oy.min() >= 0 and oy.max() <= 29
        assert set(np.unique(fl)) <= {0, 1}
        seen_x |= set(ox.tolist())
        seen_f |= set(fl.tolist())
    assert seen_x == set(range(30)) and seen_f == {0, 1}
    m = O.dropout_mask(spec, 3, O.TAG_DROP6, 4096)
    assert m.shape == (128, 4096) and set(np.unique(m)) == {0.0, 1.0}
    assert abs(m.mean() - 0.5) < 5e-3
    # different step / tag => different mask; same arguments => same mask
    assert np.array_equal(m, O.dropout_mask(spec, 3, O.TAG_DROP6, 4096))
    assert not np.array_equal(m, O.dropout_mask(spec, 4, O.TAG_DROP6, 4096))
    assert not np.array_equal(m, O.dropout_mask(spec, 3, O.TAG_DROP7, 4096))
    spec.dropout_p = 0.25
    assert abs(O.dropout_mask(spec, 3, O.TAG_DROP6, 4096).mean() - 0.75) < 5e-3


# ----------------------------------------------------------- preprocess ---

def test_preprocess_bruteforce_and_special_cases():
    b, c, h, w, ch = 3, 3, 12, 12, 7
    raw = rng.integers(0, 256, size=(b, c, h, w), dtype=np.uint8)
    mean = rng.uniform(100, 140, size=(c, h, w))
    ox = np.array([0, 5, 2]); oy = np.array([0, 1, 5]); fl = np.array([0, 1, 1])
    out = O.preprocess(raw, mean, ox, oy, fl, ch, ch)
    for n in range(b):
        for k in range(c):
            for y in range(ch):
                for x in range(ch):
                    sx = ox[n] + (ch - 1 - x if fl[n] else x)
                    sy = oy[n] + y
                    assert out[n, k, y, x] == float(raw[n, k, sy, sx]) - mean[k, sy, sx]
    # crop at (0,0), no flip = top-left block of raw - mean
    assert np.array_equal(out[0], raw[0, :, :ch, :ch].astype(np.float64) - mean[:, :ch, :ch])
    # flipping twice is the identity
    once = O.preprocess(raw, mean, ox, oy, np.ones(b, int), ch, ch)
    assert np.array_equal(once[:, :, :, ::-1], O.preprocess(raw, mean, ox, oy, np.zeros(b, int), ch, ch))


# ----------------------------------------------------------------- conv ---

def direct_conv(x, w, b, stride, pad, groups):
    n, cin, h, wd = x.shape
    cout, cg, k, _ = w.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    og = cout // groups
    y = np.zeros((n, cout, ho, wo))
    for i in range(n):
        for o in range(cout):
            g = o // og
            for yy in range(ho):
                for xx in range(wo):
                    acc = b[o]
                    for c in range(cg):
                        for r in range(k):
                            for s in range(k):
                                iy, ix = yy * stride + r - pad, xx * stride + s - pad
                                if 0 <= iy < h and 0 <= ix < wd:
                                    acc += w[o, c, r, s] * x[i, g * cg + c, iy, ix]
                    y[i, o, yy, xx] = acc
    return y


CONV_CASES = [
    # n, cin, h, w, cout, k, stride, pad, groups
    (2, 3, 15, 15, 4, 11, 4, 0, 1),
    (2, 4, 7, 7, 6, 5, 1, 2, 2),
    (1, 4, 5, 6, 4, 3, 1, 1, 1),
    (2, 6, 5, 5, 4, 3, 1, 1, 2),
    (1, 2, 9, 8, 2, 3, 2, 1, 1),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_forward_bruteforce(case):
    n, cin, h, w, cout, k, st, pd, g = case
    x = rng.standard_normal((n, cin, h, w))
    wt = rng.standard_normal((cout, cin // g, k, k))
    b = rng.standard_normal(cout)
    np.testing.assert_allclose(O.conv_forward(x, wt, b, st, pd, g), direct_conv(x, wt, b, st, pd, g), rtol=1e-12, atol=1e-12)


def test_conv_special_cases():
    x = rng.standard_normal((2, 5, 6, 7))
    # 1x1 stride-1 conv is a matrix product over channels
    w = rng.standard_normal((4, 5, 1, 1))
    want = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(O.conv_forward(x, w, np.zeros(4), 1, 0, 1), want, rtol=1e-12, atol=1e-12)
    # a delta kernel at tap (0, 2) with pad 1 shifts the picture: y[i,j] = x[i-1, j+1]
    wd = np.zeros((5, 1, 3, 3)); wd[:, 0, 0, 2] = 1.0
    y = O.conv_forward(x, wd, None, 1, 1, 5)
    want = np.zeros_like(x); want[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(y, want)
    # groups = g equals g independent convolutions, concatenated
    w2 = rng.standard_normal((6, 2, 3, 3)); xb = rng.standard_normal((2, 4, 6, 6)); b2 = rng.standard_normal(6)
    parts = [O.conv_forward(xb[:, 2 * g:2 * g + 2], w2[3 * g:3 * g + 3], b2[3 * g:3 * g + 3], 1, 1, 1) for g in range(2)]
    np.testing.assert_allclose(O.conv_forward(xb, w2, b2, 1, 1, 2), np.concatenate(parts, 1), rtol=1e-13)


@pytest.mark.parametrize("case", CONV_CASES + [(3, 8, 13, 13, 12, 3, 1, 1, 2), (9, 3, 31, 31, 8, 7, 2, 0, 1)])
def test_conv_all_three_match_torch_cpu_float64(case):
    n, cin, h, w, cout, k, st, pd, g = case
    x = rng.standard_normal((n, cin, h, w)); wt = rng.standard_normal((cout, cin // g, k, k)); b = rng.standard_normal(cout)
    xt = torch.tensor(x, requires_grad=True); wtt = torch.tensor(wt, requires_grad=True); bt = torch.tensor(b, requires_grad=True)
    yt = F.conv2d(xt, wtt, bt, stride=st, padding=pd, groups=g)
    y = O.conv_forward(x, wt, b, st, pd, g, chunk=4)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-11)
    dy = rng.standard_normal(y.shape)
    yt.backward(torch.tensor(dy))
    dw, db = O.conv_backward_weight(x, dy, k, st, pd, g, chunk=4)
    dx = O.conv_backward_data(dy, wt, (h, w), st, pd, g, chunk=4)
    np.testing.assert_allclose(dw, wtt.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identities(case):
    n, cin, h, w, cout, k, st, pd, g = case
    x = rng.standard_normal((n, cin, h, w)); wt = rng.standard_normal((cout, cin // g, k, k))
    y = O.conv_forward(x, wt, None, st, pd, g)
    dy = rng.standard_normal(y.shape)
    lhs = float((y * dy).sum())
    dx = O.conv_backward_data(dy, wt, (h, w), st, pd, g)
    dw, db = O.conv_backward_weight(x, dy, k, st, pd, g)
    assert abs(lhs - float((x * dx).sum())) <= 1e-10 * max(1.0, abs(lhs))
    assert abs(lhs - float((wt * dw).sum())) <= 1e-10 * max(1.0, abs(lhs))
    np.testing.assert_allclose(db, dy.sum((0, 2, 3)), rtol=1e-12)


def test_conv_finite_differences():
    n, cin, h, w, cout, k, st, pd, g = 2, 4, 7, 7, 6, 5, 1, 2, 2
    x = rng.standard_normal((n, cin, h, w)); wt = rng.standard_normal((cout, cin // g, k, k)); b = rng.standard_normal(cout)
    dy = rng.standard_normal((n, cout, h, w))
    f = lambda x_, w_: float((O.conv_forward(x_, w_, b, st, pd, g) * dy).sum())
    dx = O.conv_backward_data(dy, wt, (h, w), st, pd, g); dw, _ = O.conv_backward_weight(x, dy, k, st, pd, g)
    eps = 1e-5
    for _ in range(10):
        i = tuple(rng.integers(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy(); xp[i] += eps; xm[i] -= eps
        assert abs((f(xp, wt) - f(xm, wt)) / (2 * eps) - dx[i]) <= 1e-6 * max(1, abs(dx[i]))
        j = tuple(rng.integers(0, s) for s in wt.shape)
        wp, wm = wt.copy(), wt.copy(); wp[j] += eps; wm[j] -= eps
        assert abs((f(x, wp) - f(x, wm)) / (2 * eps) - dw[j]) <= 1e-6 * max(1, abs(dw[j]))


# ------------------------------------------------------------------ LRN ---

def test_lrn_closed_forms():
    a = np.abs(rng.standard_normal((2, 9, 3, 3))) * 10
    b, s = O.lrn_forward(a, 5, 2.0, 0.0, 0.75)
    np.testing.assert_allclose(b, a * 2.0 ** -0.75, rtol=1e-14)
    b, s = O.lrn_forward(a, 1, 2.0, 1e-2, 0.75)
    np.testing.assert_allclose(b, a / (2.0 + 1e-2 * a * a) ** 0.75, rtol=1e-13)
    c = np.full((1, 9, 2, 2), 3.0)
    b, s = O.lrn_forward(c, 5, 2.0, 1e-2, 0.75)
    np.testing.assert_allclose(b[:, 2:7], 3.0 / (2.0 + 5 * 1e-2 * 9.0) ** 0.75, rtol=1e-13)
    # edges: channel 0 sees 3 channels, channel 1 sees 4
    np.testing.assert_allclose(b[:, 0], 3.0 / (2.0 + 3 * 1e-2 * 9.0) ** 0.75, rtol=1e-13)
    np.testing.assert_allclose(b[:, 1], 3.0 / (2.0 + 4 * 1e-2 * 9.0) ** 0.75, rtol=1e-13)
    np.testing.assert_allclose(b[:, 8], 3.0 / (2.0 + 3 * 1e-2 * 9.0) ** 0.75, rtol=1e-13)


def test_lrn_bruteforce_window():
    a = rng.standard_normal((1, 7, 2, 2))
    b, s = O.lrn_forward(a, 5, 2.0, 0.3, 0.75)
    for i in range(7):
        tot = sum(a[0, j] ** 2 for j in range(max(0, i - 2), min(6, i + 2) + 1))
        np.testing.assert_allclose(s[0, i], 2.0 + 0.3 * tot, rtol=1e-13)


def test_lrn_matches_torch_with_alpha_times_n_and_backward():
    # torch divides alpha by the window size, so alpha*n there equals alpha here
    a = rng.standard_normal((2, 11, 4, 5)) * 3
    at = torch.tensor(a, requires_grad=True)
    bt = F.local_response_norm(at, 5, alpha=0.05 * 5, beta=0.75, k=2.0)
    b, s = O.lrn_forward(a, 5, 2.0, 0.05, 0.75)
    np.testing.assert_allclose(b, bt.detach().numpy(), rtol=1e-12, atol=1e-13)
    dy = rng.standard_normal(a.shape)
    bt.backward(torch.tensor(dy))
    np.testing.assert_allclose(O.lrn_backward(dy, a, s, 5, 0.05, 0.75), at.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_lrn_backward_finite_differences():
    a = rng.standard_normal((1, 8, 2, 2)) * 2; dy = rng.standard_normal(a.shape)
    f = lambda a_: float((O.lrn_forward(a_, 5, 2.0, 0.1, 0.75)[0] * dy).sum())
    _, s = O.lrn_forward(a, 5, 2.0, 0.1, 0.75)
    da = O.lrn_backward(dy, a, s, 5, 0.1, 0.75)
    for _ in range(12):
        i = tuple(rng.integers(0, n) for n in a.shape)
        ap, am = a.copy(), a.copy(); ap[i] += 1e-5; am[i] -= 1e-5
        assert abs((f(ap) - f(am)) / 2e-5 - da[i]) < 1e-7


# ----------------------------------------------------------------- pool ---

def test_maxpool_bruteforce_ties_and_backward():
    x = rng.standard_normal((2, 3, 9, 8))
    x[0, 0, :4, :4] = 0.0          # all-equal windows
    x[1, 2] = np.round(x[1, 2])    # many ties
    y, arg = O.maxpool_forward(x, 3, 2)
    n, c, h, w = x.shape
    ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
    assert y.shape == (n, c, ho, wo) and arg.dtype == np.int32
    for i in range(n):
        for j in range(c):
            for yy in range(ho):
                for xx in range(wo):
                    best, bi = None, -1
                    for r in range(3):
                        for s in range(3):
                            v = x[i, j, 2 * yy + r, 2 * xx + s]
                            if best is None or v > best:
                                best, bi = v, (2 * yy + r) * w + 2 * xx + s
                    assert y[i, j, yy, xx] == best and arg[i, j, yy, xx] == bi
    assert arg[0, 0, 0, 0] == 0  # all-zero window -> top-left tap
    dy = rng.standard_normal(y.shape)
    dx = O.maxpool_backward(dy, arg, (h, w))
    np.testing.assert_allclose(dx.sum(), dy.sum(), rtol=1e-12)
    mask = np.zeros((n, c, h * w), bool)
    for i in range(n):
        for j in range(c):
            mask[i, j, arg[i, j].ravel()] = True
    assert np.all(dx.reshape(n, c, -1)[~mask] == 0)


def test_maxpool_matches_torch_on_tie_free_input():
    x = rng.standard_normal((2, 4, 13, 13))
    xt = torch.tensor(x, requires_grad=True)
    yt, it = F.max_pool2d(xt, 3, 2, return_indices=True)
    y, arg = O.maxpool_forward(x, 3, 2)
    assert np.array_equal(y, yt.detach().numpy()) and np.array_equal(arg, it.numpy().astype(np.int32))
    dy = rng.standard_normal(y.shape)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(O.maxpool_backward(dy, arg, (13, 13)), xt.grad.numpy(), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------- fc / softmax -----

def test_fc_adjoint_and_definition():
    x = rng.standard_normal((5, 7)); w = rng.standard_normal((4, 7)); b = rng.standard_normal(4)
    y = O.fc_forward(x, w, b)
    for n in range(5):
        for o in range(4):
            assert abs(y[n, o] - (sum(x[n, i] * w[o, i] for i in range(7)) + b[o])) < 1e-12
    dy = rng.standard_normal(y.shape)
    dx, dw, db = O.fc_backward(x, w, dy)
    lhs = float(((y - b) * dy).sum())
    assert abs(lhs - float((x * dx).sum())) < 1e-10 and abs(lhs - float((w * dw).sum())) < 1e-10
    np.testing.assert_allclose(db, dy.sum(0))


def test_softmax_xent_properties_and_torch():
    z = rng.standard_normal((6, 10)) * 5; lab = rng.integers(0, 10, 6)
    loss, p, dz = O.softmax_xent(z, lab)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(dz.sum(1), 0.0, atol=1e-15)
    l0, _, _ = O.softmax_xent(np.zeros((4, 1000)), np.array([0, 5, 999, 7]))
    assert abs(l0 - math.log(1000)) < 1e-12
    zt = torch.tensor(z, requires_grad=True)
    lt = F.cross_entropy(zt, torch.tensor(lab))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=1e-11, atol=1e-14)
    # large logits do not overflow
    lbig, pbig, _ = O.softmax_xent(np.array([[1000.0, 0.0, -1000.0]]), np.array([0]))
    assert np.isfinite(lbig) and abs(pbig.sum() - 1) < 1e-14


# --------------------------------------------------------------- update ---

def test_update_closed_forms():
    w, v, g = 2.0, 0.5, -3.0
    wn, vn = O.sgd_update(w, v, g, 0.01, 0.9, 5e-4)
    assert abs(vn - (0.9 * 0.5 - 0.01 * (-3.0 + 5e-4 * 2.0))) < 1e-15 and abs(wn - (2.0 + vn)) < 1e-15
    # the 2012 paper's form: v <- 0.9 v - 0.0005*lr*w - lr*g
    assert abs(vn - (0.9 * v - 5e-4 * 0.01 * w - 0.01 * g)) < 1e-15
    wa = rng.standard_normal(9); ga = rng.standard_normal(9)
    wn, vn = O.sgd_update(wa, np.ones(9), ga, 0.1, 0.0, 0.0)
    np.testing.assert_allclose(wn, wa - 0.1 * ga, rtol=1e-14)


# ----------------------------------------------------------- whole net ----

def _mini_problem(batch, seed=0, bias=0.0, std=0.01):
    spec = oracle_spec(S.MINI, batch, seed=seed)
    params = to64(S.make_params(O.param_shapes(spec), S.SEED_BASE + 1, bias_value=bias, std=std))
    x, lab = S.make_float_batch(batch, 3, 63, 63, 10, S.SEED_BASE + 1)
    return spec, params, x.astype(np.float64), lab


def test_architecture_census_and_param_count():
    spec = oracle_spec(S.ALEXNET, 128)
    assert len(spec.conv) == 5 and sum(c.pool for c in spec.conv) == 3 and len(spec.fc) == 3
    stages, flat = O.layer_shapes(spec)
    assert [s["conv"] for s in stages] == [(96, 55, 55), (256, 27, 27), (384, 13, 13), (384, 13, 13), (256, 13, 13)]
    assert flat == 9216
    shapes = O.param_shapes(spec)
    assert sum(int(np.prod(s)) for s in shapes.values()) == 60965224
    assert O.n_weight_elems(spec) == 60965224 - (96 + 256 + 384 + 384 + 256 + 4096 + 4096 + 1000)
    mini = oracle_spec(S.MINI, 4)
    assert O.layer_shapes(mini)[1] == 128
    assert O.param_shapes(mini)["fc6.w"] == (256, 128)


def test_initial_loss_is_log_classes():
    spec, params, x, lab = _mini_problem(4)
    loss, *_ = O.train_step(spec, params, {k: np.zeros_like(v) for k, v in params.items()}, x, lab, 0)
    assert abs(loss - math.log(10)) < 1e-3


def _torch_net(spec, params, x, lab, masks):
    tp = {k: torch.tensor(v, requires_grad=True) for k, v in params.items()}
    h = torch.tensor(x)
    for i, cv in enumerate(spec.conv):
        h = F.relu(F.conv2d(h, tp[f"conv{i+1}.w"], tp[f"conv{i+1}.b"], stride=cv.stride, padding=cv.pad, groups=cv.groups))
        if cv.lrn:
            h = F.local_response_norm(h, spec.lrn_n, alpha=spec.lrn_alpha * spec.lrn_n, beta=spec.lrn_beta, k=spec.lrn_k)
        if cv.pool:
            h = F.max_pool2d(h, 3, 2)
    h = h.flatten(1)
    for j in range(3):
        h = F.linear(h, tp[f"fc{6+j}.w"], tp[f"fc{6+j}.b"])
        if j < 2:
            h = F.relu(h) * torch.tensor(masks[j])
    loss = F.cross_entropy(h, torch.tensor(lab).long())
    loss.backward()
    return loss.item(), {k: v.grad.numpy() for k, v in tp.items()}


def test_whole_step_gradients_match_torch_autograd():
    # larger weights and non-zero biases so every layer carries signal
    spec, params, x, lab = _mini_problem(3, seed=5, bias=0.1, std=0.08)
    masks = [O.dropout_mask(spec, 2, t, w) for t, w in ((O.TAG_DROP6, 256), (O.TAG_DROP7, 256))]
    loss, grads, _ = O.loss_and_grads(spec, params, x, lab, masks)
    tl, tg = _torch_net(spec, params, x, lab, masks)
    assert abs(loss - tl) < 1e-12
    for k in grads:
        assert np.linalg.norm(tg[k]) > 0, k
        np.testing.assert_allclose(grads[k], tg[k], rtol=1e-8, atol=1e-12 * max(1.0, np.abs(tg[k]).max()), err_msg=k)


def test_whole_step_finite_differences():
    spec, params, x, lab = _mini_problem(2, seed=5, bias=0.1, std=0.08)
    masks = [O.dropout_mask(spec, 0, t, w) for t, w in ((O.TAG_DROP6, 256), (O.TAG_DROP7, 256))]
    loss, grads, _ = O.loss_and_grads(spec, params, x, lab, masks)
    r = np.random.default_rng(3)
    eps = 1e-6
    checked = 0
    for k in ["conv1.w", "conv2.w", "conv3.b", "conv5.w", "fc6.w", "fc7.b", "fc8.w"]:
        for _ in range(3):
            i = tuple(r.integers(0, n) for n in params[k].shape)
            pp = {a: b.copy() for a, b in params.items()}; pm = {a: b.copy() for a, b in params.items()}
            pp[k][i] += eps; pm[k][i] -= eps
            lp = O.loss_and_grads(spec, pp, x, lab, masks)[0]; lm = O.loss_and_grads(spec, pm, x, lab, masks)[0]
            fd = (lp - lm) / (2 * eps)
            second = abs(lp - 2 * loss + lm) / eps ** 2  # kinks show up as a huge second difference
            if second > 1e3:
                continue
            assert abs(fd - grads[k][i]) <= 1e-6 * max(1.0, abs(grads[k][i])) + 1e-8, (k, i, fd, grads[k][i])
            checked += 1
    assert checked >= 15


def test_train_step_applies_update_and_decay_only_on_weights():
    spec, params, x, lab = _mini_problem(2, bias=0.3)
    mom = to64(S.make_random_like(O.param_shapes(spec), 11, std=0.01))
    loss, newp, newv, grads, _ = O.train_step(spec, params, mom, x, lab, 4)
    for k in params:
        wd = 5e-4 if k.endswith(".w") else 0.0
        v = 0.9 * mom[k] - 0.01 * (grads[k] + wd * params[k])
        np.testing.assert_allclose(newv[k], v, rtol=1e-13, atol=1e-18)
        np.testing.assert_allclose(newp[k], params[k] + v, rtol=1e-13, atol=1e-18)


def test_inference_scales_dropout_layers_by_keep_probability():
    spec, params, x, lab = _mini_problem(2, bias=0.1, std=0.08)
    p = O.forward(spec, params, x)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=1e-14)
    ones = [np.ones((2, 256)), np.ones((2, 256))]
    half = {k: v.copy() for k, v in params.items()}
    # keep-probability scaling of fc6/fc7 activations == halving fc7/fc8 weights with all-ones masks
    half["fc7.w"] *= 0.5; half["fc8.w"] *= 0.5
    z, _ = O._forward_stack(spec, half, x, ones, train=True)
    e = np.exp(z - z.max(1, keepdims=True)); q = e / e.sum(1, keepdims=True)
    np.testing.assert_allclose(p, q, rtol=1e-12)


# ---------------------------------------------------- two replicas (2.2) --

def test_identical_replicas_stay_identical_and_unchanged():
    a = rng.standard_normal(1000)
    assert np.array_equal(O.average_replicas(a, a.copy()), a)


def test_two_half_batches_plus_average_equal_one_full_batch():
    """Section 3 states batch 256 on one GPU is equivalent to 2 x 128: the
    update is affine in the gradient and the loss is a minibatch mean."""
    b = 2
    specA = oracle_spec(S.MINI, b, seed=1); specB = oracle_spec(S.MINI, b, seed=2); specAB = oracle_spec(S.MINI, 2 * b)
    params = to64(S.make_params(O.param_shapes(specA), 3, bias_value=0.1, std=0.08))
    mom = to64(S.make_random_like(O.param_shapes(specA), 4, std=0.01))
    xa, la = S.make_float_batch(b, 3, 63, 63, 10, 100); xb, lb = S.make_float_batch(b, 3, 63, 63, 10, 200)
    _, pa, va, ga, ca = O.train_step(specA, params, mom, xa, la, 0)
    _, pb, vb, gb, cb = O.train_step(specB, params, mom, xb, lb, 0)
    masks = [np.concatenate([ca["masks"][j], cb["masks"][j]]) for j in range(2)]
    _, pab, vab, gab, _ = O.train_step(specAB, params, mom, np.concatenate([xa, xb]), np.concatenate([la, lb]), 0, masks=masks)
    for k in params:
        np.testing.assert_allclose(O.average_replicas(pa[k], pb[k]), pab[k], rtol=1e-10, atol=1e-15, err_msg=k)
        np.testing.assert_allclose(O.average_replicas(va[k], vb[k]), vab[k], rtol=1e-10, atol=1e-15, err_msg=k)


def test_gradient_exchange_equals_parameter_exchange_for_identical_replicas():
    """Update-then-average (Section 2.2) and average-the-gradients-then-update agree when both
    replicas start from the same weights and momentum, and agree with one step on the joint batch."""
    b = 2
    specA = oracle_spec(S.MINI, b, seed=1); specB = oracle_spec(S.MINI, b, seed=2); specAB = oracle_spec(S.MINI, 2 * b)
    params = to64(S.make_params(O.param_shapes(specA), 3, bias_value=0.1, std=0.08))
    mom = to64(S.make_random_like(O.param_shapes(specA), 4, std=0.01))
    xa, la = S.make_float_batch(b, 3, 63, 63, 10, 100); xb, lb = S.make_float_batch(b, 3, 63, 63, 10, 200)
    _, pa, va, ga, ca = O.train_step(specA, params, mom, xa, la, 0)
    _, pb, vb, gb, cb = O.train_step(specB, params, mom, xb, lb, 0)
    masks = [np.concatenate([ca["masks"][j], cb["masks"][j]]) for j in range(2)]
    _, pab, vab, _, _ = O.train_step(specAB, params, mom, np.concatenate([xa, xb]), np.concatenate([la, lb]), 0, masks=masks)
    for k in params:
        wd = specA.weight_decay if k.endswith(".w") else 0.0
        (wa2, va2), (wb2, vb2) = O.averaged_gradient_update(params[k], mom[k], ga[k], params[k], mom[k], gb[k],
                                                            specA.lr, specA.momentum, wd)
        assert np.array_equal(wa2, wb2) and np.array_equal(va2, vb2)
        np.testing.assert_allclose(wa2, O.average_replicas(pa[k], pb[k]), rtol=1e-12, atol=1e-15, err_msg=k)
        np.testing.assert_allclose(va2, O.average_replicas(va[k], vb[k]), rtol=1e-12, atol=1e-15, err_msg=k)
        np.testing.assert_allclose(wa2, pab[k], rtol=1e-10, atol=1e-15, err_msg=k)


def test_gradient_exchange_by_hand_for_replicas_that_differ():
    # lr 0.5, mu 0.5, wd 0.25; replica a: w 2, v 4, g 1; replica b: w -1, v 0, g 3 -> mean gradient 2
    (wa, va), (wb, vb) = O.averaged_gradient_update(np.array([2.0]), np.array([4.0]), np.array([1.0]),
                                                    np.array([-1.0]), np.array([0.0]), np.array([3.0]), 0.5, 0.5, 0.25)
    assert va[0] == 0.5 * 4.0 - 0.5 * (2.0 + 0.25 * 2.0) and wa[0] == 2.0 + va[0]      # 0.75, 2.75
    assert vb[0] == 0.0 - 0.5 * (2.0 + 0.25 * -1.0) and wb[0] == -1.0 + vb[0]          # -0.875, -1.875
    assert (va[0], wa[0], vb[0], wb[0]) == (0.75, 2.75, -0.875, -1.875)


def test_topk_count_against_sorting_and_ties():
    scores = rng.standard_normal((50, 17))
    labels = rng.integers(0, 17, size=50)
    order = np.argsort(-scores, axis=1, kind="stable")  # continuous draws: no ties
    for k in (1, 3, 5, 17):
        want = sum(int(labels[i] in order[i, :k]) for i in range(50))
        assert O.topk_correct(scores, labels, k) == want
    assert O.topk_correct(scores, labels, 17) == 50
    tied = np.array([[1.0, 1.0, 1.0, 0.0], [2.0, 1.0, 1.0, 1.0], [0.0, 3.0, 2.0, 1.0]])
    # row 0: nothing beats the label (tie goes to the label); row 1: label 3 is beaten by one class;
    # row 2: label 0 is beaten by three
    assert O.topk_correct(tied, np.array([2, 3, 0]), 1) == 1
    assert O.topk_correct(tied, np.array([2, 3, 0]), 2) == 2
    assert O.topk_correct(tied, np.array([2, 3, 0]), 4) == 3


def test_center_crop_offsets():
    spec = oracle_spec(S.ALEXNET, 3)
    ox, oy, fl = O.center_crop_params(spec)
    assert ox.tolist() == [14, 14, 14] and oy.tolist() == [14, 14, 14] and fl.tolist() == [0, 0, 0]  # (256-227)//2
    raw = np.arange(3 * 3 * 256 * 256, dtype=np.int64).reshape(3, 3, 256, 256) % 251
    out = O.preprocess(raw.astype(np.uint8), np.zeros((3, 256, 256)), ox, oy, fl, 227, 227)
    assert np.array_equal(out, raw[:, :, 14:241, 14:241].astype(np.float64))


def test_flatten_roundtrip_and_order():
    spec = oracle_spec(S.MINI, 2)
    shapes = O.param_shapes(spec)
    names = list(shapes)
    assert names[:8] == [f"conv{i}.w" for i in range(1, 6)] + ["fc6.w", "fc7.w", "fc8.w"]
    assert names[8:] == [f"conv{i}.b" for i in range(1, 6)] + ["fc6.b", "fc7.b", "fc8.b"]
    p = to64(S.make_random_like(shapes, 1))
    flat = O.flatten_params(spec, p)
    back = O.unflatten_params(spec, flat)
    assert all(np.array_equal(back[k], p[k]) for k in p)
