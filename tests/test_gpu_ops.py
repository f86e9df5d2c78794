"""Per-operator GPU parity on seeded synthetic inputs (including tie-heavy
ones), each through its own C-ABI entry point."""
import numpy as np
import pytest

import synthetic_inputs as S
from gpu_common import cuda
from helpers import oracle_spec, rel_l2
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu
OP_RTOL = 2e-5  # one fp32 operator against float64 on identical inputs


def _tie_heavy(shape, seed):
    """Values on a coarse grid with zero blocks: every pooling window has ties."""
    rng = np.random.default_rng(seed)
    x = np.round(rng.standard_normal(shape) * 2).astype(np.float32) / 2
    x[..., : shape[-2] // 2, : shape[-1] // 3] = 0.0
    return np.maximum(x, 0)


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 3), (S.ODD, 3), (S.ALEXNET, 128)])
def test_pool_forward_backward_bit_exact_decisions(lib, wl, batch):
    net = lib.AlexNet(wl, batch)
    spec = oracle_spec(wl, batch)
    stages, _ = O.layer_shapes(spec)
    for li, (cv, st) in enumerate(zip(spec.conv, stages), start=1):
        if not cv.pool:
            continue
        c, h, w = st["conv"]
        for kind, x in (("ties", _tie_heavy((batch, c, h, w), 100 + li)), ("normal", S.make_normal((batch, c, h, w), 200 + li))):
            y, arg = net.pool_forward(li, x)
            want_y, want_a = O.maxpool_forward(x, 3, 2)
            assert np.array_equal(y.cpu().numpy(), want_y), (li, kind)
            assert np.array_equal(arg.cpu().numpy(), want_a), (li, kind)
            dy = S.make_normal(want_y.shape, 300 + li)
            dx = net.pool_backward(li, x, dy, relu_gate=False).cpu().numpy()
            want_dx = O.maxpool_backward(dy, want_a, (h, w))
            assert rel_l2(dx, want_dx) <= OP_RTOL, (li, kind)
            assert np.all(dx[want_dx == 0] == 0)
            dxg = net.pool_backward(li, x, dy, relu_gate=True).cpu().numpy()
            assert rel_l2(dxg, want_dx * (x > 0)) <= OP_RTOL, (li, kind)
    net.close()


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 3), (S.ODD, 3), (S.ALEXNET, 16)])
def test_lrn_forward_backward(lib, wl, batch):
    net = lib.AlexNet(wl, batch)
    spec = oracle_spec(wl, batch)
    stages, _ = O.layer_shapes(spec)
    for li, (cv, st) in enumerate(zip(spec.conv, stages), start=1):
        if not cv.lrn:
            continue
        c, h, w = st["conv"]
        # large activations so the normalisation term matters: alpha*sum(a^2) ~ O(1)
        a = np.maximum(S.make_normal((batch, c, h, w), 400 + li, std=60.0), 0)
        b = net.lrn_forward(li, a).cpu().numpy()
        want_b, s = O.lrn_forward(a, spec.lrn_n, spec.lrn_k, spec.lrn_alpha, spec.lrn_beta)
        assert float(s.max()) > 2.5
        assert rel_l2(b, want_b) <= OP_RTOL, li
        db = S.make_normal(a.shape, 500 + li)
        want_da = O.lrn_backward(db, a, s, spec.lrn_n, spec.lrn_alpha, spec.lrn_beta)
        da = net.lrn_backward(li, a, db, relu_gate=False).cpu().numpy()
        assert rel_l2(da, want_da) <= OP_RTOL, li
        dag = net.lrn_backward(li, a, db, relu_gate=True).cpu().numpy()
        assert rel_l2(dag, want_da * (a > 0)) <= OP_RTOL, li
    net.close()


def _lrn_tie_heavy(shape, seed):
    """Post-ReLU activations whose *normalised* values tie exactly inside pooling windows: zero blocks
    (all-zero windows: the first tap must win), and whole pixels (all channels) copied onto their right
    and lower neighbours, so that equal channel vectors give bit-equal normalised values in one window."""
    rng = np.random.default_rng(seed)
    a = np.maximum(rng.standard_normal(shape).astype(np.float32) * 40.0, 0)
    n, c, h, w = shape
    a[:, :, : h // 3, : w // 2] = 0.0
    a[:, :, 1::4, :] = a[:, :, 0:h - 1:4, :][:, :, : a[:, :, 1::4, :].shape[2], :]   # row y+1 := row y
    a[:, :, :, 2::5] = a[:, :, :, 1:w - 1:5][:, :, :, : a[:, :, :, 2::5].shape[3]]   # column x+1 := column x
    return a


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 3), (S.TINY, 2), (S.ALEXNET, 128)])
def test_fused_lrn_pool_kernels_of_the_training_step(lib, wl, batch):
    """The kernels a training step runs for conv1 and conv2 -- normalisation + pool in one pass, and pool
    adjoint + normalisation adjoint + ReLU gate + bias sums in one pass -- through entry points of their
    own, at the layers' real shapes.
    Forward: the pooled values and winning taps must be, bit for bit, the oracle's first-maximum pool of the
    fp32 normalised tensor (which the separate normalisation kernel gives, itself within 2e-5 of the float64
    normalisation); the inputs tie exactly in most windows.
    Backward: against the float64 adjoints evaluated with those same winners."""
    net = lib.AlexNet(wl, batch)
    spec = oracle_spec(wl, batch)
    stages, _ = O.layer_shapes(spec)
    ran = 0
    for li, (cv, st) in enumerate(zip(spec.conv, stages), start=1):
        if not (cv.lrn and cv.pool):
            continue
        c, h, w = st["conv"]
        for kind, a in (("ties", _lrn_tie_heavy((batch, c, h, w), 900 + li)),
                        ("normal", np.maximum(S.make_normal((batch, c, h, w), 910 + li, std=60.0), 0))):
            try:
                y, arg = net.lrn_pool_forward(li, a)
            except lib.AlexNetError as e:
                assert e.code == lib.ENOTIMPL and c % 4, (li, str(e))  # only channel counts the kernel cannot take
                continue
            ran += 1
            y, arg = y.cpu().numpy(), arg.cpu().numpy()
            b32 = net.lrn_forward(li, a).cpu().numpy()
            want_b, s = O.lrn_forward(a, spec.lrn_n, spec.lrn_k, spec.lrn_alpha, spec.lrn_beta)
            assert rel_l2(b32, want_b) <= OP_RTOL, (li, kind)
            want_y, want_arg = O.maxpool_forward(b32, 3, 2)
            if kind == "ties":  # the input really ties: most windows hold their maximum more than once
                taps = np.stack([b32[:, :, r:r + 2 * want_y.shape[2]:2, q:q + 2 * want_y.shape[3]:2]
                                 for r in range(3) for q in range(3)])
                assert ((taps == want_y[None]).sum(0) > 1).mean() > 0.3
            assert np.array_equal(y, want_y), (li, kind, "pooled values", int((y != want_y).sum()), y.size,
                                               float(np.abs(y - want_y).max()), float(np.abs(want_y).max()))
            assert np.array_equal(arg, want_arg), (li, kind, "winning taps")
            assert rel_l2(y, O.maxpool_forward(want_b, 3, 2)[0]) <= OP_RTOL, (li, kind)
            dy = S.make_normal(want_y.shape, 920 + li)
            for gate in (True, False):
                da, db = net.pool_lrn_backward(li, a, dy, relu_gate=gate)
                da, db = da.cpu().numpy(), db.cpu().numpy()
                d = O.maxpool_backward(dy, want_arg, (h, w))
                want_da = O.lrn_backward(d, a, s, spec.lrn_n, spec.lrn_alpha, spec.lrn_beta)
                if gate:
                    want_da = want_da * (a > 0)
                assert rel_l2(da, want_da) <= OP_RTOL, (li, kind, gate, rel_l2(da, want_da))
                assert rel_l2(db, want_da.sum((0, 2, 3))) <= OP_RTOL, (li, kind, gate)
                if gate:
                    assert np.all(da[a <= 0] == 0)
                # and the two-kernel route of the single operators gives the same numbers
                d32 = net.pool_backward(li, b32, dy, relu_gate=False)
                da2 = net.lrn_backward(li, a, d32, relu_gate=gate).cpu().numpy()
                assert rel_l2(da, da2) <= 1e-6, (li, kind, gate)
    assert ran >= 2 or wl is not S.ALEXNET
    net.close()


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 7), (S.ODD, 3), (S.ALEXNET, 128)])
def test_dense_layers_alone(lib, wl, batch):
    net = lib.AlexNet(wl, batch)
    spec = oracle_spec(wl, batch)
    _, flat = O.layer_shapes(spec)
    fin = flat
    for j, fo in enumerate(spec.fc):
        layer = 6 + j
        x = S.make_normal((batch, fin), 600 + j)
        w = S.make_normal((fo, fin), 610 + j, std=0.05)
        b = S.make_normal((fo,), 620 + j)
        dy = S.make_normal((batch, fo), 630 + j)
        y = net.fc_forward(layer, x, w, b, relu=False).cpu().numpy()
        want = O.fc_forward(x, w, b)
        assert rel_l2(y, want) <= OP_RTOL, layer
        yr = net.fc_forward(layer, x, w, b, relu=True).cpu().numpy()
        assert rel_l2(yr, np.maximum(want, 0)) <= OP_RTOL
        dx, dw, db = net.fc_backward(layer, x, w, dy)
        wdx, wdw, wdb = O.fc_backward(x, w, dy)
        assert rel_l2(dx.cpu().numpy(), wdx) <= OP_RTOL and rel_l2(dw.cpu().numpy(), wdw) <= OP_RTOL, layer
        assert rel_l2(db.cpu().numpy(), wdb) <= OP_RTOL
        fin = fo
    net.close()


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.ALEXNET, 128)])
def test_softmax_cross_entropy(lib, wl, batch):
    net = lib.AlexNet(wl, batch)
    classes = wl["fc"][-1]
    z = S.make_normal((batch, classes), 700, std=4.0)
    z[0, :] = 80.0 * np.sign(z[0, :])  # large logits must not overflow
    labels = np.random.default_rng(701).integers(0, classes, batch).astype(np.int32)
    dz, loss = net.softmax_xent(z, labels)
    want_loss, p, want_dz = O.softmax_xent(z, labels)
    assert abs(float(loss.cpu().item()) - want_loss) <= 1e-5 * abs(want_loss)
    assert rel_l2(dz.cpu().numpy(), want_dz) <= OP_RTOL
    np.testing.assert_allclose(dz.cpu().numpy().sum(1), 0.0, atol=1e-6)
    net.close()


def test_update_and_average_alone(lib):
    """Momentum / weight-decay update through forward_backward + apply_update,
    and the two-replica mean, on parameters and momentum with every region non-zero."""
    batch = 4
    net = lib.AlexNet(S.MINI, batch, seed=9)
    spec = oracle_spec(S.MINI, batch, seed=9)
    shapes = O.param_shapes(spec)
    p = S.make_random_like(shapes, 800, std=0.05)
    m = S.make_random_like(shapes, 801, std=0.01)
    net.set_params(p); net.set_momentum(m)
    x, labels = S.make_float_batch(batch, 3, 63, 63, 10, 802)
    net.set_input(cuda(x), 1)
    net.forward_backward(cuda(labels), 3, slot=1)
    g = net.get_grads()
    net.apply_update()
    pn, mn = net.get_params(), net.get_momentum()
    for k in shapes:
        wd = spec.weight_decay if k.endswith(".w") else 0.0
        wp, wv = O.sgd_update(p[k], m[k], g[k], spec.lr, spec.momentum, wd)
        assert rel_l2(pn[k], wp) <= 1e-6 and rel_l2(mn[k], wv) <= 1e-6, k
    net.close()
