"""GPU parity: every call goes through the C ABI and is compared with the
float64 oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

import synthetic_inputs as S
from gpu_common import LOSS_RTOL, TENSOR_RTOL, build_pair, cuda, run_step_and_compare
from helpers import oracle_spec, rel_l2, to64
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu


def stage_io_shapes(spec):
    stages, _ = O.layer_shapes(spec)
    return stages


# ------------------------------------------------------------ layouts -------
def test_layout_roundtrip_is_bit_exact(lib):
    x = S.make_normal((3, 5, 7, 6), 1)
    y = lib.nchw_to_nhwc(cuda(x))
    assert np.array_equal(y.cpu().numpy(), np.transpose(x, (0, 2, 3, 1)))
    assert np.array_equal(lib.nhwc_to_nchw(y).cpu().numpy(), x)


def test_param_roundtrip_is_bit_exact(lib):
    net, spec, p64, _ = build_pair(lib, S.MIDI, 2, seed=3, bias=0.25, mom_std=0.1)
    got = net.get_params()
    for k in p64:
        assert np.array_equal(got[k].astype(np.float64), p64[k]), k
    mom = net.get_momentum()
    assert all(np.abs(v).sum() > 0 for v in mom.values())


# ---------------------------------------------------- single conv layers ----
def conv_flags(lib, direct):
    """ALEXNET_FLAG_DIRECT_CONV in the configuration keeps the 3x3 and 5x5 unit-stride stages on the direct
    implicit GEMM instead of the tile-transform path."""
    return lib.FLAG_DIRECT_CONV if direct else 0


@pytest.mark.parametrize("direct", [False, True], ids=["transformed3x3", "direct3x3"])
@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 5), (S.PADS, 3), (S.ODD, 3)])
def test_conv_layers_alone(lib, wl, batch, direct):
    net = lib.AlexNet(wl, batch, flags=conv_flags(lib, direct))
    spec = oracle_spec(wl, batch)
    for li, (cv, st) in enumerate(zip(spec.conv, stage_io_shapes(spec)), start=1):
        cin, h, w = st["in"]
        cout, ho, wo = st["conv"]
        x = S.make_normal((batch, cin, h, w), 10 + li)
        wt = S.make_normal((cout, cin // cv.groups, cv.k, cv.k), 20 + li, std=0.05)
        b = S.make_normal((cout,), 30 + li)
        dy = S.make_normal((batch, cout, ho, wo), 40 + li)
        y = net.conv_forward(li, x, wt, b, relu=False).cpu().numpy().reshape(batch, cout, ho, wo)
        y_ref = O.conv_forward(x, wt, b, cv.stride, cv.pad, cv.groups)
        assert rel_l2(y, y_ref) <= TENSOR_RTOL, (li, rel_l2(y, y_ref))
        yr = net.conv_forward(li, x, wt, b, relu=True).cpu().numpy().reshape(y_ref.shape)
        assert rel_l2(yr, np.maximum(y_ref, 0)) <= TENSOR_RTOL
        dx = net.conv_backward_data(li, dy, wt, x.shape).cpu().numpy()
        dx_ref = O.conv_backward_data(dy, wt, (h, w), cv.stride, cv.pad, cv.groups)
        assert rel_l2(dx, dx_ref) <= TENSOR_RTOL, (li, rel_l2(dx, dx_ref))
        dw, db = net.conv_backward_weight(li, x, dy, wt.shape)
        dw_ref, db_ref = O.conv_backward_weight(x, dy, cv.k, cv.stride, cv.pad, cv.groups)
        assert rel_l2(dw.cpu().numpy(), dw_ref) <= TENSOR_RTOL, (li, rel_l2(dw.cpu().numpy(), dw_ref))
        assert rel_l2(db.cpu().numpy(), db_ref) <= TENSOR_RTOL
    net.close()


def test_3x3_and_5x5_stages_take_the_transform_path_by_default(lib):
    """Same inputs through a default handle and through one created with ALEXNET_FLAG_DIRECT_CONV: both
    within the bar of the oracle, but not bit-identical where the default handle takes the transformed
    path -- different arithmetic -- and bit-identical elsewhere."""
    wl, batch = S.MIDI, 5
    a = lib.AlexNet(wl, batch)
    b = lib.AlexNet(wl, batch, flags=lib.FLAG_DIRECT_CONV)
    spec = oracle_spec(wl, batch)
    for li, (cv, st) in enumerate(zip(spec.conv, stage_io_shapes(spec)), start=1):
        cin, h, w = st["in"]
        cout, ho, wo = st["conv"]
        x = S.make_normal((batch, cin, h, w), 110 + li)
        wt = S.make_normal((cout, cin // cv.groups, cv.k, cv.k), 120 + li, std=0.05)
        bias = S.make_normal((cout,), 130 + li)
        dy = S.make_normal((batch, cout, ho, wo), 140 + li)
        outs = []
        for net in (a, b):
            y = net.conv_forward(li, x, wt, bias, relu=False).cpu().numpy()
            dx = net.conv_backward_data(li, dy, wt, x.shape).cpu().numpy()
            dw, _ = net.conv_backward_weight(li, x, dy, wt.shape)
            outs.append((y, dx, dw.cpu().numpy()))
        same = [np.array_equal(p, q) for p, q in zip(*outs)]  # forward, data gradient, weight gradient
        if cv.k in (3, 5) and cv.stride == 1:  # 5x5 as four 3x3 sub-kernels
            want_same = [False, False, False]
        else:
            want_same = [True, True, True]
        assert same == want_same, (li, same)
        for p, q in zip(*outs):
            assert rel_l2(p, q) <= 1e-5, li
    a.close()
    b.close()


def test_whole_step_with_paddings_0_1_2_and_ragged_tiles(lib):
    run_step_and_compare(lib, S.PADS, 3, seed=14, bias=0.05, std=0.08, use_raw=False, steps=2, mom_std=0.01)


@pytest.mark.parametrize("wl,batch", [(S.TINY, 1), (S.TINY, 2), (S.MINI, 1)])
def test_whole_step_at_degenerate_sizes(lib, wl, batch):
    """Batch 1 and 2, maps that shrink to 3x3 and 1x1 (one 4x4 tile per picture on the transformed path,
    one pixel per picture on the direct one), dense layers narrower than a GEMM tile."""
    run_step_and_compare(lib, wl, batch, seed=15, bias=0.1, std=0.3, use_raw=False, steps=2, mom_std=0.01)


def test_whole_step_with_sizes_that_are_no_multiples_of_four(lib):
    """Channel counts 6, 10, 9, 15, 7 (3 and 5 per group), dense widths 13, 11, 3: the 4-byte forms of the
    GEMM loaders, normalisation, pooling and column sums, parameter blocks that start off 16-byte boundaries,
    and one update at the end of the step instead of the early dense-layer update."""
    run_step_and_compare(lib, S.ODD, 5, seed=16, bias=0.1, std=0.2, use_raw=False, steps=2, mom_std=0.01)


def midi_with_odd_dense_widths():
    return dict(S.MIDI, name="midi_odd_fc", fc=[201, 135, 37])


def test_whole_step_with_transformed_stages_and_odd_dense_widths(lib):
    """Aligned convolution stages (tile-transform path) over dense layers of odd width: the parameter count is
    no multiple of four, so the step updates everything at its end and transforms the taps on the caller's
    stream."""
    wl = midi_with_odd_dense_widths()
    probe = lib.AlexNet(wl, 4)
    assert sum(int(np.prod(s)) for k, s in probe.shapes.items() if k.endswith(".w")) % 4 != 0
    probe.close()
    run_step_and_compare(lib, wl, 4, seed=17, bias=0.05, std=0.02, use_raw=True, steps=2, mom_std=0.01)


@pytest.mark.parametrize("wl", [S.ODD, None], ids=["odd", "midi_odd_fc"])
def test_train_step_equals_its_parts_without_the_early_update(lib, wl):
    wl = wl or midi_with_odd_dense_widths()
    batch, classes = 5, wl["fc"][-1]
    a, _, _, _ = build_pair(lib, wl, batch, seed=S.SEED_BASE + 4, pseed=4, std=0.1, bias=0.1)
    b, _, _, _ = build_pair(lib, wl, batch, seed=S.SEED_BASE + 4, pseed=4, std=0.1, bias=0.1)
    mean = cuda(S.make_mean_image(3, wl["raw"], wl["raw"], S.SEED_BASE + 7))
    for step in range(3):
        raw, labels = S.make_raw_batch(batch, 3, wl["raw"], wl["raw"], classes, S.SEED_BASE + 40 + step)
        raw, labels = cuda(raw), cuda(labels)
        a.preprocess(raw, mean, step, step % 2)
        b.preprocess(raw, mean, step, step % 2)
        la = float(a.train_step(labels, step, slot=step % 2).cpu().item())
        lb = float(b.forward_backward(labels, step, slot=step % 2).cpu().item())
        b.apply_update()
        assert la == lb, (step, la, lb)
    a.check()
    b.check()
    pa, pb, ma, mb = a.get_params(), b.get_params(), a.get_momentum(), b.get_momentum()
    for k in pa:
        assert np.array_equal(pa[k], pb[k]), k
        assert np.array_equal(ma[k], mb[k]), k
    assert any(np.abs(v).max() > 0 for v in ma.values())
    a.close()
    b.close()


def test_mini_three_steps_with_direct_3x3_stages(lib):
    run_step_and_compare(lib, S.MINI, 6, seed=12, bias=0.1, std=0.08, use_raw=False, steps=3, mom_std=0.01,
                         flags=lib.FLAG_DIRECT_CONV)


# --------------------------------------------------------- preprocess -------
def test_preprocess_crop_flip_exact(lib):
    batch = 9
    net, spec, _, _ = build_pair(lib, S.MIDI, batch, seed=77)
    raw, _ = S.make_raw_batch(batch, 3, 80, 80, 37, 5)
    mean = S.make_mean_image(3, 80, 80, 6)
    for step, slot in [(0, 0), (5, 1), (123456789012, 0)]:
        net.preprocess(cuda(raw), cuda(mean), step, slot)
        ox, oy, fl = O.crop_flip_params(spec, step)
        assert np.array_equal(net.tensor(lib.T_CROP_X, slot), ox)
        assert np.array_equal(net.tensor(lib.T_CROP_Y, slot), oy)
        assert np.array_equal(net.tensor(lib.T_FLIP, slot), fl)
        want = O.preprocess(raw, mean, ox, oy, fl, 67, 67).astype(np.float32)  # exact in f64, one rounding
        got = net.tensor(lib.T_INPUT, slot).reshape(want.shape)
        assert np.array_equal(got, want)
    assert len(set(ox.tolist())) > 1 and set(fl.tolist()) == {0, 1}
    net.close()


# ------------------------------------------------------- whole step ---------
def test_mini_alexnet_step_batch4(lib):
    """Workload 1: mini-AlexNet, one SGD step, batch 4, weights N(0, 0.01^2), zero biases."""
    loss = run_step_and_compare(lib, S.MINI, 4, seed=11, bias=0.0, std=0.01, use_raw=False)
    assert abs(loss - math.log(10)) < 1e-2


def test_mini_alexnet_three_steps_with_signal_everywhere(lib):
    run_step_and_compare(lib, S.MINI, 6, seed=12, bias=0.1, std=0.08, use_raw=False, steps=3, mom_std=0.01)


def test_midi_net_with_preprocess_ragged_tiles(lib):
    # raw uint8 pixels are O(100); small conv1 weights keep the activations moderate
    run_step_and_compare(lib, S.MIDI, 7, seed=13, bias=0.05, std=0.02, use_raw=True, steps=2, mom_std=0.01)


def test_inference_forward(lib):
    batch = 5
    net, spec, p64, _ = build_pair(lib, S.MIDI, batch, seed=3, bias=0.1, std=0.05)
    x, _ = S.make_float_batch(batch, 3, 67, 67, 37, 99)
    p = net.forward(cuda(x)).cpu().numpy()
    want = O.forward(spec, p64, x.astype(np.float64))
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=1e-5)
    assert rel_l2(p, want) <= TENSOR_RTOL
    net.close()


# --------------------------------------------------- two replicas (2.2) -----
def test_average_replicas_bit_identical_and_correct(lib):
    batch = 4
    a, spec, p64, m64 = build_pair(lib, S.MINI, batch, seed=1, bias=0.1, std=0.08, mom_std=0.01)
    b, _, _, _ = build_pair(lib, S.MINI, batch, seed=2, bias=0.1, std=0.08, mom_std=0.01)
    # identical replicas stay identical and unchanged
    lib.average_replicas(a, b)
    pa, pb = a.get_params(), b.get_params()
    for k in pa:
        assert np.array_equal(pa[k], pb[k]) and np.array_equal(pa[k].astype(np.float64), p64[k]), k
    # one step on different minibatches, then exchange-and-average
    xa, la = S.make_float_batch(batch, 3, 63, 63, 10, 100)
    xb, lb = S.make_float_batch(batch, 3, 63, 63, 10, 200)
    a.set_input(cuda(xa), 0); b.set_input(cuda(xb), 0)
    a.train_step(cuda(la), 0); b.train_step(cuda(lb), 0)
    pa0, pb0, ma0, mb0 = a.get_params(), b.get_params(), a.get_momentum(), b.get_momentum()
    assert any(not np.array_equal(pa0[k], pb0[k]) for k in pa0)
    lib.average_replicas(a, b)
    pa, pb, ma, mb = a.get_params(), b.get_params(), a.get_momentum(), b.get_momentum()
    for k in pa:
        assert np.array_equal(pa[k], pb[k]) and np.array_equal(ma[k], mb[k]), k
        # 0.5*(x+y) in fp32 is one rounding of the exact mean
        assert np.array_equal(pa[k], (0.5 * (pa0[k].astype(np.float64) + pb0[k])).astype(np.float32).astype(np.float64).astype(np.float32)) or \
            rel_l2(pa[k], O.average_replicas(pa0[k], pb0[k])) <= 1e-7, k
        assert rel_l2(ma[k], O.average_replicas(ma0[k], mb0[k])) <= 1e-7, k
    # 2 x batch + average == one step on the concatenated batch (Section 3)
    specA = oracle_spec(S.MINI, batch, seed=1); specB = oracle_spec(S.MINI, batch, seed=2)
    masks = [np.concatenate([O.dropout_mask(specA, 0, t, 256), O.dropout_mask(specB, 0, t, 256)]) for t in (O.TAG_DROP6, O.TAG_DROP7)]
    spec2 = oracle_spec(S.MINI, 2 * batch)
    _, p2, m2, _, _ = O.train_step(spec2, p64, m64, np.concatenate([xa, xb]).astype(np.float64), np.concatenate([la, lb]), 0, masks=masks)
    for k in pa:
        assert rel_l2(pa[k], p2[k]) <= TENSOR_RTOL and rel_l2(ma[k], m2[k]) <= TENSOR_RTOL, k
    a.close(); b.close()


def test_out_of_range_label_is_reported(lib):
    net, spec, _, _ = build_pair(lib, S.MINI, 4, seed=1)
    x, labels = S.make_float_batch(4, 3, 63, 63, 10, 1)
    net.set_input(cuda(x), 0)
    labels[2] = 10
    net.forward_backward(cuda(labels), 0)
    with pytest.raises(lib.AlexNetError) as e:
        net.check()
    assert e.value.code == lib.ELABEL
    net.check()  # flag is cleared once reported
    net.close()


def test_binding_refuses_wrong_tensors_before_the_library_sees_them(lib):
    net = lib.AlexNet(S.MIDI, 4)
    good_raw = torch.zeros(4, 3, 80, 80, dtype=torch.uint8, device="cuda")
    mean = torch.zeros(3, 80, 80, dtype=torch.float32, device="cuda")
    net.preprocess(good_raw, mean, 0, 0)
    with pytest.raises(ValueError, match="at least"):
        net.preprocess(good_raw[:3], mean, 0, 0)                       # one picture short
    with pytest.raises(ValueError, match="uint8"):
        net.preprocess(good_raw.float(), mean, 0, 0)
    with pytest.raises(ValueError, match="device"):
        net.preprocess(good_raw.cpu(), mean, 0, 0)
    with pytest.raises(ValueError, match="contiguous"):
        net.preprocess(good_raw.permute(0, 1, 3, 2), mean, 0, 0)
    with pytest.raises(ValueError, match="int32"):
        net.train_step(torch.zeros(4, dtype=torch.int64, device="cuda"), 0)
    with pytest.raises(ValueError, match="at least"):
        net.set_input(torch.zeros(4, 3, 66, 67, device="cuda"))
    net.check()
    net.close()
