"""GPU parity of the bf16 matrix products (precision = 1).

Two comparisons per product: against the float64 oracle fed with operands
rounded to bfloat16 (round to nearest even) -- products of bf16 values are
exact in fp32, so only the fp32 accumulation order remains and the bar is
tight; and against the oracle on the unrounded operands, to the 2e-2
per-tensor bar of the bf16 configuration."""
import math

import numpy as np
import pytest

import synthetic_inputs as S
from gpu_common import BF16_OWN_DECISIONS_RTOL, build_pair, cuda, run_step_and_compare
from helpers import oracle_spec, rel_l2
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu

BF16_RTOL = 2e-2      # per-tensor relative L2 against the float64 oracle
BF16_LOSS_RTOL = 1e-2
EXACT_RTOL = 2e-5     # against the oracle on bf16-rounded operands (fp32 accumulation only)


def round_bf16(a):
    """float32 -> nearest bfloat16 (ties to even) -> float64."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def test_round_bf16_helper():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5, 0.0], np.float32)  # 1 + 2^-8 is a tie -> even (1.0)
    r = round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625 and r[4] == 0.0
    assert abs(r[3] - x[3]) <= abs(x[3]) * 2.0 ** -8


def _kind(got, exact, plain):
    """Which arithmetic produced `got`: ('bf16'|'fp32', error against that reference)."""
    e_bf, e_fp = rel_l2(got, exact), rel_l2(got, plain)
    return ("bf16", e_bf, e_fp) if e_bf < e_fp else ("fp32", e_fp, e_fp)


@pytest.mark.parametrize("wl,batch", [(S.MINI, 4), (S.MIDI, 5), (S.MINI, 32)])
def test_bf16_conv_layers_alone(lib, wl, batch):
    net = lib.AlexNet(wl, batch, precision=1)
    spec = oracle_spec(wl, batch)
    stages, _ = O.layer_shapes(spec)
    used = {}
    for li, (cv, st) in enumerate(zip(spec.conv, stages), start=1):
        cin, h, w = st["in"]
        cout, ho, wo = st["conv"]
        x = S.make_normal((batch, cin, h, w), 10 + li)
        wt = S.make_normal((cout, cin // cv.groups, cv.k, cv.k), 20 + li, std=0.05)
        b = S.make_normal((cout,), 30 + li)
        dy = S.make_normal((batch, cout, ho, wo), 40 + li)
        xr, wr, dyr = round_bf16(x), round_bf16(wt), round_bf16(dy)

        y = net.conv_forward(li, x, wt, b, relu=False).cpu().numpy().reshape(batch, cout, ho, wo)
        k, e, e_plain = _kind(y, O.conv_forward(xr, wr, b, cv.stride, cv.pad, cv.groups),
                              O.conv_forward(x, wt, b, cv.stride, cv.pad, cv.groups))
        assert e <= EXACT_RTOL and e_plain <= BF16_RTOL, ("fwd", li, k, e, e_plain)
        used[("fwd", li)] = k

        dx = net.conv_backward_data(li, dy, wt, x.shape).cpu().numpy()
        k, e, e_plain = _kind(dx, O.conv_backward_data(dyr, wr, (h, w), cv.stride, cv.pad, cv.groups),
                              O.conv_backward_data(dy, wt, (h, w), cv.stride, cv.pad, cv.groups))
        assert e <= EXACT_RTOL and e_plain <= BF16_RTOL, ("bwd_data", li, k, e, e_plain)
        used[("bwd_data", li)] = k

        dw, db = net.conv_backward_weight(li, x, dy, wt.shape)
        dw_r, _ = O.conv_backward_weight(xr, dyr, cv.k, cv.stride, cv.pad, cv.groups)
        dw_p, db_p = O.conv_backward_weight(x, dy, cv.k, cv.stride, cv.pad, cv.groups)
        k, e, e_plain = _kind(dw.cpu().numpy(), dw_r, dw_p)
        assert e <= EXACT_RTOL and e_plain <= BF16_RTOL, ("bwd_weight", li, k, e, e_plain)
        assert rel_l2(db.cpu().numpy(), db_p) <= 1e-5  # the bias gradient is an fp32 column sum
        used[("bwd_weight", li)] = k
    print(used)
    # every product of layers 2..5 reads 16 bytes at a time here, and so does the first layer's
    # forward and weight gradient (whole kernel rows); those must have taken the bf16 kernels
    for li in range(2, 6):
        for op in ("fwd", "bwd_data", "bwd_weight"):
            assert used[(op, li)] == "bf16", (op, li)
    assert used[("fwd", 1)] == "bf16" and used[("bwd_weight", 1)] == "bf16"
    net.close()


def test_bf16_dense_layers_alone(lib):
    batch, wl = 7, S.MIDI
    net = lib.AlexNet(wl, batch, precision=1)
    shapes = net.shapes
    for li in (6, 7, 8):
        out, inn = shapes[f"fc{li}.w"]
        x = S.make_normal((batch, inn), 60 + li)
        w = S.make_normal((out, inn), 70 + li, std=0.05)
        b = S.make_normal((out,), 80 + li)
        dy = S.make_normal((batch, out), 90 + li)
        xr, wr, dyr = round_bf16(x), round_bf16(w), round_bf16(dy)
        y = net.fc_forward(li, x, w, b).cpu().numpy()
        k, e, e_plain = _kind(y, O.fc_forward(xr, wr, b), O.fc_forward(x, w, b))
        assert e <= EXACT_RTOL and e_plain <= BF16_RTOL, ("fc fwd", li, k, e, e_plain)
        assert k == "bf16" or inn % 4, li
        dx, dw, db = (t.cpu().numpy() for t in net.fc_backward(li, x, w, dy))
        dx_r, dw_r, _ = O.fc_backward(xr, wr, dyr)  # dx pairs dy with w, dw pairs dy with x
        dx_p, dw_p, db_p = O.fc_backward(x, w, dy)
        kx, ex, ex_plain = _kind(dx, dx_r, dx_p)
        kw, ew, ew_plain = _kind(dw, dw_r, dw_p)
        assert ex <= EXACT_RTOL and ex_plain <= BF16_RTOL, ("fc bwd_data", li, kx, ex, ex_plain)
        assert ew <= EXACT_RTOL and ew_plain <= BF16_RTOL, ("fc bwd_weight", li, kw, ew, ew_plain)
        if out % 4 == 0 and inn % 4 == 0:
            assert kx == "bf16" and kw == "bf16", (li, kx, kw)
        assert rel_l2(db, db_p) <= 1e-5
    net.close()




def test_bf16_mini_alexnet_step(lib):
    errs, own = {}, {}
    loss = run_step_and_compare(lib, S.MINI, 4, seed=11, bias=0.0, std=0.01, use_raw=False, precision=1, direct=True, direct_tol=BF16_OWN_DECISIONS_RTOL, direct_report=own,
                                loss_rtol=BF16_LOSS_RTOL, tol=BF16_RTOL, report=errs)
    print(errs, 'decision-free:', own)
    assert abs(loss - math.log(10)) < 1e-2


def test_bf16_mini_three_steps_with_signal_everywhere(lib):
    errs, own = {}, {}
    run_step_and_compare(lib, S.MINI, 6, seed=12, bias=0.1, std=0.08, use_raw=False, steps=3, mom_std=0.01,
                         precision=1, direct=True, direct_tol=BF16_OWN_DECISIONS_RTOL, direct_report=own, loss_rtol=BF16_LOSS_RTOL, tol=BF16_RTOL, report=errs)
    print(errs, 'decision-free:', own)


def test_bf16_midi_net_with_preprocess(lib):
    errs, own = {}, {}
    run_step_and_compare(lib, S.MIDI, 7, seed=13, bias=0.05, std=0.02, use_raw=True, steps=2, mom_std=0.01,
                         precision=1, direct=True, direct_tol=BF16_OWN_DECISIONS_RTOL, direct_report=own, loss_rtol=BF16_LOSS_RTOL, tol=BF16_RTOL, report=errs)
    print(errs, 'decision-free:', own)


def test_bf16_falls_back_to_fp32_products_where_sizes_are_no_multiples_of_four(lib):
    """The bf16 kernels exist for 16-byte loads only; a net whose every operand is unaligned runs the fp32
    kernels under precision = 1 and meets the fp32 bar."""
    run_step_and_compare(lib, S.ODD, 5, seed=16, bias=0.1, std=0.2, use_raw=False, steps=2, mom_std=0.01, precision=1)


def test_bf16_and_fp32_replicas_stay_close(lib):
    """Same data, same parameters: the bf16 step lands within the bf16 bar of the fp32 step."""
    batch, wl = 6, S.MIDI
    a, _, _, _ = build_pair(lib, wl, batch, seed=5, bias=0.05, std=0.03)
    b, _, _, _ = build_pair(lib, wl, batch, seed=5, bias=0.05, std=0.03, precision=1)
    x, labels = S.make_float_batch(batch, 3, 67, 67, 37, 123)
    for net in (a, b):
        net.set_input(cuda(x), 0)
    la = float(a.forward_backward(cuda(labels), 0, slot=0).cpu().item())
    lb = float(b.forward_backward(cuda(labels), 0, slot=0).cpu().item())
    assert abs(la - lb) <= BF16_LOSS_RTOL * abs(la)
    ga, gb = a.get_grads(), b.get_grads()
    differ = 0
    for k in ga:
        differ += int(not np.array_equal(ga[k], gb[k]))
    assert differ > 0, "the bf16 replica must actually compute in bf16"
    a.close()
    b.close()


def mini_with_widths_of_eight():
    """`mini` with 16 classes: every dense width is a multiple of eight, so a bf16 handle keeps bf16 copies of
    the dense layers' operands too (with 10 classes only its convolutions do)."""
    wl = dict(S.MINI)
    wl["name"] = "mini16"
    wl["fc"] = [256, 256, 16]
    return wl


def test_bf16_three_steps_with_every_operand_stored_as_bf16(lib):
    errs, own = {}, {}
    run_step_and_compare(lib, mini_with_widths_of_eight(), 6, seed=14, bias=0.1, std=0.08, use_raw=False, steps=3,
                         mom_std=0.01, precision=1, direct=True, direct_tol=BF16_OWN_DECISIONS_RTOL, direct_report=own,
                         loss_rtol=BF16_LOSS_RTOL, tol=BF16_RTOL, report=errs)
    print(errs, 'decision-free:', own)


@pytest.mark.parametrize("wl", [None, S.MIDI], ids=["mini16", "midi"])
def test_bf16_train_step_equals_its_parts(lib, wl):
    """alexnet_train_step makes the bf16 copies of the weights on the handle's own stream (events before the
    first convolution that reads them, before fc6 and before the first data gradient) and forks the dense-layer
    update; forward_backward + apply_update make them in line.  Same kernels on the same values: three steps
    either way must leave the same bits."""
    wl = wl or mini_with_widths_of_eight()
    batch, classes = 6, wl["fc"][-1]
    a, _, _, _ = build_pair(lib, wl, batch, seed=S.SEED_BASE + 4, pseed=4, std=0.1, bias=0.1, precision=1)
    b, _, _, _ = build_pair(lib, wl, batch, seed=S.SEED_BASE + 4, pseed=4, std=0.1, bias=0.1, precision=1)
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
