"""GPU parity of the rows beyond the training step proper: the gradient-exchange
variant of the two-replica update, and the validation pass (central crop, top-k count)."""
import numpy as np
import pytest
import torch

import synthetic_inputs as S
from gpu_common import LOSS_RTOL, TENSOR_RTOL, build_pair, cuda
from helpers import oracle_spec, rel_l2, to64
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu

ELEMENTWISE_RTOL = 1e-6  # a handful of fp32 roundings per element


def _two_replicas(lib, wl, batch, same_state):
    a, spec_a, p64, m64 = build_pair(lib, wl, batch, seed=21, bias=0.1, std=0.05, mom_std=0.01)
    if same_state:
        b, spec_b, _, _ = build_pair(lib, wl, batch, seed=22, bias=0.1, std=0.05, mom_std=0.01)
        pb64, mb64 = p64, m64
    else:
        b, spec_b, pb64, mb64 = build_pair(lib, wl, batch, seed=22, bias=0.05, std=0.04, pseed=9, mom_std=0.02)
    return a, b, spec_a, spec_b, p64, m64, pb64, mb64


@pytest.mark.parametrize("same_state", [True, False])
def test_gradient_exchange_update_matches_oracle(lib, same_state):
    wl, batch = S.MIDI, 5
    a, b, spec_a, spec_b, pa, ma, pb, mb = _two_replicas(lib, wl, batch, same_state)
    xa, la = S.make_float_batch(batch, 3, 67, 67, 37, 301)
    xb, lb = S.make_float_batch(batch, 3, 67, 67, 37, 302)
    a.set_input(cuda(xa), 0)
    b.set_input(cuda(xb), 0)
    a.forward_backward(cuda(la), 0, slot=0)
    b.forward_backward(cuda(lb), 0, slot=0)
    ga, gb = a.get_grads(), b.get_grads()  # the library's own fp32 gradients feed the oracle's update
    lib.average_gradients_update(a, b)
    wa, va, wb, vb = a.get_params(), a.get_momentum(), b.get_params(), b.get_momentum()
    for k in pa:
        wd = spec_a.weight_decay if k.endswith(".w") else 0.0
        (wa_r, va_r), (wb_r, vb_r) = O.averaged_gradient_update(pa[k], ma[k], ga[k], pb[k], mb[k], gb[k], spec_a.lr,
                                                                spec_a.momentum, wd)
        for got, want, what in ((wa[k], wa_r, "w a"), (va[k], va_r, "v a"), (wb[k], wb_r, "w b"), (vb[k], vb_r, "v b")):
            assert rel_l2(got, want) <= ELEMENTWISE_RTOL, (k, what, rel_l2(got, want))
        if same_state:
            assert np.array_equal(wa[k], wb[k]) and np.array_equal(va[k], vb[k]), k
    a.close()
    b.close()


def test_gradient_exchange_equals_parameter_exchange(lib):
    """Same start, same minibatches: update + average_replicas and average_gradients_update agree to rounding."""
    wl, batch = S.MIDI, 4
    xa, la = S.make_float_batch(batch, 3, 67, 67, 37, 311)
    xb, lb = S.make_float_batch(batch, 3, 67, 67, 37, 312)
    results = []
    for mode in ("params", "grads"):
        a, b, *_ = _two_replicas(lib, wl, batch, True)
        a.set_input(cuda(xa), 0)
        b.set_input(cuda(xb), 0)
        a.forward_backward(cuda(la), 3, slot=0)
        b.forward_backward(cuda(lb), 3, slot=0)
        if mode == "params":
            a.apply_update()
            b.apply_update()
            lib.average_replicas(a, b)
        else:
            lib.average_gradients_update(a, b)
        results.append((a.get_params(), a.get_momentum(), b.get_params()))
        a.close()
        b.close()
    (p1, m1, q1), (p2, m2, q2) = results
    for k in p1:
        assert np.array_equal(p1[k], q1[k]) and np.array_equal(p2[k], q2[k]), k
        assert rel_l2(p2[k], p1[k]) <= ELEMENTWISE_RTOL and rel_l2(m2[k], m1[k]) <= 1e-5, k


def test_center_crop_and_topk_validation(lib):
    wl, batch = S.MIDI, 9
    net, spec, p64, _ = build_pair(lib, wl, batch, seed=4, bias=0.1, std=0.05)
    raw, labels = S.make_raw_batch(batch, 3, 80, 80, 37, 55)
    mean = S.make_mean_image(3, 80, 80, 56)
    net.preprocess_center(cuda(raw), cuda(mean), 1)
    ox, oy, fl = O.center_crop_params(spec)
    assert np.array_equal(net.tensor(lib.T_CROP_X, 1), ox) and np.array_equal(net.tensor(lib.T_CROP_Y, 1), oy)
    assert np.array_equal(net.tensor(lib.T_FLIP, 1), fl)
    x64 = O.preprocess(raw, mean, ox, oy, fl, 67, 67)
    assert np.array_equal(net.tensor(lib.T_INPUT, 1).reshape(x64.shape), x64.astype(np.float32))
    ks = [1, 3, 5, 37]
    counts = torch.zeros(len(ks), dtype=torch.int32, device="cuda")
    net.validate(cuda(labels), ks, counts, slot=1)
    net.validate(cuda(labels), ks, counts, slot=1)  # counts accumulate over batches
    net.check()
    probs = O.forward(spec, p64, x64)
    want = [2 * O.topk_correct(probs, labels, k) for k in ks]
    # the ranks must not hinge on fp32 rounding: every label's score is well separated from the others here
    own = probs[np.arange(batch), labels][:, None]
    gap = np.abs(probs - own) / own
    gap[np.arange(batch), labels] = 1.0
    assert gap.min() > 1e-5
    assert counts.cpu().tolist() == want, (counts.cpu().tolist(), want)
    assert want[-1] == 2 * batch
    net.close()


def test_topk_ties_go_to_the_label(lib):
    """All-equal scores: nothing scores strictly higher than the label, so every picture counts for every k."""
    wl, batch = S.MINI, 4
    net = lib.AlexNet(wl, batch)
    zero = {k: np.zeros(s, np.float32) for k, s in net.shapes.items()}
    net.set_params(zero)
    x, labels = S.make_float_batch(batch, 3, 63, 63, 10, 77)
    net.set_input(cuda(x), 0)
    counts = torch.zeros(2, dtype=torch.int32, device="cuda")
    net.validate(cuda(labels), [1, 5], counts, slot=0)
    assert counts.cpu().tolist() == [batch, batch]
    bad = labels.copy()
    bad[1] = 10
    net.validate(cuda(bad), [1], counts[:1], slot=0)
    with pytest.raises(lib.AlexNetError) as e:
        net.check()
    assert e.value.code == lib.ELABEL
    net.close()
