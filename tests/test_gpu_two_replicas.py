"""Workload 5: consecutive steps of two same-GPU replicas with on-device
preprocessing on a side stream, exchange-and-average after every step
(paper Section 2.2), checked against the oracle on the first steps."""
import numpy as np
import pytest
import torch

import synthetic_inputs as S
from gpu_common import LOSS_RTOL, TENSOR_RTOL, cuda
from helpers import oracle_spec, rel_l2, to64
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu


def _run(lib, wl, batch, steps, overlap, seeds=(101, 202), bias=0.05, std=0.03, snapshots=None):
    """Runs `steps` two-replica iterations; returns per-step losses and the final state of replica A.
    After every averaging step the two replicas' parameter and momentum vectors are compared on the device
    (bit for bit, no host synchronisation); `snapshots` (a list) also receives replica A's state after every
    step, which synchronises."""
    classes = wl["fc"][-1]
    nets = [lib.AlexNet(wl, batch, seed=s) for s in seeds]
    shapes = nets[0].shapes
    p32 = S.make_params(shapes, S.SEED_BASE + 5, bias_value=bias, std=std)
    for n in nets:
        n.set_params(p32)
    mean = cuda(S.make_mean_image(wl["in_c"], wl["raw"], wl["raw"], S.SEED_BASE + 7))
    data = [[S.make_raw_batch(batch, wl["in_c"], wl["raw"], wl["raw"], classes, S.SEED_BASE + 5 + 1000 * r + k)
             for k in range(steps)] for r in range(2)]
    raws = [[cuda(d[0]) for d in data[r]] for r in range(2)]
    labels = [[cuda(d[1]) for d in data[r]] for r in range(2)]
    compute = torch.cuda.Stream()
    side = torch.cuda.Stream() if overlap else compute
    ready = [[torch.cuda.Event() for _ in range(2)] for _ in range(2)]
    freed = [torch.cuda.Event() for _ in range(2)]
    losses = torch.zeros(steps, 2, device="cuda")
    differ = torch.zeros(steps, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for r in range(2):
        nets[r].preprocess(raws[r][0], mean, 0, 0, stream=side)
        ready[r][0].record(side)
    for k in range(steps):
        s = k % 2
        if k + 1 < steps:
            if k > 0:
                side.wait_event(freed[1 - s])
            for r in range(2):
                nets[r].preprocess(raws[r][k + 1], mean, k + 1, 1 - s, stream=side)
                ready[r][1 - s].record(side)
        for r in range(2):
            compute.wait_event(ready[r][s])
            nets[r].train_step(labels[r][k], k, slot=s, stream=compute)
            with torch.cuda.stream(compute):
                losses[k, r].copy_(nets[r].loss[0])
        freed[s].record(compute)
        lib.average_replicas(nets[0], nets[1], stream=compute)
        with torch.cuda.stream(compute):  # "checked bit-identical after averaging", every step
            differ[k] = (nets[0].params != nets[1].params).sum() + (nets[0].momentum != nets[1].momentum).sum()
        if snapshots is not None:
            compute.synchronize()
            snapshots.append((nets[0].get_params(), nets[0].get_momentum()))
    torch.cuda.synchronize()
    assert int(differ.sum().item()) == 0, differ.cpu().numpy()
    for n in nets:
        n.check()
    pa, pb = nets[0].get_params(), nets[1].get_params()
    ma, mb = nets[0].get_momentum(), nets[1].get_momentum()
    for k in pa:  # "2 AlexNets sharing the same parameters": bit-identical after averaging
        assert np.all(np.isfinite(pa[k])), k
        assert np.array_equal(pa[k], pb[k]) and np.array_equal(ma[k], mb[k]), k
    for n in nets:
        n.close()
    return losses.cpu().numpy(), pa, ma, p32, data


def test_two_replicas_midi_matches_oracle_and_overlap_is_bit_equal(lib):
    wl, batch, steps = S.MIDI, 6, 4
    snaps = []
    l1, p1, m1, p32, data = _run(lib, wl, batch, steps, overlap=True, snapshots=snaps)
    l0, p0, m0, _, _ = _run(lib, wl, batch, steps, overlap=False)
    assert np.array_equal(l1, l0)
    for k in p1:  # side-stream preprocessing must not change a single bit
        assert np.array_equal(p1[k], p0[k]) and np.array_equal(m1[k], m0[k]), k
    # oracle: both replicas step, then both take the mean (weights, biases and momentum).  Every step starts from
    # the state the library left (float32 values, exact in float64), so the stated bars apply to each step
    # and differences do not pile up over the steps.
    specs = [oracle_spec(wl, batch, seed=s) for s in (101, 202)]
    p = to64(p32)
    m = {k: np.zeros_like(v) for k, v in p.items()}
    for k in range(steps):
        outs = []
        for r in range(2):
            raw, lab = data[r][k]
            mean = S.make_mean_image(wl["in_c"], wl["raw"], wl["raw"], S.SEED_BASE + 7)
            ox, oy, fl = O.crop_flip_params(specs[r], k)
            x = O.preprocess(raw, mean, ox, oy, fl, wl["crop"], wl["crop"])
            loss, pn, mn, _, _ = O.train_step(specs[r], p, m, x, lab, k)
            assert abs(l1[k, r] - loss) <= LOSS_RTOL * abs(loss), (k, r, l1[k, r], loss)
            outs.append((pn, mn))
        p_ref = {kk: O.average_replicas(outs[0][0][kk], outs[1][0][kk]) for kk in p}
        m_ref = {kk: O.average_replicas(outs[0][1][kk], outs[1][1][kk]) for kk in m}
        p_gpu, m_gpu = snaps[k]
        for kk in p_ref:
            assert rel_l2(p_gpu[kk], p_ref[kk]) <= TENSOR_RTOL, (k, kk)
            assert rel_l2(m_gpu[kk], m_ref[kk]) <= TENSOR_RTOL, (k, kk, rel_l2(m_gpu[kk], m_ref[kk]))
        p, m = to64(p_gpu), to64(m_gpu)
    for kk in p1:
        assert np.array_equal(p1[kk], snaps[-1][0][kk]) and np.array_equal(m1[kk], snaps[-1][1][kk]), kk


@pytest.mark.timeout(600)
def test_two_replicas_alexnet_20_steps(lib):
    """Full size: 20 consecutive fp32 batch-128 steps on two replicas; losses stay finite
    and near log(1000), replicas end bit-identical, overlap on/off gives the same bits."""
    l1, p1, m1, _, _ = _run(lib, S.ALEXNET, 128, 20, overlap=True, bias=0.0, std=0.01)
    assert np.all(np.isfinite(l1)) and abs(l1[0].mean() - np.log(1000)) < 0.1
    l0, p0, m0, _, _ = _run(lib, S.ALEXNET, 128, 20, overlap=False, bias=0.0, std=0.01)
    assert np.array_equal(l1, l0)
    for k in p1:
        assert np.array_equal(p1[k], p0[k]), k
