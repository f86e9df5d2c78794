"""The loading thread (Section 2.1): training fed through pinned staging and a copy stream must be
bit-identical to training on pictures already resident on the GPU, and match the oracle."""
import numpy as np
import pytest
import torch

import synthetic_inputs as S
from gpu_common import LOSS_RTOL, build_pair, cuda
from helpers import to64
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("depth,shared_stream", [(2, True), (3, True), (3, False)])
def test_loader_matches_resident_training_bit_for_bit(lib, depth, shared_stream):
    """shared_stream: the loading thread issues its host-to-device copies on the caller's side stream
    (the recommended set-up) instead of a stream of the loader's own."""
    wl, batch, steps, count = S.MIDI, 6, 7, 15   # 15 pictures: minibatches wrap around the data set
    raw, labels = S.make_raw_batch(count, 3, 80, 80, 37, 500)
    mean = cuda(S.make_mean_image(3, 80, 80, 501))

    def batch_ids(k):
        return [(k * batch + i) % count for i in range(batch)]

    # (1) resident path
    ref, spec, p64, m64 = build_pair(lib, wl, batch, seed=31, bias=0.05, std=0.03, mom_std=0.01)
    ref_losses = []
    for k in range(steps):
        ids = batch_ids(k)
        ref.preprocess(cuda(raw[ids]), mean, k, k % 2)
        ref_losses.append(float(ref.train_step(cuda(labels[ids]), k, slot=k % 2).cpu().item()))
    ref.check()

    # (2) through the loader, preprocessing on a side stream
    net, _, _, _ = build_pair(lib, wl, batch, seed=31, bias=0.05, std=0.03, mom_std=0.01)
    compute, side = torch.cuda.Stream(), torch.cuda.Stream()
    loader = lib.Loader(net, torch.from_numpy(raw), torch.from_numpy(labels), depth=depth,
                        copy_stream=side if shared_stream else None)
    torch.cuda.synchronize()
    losses = []
    lab = loader.stage(0, mean, side, compute)
    for k in range(steps):
        nxt = loader.stage(k + 1, mean, side, compute) if k + 1 < steps else None
        loss = net.train_step(lab, k, slot=k % 2, stream=compute)
        loader.done(k, compute)
        with torch.cuda.stream(compute):
            losses.append(loss.clone())
        lab = nxt
    torch.cuda.synchronize()
    net.check()
    got = [float(l.cpu().item()) for l in losses]
    assert got == ref_losses, (got, ref_losses)
    pa, pb = ref.get_params(), net.get_params()
    for name in pa:
        assert np.array_equal(pa[name], pb[name]), name

    # (3) the first step against the oracle
    ids = batch_ids(0)
    ox, oy, fl = O.crop_flip_params(spec, 0)
    x64 = O.preprocess(raw[ids], mean.cpu().numpy(), ox, oy, fl, 67, 67)
    loss_ref, *_ = O.train_step(spec, p64, m64, x64, labels[ids], 0)
    assert abs(got[0] - loss_ref) <= LOSS_RTOL * abs(loss_ref)

    # calls out of order are refused, not left hanging
    with pytest.raises(lib.AlexNetError):
        loader.stage(steps + 5, mean, side, compute)
    with pytest.raises(lib.AlexNetError):
        loader.done(steps + 5, compute)
    loader.close()
    net.close()
    ref.close()
