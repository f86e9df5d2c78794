"""The entry point that allocates nothing (alexnet_softmax_xent_static) against the handle-based
alexnet_softmax_xent: same kernels, so the same bits, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

import synthetic_inputs as S
from oracle import alexnet_oracle as O

pytestmark = pytest.mark.gpu


def test_static_softmax_matches_the_handle_based_call_twice_in_a_row(lib):
    classes = 1000
    for batch, seed in ((128, 1), (37, 2)):  # the second call is smaller: stale rows of the first stay in the scratch
        net = lib.AlexNet(S.ALEXNET, batch)
        z = S.make_normal((batch, classes), 7000 + seed, std=4.0)
        labels = np.random.default_rng(7100 + seed).integers(0, classes, batch).astype(np.int32)
        want_dz, want_loss = net.softmax_xent(z, labels)
        zt, lt = torch.from_numpy(z).cuda(), torch.from_numpy(labels).cuda()
        dz = torch.full((batch, classes), float("nan"), dtype=torch.float32, device="cuda")
        loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        bad = torch.full((1,), 7, dtype=torch.int32, device="cuda")
        before = torch.cuda.memory_allocated()
        lib.softmax_xent_static(zt, lt, dz, loss, bad)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert np.array_equal(dz.cpu().numpy(), want_dz.cpu().numpy()), batch
        assert float(loss.cpu().item()) == float(want_loss.cpu().item()), batch
        assert int(bad.cpu().item()) == 0
        ref_loss, _, ref_dz = O.softmax_xent(z, labels)
        assert abs(float(loss.cpu().item()) - ref_loss) <= 1e-5 * abs(ref_loss)
        assert np.linalg.norm(dz.cpu().numpy() - ref_dz) <= 2e-5 * np.linalg.norm(ref_dz)
        net.close()
    # a label out of range raises the flag for that call only; the next call clears it
    z = torch.from_numpy(S.make_normal((5, 10), 7200)).cuda()
    dz = torch.empty(5, 10, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    lib.softmax_xent_static(z, torch.tensor([0, 1, 10, 3, 4], dtype=torch.int32).cuda(), dz, loss, bad)
    assert int(bad.cpu().item()) == 1
    lib.softmax_xent_static(z, torch.tensor([0, 1, 9, 3, 4], dtype=torch.int32).cuda(), dz, loss, bad)
    assert int(bad.cpu().item()) == 0
    # sizes beyond the built-in scratch are refused on the host, before any launch
    big = torch.zeros(4097, 2, dtype=torch.float32, device="cuda")
    with pytest.raises(lib.AlexNetError) as e:
        lib.softmax_xent_static(big, torch.zeros(4097, dtype=torch.int32).cuda(), torch.empty_like(big), loss)
    assert e.value.code == lib.ENOMEM and "4096" in str(e.value)
