"""Shared set-up of the GPU parity tests: same seeded inputs to the oracle and
to the HIP library."""
import numpy as np
import torch

import synthetic_inputs as S
from helpers import oracle_spec, to64
from oracle import alexnet_oracle as O

# Tolerances of the fp32 path: loss relative error and per-tensor relative L2.
LOSS_RTOL = 1e-4
TENSOR_RTOL = 1e-3


def build_pair(binding, wl, batch, seed, bias=0.0, std=0.01, pseed=1, mom_std=0.0):
    """Returns (net, spec, params64, mom64): a HIP replica and the oracle's
    view of the same float32 parameters."""
    net = binding.AlexNet(wl, batch, seed=seed)
    spec = oracle_spec(wl, batch, seed=seed)
    shapes = O.param_shapes(spec)
    assert {k: tuple(v) for k, v in shapes.items()} == {k: tuple(v) for k, v in net.shapes.items()}
    assert list(shapes) == list(net.shapes)
    p32 = S.make_params(shapes, S.SEED_BASE + pseed, bias_value=bias, std=std)
    net.set_params(p32)
    if mom_std > 0:
        m32 = S.make_random_like(shapes, S.SEED_BASE + pseed + 50, std=mom_std)
    else:
        m32 = {k: np.zeros(s, np.float32) for k, s in shapes.items()}
    net.set_momentum(m32)
    return net, spec, to64(p32), to64(m32)


def cuda(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)
