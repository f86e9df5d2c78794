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


def validated_decisions(binding, net, spec, tau=1e-4, max_frac=1e-4, report=None):
    """Returns a function for the oracle's `decisions` hook.

    ReLU gates and pooling winners are discrete choices of the forward pass;
    where a pre-activation is zero, or two taps are equal, to within fp32
    rounding, the fp32 library and the float64 oracle may legitimately choose
    differently, and either choice is a valid (sub)gradient.  The hook takes
    the library's choices, checks each one against the oracle's own forward
    pass -- they must agree everywhere except where the oracle's margin is
    below tau x the tensor's rms, and on at most max_frac of the units -- and
    only then lets the oracle's backward pass use them."""
    def hook(cache):
        dec = {}
        nconv = len(spec.conv)
        for i, cv in enumerate(spec.conv, start=1):
            name = f"conv{i}"
            z = cache[name + ".z"]
            gate = net.tensor(binding.T_CONV_ACT, i).reshape(z.shape) > 0
            diff = gate != (z > 0)
            scale = float(np.sqrt(np.mean(z * z)))
            assert diff.mean() <= max_frac, (name, "gate mismatches", diff.mean())
            assert not diff.any() or np.abs(z[diff]).max() <= tau * scale, (name, np.abs(z[diff]).max(), scale)
            dec[name + ".gate"] = gate
            nflip = int(diff.sum())
            if cv.pool:
                src = cache[name + ".lrn"] if cv.lrn else cache[name + ".act"]
                arg_o = cache[name + ".argmax"]
                arg_g = net.tensor(binding.T_ARGMAX, i).reshape(arg_o.shape)
                d = arg_g != arg_o
                assert d.mean() <= max_frac, (name, "argmax mismatches", d.mean())
                if d.any():
                    n_, c_, h_, w_ = src.shape
                    flat = src.reshape(n_, c_, h_ * w_)
                    nn, cc = np.nonzero(d)[0], np.nonzero(d)[1]
                    v_g = flat[nn, cc, arg_g[d]]
                    v_o = flat[nn, cc, arg_o[d]]
                    s2 = float(np.sqrt(np.mean(src * src)))
                    assert np.abs(v_g - v_o).max() <= tau * s2, (name, "argmax not a near-tie")
                dec[name + ".argmax"] = arg_g
                nflip += int(d.sum())
            if report is not None:
                report[name] = nflip
        for j in range(len(spec.fc) - 1):
            name = f"fc{nconv + 1 + j}"
            z = cache[name + ".z"]
            gate = net.tensor(binding.T_FC_ACT, nconv + 1 + j).reshape(z.shape) > 0
            want = cache[name + ".act"] > 0
            diff = gate != want
            scale = float(np.sqrt(np.mean(z * z)))
            assert diff.mean() <= max_frac, (name, diff.mean())
            assert not diff.any() or np.abs(z[diff]).max() <= tau * scale, name
            dec[name + ".gate"] = gate
            if report is not None:
                report[name] = int(diff.sum())
        return dec
    return hook
