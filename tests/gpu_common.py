"""Shared set-up of the GPU parity tests: same seeded inputs to the oracle and
to the HIP library."""
import numpy as np
import torch

import synthetic_inputs as S
from helpers import oracle_spec, rel_l2, to64
from oracle import alexnet_oracle as O

# Tolerances of the fp32 path: loss relative error and per-tensor relative L2.
LOSS_RTOL = 1e-4
TENSOR_RTOL = 1e-3


# ReLU gates and pooling winners: a bf16 forward pass moves pre-activations by ~1e-3 of their
# scale, so more of them change side than in fp32; the window in which the library's choices may
# differ from the oracle's is derived from the forward error measured in the same run
# (gpu_common.validated_decisions), so it widens by itself.  With those validated choices held fixed the
# gradients meet the 2e-2 bar; against the oracle's own choices (nothing of the library's enters the oracle)
# about 0.1 % of the units gate differently and each such unit moves its gradient tensor and every one
# below it: measured 3-16 % on these nets and 5-22 % at batch 256, so that comparison only guards against
# gross errors.
BF16_OWN_DECISIONS_RTOL = 0.5


def build_pair(binding, wl, batch, seed, bias=0.0, std=0.01, pseed=1, mom_std=0.0, precision=0, flags=0):
    """Returns (net, spec, params64, mom64): a HIP replica and the oracle's
    view of the same float32 parameters."""
    net = binding.AlexNet(wl, batch, seed=seed, precision=precision, flags=flags)
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


# A discrete choice of the library may differ from the oracle's only inside this many times the
# forward error measured on the same tensor in the same run.
WINDOW_C = 4.0


def flip_cap(n_window, c=WINDOW_C):
    """How many of the `n_window` units whose oracle margin lies inside the window may change side.
    A unit changes side only if the library's forward error exceeds its margin in the right direction:
    for margins spread evenly over a window c times the largest error that is at most 1/c of them, half
    of those by sign, so n/(2c) are expected; three standard deviations and two units on top."""
    mean = n_window / (2.0 * c)
    return int(np.ceil(mean + 3.0 * np.sqrt(mean) + 2.0))


def validated_decisions(binding, net, spec, c=WINDOW_C, report=None):
    """Returns a function for the oracle's `decisions` hook.

    ReLU gates and pooling winners are discrete choices of the forward pass; where a pre-activation
    is zero, or two taps are equal, to within the forward pass's rounding error, the library and the
    float64 oracle may legitimately choose differently, and either choice is a valid (sub)gradient.
    The hook takes the library's choices and checks each one against the oracle's own forward pass
    before the oracle's backward pass may use them.  Nothing here is a free parameter of the test:

      * eps = the largest |library - oracle| over the units of that tensor on which both made the
        same choice (measured in this run);
      * a gate may differ only where the oracle's pre-activation satisfies |z| <= c * eps, a pooling
        winner only where the oracle's margin between its winner and the library's is <= c * eps;
      * the number of differing choices per tensor is capped by flip_cap() of the number of oracle
        units inside that window.

    report[<layer>] = (differing gates, differing winners, units inside the gate window, eps)."""
    def hook(cache):
        dec = {}
        nconv = len(spec.conv)
        for i, cv in enumerate(spec.conv, start=1):
            name = f"conv{i}"
            z, act_o = cache[name + ".z"], cache[name + ".act"]
            act_g = net.tensor(binding.T_CONV_ACT, i).reshape(z.shape)
            gate = act_g > 0
            diff = gate != (z > 0)
            eps = float(np.abs(act_g - act_o)[~diff].max())
            inside = int((np.abs(z) <= c * eps).sum())
            nflip = int(diff.sum())
            assert not diff.any() or np.abs(z[diff]).max() <= c * eps, (name, "a gate differs outside the window",
                                                                       float(np.abs(z[diff]).max()), eps)
            assert nflip <= flip_cap(inside, c), (name, "too many gates differ", nflip, inside)
            dec[name + ".gate"] = gate
            nwin = 0
            if cv.pool:
                src_o = cache[name + ".lrn"] if cv.lrn else act_o
                src_g = net.tensor(binding.T_LRN, i).reshape(z.shape) if cv.lrn else act_g
                eps_p = float(np.abs(src_g - src_o)[~diff].max())
                arg_o = cache[name + ".argmax"]
                arg_g = net.tensor(binding.T_ARGMAX, i).reshape(arg_o.shape)
                d = arg_g != arg_o
                nwin = int(d.sum())
                n_, c_, h_, w_ = src_o.shape
                flat = src_o.reshape(n_, c_, h_ * w_)
                # oracle margin of every window: its largest tap minus its second largest
                ho, wo = arg_o.shape[2], arg_o.shape[3]
                best = second = None
                for r in range(3):
                    for q in range(3):
                        tap = src_o[:, :, r:r + 2 * ho:2, q:q + 2 * wo:2]
                        if best is None:
                            best, second = tap.copy(), np.full(tap.shape, -np.inf)
                        else:
                            second = np.maximum(second, np.minimum(best, tap))
                            best = np.maximum(best, tap)
                inside_p = int(((best - second <= c * eps_p) & (best > 0)).sum())
                del best, second
                if d.any():
                    nn, cc = np.nonzero(d)[0], np.nonzero(d)[1]
                    margin = flat[nn, cc, arg_o[d]] - flat[nn, cc, arg_g[d]]
                    assert margin.min() >= 0, (name, "the oracle's winner is not a maximum")
                    assert margin.max() <= c * eps_p, (name, "a pooling winner differs outside the window",
                                                       float(margin.max()), eps_p)
                    # the library's winner must be a tap of the same window
                    yy, xx = np.nonzero(d)[2], np.nonzero(d)[3]
                    gy, gx = arg_g[d] // w_, arg_g[d] % w_
                    assert np.all((gy >= 2 * yy) & (gy < 2 * yy + 3) & (gx >= 2 * xx) & (gx < 2 * xx + 3)), name
                assert nwin <= flip_cap(inside_p, c), (name, "too many pooling winners differ", nwin, inside_p)
                dec[name + ".argmax"] = arg_g
            if report is not None:
                report[name] = (nflip, nwin, inside, eps)
        for j in range(len(spec.fc) - 1):
            name = f"fc{nconv + 1 + j}"
            z, act_o = cache[name + ".z"], cache[name + ".act"]
            act_g = net.tensor(binding.T_FC_ACT, nconv + 1 + j).reshape(z.shape)
            gate = act_g > 0
            diff = gate != (act_o > 0)
            eps = float(np.abs(act_g - act_o)[~diff].max())
            inside = int((np.abs(z) <= c * eps).sum())
            nflip = int(diff.sum())
            assert not diff.any() or np.abs(z[diff]).max() <= c * eps, (name, "a gate differs outside the window")
            assert nflip <= flip_cap(inside, c), (name, "too many gates differ", nflip, inside)
            dec[name + ".gate"] = gate
            if report is not None:
                report[name] = (nflip, 0, inside, eps)
        return dec
    return hook


# ------------------------------------------------------- whole step ---------
def check_forward(lib, net, spec, cache, batch, tol=TENSOR_RTOL):
    """Forward tensors are continuous in the inputs: compared directly."""
    for i, cv in enumerate(spec.conv, start=1):
        a = net.tensor(lib.T_CONV_ACT, i).reshape(cache[f"conv{i}.act"].shape)
        assert rel_l2(a, cache[f"conv{i}.act"]) <= tol, ("act", i)
        if cv.lrn:
            assert rel_l2(net.tensor(lib.T_LRN, i).reshape(a.shape), cache[f"conv{i}.lrn"]) <= tol, ("lrn", i)
        if cv.pool:
            pv = net.tensor(lib.T_POOL, i).reshape(cache[f"conv{i}.pool"].shape)
            assert rel_l2(pv, cache[f"conv{i}.pool"]) <= tol, ("pool", i)
    for j in (6, 7):
        a = net.tensor(lib.T_FC_ACT, j).reshape(batch, -1)
        mask = cache["masks"][j - 6]
        assert np.all(a[mask == 0] == 0), "dropout mask must match the generator bit for bit"
        assert rel_l2(a, cache[f"fc{j}.act"]) <= tol, ("fc act", j)
    assert rel_l2(net.tensor(lib.T_FC_ACT, 8).reshape(batch, -1), cache["logits"]) <= tol


def run_step_and_compare(lib, wl, batch, seed, bias, std, use_raw, steps=1, mom_std=0.0, direct=True, precision=0,
                         loss_rtol=LOSS_RTOL, tol=TENSOR_RTOL, direct_tol=None, report=None, flags=0, flip_report=None, direct_report=None):
    """Runs `steps` SGD steps in the library and in the oracle and compares loss,
    forward tensors, gradients, updated weights and momentum.

    direct=True additionally compares against the oracle's own forward
    decisions (no information from the library enters the oracle at all)."""
    net, spec, p64, m64 = build_pair(lib, wl, batch, seed=seed, bias=bias, std=std, mom_std=mom_std,
                                     precision=precision, flags=flags)
    direct_tol = tol if direct_tol is None else direct_tol
    classes = wl["fc"][-1]
    for step in range(steps):
        if use_raw:
            raw, labels = S.make_raw_batch(batch, wl["in_c"], wl["raw"], wl["raw"], classes, S.SEED_BASE + 100 + step)
            mean = S.make_mean_image(wl["in_c"], wl["raw"], wl["raw"], S.SEED_BASE + 7)
            net.preprocess(cuda(raw), cuda(mean), step, step % 2)
            ox, oy, fl = O.crop_flip_params(spec, step)
            x64 = O.preprocess(raw, mean, ox, oy, fl, wl["crop"], wl["crop"])
        else:
            x32, labels = S.make_float_batch(batch, wl["in_c"], wl["crop"], wl["crop"], classes, S.SEED_BASE + 1 + step)
            net.set_input(cuda(x32), step % 2)
            x64 = x32.astype(np.float64)
        loss = net.forward_backward(cuda(labels), step, slot=step % 2)
        net.check()
        got_loss = float(loss.cpu().item())
        g = net.get_grads()
        flips = {}
        loss_ref, p_new, m_new, g_ref, cache = O.train_step(
            spec, p64, m64, x64, labels, step, decisions=validated_decisions(lib, net, spec, report=flips))
        assert abs(got_loss - loss_ref) <= loss_rtol * abs(loss_ref), (step, got_loss, loss_ref)
        if flip_report is not None:
            flip_report[step] = flips
        check_forward(lib, net, spec, cache, batch, tol)
        net.apply_update()
        pn, mn = net.get_params(), net.get_momentum()
        for k in g_ref:
            assert np.linalg.norm(g_ref[k]) > 0, k
            assert rel_l2(g[k], g_ref[k]) <= tol, ("grad", k, rel_l2(g[k], g_ref[k]))
            if report is not None:
                report[k] = max(report.get(k, 0.0), rel_l2(g[k], g_ref[k]))
            assert rel_l2(pn[k], p_new[k]) <= tol, ("param", k)
            assert rel_l2(mn[k], m_new[k]) <= tol, ("momentum", k, rel_l2(mn[k], m_new[k]))
        if direct:
            _, _, _, g_own, _ = O.train_step(spec, p64, m64, x64, labels, step)
            for k in g_own:
                e_own = rel_l2(g[k], g_own[k])
                if direct_report is not None:
                    direct_report[k] = max(direct_report.get(k, 0.0), e_own)
                assert e_own <= direct_tol, ("grad vs oracle's own decisions", k, e_own, flips)
        # continue from the library's own fp32 state so that errors do not pile up across steps
        p64, m64 = to64(pn), to64(mn)
    net.close()
    return got_loss
