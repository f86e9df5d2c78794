"""CPU-only pins for the oracle's `decisions=` hook (fixed ReLU gates and pooling winners in the
backward pass).  The GPU parity tests hand the library's own discrete choices to the oracle's
backward pass through that hook, so what the hook computes is pinned here against things that are
not the oracle: torch autograd on a network whose discrete choices are frozen constants, a
hand-derived single flip, and one-sided finite differences of the true loss at a kink."""
import numpy as np
import torch
import torch.nn.functional as F

import synthetic_inputs as S
from helpers import oracle_spec, to64
from oracle import alexnet_oracle as O


def _problem(batch=3, seed=5, bias=0.1, std=0.08):
    spec = oracle_spec(S.MINI, batch, seed=seed)
    params = to64(S.make_params(O.param_shapes(spec), S.SEED_BASE + 1, bias_value=bias, std=std))
    x, lab = S.make_float_batch(batch, 3, 63, 63, 10, S.SEED_BASE + 1)
    masks = [O.dropout_mask(spec, 2, t, w) for t, w in ((O.TAG_DROP6, 256), (O.TAG_DROP7, 256))]
    return spec, params, x.astype(np.float64), lab, masks


def _own_decisions(spec, cache):
    dec = {}
    for i, cv in enumerate(spec.conv, start=1):
        dec[f"conv{i}.gate"] = cache[f"conv{i}.act"] > 0
        if cv.pool:
            dec[f"conv{i}.argmax"] = cache[f"conv{i}.argmax"].copy()
    for j in (6, 7):
        dec[f"fc{j}.gate"] = cache[f"fc{j}.act"] > 0
    return dec


def _frozen_torch_net(spec, params, x, lab, masks, dec):
    """The forward values are the true network's (ReLU, max-pool, computed by torch); the derivative of
    every discrete operator is replaced by that of its frozen form: ReLU by `z * gate`, a pool by a
    gather of the given taps (value = true.detach() + frozen - frozen.detach()).  Autograd of this
    function is what "the backward pass with the decisions held fixed" means."""
    def with_grad_of(true, frozen):
        return true.detach() + frozen - frozen.detach()

    tp = {k: torch.tensor(v, requires_grad=True) for k, v in params.items()}
    h = torch.tensor(x)
    for i, cv in enumerate(spec.conv, start=1):
        z = F.conv2d(h, tp[f"conv{i}.w"], tp[f"conv{i}.b"], stride=cv.stride, padding=cv.pad, groups=cv.groups)
        h = with_grad_of(F.relu(z), z * torch.tensor(dec[f"conv{i}.gate"].astype(np.float64)))
        if cv.lrn:
            h = F.local_response_norm(h, spec.lrn_n, alpha=spec.lrn_alpha * spec.lrn_n, beta=spec.lrn_beta, k=spec.lrn_k)
        if cv.pool:
            arg = torch.tensor(dec[f"conv{i}.argmax"].astype(np.int64))
            n, c, ho, wo = arg.shape
            h = with_grad_of(F.max_pool2d(h, 3, 2), h.flatten(2).gather(2, arg.flatten(2)).reshape(n, c, ho, wo))
    h = h.flatten(1)
    for j in range(3):
        z = F.linear(h, tp[f"fc{6+j}.w"], tp[f"fc{6+j}.b"])
        # fc gate = ReLU gate AND dropout keep (the stored activation is positive exactly there)
        if j < 2:
            h = with_grad_of(F.relu(z) * torch.tensor(masks[j]), z * torch.tensor(dec[f"fc{6+j}.gate"].astype(np.float64)))
        else:
            h = z
    loss = F.cross_entropy(h, torch.tensor(lab).long())
    loss.backward()
    return {k: v.grad.numpy() for k, v in tp.items()}


def test_own_decisions_reproduce_the_plain_backward_bit_for_bit():
    spec, params, x, lab, masks = _problem()
    loss0, g0, cache = O.loss_and_grads(spec, params, x, lab, masks)
    loss1, g1, _ = O.loss_and_grads(spec, params, x, lab, masks, decisions=_own_decisions(spec, cache))
    assert loss0 == loss1
    for k in g0:
        assert np.array_equal(g0[k], g1[k]), k
    # the callable form sees the same forward pass
    seen = {}

    def hook(c):
        seen["z"] = c["conv3.z"]
        return _own_decisions(spec, c)

    _, g2, c2 = O.loss_and_grads(spec, params, x, lab, masks, decisions=hook)
    assert np.array_equal(seen["z"], c2["conv3.z"])
    for k in g0:
        assert np.array_equal(g0[k], g2[k]), k
    # and through train_step
    mom = {k: np.zeros_like(v) for k, v in params.items()}
    spec2 = oracle_spec(S.MINI, 3, seed=5)
    _, p_a, v_a, g_a, c_a = O.train_step(spec2, params, mom, x, lab, 2)
    _, p_b, v_b, g_b, _ = O.train_step(spec2, params, mom, x, lab, 2, decisions=lambda c: _own_decisions(spec2, c))
    for k in g_a:
        assert np.array_equal(g_a[k], g_b[k]) and np.array_equal(p_a[k], p_b[k]) and np.array_equal(v_a[k], v_b[k])


def test_foreign_decisions_equal_autograd_of_the_frozen_network():
    """Many gates flipped and many pooling winners moved inside their windows (valid choices or
    not): the backward pass with those decisions is the gradient of the frozen network.  A wrong
    sign, a gate applied at the wrong layer, an argmax read in another index convention, or a
    decision silently ignored, fails here."""
    spec, params, x, lab, masks = _problem()
    _, g_plain, cache = O.loss_and_grads(spec, params, x, lab, masks)
    dec = _own_decisions(spec, cache)
    r = np.random.default_rng(11)
    stages, _ = O.layer_shapes(spec)
    for i, cv in enumerate(spec.conv, start=1):
        gate = dec[f"conv{i}.gate"]
        flip = r.random(gate.shape) < 0.02
        dec[f"conv{i}.gate"] = gate ^ flip
        if cv.pool:
            arg = dec[f"conv{i}.argmax"]
            _, hin, win = stages[i - 1]["conv"]
            n, c, ho, wo = arg.shape
            yy = (np.arange(ho) * 2)[:, None] + r.integers(0, 3, size=arg.shape)
            xx = (np.arange(wo) * 2)[None, :] + r.integers(0, 3, size=arg.shape)
            moved = r.random(arg.shape) < 0.05
            dec[f"conv{i}.argmax"] = np.where(moved, yy * win + xx, arg).astype(np.int32)
            assert dec[f"conv{i}.argmax"].max() < hin * win
    for j in (6, 7):
        gate = dec[f"fc{j}.gate"]
        dec[f"fc{j}.gate"] = gate ^ (r.random(gate.shape) < 0.05)
    _, g_dec, _ = O.loss_and_grads(spec, params, x, lab, masks, decisions=dec)
    want = _frozen_torch_net(spec, params, x, lab, masks, dec)
    changed = 0
    for k in g_dec:
        np.testing.assert_allclose(g_dec[k], want[k], rtol=1e-8, atol=1e-12 * max(1.0, np.abs(want[k]).max()), err_msg=k)
        changed += int(not np.allclose(g_dec[k], g_plain[k], rtol=1e-6, atol=0))
    assert changed >= 14  # every tensor below fc8 feels the foreign decisions


def test_single_dense_gate_flip_changes_gradients_by_the_hand_derived_amount():
    """Open the gate of one fc7 unit u for one picture n that the forward pass had closed.
    By the chain rule: fc8's gradients do not change (they see activations, not gates);
    d7[n,u] goes from 0 to e = dz8[n,:] . W8[:,u]; so fc7.w[u,:] gains e * a6[n,:], fc7.b[u] gains e,
    d6[n,:] gains e * W7[u,:] * gate6[n,:], fc6.w gains that outer a5[n,:], fc6.b gains it."""
    spec, params, x, lab, masks = _problem()
    _, g0, cache = O.loss_and_grads(spec, params, x, lab, masks)
    gate7 = cache["fc7.act"] > 0
    n, u = [(int(a), int(b)) for a, b in zip(*np.nonzero(~gate7))][7]
    dec = {"fc7.gate": gate7.copy()}
    dec["fc7.gate"][n, u] = True
    _, g1, _ = O.loss_and_grads(spec, params, x, lab, masks, decisions=dec)
    b = x.shape[0]
    p = cache["probs"].copy()
    p[np.arange(b), lab] -= 1.0
    dz8 = p / b
    e = float(dz8[n] @ params["fc8.w"][:, u])
    assert e != 0.0
    a6, a5 = cache["fc7.in"], cache["fc6.in"]
    gate6 = cache["fc6.act"] > 0
    assert np.array_equal(g1["fc8.w"], g0["fc8.w"]) and np.array_equal(g1["fc8.b"], g0["fc8.b"])
    dw7 = np.zeros_like(g0["fc7.w"]); dw7[u] = e * a6[n]
    db7 = np.zeros_like(g0["fc7.b"]); db7[u] = e
    d6 = e * params["fc7.w"][u] * gate6[n]
    np.testing.assert_allclose(g1["fc7.w"] - g0["fc7.w"], dw7, rtol=1e-9, atol=1e-16)
    np.testing.assert_allclose(g1["fc7.b"] - g0["fc7.b"], db7, rtol=1e-9, atol=1e-16)
    np.testing.assert_allclose(g1["fc6.w"] - g0["fc6.w"], np.outer(d6, a5[n]), rtol=1e-7, atol=1e-15)
    np.testing.assert_allclose(g1["fc6.b"] - g0["fc6.b"], d6, rtol=1e-7, atol=1e-15)
    assert np.linalg.norm(g1["conv5.w"] - g0["conv5.w"]) > 0


def test_single_argmax_move_between_tied_taps_moves_exactly_that_gradient():
    """conv5's pool: move one winner from its tap p to another tap q of the same window.  The pooled
    gradient d[n,c,y,x] then lands on q instead of p; with both gates open the change of conv5's bias
    gradient is 0 (the sum over the plane is the same) and that of d(conv5 pre-activation) is
    +d at q, -d at p: checked through conv5.b (unchanged) and through the closed-gate variant, where
    the bias gradient loses exactly d."""
    spec, params, x, lab, masks = _problem()
    _, g0, cache = O.loss_and_grads(spec, params, x, lab, masks, want_dx=False)
    arg = cache["conv5.argmax"]
    gate = cache["conv5.act"] > 0
    # gradient that arrives at the pooled output of conv5: fc6's data gradient reshaped
    p = cache["probs"].copy(); p[np.arange(x.shape[0]), lab] -= 1.0
    d8 = p / x.shape[0]
    d7 = (d8 @ params["fc8.w"]) * (cache["fc7.act"] > 0)
    d6 = (d7 @ params["fc7.w"]) * (cache["fc6.act"] > 0)
    dpool = (d6 @ params["fc6.w"]).reshape(cache["flat_shape"])
    win = cache["conv5.pool_in_hw"][1]
    n, c, y, xx = 1, 3, 0, 1
    pidx = int(arg[n, c, y, xx])
    taps = [(2 * y + r) * win + (2 * xx + s) for r in range(3) for s in range(3)]
    assert pidx in taps
    assert gate.reshape(gate.shape[0], gate.shape[1], -1)[n, c, pidx], "the winner of a positive window is open"
    q = [t for t in taps if t != pidx][0]
    dval = float(dpool[n, c, y, xx])
    assert dval != 0.0
    for q_open in (True, False):
        dec = {"conv5.argmax": arg.copy(), "conv5.gate": gate.copy()}
        dec["conv5.argmax"][n, c, y, xx] = q
        dec["conv5.gate"].reshape(gate.shape[0], gate.shape[1], -1)[n, c, q] = q_open
        _, g1, _ = O.loss_and_grads(spec, params, x, lab, masks, decisions=dec)
        # other windows that also chose q keep their gradient only if q is open
        others = float(sum(dpool[n, c, yy, xc] for yy in range(arg.shape[2]) for xc in range(arg.shape[3])
                           if (yy, xc) != (y, xx) and arg[n, c, yy, xc] == q))
        was_open = bool(gate.reshape(gate.shape[0], gate.shape[1], -1)[n, c, q])
        want = g0["conv5.b"].copy()
        want[c] += -dval + (dval if q_open else 0.0) + (others if (q_open and not was_open) else 0.0) \
            - (others if (was_open and not q_open) else 0.0)
        np.testing.assert_allclose(g1["conv5.b"], want, rtol=1e-9, atol=1e-16)
        for k in ("fc6.w", "fc7.w", "fc8.w", "fc6.b"):
            assert np.array_equal(g1[k], g0[k]), k


def test_one_sided_finite_differences_at_a_relu_kink():
    """Put one conv3 pre-activation exactly on zero by moving its channel's bias.  The loss then has
    a kink along that bias: its right derivative is the gradient with that unit's gate open, its left
    derivative the gradient with the gate closed -- the two answers a fp32 and a float64 forward
    pass may give for a unit within rounding of zero.  Both are checked against one-sided differences
    of the true loss (plain forward pass, no decisions)."""
    spec, params, x, lab, masks = _problem(batch=2)
    masks = [m[:2] for m in masks]
    _, _, cache = O.loss_and_grads(spec, params, x, lab, masks)
    z = cache["conv3.z"]
    n, c, yy, xx = 1, 5, 2, 3
    params = {k: v.copy() for k, v in params.items()}
    params["conv3.b"][c] -= z[n, c, yy, xx]
    loss0, _, cache = O.loss_and_grads(spec, params, x, lab, masks)
    z = cache["conv3.z"]
    assert abs(z[n, c, yy, xx]) < 1e-15
    h = 1e-7
    others = np.abs(np.delete(z[:, c].ravel(), np.ravel_multi_index((n, yy, xx), z[:, c].shape)))
    assert others.min() > 10 * h, "no other unit of the channel changes side inside the step"
    base_gate = z > 0
    grads = {}
    for is_open in (True, False):
        gate = base_gate.copy()
        gate[n, c, yy, xx] = is_open
        grads[is_open] = O.loss_and_grads(spec, params, x, lab, masks, decisions={"conv3.gate": gate})[1]["conv3.b"][c]

    def loss_at(delta):
        p = {k: v.copy() for k, v in params.items()}
        p["conv3.b"][c] += delta
        return O.loss_and_grads(spec, p, x, lab, masks)[0]

    right = (loss_at(h) - loss0) / h
    left = (loss0 - loss_at(-h)) / h
    assert abs(grads[True] - grads[False]) > 1e3 * 1e-9, "the kink must be visible"
    scale = max(abs(grads[True]), abs(grads[False]))
    assert abs(right - grads[True]) <= 2e-5 * scale + 1e-10, (right, grads[True])
    assert abs(left - grads[False]) <= 2e-5 * scale + 1e-10, (left, grads[False])
    # and the wrong pairing is told apart
    assert abs(right - grads[False]) > 10 * abs(right - grads[True])
