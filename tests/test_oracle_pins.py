"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types the oracle's own formulas: the expected values
come from a hand-derived trace (tests/golden), from PyTorch CPU library
routines in fp64 (nn.functional.linear / conv2d, autograd, optim.SGD,
cross_entropy, .to(bfloat16)), from central finite differences, and from the
delay structure the paper states (Eq. 7; the 2(D-h) remark after Eq. 8).
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as orc
import partime_streams as ps

torch.set_num_threads(2)
GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers

def t64(a):
    return torch.tensor(np.asarray(a), dtype=torch.float64)


def act_fn(act):
    return {ps.ACT_ID: lambda v: v, ps.ACT_RELU: torch.relu,
            ps.ACT_GELU: lambda v: F.gelu(v, approximate="none")}[act]


def torch_layer(l, W, b, u):
    """One layer on a batch u [S, ...] with library routines, fp64."""
    if l.kind == ps.DENSE:
        z = F.linear(u, W, b)
    elif l.kind == ps.CONV3X3:
        z = F.conv2d(u.reshape(-1, l.c_in, l.h, l.w), W, b, stride=1, padding=1).reshape(u.shape[0], -1)
    else:
        z = F.linear(u.reshape(-1, l.c_in, l.h * l.w).mean(dim=2), W, b)
    return act_fn(l.act)(z)


def torch_forward(layers, Ws, bs, x):
    u, outs = x, []
    for l, W, b in zip(layers, Ws, bs):
        u = torch_layer(l, W, b, u)
        if getattr(l, "skip_from", -1) >= 0:     # residual connection: an earlier layer's output is added
            u = u + outs[l.skip_from]
        outs.append(u)
    return u


def torch_loss(loss, o, tgt):
    if loss == ps.LOSS_MSE:
        return F.mse_loss(o, tgt, reduction="mean")          # mean over streams and outputs
    return F.cross_entropy(o, tgt.long(), reduction="mean")  # mean over streams


def rand_stream(T, S, d, seed):
    return np.random.default_rng(seed).standard_normal((T, S, d)).astype(np.float32)


def make(widths, act, loss, lr, seed=0, S=1, balance=None, k=0, bf16=False):
    layers = ps.mlp(widths, act)
    Ws, bs = ps.init_weights(layers, seed)
    o = orc.Oracle(layers, Ws, bs, balance=balance, n_streams=S, w_bf16=bf16, loss=loss, lr=lr, target_delay=k)
    return layers, Ws, bs, o


def targets_for(loss, T, S, n_out, seed):
    rng = np.random.default_rng(seed + 77)
    if loss == ps.LOSS_CE:
        return rng.integers(0, n_out, size=(T, S)).astype(np.int32)
    return rng.standard_normal((T, S, n_out)).astype(np.float32)


# ----------------------------------------------------------------------------- hand trace

def test_hand_trace_two_stages():
    rows = [l.split() for l in open(os.path.join(GOLD, "hand_trace_d2.txt")) if l.strip() and not l.startswith("#")]
    layers = ps.mlp([1, 1, 1], ps.ACT_ID)
    o = orc.Oracle(layers, [np.ones((1, 1))] * 2, [np.zeros(1)] * 2, loss=ps.LOSS_MSE, lr=0.125)
    for r in rows:
        t, out, loss, err2, w1, b1, w2, b2 = (float(v) for v in r)
        assert o.tick == int(t)
        y, l = o.step(np.ones((1, 1, 1)), np.zeros((1, 1, 1)))
        assert y[0, 0, 0] == out and l[0] == loss
        assert o.get_buffer("err", 1, int(t) & 1)[0, 0] == err2
        (W1, B1), (W2, B2) = o.get_weights(0), o.get_weights(1)
        assert (W1[0, 0], B1[0], W2[0, 0], B2[0]) == (w1, b1, w2, b2)


# ----------------------------------------------------------------------------- bf16 rounding

def test_bf16_round_to_nearest_even_matches_library_cast():
    lowers = np.array([0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff], dtype=np.uint32)
    upper = np.arange(1 << 16, dtype=np.uint32)
    bits = ((upper[:, None] << 16) | lowers[None, :]).reshape(-1)
    vals = bits.view(np.float32)
    finite = np.isfinite(vals)
    want = torch.from_numpy(vals.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    # through the oracle's weight store: a 1 x n layer with bf16 storage rounds what it is given
    n = vals.size
    layers = [ps.LayerSpec(ps.DENSE, ps.ACT_ID, n, 1)]
    o = orc.Oracle(layers, [np.where(finite, vals, 0).reshape(1, n)], [np.zeros(1)], w_bf16=True)
    got = o.get_weights(0)[0].reshape(-1)
    assert np.array_equal(got[finite].view(np.uint32), want[finite].view(np.uint32))
    assert np.isnan(orc.round_bf16(float("nan")))
    assert orc.round_bf16(float("inf")) == float("inf")


# ----------------------------------------------------------------------------- Eq. 7: delayed forward

@pytest.mark.parametrize("act", [ps.ACT_RELU, ps.ACT_GELU])
@pytest.mark.parametrize("widths,balance", [([7, 9, 8, 6, 5], None), ([7, 9, 8, 6, 5], [2, 1, 1]), ([5, 4], None)])
def test_frozen_weights_output_is_sequential_forward_of_delayed_sample(act, widths, balance):
    S, T = 2, 12
    layers, Ws, bs, o = make(widths, act, ps.LOSS_MSE, 0.0, seed=3, S=S, balance=balance)
    D = o.depth
    x = rand_stream(T, S, widths[0], 5)
    out, _ = o.step(x, np.zeros((T, S, widths[-1]), np.float32))
    ref = torch_forward(layers, [t64(W) for W in Ws], [t64(b) for b in bs], t64(x).reshape(T * S, -1)).reshape(T, S, -1)
    np.testing.assert_allclose(out[D - 1:], ref[:T - D + 1].numpy(), rtol=2e-6, atol=2e-7)
    # inference-only ticks give the same stream of outputs and never touch the weights
    o2 = make(widths, act, ps.LOSS_MSE, 0.5, seed=3, S=S, balance=balance)[3]
    out2 = o2.infer(x)
    assert np.array_equal(out2, out)
    for i in range(len(layers)):
        assert np.array_equal(o2.get_weights(i)[0], Ws[i])


def test_constant_input_reaches_sequential_output_after_depth_ticks():
    widths = [6, 6, 6, 6, 3]
    layers, Ws, bs, o = make(widths, ps.ACT_RELU, ps.LOSS_MSE, 0.0, seed=1)
    x = np.repeat(rand_stream(1, 1, 6, 2), 6, axis=0)
    out, _ = o.step(x, np.zeros((6, 1, 3), np.float32))
    ref = torch_forward(layers, [t64(W) for W in Ws], [t64(b) for b in bs], t64(x[0]))
    np.testing.assert_allclose(out[3], ref.numpy(), rtol=2e-6, atol=2e-7)
    assert np.array_equal(out[3], out[4]) and np.array_equal(out[4], out[5])


# ----------------------------------------------------------------------------- depth 1 == online SGD

@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
@pytest.mark.parametrize("act", [ps.ACT_RELU, ps.ACT_GELU])
@pytest.mark.parametrize("S,k", [(1, 0), (3, 0), (2, 2)])
def test_depth_one_is_plain_online_sgd(loss, act, S, k):
    widths, T, lr = [6, 8, 7, 4], 25, 0.05
    layers, Ws, bs, o = make(widths, act, loss, lr, seed=11, S=S, balance=[3], k=k)
    x = rand_stream(T, S, widths[0], 9)
    tg = targets_for(loss, T, S, widths[-1], 9)
    out, lo = o.step(x, tg)

    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    opt = torch.optim.SGD(params, lr=lr)
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        np.testing.assert_allclose(out[t], y.detach().numpy(), rtol=5e-5, atol=5e-6)
        if t < k:                      # no target has arrived yet: nothing to learn from
            assert lo[t] == 0.0
            continue
        L = torch_loss(loss, y, t64(tg[t - k]) if loss == ps.LOSS_MSE else torch.tensor(tg[t - k]))
        np.testing.assert_allclose(lo[t], L.item(), rtol=5e-5, atol=1e-6)
        opt.zero_grad()
        L.backward()
        opt.step()
    for i in range(len(layers)):
        W, b = o.get_weights(i)
        np.testing.assert_allclose(W, params[2 * i].detach().numpy(), rtol=1e-4, atol=2e-6)
        np.testing.assert_allclose(b, params[2 * i + 1].detach().numpy(), rtol=1e-4, atol=2e-6)


# ----------------------------------------------------------------------------- Adam (Sec. V-D trains with it)

@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
@pytest.mark.parametrize("S,k", [(1, 0), (3, 2)])
def test_depth_one_with_adam_is_torch_adam(loss, S, k):
    """One stage holding the whole network has no delays, so the oracle's Adam must walk with torch.optim.Adam
    (same betas, eps, bias correction; one optimiser step per tick)."""
    widths, T, lr, betas, eps = [6, 8, 7, 4], 30, 0.01, (0.9, 0.999), 1e-8
    layers = ps.mlp(widths, ps.ACT_GELU)
    Ws, bs = ps.init_weights(layers, 12)
    o = orc.Oracle(layers, Ws, bs, balance=[3], n_streams=S, loss=loss, lr=lr, target_delay=k, adam=(*betas, eps))
    x = rand_stream(T, S, widths[0], 10)
    tg = targets_for(loss, T, S, widths[-1], 10)
    out, lo = o.step(x, tg)
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    # the oracle takes its parameters as fp32 values: hand torch the same numbers
    opt = torch.optim.Adam(params, lr=float(np.float32(lr)), betas=tuple(float(np.float32(v)) for v in betas),
                           eps=float(np.float32(eps)))
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        np.testing.assert_allclose(out[t], y.detach().numpy(), rtol=2e-4, atol=2e-5)
        opt.zero_grad()
        if t < k:
            # no target yet: the gradient is held at zero, but the tick still counts as an optimiser step
            for q in params:
                q.grad = torch.zeros_like(q)
        else:
            L = torch_loss(loss, y, t64(tg[t - k]) if loss == ps.LOSS_MSE else torch.tensor(tg[t - k]))
            L.backward()
        opt.step()
    for i in range(len(layers)):
        W, b = o.get_weights(i)
        np.testing.assert_allclose(W, params[2 * i].detach().numpy(), rtol=5e-4, atol=1e-5)
        np.testing.assert_allclose(b, params[2 * i + 1].detach().numpy(), rtol=5e-4, atol=1e-5)
        mW, vW, mb, vb = o.get_moments(i)
        st = opt.state[params[2 * i]]
        np.testing.assert_allclose(mW, st["exp_avg"].numpy(), rtol=1e-3, atol=1e-7)
        np.testing.assert_allclose(vW, st["exp_avg_sq"].numpy(), rtol=1e-3, atol=1e-9)


def test_adam_first_step_has_the_closed_form():
    """With zero moments the first bias-corrected step is lr * g / (|g| + eps): a step of size lr against the
    sign of the gradient wherever |g| >> eps."""
    layers = [ps.LayerSpec(ps.DENSE, ps.ACT_ID, 2, 1)]
    W, b = np.array([[0.5, -0.25]], dtype=np.float32), np.array([0.125], dtype=np.float32)
    o = orc.Oracle(layers, [W], [b], loss=ps.LOSS_MSE, lr=0.1, adam=(0.9, 0.999, 1e-8))
    x = np.array([[[1.0, 2.0]]], dtype=np.float32)            # z = 0.5 - 0.5 + 0.125 = 0.125; target 1 -> g = 2 (z - 1) = -1.75
    o.step(x, np.ones((1, 1, 1), dtype=np.float32))
    W1, b1 = o.get_weights(0)
    np.testing.assert_allclose(W1, W + 0.1, rtol=0, atol=1e-7)  # dL/dW = g x = (-1.75, -3.5): both negative -> +lr
    np.testing.assert_allclose(b1, b + 0.1, rtol=0, atol=1e-7)
    mW, vW, mb, vb = o.get_moments(0)
    # the betas are fp32 values at the boundary (like the learning rate): 1 - beta is formed from those
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    np.testing.assert_allclose(mW, (1 - b1) * np.array([[-1.75, -3.5]]), rtol=1e-6)
    np.testing.assert_allclose(vW, (1 - b2) * np.array([[-1.75, -3.5]]) ** 2, rtol=1e-6)


def test_adam_counts_the_fill_ticks_of_every_stage_as_steps():
    """Two scalar stages (identity, w = 1, x = 1, target 0, squared error): the last stage sees its first gradient
    (2) at tick 1, the first stage (through the error published then) at tick 2; the ticks before carry a zero gradient
    but count as optimiser steps, so the bias corrections of those first real steps are those of step 2 and step 3.
    torch.optim.Adam, stepped with the same gradient sequences, must land on the same weights."""
    layers = [ps.LayerSpec(ps.DENSE, ps.ACT_ID, 1, 1), ps.LayerSpec(ps.DENSE, ps.ACT_ID, 1, 1)]
    one, zero = np.ones((1, 1), dtype=np.float32), np.zeros(1, dtype=np.float32)
    lr, betas, eps = 0.01, (0.9, 0.999), 1e-8
    x, tg = np.ones((3, 1, 1), dtype=np.float32), np.zeros((3, 1, 1), dtype=np.float32)

    def torch_walk(grads):
        q = torch.ones(1, dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([q], lr=float(np.float32(lr)), betas=tuple(float(np.float32(v)) for v in betas),
                               eps=float(np.float32(eps)))
        for g in grads:
            q.grad = torch.full_like(q, g)
            opt.step()
        return q.item()

    o = orc.Oracle(layers, [one.copy(), one.copy()], [zero.copy(), zero.copy()], loss=ps.LOSS_MSE, lr=lr, target_delay=0,
                   adam=(*betas, eps))
    o.step(x[:2], tg[:2])
    assert o.get_weights(0)[0][0, 0] == 1.0                       # no gradient has reached the first stage yet
    w2 = o.get_weights(1)[0][0, 0]
    np.testing.assert_allclose(w2, torch_walk([0.0, 2.0]), rtol=1e-6)
    # (had the fill tick not counted, the first real step would be a full lr)
    assert abs((1.0 - w2) / lr - 1.0) > 0.2
    o.step(x[2:], tg[2:])
    np.testing.assert_allclose(o.get_weights(0)[0][0, 0], torch_walk([0.0, 0.0, 2.0]), rtol=1e-6)


def test_delay_lines_of_a_skip_by_age():
    """Test access to the delay lines: with frozen weights the entry of age j of the skipped tensor is the source layer's
    output for the sample that entered the pipeline j ticks before the last one (Eq. 7 at the source's stage), computed
    here with torch; an entry written and read back is unchanged and ages by one per tick."""
    widths, S = [5, 6, 6, 6, 6, 3], 2
    layers = ps.mlp(widths, ps.ACT_GELU)
    layers[3].skip_from = 0                                   # crosses three stage boundaries
    Ws, bs = ps.init_weights(layers, 31)
    o = orc.Oracle(layers, Ws, bs, n_streams=S, loss=ps.LOSS_MSE, lr=0.0)
    assert [o.skip_delay(i) for i in range(5)] == [0, 0, 0, 3, 0]
    T = 7
    x = rand_stream(T, S, 5, 3)
    o.step(x, targets_for(ps.LOSS_MSE, T, S, 3, 3))
    for age in range(3):
        # the source is layer 0 = stage 0: its output at tick t belongs to the sample of tick t
        want = torch.nn.functional.gelu(t64(x[T - 1 - age]) @ t64(Ws[0]).T + t64(bs[0])).numpy()
        np.testing.assert_allclose(o.get_lane(0, 3, age), want, rtol=1e-6, atol=1e-7)
    a1 = o.get_lane(0, 3, 1)
    o.set_lane(0, 3, 1, a1 * 2)
    assert np.array_equal(o.get_lane(0, 3, 1), a1 * 2)
    o.step(x[:1], targets_for(ps.LOSS_MSE, 1, S, 3, 4))
    assert np.array_equal(o.get_lane(0, 3, 2), a1 * 2)


# ----------------------------------------------------------------------------- Eq. 9 at steady state

@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
@pytest.mark.parametrize("balance", [None, [2, 1], [1, 2]])
def test_steady_state_gradient_is_true_gradient(loss, balance):
    """Constant (x, target) and frozen weights: every stale quantity equals the fresh one, so
    the stage gradients of Eq. 9 must equal the exact gradient of the sequential network."""
    widths, S = [3, 4, 3, 2], 2
    layers, Ws, bs, o = make(widths, ps.ACT_GELU, loss, 0.0, seed=21, S=S, balance=balance)
    T = 2 * o.depth + 1
    x1 = rand_stream(1, S, 3, 4)
    tg1 = targets_for(loss, 1, S, 2, 4)
    o.step(np.repeat(x1, T, axis=0), np.repeat(tg1, T, axis=0))

    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    tgt = t64(tg1[0]) if loss == ps.LOSS_MSE else torch.tensor(tg1[0])

    def L_of(ps_):
        return torch_loss(loss, torch_forward(layers, ps_[0::2], ps_[1::2], t64(x1[0])), tgt)

    grads = torch.autograd.grad(L_of(params), params)
    for i in range(len(layers)):
        dW, db = o.get_grads(i)
        np.testing.assert_allclose(dW, grads[2 * i].numpy(), rtol=1e-6, atol=1e-9)
        np.testing.assert_allclose(db, grads[2 * i + 1].numpy(), rtol=1e-6, atol=1e-9)
    # brute-force central finite differences on every parameter
    eps = 1e-5
    base = [p.detach().clone() for p in params]
    for i in range(len(layers)):
        dW, db = o.get_grads(i)
        for j, got in ((2 * i, dW), (2 * i + 1, db)):
            fd = np.zeros(got.size)
            for e in range(got.size):
                vals = []
                for sgn in (+1, -1):
                    q = [b.clone() for b in base]
                    q[j].view(-1)[e] += sgn * eps
                    vals.append(L_of(q).item())
                fd[e] = (vals[0] - vals[1]) / (2 * eps)
            np.testing.assert_allclose(got.reshape(-1), fd, rtol=1e-6, atol=1e-8)


# ----------------------------------------------------------------------------- delays: 2(D-h)

def test_forward_and_error_delays_per_stage():
    """Frozen ReLU net, fast-changing stream: the error that stage h (1-based) publishes at tick t
    is the loss gradient of the sample that ENTERED at tick t-(2D-h-1), pulled back through the
    Jacobian of stage j (j = D..h) evaluated at the sample stage j was processing when it handled
    that error; the weight gradient pairs it with the stage's input of THIS tick, i.e. sample
    t-(h-1).  The gap between the two sample indices is 2(D-h) (remark after Eq. 8)."""
    widths = [5, 6, 7, 6, 4]
    D, T = 4, 16
    layers, Ws, bs, o = make(widths, ps.ACT_RELU, ps.LOSS_MSE, 0.0, seed=31)
    Wt, bt = [t64(W) for W in Ws], [t64(b) for b in bs]
    x = rand_stream(T, 1, 5, 6)
    tg = targets_for(ps.LOSS_MSE, T, 1, 4, 6)

    def stage_pre(j, sample):          # pre-activation of stage j (1-based) for a given sample, and its input
        u = t64(x[sample])
        for i in range(j - 1):
            u = torch_layer(layers[i], Wt[i], bt[i], u)
        return F.linear(u, Wt[j - 1], bt[j - 1]), u

    def relu_mask(j, z):
        return (z > 0).double() if layers[j - 1].act == ps.ACT_RELU else torch.ones_like(z)

    k = 0
    for t in range(T):
        o.step(x[t:t + 1], tg[t:t + 1])
        for h in range(1, D + 1):
            s_loss = t - (2 * D - h - 1)          # sample whose loss arrives at stage h now
            if s_loss < 0:
                continue
            # loss gradient of that sample: it left the last stage at tick s_loss + D - 1 against target of that tick
            zD, _ = stage_pre(D, s_loss)
            g = 2.0 * (zD - t64(tg[s_loss + D - 1 - k])) / widths[-1]
            for j in range(D, h, -1):             # stages above h: Jacobian w.r.t. their input
                zj, _ = stage_pre(j, t - 2 * j + h + 1)
                g = (g * relu_mask(j, zj)) @ Wt[j - 1]
            zh, uh = stage_pre(h, t - (h - 1))    # this tick's own forward: sample t-(h-1)
            assert (t - (h - 1)) - s_loss == 2 * (D - h)
            delta = g * relu_mask(h, zh)
            dW, db = o.get_grads(h - 1)
            np.testing.assert_allclose(dW, (delta.T @ uh).numpy(), rtol=1e-5, atol=1e-7)
            np.testing.assert_allclose(db, delta[0].numpy(), rtol=1e-5, atol=1e-7)
            if h > 1:
                np.testing.assert_allclose(o.get_buffer("err", h - 1, t & 1), (delta @ Wt[h - 1]).numpy(),
                                           rtol=1e-5, atol=1e-7)


# ----------------------------------------------------------------------------- order of stages in a tick

@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_stage_order_inside_a_tick_is_irrelevant(loss):
    widths, T, S = [6, 7, 8, 7, 5], 30, 2
    x = rand_stream(T, S, 6, 8)
    tg = targets_for(loss, T, S, 5, 8)
    res = []
    for order in (None, [3, 2, 1, 0], [2, 0, 3, 1]):
        o = make(widths, ps.ACT_RELU, loss, 0.05, seed=41, S=S, k=3)[3]
        out, lo = o.step(x, tg, order=order)
        res.append((out, lo, [o.get_weights(i) for i in range(4)]))
    for out, lo, ws in res[1:]:
        assert np.array_equal(out, res[0][0]) and np.array_equal(lo, res[0][1])
        for (W, b), (W0, b0) in zip(ws, res[0][2]):
            assert np.array_equal(W, W0) and np.array_equal(b, b0)


def test_chunked_calls_equal_one_call():
    widths, T = [6, 7, 5, 4], 20
    x = rand_stream(T, 1, 6, 12)
    tg = targets_for(ps.LOSS_CE, T, 1, 4, 12)
    a = make(widths, ps.ACT_GELU, ps.LOSS_CE, 0.05, seed=5, k=2)[3]
    b = make(widths, ps.ACT_GELU, ps.LOSS_CE, 0.05, seed=5, k=2)[3]
    oa, la = a.step(x, tg)
    parts = [b.step(x[i:j], tg[i:j]) for i, j in ((0, 1), (1, 2), (2, 9), (9, 20))]
    assert np.array_equal(oa, np.concatenate([p[0] for p in parts]))
    assert np.array_equal(la, np.concatenate([p[1] for p in parts]))


# ----------------------------------------------------------------------------- fill ticks and kinks

def test_nothing_is_learned_before_the_pipeline_is_full():
    widths, D = [4, 5, 6, 3], 3
    for k in (0, 2, 4):
        layers, Ws, bs, o = make(widths, ps.ACT_RELU, ps.LOSS_MSE, 0.1, seed=2, k=k)
        fill = max(D - 1, k)
        x = rand_stream(fill, 1, 4, 3)
        _, lo = o.step(x, targets_for(ps.LOSS_MSE, fill, 1, 3, 3))
        assert np.all(lo == 0)
        for i in range(3):
            assert np.array_equal(o.get_weights(i)[0], Ws[i]) and np.array_equal(o.get_weights(i)[1], bs[i])
        _, lo = o.step(rand_stream(1, 1, 4, 4), targets_for(ps.LOSS_MSE, 1, 1, 3, 4))
        assert lo[0] > 0 and not np.array_equal(o.get_weights(2)[0], Ws[2])


def test_relu_derivative_at_zero_is_zero():
    layers = ps.mlp([2, 2, 1], ps.ACT_RELU)
    Ws = [np.zeros((2, 2), np.float32), np.ones((1, 2), np.float32)]
    bs = [np.zeros(2, np.float32), np.zeros(1, np.float32)]
    o = orc.Oracle(layers, Ws, bs, loss=ps.LOSS_MSE, lr=1.0)
    o.step(np.ones((4, 1, 2), np.float32), np.ones((4, 1, 1), np.float32))
    assert np.array_equal(o.get_weights(0)[0], Ws[0]) and np.array_equal(o.get_weights(0)[1], bs[0])
    assert not np.array_equal(o.get_weights(1)[1], bs[1])


# ----------------------------------------------------------------------------- conv / pooled head

def conv_net():
    return [ps.LayerSpec(ps.CONV3X3, ps.ACT_GELU, c_in=2, c_out=3, h=5, w=4),
            ps.LayerSpec(ps.CONV3X3, ps.ACT_GELU, c_in=3, c_out=2, h=5, w=4),
            ps.LayerSpec(ps.GAP_DENSE, ps.ACT_ID, out_dim=3, c_in=2, h=5, w=4)]


def test_conv_pipeline_forward_and_steady_gradient():
    layers = conv_net()
    Ws, bs = ps.init_weights(layers, 7)
    S = 2
    o = orc.Oracle(layers, Ws, bs, n_streams=S, loss=ps.LOSS_CE, lr=0.0)
    T = 7
    x = rand_stream(T, S, 2 * 5 * 4, 3)
    tg = targets_for(ps.LOSS_CE, T, S, 3, 3)
    out, _ = o.step(x, tg)
    Wt, bt = [t64(W) for W in Ws], [t64(b) for b in bs]
    ref = torch_forward(layers, Wt, bt, t64(x).reshape(T * S, -1)).reshape(T, S, -1)
    np.testing.assert_allclose(out[2:], ref[:T - 2].numpy(), rtol=2e-6, atol=2e-7)
    # steady state: exact gradient
    o.reset()
    o.step(np.repeat(x[:1], T, axis=0), np.repeat(tg[:1], T, axis=0))
    params = [p.clone().requires_grad_(True) for pair in zip(Wt, bt) for p in pair]
    L = torch_loss(ps.LOSS_CE, torch_forward(layers, params[0::2], params[1::2], t64(x[0])), torch.tensor(tg[0]))
    grads = torch.autograd.grad(L, params)
    for i in range(3):
        dW, db = o.get_grads(i)
        np.testing.assert_allclose(dW, grads[2 * i].numpy(), rtol=1e-6, atol=2e-9)  # inter-stage vectors are fp32 between ticks
        np.testing.assert_allclose(db, grads[2 * i + 1].numpy(), rtol=1e-6, atol=2e-9)  # inter-stage vectors are fp32 between ticks


def test_conv_depth_one_is_online_sgd():
    layers = conv_net()
    Ws, bs = ps.init_weights(layers, 8)
    o = orc.Oracle(layers, Ws, bs, balance=[3], loss=ps.LOSS_CE, lr=0.1)
    T = 10
    x = rand_stream(T, 1, 40, 5)
    tg = targets_for(ps.LOSS_CE, T, 1, 3, 5)
    out, lo = o.step(x, tg)
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    opt = torch.optim.SGD(params, lr=0.1)
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        L = torch_loss(ps.LOSS_CE, y, torch.tensor(tg[t]))
        np.testing.assert_allclose(lo[t], L.item(), rtol=5e-5)
        opt.zero_grad(); L.backward(); opt.step()
    for i in range(3):
        np.testing.assert_allclose(o.get_weights(i)[0], params[2 * i].detach().numpy(), rtol=1e-4, atol=2e-6)


def test_conv_depth_one_with_adam_is_torch_adam():
    """The update rule does not depend on the kind of layer: a conv net with its pooled head in one stage, trained
    with Adam, walks with torch.optim.Adam (moments of the conv kernels included)."""
    layers = conv_net()
    Ws, bs = ps.init_weights(layers, 8)
    lr, betas, eps = 0.01, (0.9, 0.999), 1e-8
    o = orc.Oracle(layers, Ws, bs, balance=[3], loss=ps.LOSS_CE, lr=lr, adam=(*betas, eps))
    T = 12
    x = rand_stream(T, 1, 40, 5)
    tg = targets_for(ps.LOSS_CE, T, 1, 3, 5)
    out, lo = o.step(x, tg)
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    opt = torch.optim.Adam(params, lr=float(np.float32(lr)), betas=tuple(float(np.float32(v)) for v in betas),
                           eps=float(np.float32(eps)))
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        L = torch_loss(ps.LOSS_CE, y, torch.tensor(tg[t]))
        np.testing.assert_allclose(lo[t], L.item(), rtol=2e-4)
        opt.zero_grad(); L.backward(); opt.step()
    for i in range(3):
        W, b = o.get_weights(i)
        np.testing.assert_allclose(W, params[2 * i].detach().numpy(), rtol=5e-4, atol=1e-5)
        np.testing.assert_allclose(b, params[2 * i + 1].detach().numpy(), rtol=5e-4, atol=1e-5)
        mW, vW, mb, vb = o.get_moments(i)
        st = opt.state[params[2 * i]]
        np.testing.assert_allclose(mW, st["exp_avg"].numpy(), rtol=1e-3, atol=1e-7)
        np.testing.assert_allclose(vW, st["exp_avg_sq"].numpy(), rtol=1e-3, atol=1e-9)


# ----------------------------------------------------------------------------- bf16 storage

def test_bf16_storage_depth_one_tracks_library_bf16_sgd():
    """Weights held in bf16, arithmetic in high precision, round-to-nearest-even on every store:
    reproduced with torch by casting the parameters through bfloat16 after every SGD step."""
    widths, T, lr = [8, 8, 4], 15, 0.05
    layers, Ws, bs, o = make(widths, ps.ACT_GELU, ps.LOSS_MSE, lr, seed=13, balance=[2], bf16=True)
    x = rand_stream(T, 1, 8, 2)
    tg = targets_for(ps.LOSS_MSE, T, 1, 4, 2)
    out, lo = o.step(x, tg)
    rb = lambda a: torch.tensor(a).to(torch.bfloat16).to(torch.float64)
    Wp = [rb(W).requires_grad_(True) for W in Ws]
    bp = [t64(b).requires_grad_(True) for b in bs]
    for t in range(T):
        y = torch_forward(layers, Wp, bp, t64(x[t]))
        np.testing.assert_allclose(out[t], y.detach().numpy(), rtol=1e-5, atol=1e-6)
        L = torch_loss(ps.LOSS_MSE, y, t64(tg[t]))
        gs = torch.autograd.grad(L, Wp + bp)
        with torch.no_grad():
            for i in range(2):
                Wp[i].copy_((Wp[i] - lr * gs[i]).to(torch.float32).to(torch.bfloat16).to(torch.float64))
                bp[i].copy_((bp[i] - lr * gs[2 + i]).to(torch.float32).to(torch.float64))
    for i in range(2):
        W, _ = o.get_weights(i)
        # a stored value may differ by one bf16 step only where the exact value sits on a rounding boundary
        diff = np.abs(W - Wp[i].detach().numpy())
        assert np.mean(diff == 0) > 0.97 and np.all(diff <= np.abs(W) * 2.0 ** -7 + 1e-30)


# ----------------------------------------------------------------------------- bf16 operands (multi-stream)

def test_bf16_operand_rounding_depth_one_against_autograd_with_rounding_hooks():
    """Multi-stream bf16 configuration: what enters a product (layer inputs, deltas) is bf16.  Reproduced
    with torch autograd: inputs pass through a straight-through bf16 cast, the gradient arriving at every
    pre-activation is cast to bf16 by a hook.  S is a power of two so that the 1/S of the mean commutes
    with the rounding."""
    widths, T, lr, S = [8, 12, 6], 6, 0.05, 4
    layers, Ws, bs, _ = make(widths, ps.ACT_GELU, ps.LOSS_MSE, lr, seed=17)
    o = orc.Oracle(layers, Ws, bs, balance=[2], n_streams=S, w_bf16=True, loss=ps.LOSS_MSE, lr=lr, operands_bf16=True)
    x = rand_stream(T, S, 8, 3)
    tg = targets_for(ps.LOSS_MSE, T, S, 6, 3)
    rb = lambda a: a.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    st = lambda v: v + (rb(v) - v).detach()                       # forward: rounded, backward: identity
    Wp = [rb(t64(W)).requires_grad_(True) for W in Ws]
    bp = [t64(b).requires_grad_(True) for b in bs]
    for t in range(T):
        out_t, lo_t = o.step(x[t:t + 1], tg[t:t + 1])
        u = st(t64(x[t]))
        zs = []
        for i, l in enumerate(layers):
            z = F.linear(u, Wp[i], bp[i])
            z.register_hook(lambda g: rb(g * S) / S)               # delta (per-stream scale) rounded to bf16
            zs.append(z)
            u = act_fn(l.act)(z)
            if i + 1 < len(layers):
                u = st(u)
        np.testing.assert_allclose(out_t[0], u.detach().numpy(), rtol=1e-5, atol=1e-6)
        L = torch_loss(ps.LOSS_MSE, u, t64(tg[t]))
        np.testing.assert_allclose(lo_t[0], L.item(), rtol=1e-5)
        gs = torch.autograd.grad(L, Wp + bp)
        for i in range(2):
            dW, db = o.get_grads(i)
            np.testing.assert_allclose(dW, gs[i].numpy(), rtol=1e-6, atol=1e-12)
            np.testing.assert_allclose(db, gs[2 + i].numpy(), rtol=1e-6, atol=1e-12)
        with torch.no_grad():
            for i in range(2):
                Wp[i].copy_(rb(Wp[i] - lr * gs[i]))
                bp[i].copy_((bp[i] - lr * gs[2 + i]).to(torch.float32).to(torch.float64))


def test_kink_margin_diagnostic_reports_smallest_relu_preactivation():
    """The diagnostic the GPU parity tests use to detect ReLU decisions within rounding distance: for a one-stage
    net with known pre-activations it returns min |z| over the units that carry a non-zero error signal."""
    layers = [ps.LayerSpec(ps.DENSE, ps.ACT_RELU, 2, 3)]
    W = np.array([[1.0, 0.0], [0.0, -2.0], [0.5, 0.5]], dtype=np.float32)
    b = np.array([0.0, 0.0, -0.5], dtype=np.float32)
    ref = orc.Oracle(layers, [W], [b], loss=ps.LOSS_MSE, lr=0.0)
    assert ref.take_kink_margin() > 1e299                      # nothing seen yet
    x = np.array([[[0.25, 0.75]]], dtype=np.float32)           # z = (0.25, -1.5, 0.0)
    ref.step(x, np.ones((1, 1, 3), dtype=np.float32))
    assert ref.take_kink_margin() == 0.0                       # third unit sits exactly on the kink
    assert ref.take_kink_margin() > 1e299                      # taking it resets it
    x = np.array([[[0.25, 0.5]]], dtype=np.float32)            # z = (0.25, -1.0, -0.125)
    ref.step(x, np.ones((1, 1, 3), dtype=np.float32))
    assert ref.take_kink_margin() == 0.125


def test_kink_band_records_units_near_zero_and_takes_the_chosen_one_sided_derivative():
    """The band diagnostic of the GPU parity tests on a one-stage net with hand-set pre-activations (all values dyadic):
    units inside the band with a non-zero error signal are recorded, side 0 leaves ReLU'(z) = [z > 0], side +1 / -1
    takes 1 / 0 for exactly those units; everything else is untouched."""
    layers = [ps.LayerSpec(ps.DENSE, ps.ACT_RELU, 2, 4)]
    W = np.array([[1.0, 0.0], [0.0, -2.0], [0.5, 0.5], [0.25, 0.0]], dtype=np.float32)
    b = np.array([0.0, 0.0, -0.5 + 2.0 ** -20, -0.0625 - 2.0 ** -20], dtype=np.float32)
    x = np.array([[[0.25, 0.75]]], dtype=np.float32)           # z = (0.25, -1.5, +2^-20, -2^-20)
    y = np.zeros((1, 1, 4), dtype=np.float32)                  # MSE: g = 2 (o - y) / 4 = o / 2
    y[0, 0, 3] = 1.0                                           # unit 3 has o = 0, so g = -0.5 (non-zero)
    y[0, 0, 1] = 0.0                                           # unit 1: o = 0, y = 0: g = 0, never recorded
    # sizes of the units' terms, sum |w u| + |b|: 0.25, 1.5, 1 - 2^-20, 0.125 + 2^-20; the band is relative to them
    grads = {}
    for side in (0, 1, -1):
        ref = orc.Oracle(layers, [W], [b], loss=ps.LOSS_MSE, lr=0.0)
        ref.set_kink_band(2.0 ** -16, side)                    # unit 3: 2^-20 < 2^-16 * 0.125 = 2^-19
        ref.step(x, y)
        cnt, ev = ref.take_kink_events()
        assert cnt == 2 and ev.tolist() == [[0, 0, 2], [0, 0, 3]]        # (tick, layer, unit); unit 0 and 1 are far / silent
        assert ref.take_kink_events()[0] == 0                            # taking them resets the count
        grads[side] = ref.get_grads(0)[1]                                # db = delta
    g2, g3 = 2.0 ** -21, -0.5                                            # g = o / 2 for unit 2, (0 - 1) / 2 for unit 3
    assert grads[0].tolist() == [0.125, 0.0, g2, 0.0]                    # [z > 0]: unit 2 active, unit 3 not
    assert grads[1].tolist() == [0.125, 0.0, g2, g3]                     # band counted as active
    assert grads[-1].tolist() == [0.125, 0.0, 0.0, 0.0]                  # band counted as inactive
    # the band is relative to the size of the unit's own terms: 2^-18 reaches unit 2 (terms of size 1: 2^-20 < 2^-18) but
    # not unit 3 (terms of size 1/8: 2^-20 > 2^-21)
    ref = orc.Oracle(layers, [W], [b], loss=ps.LOSS_MSE, lr=0.0)
    ref.set_kink_band(2.0 ** -18, -1)
    ref.step(x, y)
    cnt, ev = ref.take_kink_events()
    assert cnt == 1 and ev.tolist() == [[0, 0, 2]] and ref.get_grads(0)[1].tolist() == [0.125, 0.0, 0.0, 0.0]
    # a band that the units are outside of changes nothing and records nothing
    ref = orc.Oracle(layers, [W], [b], loss=ps.LOSS_MSE, lr=0.0)
    ref.set_kink_band(2.0 ** -21, 1)
    ref.step(x, y)
    assert ref.take_kink_events()[0] == 0 and ref.get_grads(0)[1].tolist() == grads[0].tolist()


@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_clone_continues_exactly_like_the_original(adam):
    """A clone carries everything that crosses a tick boundary: weights, moments, both halves of the buffers, skip lanes,
    the target history and the tick; stepping both gives bit-identical results, and they do not share memory."""
    layers = skip_mlp_layers([6, 8, 8, 8, 5], {2: 1}, ps.ACT_RELU)
    Ws, bs = ps.init_weights(layers, 3)
    ref = orc.Oracle(layers, Ws, bs, loss=ps.LOSS_CE, lr=0.05, target_delay=2, balance=[1, 2, 1], adam=adam)
    x = rand_stream(16, 1, 6, 5)
    tg = targets_for(ps.LOSS_CE, 16, 1, 5, 5)
    ref.step(x[:9], tg[:9])
    twin = ref.clone()
    assert twin.tick == 9
    o1, l1 = ref.step(x[9:], tg[9:])
    w_after = ref.get_weights(0)[0].copy()
    o2, l2 = twin.step(x[9:], tg[9:])                                   # the original has moved on: no shared state
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    for i in range(len(layers)):
        for a, c in zip(ref.get_weights(i), twin.get_weights(i)):
            assert np.array_equal(a, c)
        if adam:
            for a, c in zip(ref.get_moments(i), twin.get_moments(i)):
                assert np.array_equal(a, c)
    assert np.array_equal(ref.get_weights(0)[0], w_after)


def skip_mlp_layers(widths, skips, act):
    layers = ps.mlp(widths, act)
    for dst, src in skips.items():
        layers[dst].skip_from = src
    return layers


# ----------------------------------------------------------------------------- skip connections (Sec. V-C)

def skip_mlp(widths, skips, act):
    layers = ps.mlp(widths, act)
    for dst, src in skips.items():
        layers[dst].skip_from = src
    return layers


@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_depth_one_with_skips_is_plain_online_sgd(loss):
    """All layers in one stage: no delays, so the oracle with residual connections must walk with autograd + SGD."""
    layers = skip_mlp([6, 8, 8, 8, 8, 4], {2: 0, 3: 1}, ps.ACT_GELU)     # 6-8-8-8-8-4 with skips 0->2 and 1->3
    Ws, bs = ps.init_weights(layers, 31)
    T, S, lr = 20, 2, 0.05
    o = orc.Oracle(layers, Ws, bs, balance=[5], n_streams=S, loss=loss, lr=lr)
    x, tg = rand_stream(T, S, 6, 3), targets_for(loss, T, S, 4, 3)
    out, lo = o.step(x, tg)
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    opt = torch.optim.SGD(params, lr=lr)
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        np.testing.assert_allclose(out[t], y.detach().numpy(), rtol=5e-5, atol=5e-6)
        L = torch_loss(loss, y, t64(tg[t]) if loss == ps.LOSS_MSE else torch.tensor(tg[t]))
        opt.zero_grad()
        L.backward()
        opt.step()
    for i in range(len(layers)):
        np.testing.assert_allclose(o.get_weights(i)[0], params[2 * i].detach().numpy(), rtol=1e-4, atol=2e-6)


@pytest.mark.parametrize("balance", [[1, 1, 1, 1, 1], [2, 1, 2], [1, 3, 1]])
def test_skips_across_stages_arrive_with_their_sample(balance):
    """Frozen weights: whatever the cut into stages, out[t] is the sequential forward (with its residual adds) of the
    sample that entered depth-1 ticks earlier (Eq. 7): the identity lanes delay a skipped tensor exactly as long as
    the stages it passes delay the main path."""
    layers = skip_mlp([5, 7, 7, 7, 7, 3], {2: 1, 3: 0}, ps.ACT_GELU)     # 1->2 (neighbours) and 0->3 (up to three boundaries)
    Ws, bs = ps.init_weights(layers, 32)
    o = orc.Oracle(layers, Ws, bs, balance=balance, loss=ps.LOSS_MSE, lr=0.0)
    T, D = 14, len(balance)
    x = rand_stream(T, 1, 5, 4)
    out, _ = o.step(x, np.zeros((T, 1, 3), dtype=np.float32))
    for t in range(D - 1, T):
        y = torch_forward(layers, [t64(W) for W in Ws], [t64(b) for b in bs], t64(x[t - D + 1]))
        np.testing.assert_allclose(out[t], y.numpy(), rtol=1e-5, atol=1e-6)
    np.testing.assert_array_equal(out, o_infer_again(layers, Ws, bs, balance, x))


def o_infer_again(layers, Ws, bs, balance, x):
    return orc.Oracle(layers, Ws, bs, balance=balance, loss=ps.LOSS_MSE, lr=0.0).infer(x)


@pytest.mark.parametrize("balance", [[1, 1, 1, 1], [2, 2], [1, 2, 1]])
def test_skip_gradients_at_steady_state_are_true_gradients(balance):
    """Constant (x, target), frozen weights: every stale quantity equals the fresh one, so the stage gradients must
    equal the exact gradient of the sequential network with its residual connections."""
    layers = skip_mlp([4, 6, 6, 6, 3], {2: 0}, ps.ACT_GELU)
    Ws, bs = ps.init_weights(layers, 33)
    o = orc.Oracle(layers, Ws, bs, balance=balance, n_streams=2, loss=ps.LOSS_MSE, lr=0.0)
    T = 2 * len(balance) + 2
    x1, tg1 = rand_stream(1, 2, 4, 5), targets_for(ps.LOSS_MSE, 1, 2, 3, 5)
    o.step(np.repeat(x1, T, axis=0), np.repeat(tg1, T, axis=0))
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    L = torch_loss(ps.LOSS_MSE, torch_forward(layers, params[0::2], params[1::2], t64(x1[0])), t64(tg1[0]))
    grads = torch.autograd.grad(L, params)
    for i in range(len(layers)):
        dW, db = o.get_grads(i)
        np.testing.assert_allclose(dW, grads[2 * i].numpy(), rtol=1e-6, atol=1e-9)
        np.testing.assert_allclose(db, grads[2 * i + 1].numpy(), rtol=1e-6, atol=1e-9)


def test_skip_gradient_lane_has_the_delay_of_the_stages_it_passes():
    """Scalar identity layers w0, w1, w2 in three stages, skip from stage 0's output to stage 2's output, frozen
    weights, constant input 1, a target that changes every tick.  The loss gradient formed at tick s reaches stage 0
    at tick s + 2 both over the main path (g w2 w1) and over the lane (g), so
    dW0(t) = (o(t-2) - y(t-2)) * (w2 w1 + 1) * x  with  o = w2 w1 w0 + w0  (half squared error would drop the 2;
    the mean squared error of one output gives g = 2 (o - y))."""
    layers = ps.mlp([1, 1, 1, 1], ps.ACT_ID)
    layers[2].skip_from = 0
    w0, w1, w2 = 0.5, -1.5, 0.75
    Ws = [np.array([[w]], dtype=np.float32) for w in (w0, w1, w2)]
    bs = [np.zeros(1, dtype=np.float32)] * 3
    o = orc.Oracle(layers, Ws, bs, loss=ps.LOSS_MSE, lr=0.0, target_delay=0)
    T = 10
    y = np.arange(T, dtype=np.float32).reshape(T, 1, 1) * 0.25
    x = np.ones((T, 1, 1), dtype=np.float32)
    out_const = w2 * w1 * w0 + w0
    for t in range(T):
        o.step(x[t:t + 1], y[t:t + 1])
        dW0, _ = o.get_grads(0)
        if t >= 4:      # past the fill ticks (t < 2) and the two ticks the first real gradient needs to come down
            g = 2.0 * (out_const - float(y[t - 2, 0, 0]))
            np.testing.assert_allclose(dW0[0, 0], g * (w2 * w1 + 1.0), rtol=1e-6)


# ----------------------------------------------------------------------------- skip connections between conv layers

def conv_skip_net(act=ps.ACT_GELU):
    """conv 2->3, conv 3->3, conv 3->3 (+ output of layer 0), conv 3->3 (+ output of layer 2), conv 3->2, pooled head."""
    c = [(2, 3), (3, 3), (3, 3), (3, 3), (3, 2)]
    layers = [ps.LayerSpec(ps.CONV3X3, act, c_in=a, c_out=b, h=4, w=5) for a, b in c]
    layers.append(ps.LayerSpec(ps.GAP_DENSE, ps.ACT_ID, out_dim=3, c_in=2, h=4, w=5))
    layers[2].skip_from = 0
    layers[3].skip_from = 2
    return layers


@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_conv_depth_one_with_skips_is_plain_online_sgd(loss):
    """All conv layers and the head in one stage: no delays, so residual connections between feature maps must walk
    with autograd + SGD on library convolutions."""
    layers = conv_skip_net()
    Ws, bs = ps.init_weights(layers, 51)
    T, S, lr = 12, 2, 0.1
    o = orc.Oracle(layers, Ws, bs, balance=[6], n_streams=S, loss=loss, lr=lr)
    x, tg = rand_stream(T, S, 2 * 4 * 5, 6), targets_for(loss, T, S, 3, 6)
    out, lo = o.step(x, tg)
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    opt = torch.optim.SGD(params, lr=lr)
    for t in range(T):
        y = torch_forward(layers, params[0::2], params[1::2], t64(x[t]))
        np.testing.assert_allclose(out[t], y.detach().numpy(), rtol=5e-5, atol=5e-6)
        L = torch_loss(loss, y, t64(tg[t]) if loss == ps.LOSS_MSE else torch.tensor(tg[t]))
        np.testing.assert_allclose(lo[t], L.item(), rtol=5e-5)
        opt.zero_grad()
        L.backward()
        opt.step()
    for i in range(len(layers)):
        assert np.abs(params[2 * i].detach().numpy() - Ws[i]).max() > 1e-4          # the walk is not a standstill
        np.testing.assert_allclose(o.get_weights(i)[0], params[2 * i].detach().numpy(), rtol=1e-4, atol=2e-6)
        np.testing.assert_allclose(o.get_weights(i)[1], params[2 * i + 1].detach().numpy(), rtol=1e-4, atol=2e-6)


@pytest.mark.parametrize("balance", [[1, 1, 1, 1, 1, 1], [2, 2, 2], [1, 3, 2], [3, 1, 1, 1]])
def test_conv_skips_across_stages_arrive_with_their_sample(balance):
    """Frozen weights: whatever the cut into stages, out[t] is the sequential forward, residual adds included, of the
    sample that entered depth - 1 ticks earlier (Eq. 7): a skipped feature map is delayed exactly as long as the
    stages it passes delay the main path."""
    layers = conv_skip_net()
    Ws, bs = ps.init_weights(layers, 52)
    o = orc.Oracle(layers, Ws, bs, balance=balance, loss=ps.LOSS_MSE, lr=0.0)
    T, D = 14, len(balance)
    x = rand_stream(T, 1, 40, 7)
    out, _ = o.step(x, np.zeros((T, 1, 3), dtype=np.float32))
    for t in range(D - 1, T):
        y = torch_forward(layers, [t64(W) for W in Ws], [t64(b) for b in bs], t64(x[t - D + 1]))
        np.testing.assert_allclose(out[t], y.numpy(), rtol=1e-5, atol=1e-6)
    # without the residual adds the same frames give another output: the check above sees them
    plain = conv_skip_net()
    for l in plain:
        l.skip_from = -1
    y0 = torch_forward(plain, [t64(W) for W in Ws], [t64(b) for b in bs], t64(x[T - D]))
    assert np.abs(out[T - 1] - y0.numpy()).max() > 1e-3


@pytest.mark.parametrize("balance", [[1, 1, 1, 1, 1, 1], [2, 2, 2], [1, 2, 2, 1]])
def test_conv_skip_gradients_at_steady_state_are_true_gradients(balance):
    """Constant (x, target), frozen weights: every stale quantity equals the fresh one, so the stage gradients of the
    conv kernels must equal the exact gradient of the sequential network with its residual connections, for a
    residual block that lies inside a stage and for one that crosses stage boundaries."""
    layers = conv_skip_net()
    Ws, bs = ps.init_weights(layers, 53)
    o = orc.Oracle(layers, Ws, bs, balance=balance, n_streams=2, loss=ps.LOSS_CE, lr=0.0)
    T = 2 * len(balance) + 2
    x1, tg1 = rand_stream(1, 2, 40, 8), targets_for(ps.LOSS_CE, 1, 2, 3, 8)
    o.step(np.repeat(x1, T, axis=0), np.repeat(tg1, T, axis=0))
    params = [t64(a).requires_grad_(True) for pair in zip(Ws, bs) for a in pair]
    L = torch_loss(ps.LOSS_CE, torch_forward(layers, params[0::2], params[1::2], t64(x1[0])), torch.tensor(tg1[0]))
    grads = torch.autograd.grad(L, params)
    for i in range(len(layers)):
        dW, db = o.get_grads(i)
        np.testing.assert_allclose(dW, grads[2 * i].numpy(), rtol=1e-6, atol=2e-9)
        np.testing.assert_allclose(db, grads[2 * i + 1].numpy(), rtol=1e-6, atol=2e-9)
