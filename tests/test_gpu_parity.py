"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars (stated by the build's goal): fp32 within 1e-5, bf16-stored weights and bf16 matrix-core operands within 2e-2,
applied element by element (relative to the largest element of the reference array) and in the 2-norm, to every
output row, loss, published activation / error buffer, Adam moment and to the UPDATE of every weight and bias
(W - W_before, not W).  Stored bf16 weights must also be bit-identical in all but 3 % of their elements and one bf16
step apart in the rest.  How ReLU units within rounding distance of z = 0 are treated is described in parity.py.
Every family and every full-size configuration has a negative control: a library that leaves the weights alone
(step size 0 on the GPU side only) must FAIL the same comparison.
"""
import numpy as np
import pytest
import torch

import oracle as orc
import partime_streams as ps
from paper_2210_09147_amd import Pipeline, binding as B
from parity import BF16_TOL, F32_TOL, Pair, compare, Report

pytestmark = pytest.mark.gpu

CONV_TOL = 1e-5   # fp32 matrix-core sums (up to 576 terms, fp32, another order than the oracle's fp64)


def rel(a, b):
    """The larger of the worst element error relative to the largest reference element and the 2-norm error."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(max(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30), np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)))


def movement(pair):
    """Per layer: largest change of a weight since the start, relative to the largest weight (oracle side)."""
    out = []
    for i in range(len(pair.layers)):
        W = pair.ref.get_weights(i)[0].astype(np.float64)
        out.append(float(np.abs(W - pair.Ws_stored[i]).max() / np.abs(pair.Ws_stored[i]).max()))
    return out


def run_pair(w, T, chunks=None, bf16=False, tol=None, k=None, exec_mode=B.PT_EXEC_AUTO, return_weights=False, adam=None,
             pipes=None, x=None, tg=None, min_move=None, expect_blind=False, negative=False):
    """T learning ticks on the oracle and on one or more library pipelines; every tick's output and loss, and the
    updates, moments and published buffers are compared (see parity.py).  min_move: every layer must have moved by at
    least this fraction of its largest weight, so that the update check cannot pass on weights that never change."""
    pipes = pipes or [{"exec_mode": exec_mode, "chunks": chunks}]
    if x is not None:
        assert len(x) == T + 1
    pair = Pair(w, bf16=bf16, k=k, adam=adam, tol=tol, pipes=pipes, T=T + 1, x=x, tg=tg)
    pair.Ws_stored = [pair.ref.get_weights(i)[0].astype(np.float64) for i in range(len(w.layers))]
    outs, losses = pair.run(0, T)
    fill = max(pair.D - 1, pair.k)
    for l in losses:
        assert np.all(l[:fill] == 0)
    if expect_blind:
        return pair
    # one more tick, taken from the oracle's state on both sides (weights, moments, buffers, target history, the delay
    # lines of skip connections, tick): everything at the full bar.
    # negative: under a step size that lifts every layer's update well above the storage rounding of its weights,
    # and first with a library that does not update at all, which must fail for every layer
    big = 0.1 if (bf16 or w.n_streams > 1) else 0.02
    pair.forced_tick(T, lr=pair.pick_lr(big) if negative else None, negative=negative)
    pair.assert_ok()
    if min_move is not None:
        mv = movement(pair)
        assert min(mv) >= min_move, f"weights barely move ({mv}): the update check would be blind"
    ws = [[p.weights(i) for i in range(len(w.layers))] for p in pair.pipes] if return_weights else None
    pair.close()
    # pipelines that differ only in execution mode or in how the ticks were split over calls must agree bit by bit
    for o, l in zip(outs[1:], losses[1:]):
        assert np.array_equal(outs[0], o) and np.array_equal(losses[0], l)
    if return_weights:
        for other in ws[1:]:
            for (W1, b1), (W2, b2) in zip(ws[0], other):
                assert np.array_equal(W1, W2) and np.array_equal(b1, b2)
        return outs[0], losses[0], ws[0]
    return outs[0], losses[0]


def assert_sees_updates(w, T, **kw):
    """Negative control for nets with skip connections (the others end run_pair with a forced tick that carries it): the
    same free run with a library that never updates (step size 0 on the GPU side only) must fail the update comparison
    for every layer."""
    pair = run_pair(w, T, pipes=[{"gpu_lr": 0.0}], expect_blind=True, **kw)
    for i in range(len(w.layers)):
        hits = [f for f in pair.rep.failures if f" update of W{i}" in f]
        assert hits, f"a library that never updates layer {i} passes: the comparison is blind there"
    pair.close()


@pytest.mark.parametrize("act", [ps.ACT_RELU, ps.ACT_GELU])
@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_small_ragged_mlp_fp32(act, loss):
    # sizes that are not multiples of the vector width, of a wave, or of the rows a wave takes at once
    w = ps.small_mlp([97, 131, 70, 257, 11], act, loss, lr=0.02, drift=0.05, seed=1)
    run_pair(w, 60, min_move=1e-3, negative=act == ps.ACT_RELU)


def test_single_stage_and_two_stage():
    run_pair(ps.small_mlp([33, 5], ps.ACT_ID, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=2), 30)
    run_pair(ps.small_mlp([64, 40, 3], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=2), 30)


def test_one_by_one_network():
    run_pair(ps.small_mlp([1, 1, 1], ps.ACT_ID, ps.LOSS_MSE, lr=0.125, drift=0.05, seed=4), 12)


def test_target_delay_zero_and_large():
    w = ps.small_mlp([48, 64, 64, 7], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=5)
    run_pair(w, 40, k=0)
    run_pair(w, 40, k=5)
    w2 = ps.small_mlp([48, 64, 64, 9], ps.ACT_RELU, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=5)
    run_pair(w2, 40, k=0)
    run_pair(w2, 40, k=5)


def test_chunked_calls_match_one_call_bitwise():
    # two pipelines against one oracle pass; run_pair asserts that they agree bit by bit
    w = ps.small_mlp([48, 64, 64, 7], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=6)
    run_pair(w, 40, pipes=[{}, {"chunks": [(0, 1), (1, 2), (2, 3), (3, 17), (17, 40)]}], return_weights=True)
    w2 = ps.small_mlp([48, 64, 64, 9], ps.ACT_RELU, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=6, target_delay=4)
    run_pair(w2, 40, pipes=[{}, {"chunks": [(0, 1), (1, 3), (3, 4), (4, 30), (30, 40)]}], return_weights=True)


def test_wide_rows_all_register_layouts_fp32():
    # in_dim 256..4096 exercises every rows-in-registers variant; out_dim leaves a ragged last tile
    for d in (256, 512, 1024, 2048, 4096):
        w = ps.small_mlp([d, 200, d, 37], ps.ACT_RELU, ps.LOSS_MSE, lr=0.02, drift=0.02, seed=d)
        run_pair(w, 12, min_move=1e-3)


def test_bf16_weights():
    w = ps.small_mlp([130, 257, 96, 12], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=7)
    run_pair(w, 50, bf16=True)
    for d in (512, 1024, 2048, 4096):
        w = ps.small_mlp([d, 150, d, 20], ps.ACT_RELU, ps.LOSS_MSE, lr=1e-2, drift=0.02, seed=d)
        run_pair(w, 8, bf16=True)


def test_inference_only_matches_and_keeps_weights():
    w = ps.small_mlp([97, 131, 70, 11], ps.ACT_GELU, ps.LOSS_MSE, lr=0.1, seed=8, drift=0.05)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 25)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr)
    ro = ref.infer(x)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(2, 25)) < F32_TOL
    for i in range(3):
        assert np.array_equal(p.weights(i)[0], Ws[i]) and np.array_equal(p.weights(i)[1], bs[i])
    p.close()


def test_single_tick_from_oracle_state():
    """The oracle's state mid-run handed to the library (weights, both halves of every buffer, target history, tick),
    then one tick on both: output, loss, updates and the published buffers element by element; the second tick
    uses a step size under which every layer's update is a few per cent of its weights, and a library that does
    not update must fail it."""
    w = ps.small_mlp([120, 200, 96, 140, 10], ps.ACT_RELU, ps.LOSS_MSE, lr=0.02, drift=0.05, seed=9)
    pair = Pair(w, T=34)
    pair.warm(0, 30)
    pair.forced_tick(30)
    pair.forced_tick(31, lr=pair.pick_lr(0.05), negative=True)
    pair.run(32, 34)                 # and on from there, freely
    pair.assert_ok()
    pair.close()


def test_zero_ticks_reset_and_errors():
    w = ps.small_mlp([16, 16, 4], ps.ACT_RELU, ps.LOSS_CE, lr=0.1, seed=1, drift=0.05)
    Ws, bs = ps.init_weights(w.layers, 1)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=1)
    lib = B.load()
    assert lib.partime_step(p.ctx, None, None, 0, None, None) == B.PT_OK
    assert lib.partime_step(p.ctx, None, None, 3, None, None) == B.PT_EINVAL
    assert lib.partime_step(p.ctx, None, None, -1, None, None) == B.PT_EINVAL
    x, tg = ps.make_inputs(w, 10)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    o1, l1 = p.step(xd, td)
    o1, l1 = o1.cpu().numpy(), l1.cpu().numpy()
    for i in range(2):
        p.set_weights(i, Ws[i], bs[i])
    B.partime_reset(p.ctx)
    assert p.tick == 0
    o2, l2 = p.step(xd, td)
    assert np.array_equal(o1, o2.cpu().numpy()) and np.array_equal(l1, l2.cpu().numpy())
    p.close()


def test_config0_full_trajectory():
    w = ps.workload(0)
    out, loss = run_pair(w, w.ticks, min_move=1e-3)
    assert np.isfinite(out).all()


def full_size_forced(w, warm_ticks, *, bf16=False, adam=None, tol=None, rel_step=0.02, synthetic=False, free=0,
                     err_scale=1e-3, n_forced=2):
    """A full-size workload in the launch configuration bench.py times: the oracle runs `warm_ticks` ticks (or starts
    from a synthetic full pipeline where a plain-loop warm-up would take minutes), then two consecutive ticks (both
    ping-pong halves, both row directions) are taken from the oracle's state on both sides under a step size that
    moves every layer by a few per cent, the first one with the negative control; `free` further ticks run freely."""
    pair = Pair(w, bf16=bf16, adam=adam, tol=tol, T=warm_ticks + n_forced + free)
    if synthetic and adam is not None:
        pair.synthetic_state(warm_ticks, seed=w.seed, err_scale=err_scale)     # (an Adam step needs no gradient to be sized)
    elif synthetic:
        pair.synthetic_state(warm_ticks - 1, seed=w.seed, err_scale=err_scale)
        pair.warm(warm_ticks - 1, warm_ticks)                                 # one tick for the gradients pick_lr looks at
    else:
        pair.warm(0, warm_ticks)
    lr = pair.pick_lr(rel_step)
    pair.forced_tick(warm_ticks, lr=lr, negative=True)
    if n_forced > 1:
        pair.forced_tick(warm_ticks + 1, lr=lr)
    if free:
        pair.run(warm_ticks + n_forced, warm_ticks + n_forced + free)
    pair.assert_ok()
    print(f"{w.name}: {len(pair.rep.rows)} arrays compared, worst {pair.rep.worst():.3f} x tol, "
          f"{pair.rep.events} undecided ReLU units in {pair.rep.event_ticks} ticks, largest |z - z_oracle| seen {pair.rep.z_err:.2e}")
    pair.close()


def test_config1_full_size():
    """The benchmark workload (8 x 4096 x 4096 fp32, ReLU, MSE) at full size: 2 D + 2 oracle ticks fill the pipeline
    and bring a real error signal to every stage, then two checked ticks and two free ones."""
    w = ps.workload(1)
    full_size_forced(w, 2 * w.depth + 2, free=2)


def test_config2_full_size_bf16():
    """16 x 2048 bf16 GELU, CE: a free run past the fill (no ReLU: the whole trajectory is unique), then two checked
    ticks whose step size lifts every layer's update above the bf16 spacing of its weights."""
    w = ps.workload(2)
    T0 = 2 * w.depth + 2
    pair = Pair(w, T=T0 + 2)
    pair.run(0, T0)
    lr = pair.pick_lr(0.1)
    pair.forced_tick(T0, lr=lr, negative=True)
    pair.forced_tick(T0 + 1, lr=lr)
    pair.assert_ok()
    pair.close()


# ----------------------------------------------------------------------------- persistent multi-tick kernel

PERSIST_CASES = [
    (lambda: ps.small_mlp([97, 131, 70, 257, 11], ps.ACT_GELU, ps.LOSS_CE, lr=0.02, drift=0.05, seed=1), 60, False),
    (lambda: ps.small_mlp([97, 131, 70, 257, 11], ps.ACT_RELU, ps.LOSS_MSE, lr=0.02, drift=0.05, seed=1, target_delay=0), 60, False),
    (lambda: ps.small_mlp([33, 5], ps.ACT_ID, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=2), 30, False),
    (lambda: ps.small_mlp([130, 257, 96, 12], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=7), 50, True),
    (lambda: ps.workload(0), 1000, False),
]
TWO_MODES = [{"exec_mode": B.PT_EXEC_LAUNCH_PER_TICK}, {"exec_mode": B.PT_EXEC_PERSISTENT}]


@pytest.mark.parametrize("case", range(len(PERSIST_CASES)))
def test_persistent_kernel_matches_oracle_and_launch_per_tick_bitwise(case):
    """One launch for a block of ticks with a grid barrier between ticks: same arithmetic in the same order as
    one launch per tick, so every output, loss and weight must be bit-identical (a stale read across the
    barrier would show here), and both must match the oracle (one oracle pass drives both pipelines)."""
    mk, T, bf16 = PERSIST_CASES[case]
    run_pair(mk(), T, bf16=bf16, pipes=TWO_MODES, return_weights=True)


@pytest.mark.parametrize("cfg,T,bf16", [(1, 24, False), (2, 36, True)])
def test_persistent_kernel_full_size_bitwise(cfg, T, bf16):
    """The two execution modes at full size (8 x 4096 fp32, 16 x 2048 bf16), bit by bit against each other over a run
    past the fill; the launch-per-tick mode is the one the full-size configuration tests compare with the oracle."""
    w = ps.workload(cfg)
    w.lr *= 100.0                    # every stage's weights change within the run
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, T)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    res = []
    for kw in TWO_MODES:
        p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_dtype=B.PT_BF16 if bf16 else B.PT_F32, **kw)
        o, l = p.step(xd, td)
        res.append((o.cpu().numpy(), l.cpu().numpy(), [p.weights(i) for i in range(len(w.layers))]))
        B.partime_sync(p.ctx)
        p.close()
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    for (W1, b1), (W2, b2) in zip(res[0][2], res[1][2]):
        assert np.array_equal(W1, W2) and np.array_equal(b1, b2)
    assert np.isfinite(res[0][0]).all()


def test_persistent_chunked_and_infer():
    w = ps.small_mlp([48, 64, 64, 7], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=6, target_delay=3)
    run_pair(w, 40, pipes=[{"exec_mode": B.PT_EXEC_PERSISTENT},
                           {"exec_mode": B.PT_EXEC_PERSISTENT, "chunks": [(0, 1), (1, 3), (3, 4), (4, 30), (30, 40)]}])
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 25)
    xd = torch.from_numpy(x).cuda()
    outs = []
    for mode in (B.PT_EXEC_LAUNCH_PER_TICK, B.PT_EXEC_PERSISTENT):
        p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, exec_mode=mode)
        outs.append(p.infer(xd).cpu().numpy())
        B.partime_sync(p.ctx)
        p.close()
    assert np.array_equal(outs[0], outs[1])


# ----------------------------------------------------------------------------- several streams (matrix cores)

def ms_workload(widths, act, loss, **kw):
    w = ps.small_mlp(widths, act, loss, **kw)
    w.n_streams = 32
    w.w_dtype = ps.W_BF16
    return w


@pytest.mark.parametrize("loss", [ps.LOSS_CE, ps.LOSS_MSE])
def test_multistream_small_ragged(loss):
    # 32 streams sharing bf16 weights; sizes that are not multiples of the 16/32/64/128 blockings
    w = ms_workload([100, 130, 200, 70, 12], ps.ACT_RELU, loss, lr=0.05, drift=0.05, seed=3)
    run_pair(w, 40, bf16=True, min_move=2e-2, negative=True)
    w = ms_workload([64, 1100, 40], ps.ACT_GELU, loss, lr=0.05, drift=0.05, seed=4)   # several forward tiles, one ragged
    run_pair(w, 20, bf16=True, min_move=2e-2)


def test_multistream_hidden_layer_wider_than_4096():
    """A hidden layer of 4200 units (padded to 4608): nine row tiles and nine column tiles, so every sum over partial planes
    runs past its first batch of requests and ends in a clamped, masked tail."""
    w = ms_workload([64, 4200, 40], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=41)
    run_pair(w, 8, bf16=True, negative=True)


def test_multistream_depth8_medium():
    w = ms_workload([512] * 8 + [100], ps.ACT_RELU, ps.LOSS_CE, lr=0.01, drift=0.02, seed=5)
    pair = Pair(w, T=28)
    pair.run(0, 24)                                  # 2 D + 8 ticks: a real error signal has reached the first stage
    lr = pair.pick_lr(0.1)
    pair.forced_tick(24, lr=lr, negative=True)
    pair.forced_tick(25, lr=lr)
    pair.run(26, 28)
    pair.assert_ok()
    pair.close()


def test_multistream_chunked_infer_and_state():
    w = ms_workload([96, 160, 80, 10], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=6, target_delay=2)
    run_pair(w, 30, bf16=True, pipes=[{}, {"chunks": [(0, 1), (1, 2), (2, 11), (11, 30)]}], return_weights=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 12)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_bf16=True, operands_bf16=True)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_dtype=B.PT_BF16)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(2, 12)) < BF16_TOL
    # inter-stage buffers come back in the caller's [S][size] layout
    act = B.partime_get_buffer(p.ctx, 0, 0, 1, 32 * 160).reshape(32, 160)
    assert rel(act, ref.get_buffer("act", 0, 1)) < BF16_TOL
    B.partime_set_buffer(p.ctx, 0, 0, 1, act)
    assert np.array_equal(B.partime_get_buffer(p.ctx, 0, 0, 1, 32 * 160).reshape(32, 160), act)
    p.close()


def test_multistream_inference_between_learning_calls():
    """A learning tick of the 32-stream path leaves the next tick's pre-activations behind; inference ticks take a kernel
    of their own and leave none.  Learning, inference and learning again, partly in one-tick calls, must follow the
    oracle through every switch."""
    w = ms_workload([96, 1100, 600, 10], ps.ACT_GELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=61)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 40)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_bf16=True, operands_bf16=True)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_dtype=B.PT_BF16)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    D = w.depth
    t = 0
    for kind, n in [("L", 9), ("I", 1), ("L", 1), ("L", 1), ("I", 6), ("I", 1), ("L", 7), ("I", 3), ("L", 11)]:
        if kind == "L":
            ro, rl = ref.step(x[t:t + n], tg[t:t + n])
            o, l = p.step(xd[t:t + n], td[t:t + n])
            for i in range(n):
                if t + i >= D - 1:
                    assert abs(float(l[i]) - rl[i]) <= 10 * BF16_TOL * max(abs(rl[i]), 1e-3), (t + i, float(l[i]), rl[i])
        else:
            ro = ref.infer(x[t:t + n])
            o = p.infer(xd[t:t + n])
        o = o.cpu().numpy()
        for i in range(n):
            if t + i >= D - 1:
                assert rel(o[i], ro[i]) < BF16_TOL, (kind, t + i, rel(o[i], ro[i]))
        t += n
    for i in range(len(w.layers)):
        W, b = p.weights(i)
        W0, b0 = ref.get_weights(i)
        assert rel(W, W0) < BF16_TOL and rel(b, b0) < BF16_TOL
        assert rel(W - Ws[i], W0 - Ws[i]) < 5 * BF16_TOL, (i, rel(W - Ws[i], W0 - Ws[i]))
    p.close()


@pytest.mark.parametrize("loss", [ps.LOSS_CE, ps.LOSS_MSE])
def test_multistream_adam(loss):
    # 32 streams with Adam: moments of the weights (updated in the backward launch) and of the biases (forward epilogue,
    # loss head) against the oracle's
    w = ms_workload([100, 130, 600, 70, 12], ps.ACT_GELU, loss, lr=2e-3, drift=0.05, seed=13, target_delay=2)
    run_pair(w, 24, bf16=True, adam=(0.9, 0.999, 1e-8), pipes=[{}, {"chunks": [(0, 3), (3, 4), (4, 24)]}], return_weights=True,
             min_move=2e-2, negative=True)


@pytest.mark.parametrize("balance", [[5], [2, 3], [3, 1, 1], [1, 2, 2]])
@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_multistream_several_layers_per_stage(balance, adam):
    """Exact back-propagation inside a stage (Eq. 3-5) on the 32-stream path: the fold across the tick boundary works
    for the first layer of a stage alone, the others take a forward-only matrix launch; one stage is plain SGD / Adam
    over 32 samples."""
    w = ms_workload([100, 260, 130, 600, 140, 10], ps.ACT_GELU, ps.LOSS_CE, lr=2e-3 if adam else 0.05, drift=0.05, seed=15,
                    balance=balance)
    run_pair(w, 14, bf16=True, adam=adam, negative=True)
    run_pair(w, 14, bf16=True, adam=adam, pipes=[{}, {"chunks": [(0, 1), (1, 6), (6, 14)]}], k=0, return_weights=True)


def test_multistream_several_layers_per_stage_relu_mse_infer():
    w = ms_workload([96, 160, 1100, 80, 12], ps.ACT_RELU, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=16, balance=[2, 2])
    run_pair(w, 12, bf16=True, negative=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 20)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_bf16=True, operands_bf16=True, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_dtype=B.PT_BF16, balance=w.balance)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    # learning, inference, learning again: the planes formed ahead of a tick are stale after the inference ticks
    t = 0
    for kind, n in [("L", 5), ("I", 3), ("L", 1), ("L", 4), ("I", 1), ("L", 6)]:
        if kind == "L":
            ro, _ = ref.step(x[t:t + n], tg[t:t + n])
            o, _ = p.step(xd[t:t + n], td[t:t + n])
        else:
            ro = ref.infer(x[t:t + n])
            o = p.infer(xd[t:t + n])
        o = o.cpu().numpy()
        for i in range(n):
            if t + i >= 1:
                assert rel(o[i], ro[i]) < BF16_TOL, (kind, t + i, rel(o[i], ro[i]))
        t += n
    for i in range(len(w.layers)):
        W, b = p.weights(i)
        W0, b0 = ref.get_weights(i)
        assert rel(W - Ws[i], W0 - Ws[i]) < 5 * BF16_TOL, (i, rel(W - Ws[i], W0 - Ws[i]))
    p.close()


@pytest.mark.parametrize("balance", [None, [6], [2, 2, 2], [1, 3, 2], [3, 1, 1, 1]])
@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_multistream_skip_connections(balance, adam):
    """Residual connections (Sec. V-C) on the 32-stream path: inside a stage, to the next stage and across several stages,
    with a layer that is both the target of one skip and the source of another."""
    w = ms_workload([97, 131, 131, 131, 131, 131, 11], ps.ACT_GELU, ps.LOSS_CE, lr=2e-3 if adam else 0.05, drift=0.05,
                    seed=17, balance=balance)
    for dst, src in {2: 0, 4: 1, 3: 2}.items():
        w.layers[dst].skip_from = src
    run_pair(w, 20, bf16=True, adam=adam, negative=True)
    run_pair(w, 20, bf16=True, adam=adam, pipes=[{}, {"chunks": [(0, 1), (1, 2), (2, 3), (3, 11), (11, 20)]}], k=0,
             return_weights=True)


def test_multistream_skip_connections_relu_mse_wide_and_infer():
    w = ms_workload([200, 600, 600, 600, 260, 260, 7], ps.ACT_RELU, ps.LOSS_MSE, lr=0.02, drift=0.05, seed=18, balance=[2, 2, 2])
    for dst, src in {2: 0, 4: 3}.items():
        w.layers[dst].skip_from = src
    run_pair(w, 16, bf16=True)
    assert_sees_updates(w, 16, bf16=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 8)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_bf16=True, operands_bf16=True, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_dtype=B.PT_BF16, balance=w.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(w.depth - 1, 8)) < BF16_TOL
    p.close()


def test_config4_full_size_multistream():
    """8 x 4096-wide bf16 layers (last 4096 -> 1000), 32 streams, at full size.  A tick of the plain-loop oracle is
    about 25 GFLOP here, so the pipeline is not filled tick by tick: it starts from a synthetic full state."""
    w = ps.workload(4)
    full_size_forced(w, w.depth + 1, bf16=True, synthetic=True, rel_step=0.1)


def test_full_width_multistream_two_layers_per_stage():
    """Layers of the benchmark's width as two stages of two layers (Eq. 3-5), 32 streams, from a synthetic full pipeline:
    forward-only matrix launches, kept pre-activations and in-stage deltas at 4096-wide layers; the checked tick is an
    odd one (rows walked bottom-up).  (Workload 21, all eight layers in four stages, is what bench.py times.)"""
    w = ps.workload(21)
    w.layers = ps.mlp([4096, 4096, 4096, 4096, 1000], ps.ACT_RELU)
    w.balance = [2, 2]
    full_size_forced(w, w.depth + 1, bf16=True, synthetic=True, rel_step=0.1, n_forced=1)


# ----------------------------------------------------------------------------- replay batch: 64 and more streams

def batched_workload(widths, act, loss, S, **kw):
    w = ps.small_mlp(widths, act, loss, **kw)
    w.n_streams = S
    w.w_dtype = ps.W_BF16
    return w


@pytest.fixture(params=["64", "128"])
def stream_tile(request, monkeypatch):
    """Small networks get 64-wide stream tiles by themselves; the variable forces either width where 128 divides S."""
    monkeypatch.setenv("PARTIME_RB_TN", request.param)
    return request.param


@pytest.mark.parametrize("S", [64, 128, 192])
@pytest.mark.parametrize("loss", [ps.LOSS_CE, ps.LOSS_MSE])
def test_batched_sgd(S, loss, stream_tile):
    # sizes that are not multiples of the 128-wide tiles; 64 and 192 streams always take the 64-wide stream tiles
    w = batched_workload([100, 300, 130, 12], ps.ACT_RELU, loss, S, lr=0.05, drift=0.05, seed=3)
    run_pair(w, 16, bf16=True, min_move=1e-2, negative=S == 128)


@pytest.mark.parametrize("S", [64, 256])
def test_batched_adam_gelu(S, stream_tile):
    w = batched_workload([96, 260, 140, 10], ps.ACT_GELU, ps.LOSS_CE, S, lr=2e-3, drift=0.05, seed=4, target_delay=2)
    run_pair(w, 14, bf16=True, adam=(0.9, 0.999, 1e-8), min_move=2e-2, negative=S == 64)


def test_batched_chunked_and_infer():
    w = batched_workload([96, 160, 80, 10], ps.ACT_RELU, ps.LOSS_CE, 64, lr=0.05, drift=0.05, seed=6, target_delay=2)
    run_pair(w, 14, bf16=True, pipes=[{}, {"chunks": [(0, 1), (1, 2), (2, 9), (9, 14)]}], return_weights=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 8)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=64, w_bf16=True, operands_bf16=True)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=64, w_dtype=B.PT_BF16)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(2, 8)) < BF16_TOL
    p.close()


@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_batched_unpadded_sizes(adam):
    # every padded size is a multiple of 256 and nothing is padded except the first input
    w = batched_workload([500, 512, 250, 256], ps.ACT_GELU, ps.LOSS_MSE, 128, lr=2e-3 if adam else 0.05, drift=0.05, seed=9)
    run_pair(w, 12, bf16=True, adam=adam)


def test_batched_full_width_short_run(monkeypatch):
    """Layers of the benchmark's width (4096, last one 4096 -> 1000) under a replay batch of 256 with Adam: two
    stages, one tick past the fill (the oracle needs about 15 GFLOP in plain loops per tick)."""
    monkeypatch.setenv("PARTIME_RB_TN", "128")   # the tile width of the 8-stage benchmark configuration
    w = ps.workload(12)
    w.layers = ps.mlp([4096, 4096, 1000], ps.ACT_RELU)
    full_size_forced(w, w.depth + 1, bf16=True, adam=w.adam, synthetic=True, rel_step=0.1, n_forced=1)


@pytest.mark.parametrize("balance", [[5], [2, 3], [3, 1, 1], [1, 2, 2]])
@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_batched_several_layers_per_stage(balance, adam):
    """Exact back-propagation inside a stage (Eq. 3-5) under a replay batch: one stage is plain batched SGD / Adam,
    two stages of several layers is the pipeline of the paper's Sec. V-D."""
    w = batched_workload([100, 260, 130, 200, 140, 10], ps.ACT_GELU, ps.LOSS_CE, 64, lr=2e-3 if adam else 0.05, drift=0.05,
                         seed=15, balance=balance)
    run_pair(w, 14, bf16=True, adam=adam)
    run_pair(w, 14, bf16=True, adam=adam, chunks=[(0, 1), (1, 6), (6, 14)], k=0)


def test_batched_several_layers_per_stage_relu_mse_infer_128(stream_tile):
    w = batched_workload([96, 160, 160, 80, 12], ps.ACT_RELU, ps.LOSS_MSE, 128, lr=0.05, drift=0.05, seed=16, balance=[2, 2])
    run_pair(w, 12, bf16=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 8)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=128, w_bf16=True, operands_bf16=True, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=128, w_dtype=B.PT_BF16, balance=w.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(1, 8)) < BF16_TOL
    p.close()


@pytest.mark.parametrize("balance", [None, [6], [2, 2, 2], [1, 3, 2], [3, 1, 1, 1]])
@pytest.mark.parametrize("adam", [None, (0.9, 0.999, 1e-8)])
def test_batched_skip_connections(balance, adam):
    """Residual connections under a replay batch: inside a stage, to the next stage and across several stages, with a
    layer that is both the target of one skip and the source of another."""
    w = batched_workload([97, 131, 131, 131, 131, 131, 11], ps.ACT_GELU, ps.LOSS_CE, 64, lr=2e-3 if adam else 0.05, drift=0.05,
                         seed=17, balance=balance)
    for dst, src in {2: 0, 4: 1, 3: 2}.items():
        w.layers[dst].skip_from = src
    run_pair(w, 20, bf16=True, adam=adam, negative=True)
    run_pair(w, 20, bf16=True, adam=adam, chunks=[(0, 1), (1, 2), (2, 3), (3, 11), (11, 20)], k=0)


def test_batched_skip_connections_relu_mse_128_and_infer(stream_tile):
    w = batched_workload([200, 300, 300, 300, 260, 260, 7], ps.ACT_RELU, ps.LOSS_MSE, 128, lr=0.02, drift=0.05, seed=18,
                         balance=[2, 2, 2])
    for dst, src in {2: 0, 4: 3}.items():
        w.layers[dst].skip_from = src
    run_pair(w, 16, bf16=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 8)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=128, w_bf16=True, operands_bf16=True, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=128, w_dtype=B.PT_BF16, balance=w.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(w.depth - 1, 8)) < BF16_TOL
    p.close()


def test_batched_single_stage_and_state_round_trip():
    # one stage only: no backward product, the loss head feeds the update directly (plain batched SGD / Adam)
    w = batched_workload([70, 9], ps.ACT_ID, ps.LOSS_CE, 64, lr=0.05, drift=0.05, seed=11)
    run_pair(w, 8, bf16=True)
    run_pair(w, 8, bf16=True, adam=(0.9, 0.999, 1e-8))
    # weights and moments written through the ABI are what the next ticks use (both weight orientations are refreshed)
    w = batched_workload([96, 160, 10], ps.ACT_RELU, ps.LOSS_CE, 64, lr=2e-3, drift=0.05, seed=12)
    adam = (0.9, 0.999, 1e-8)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 16)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_bf16=True, n_streams=64,
                     operands_bf16=True, adam=adam)
    ref.step(x[:8], tg[:8])
    # a fresh pipeline takes over the oracle's weights and moments after 8 ticks; activations and errors in flight are
    # zero on its side, so compare against an oracle that is reset the same way
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, n_streams=64, w_dtype=B.PT_BF16, adam=adam)
    ref2 = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_bf16=True, n_streams=64,
                      operands_bf16=True, adam=adam)
    for i in range(len(w.layers)):
        W, b = ref.get_weights(i)
        mom = ref.get_moments(i)
        B.partime_set_state(p.ctx, i, W, b)
        B.partime_set_opt_state(p.ctx, i, *mom)
        ref2.set_weights(i, W, b)
        ref2.set_moments(i, *mom)
    ro, rl = ref2.step(x[8:], tg[8:])
    o, l = p.step(torch.from_numpy(x[8:]).cuda(), torch.from_numpy(tg[8:]).cuda())
    o, l = o.cpu().numpy(), l.cpu().numpy()
    assert max(rel(o[t], ro[t]) for t in range(w.depth - 1, 8)) < BF16_TOL
    for i in range(len(w.layers)):
        W, b = p.weights(i)
        W0, b0 = ref2.get_weights(i)
        assert rel(W, W0) < BF16_TOL and rel(b, b0) < BF16_TOL
        for got, want in zip(p.moments(i), ref2.get_moments(i)):
            assert rel(got, want) < BF16_TOL
    p.close()


def test_batched_single_tick_from_oracle_state(stream_tile):
    """The oracle's state after 11 ticks (weights, moments, both halves of every inter-stage buffer, tick) handed to a
    pipeline of 128 streams: the next ticks must agree on output, loss, updates, moments and the buffers they write."""
    adam = (0.9, 0.999, 1e-8)
    w = batched_workload([100, 200, 130, 10], ps.ACT_GELU, ps.LOSS_CE, 128, lr=2e-3, drift=0.05, seed=14, target_delay=0)
    pair = Pair(w, adam=adam, T=14)
    pair.warm(0, 11)
    pair.forced_tick(11)
    pair.forced_tick(12, lr=pair.pick_lr(0.1), negative=True)
    pair.run(13, 14)
    pair.assert_ok()
    pair.close()


def test_batched_benchmark_configuration_short_run():
    """Workload 14 as bench.py runs it: all 8 stages at full width, replay batch of 64, Adam; a few ticks past the fill."""
    w = ps.workload(14)
    full_size_forced(w, w.depth + 1, bf16=True, adam=w.adam, synthetic=True, rel_step=0.1, n_forced=1)


def test_batched_wide_layers(monkeypatch):
    """Two 1024-wide layers under 1024 streams (the largest batch): several tiles along every axis."""
    monkeypatch.setenv("PARTIME_RB_TN", "128")
    w = batched_workload([1024, 1024, 100], ps.ACT_RELU, ps.LOSS_CE, 1024, lr=0.02, drift=0.05, seed=8)
    run_pair(w, 5, bf16=True)


# ----------------------------------------------------------------------------- conv stages (matrix cores, fp32)

def conv_workload(c_in, h, w, n_conv, n_classes, loss=ps.LOSS_CE, **kw):
    return ps.Workload(f"cnn{n_conv}_{h}x{w}", ps.conv_net(c_in, h, w, n_conv, n_classes), loss=loss,
                       n_classes=n_classes if loss == ps.LOSS_CE else 0, **kw)


@pytest.mark.parametrize("shape", [(3, 32, 32, 2), (3, 8, 64, 3), (5, 16, 128, 2)])
@pytest.mark.parametrize("loss", [ps.LOSS_CE, ps.LOSS_MSE])
def test_conv_pipeline_small(shape, loss):
    c_in, h, w, n_conv = shape
    wl = conv_workload(c_in, h, w, n_conv, 6, loss=loss, lr=0.05, seed=3)
    if c_in != 3:
        wl.layers[0].c_in = c_in
    if c_in == 3:
        run_pair(wl, 16, tol=CONV_TOL, min_move=1e-4, negative=shape[1] == 32)
    else:   # a generic smooth stream for the odd channel count
        x = ps.smooth_stream(15, c_in * h * w, 0.05, 1)
        tg = ps.teacher_classes(x[:, :, :64], 6, 1) if loss == ps.LOSS_CE else ps.teacher_regression(x[:, :, :64], 6, 1)
        run_pair(wl, 14, tol=CONV_TOL, x=x, tg=tg, min_move=2e-4)


@pytest.mark.parametrize("balance", [None, [2, 1, 1]])
@pytest.mark.parametrize("loss", [ps.LOSS_CE, ps.LOSS_MSE])
def test_conv_pipeline_adam(balance, loss):
    """Adam on conv kernels, biases and the pooled head (Sec. V-D trains a conv net with it); moments compared too."""
    wl = conv_workload(3, 32, 32, 3, 6, loss=loss, lr=1e-3, seed=5)
    wl.balance = balance
    run_pair(wl, 14, tol=CONV_TOL, adam=ADAM, min_move=2e-4, negative=balance is None)


def test_conv_infer_chunks_and_state():
    wl = conv_workload(3, 32, 32, 2, 5, lr=0.05, seed=4, target_delay=1)
    run_pair(wl, 12, tol=CONV_TOL, pipes=[{}, {"chunks": [(0, 1), (1, 5), (5, 12)]}], return_weights=True)
    Ws, bs = ps.init_weights(wl.layers, wl.seed)
    x, _ = ps.make_inputs(wl, 8)
    ref = orc.Oracle(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr)
    p = Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(2, 8)) < CONV_TOL
    for i in range(3):
        assert np.array_equal(p.weights(i)[0], Ws[i])
    act = B.partime_get_buffer(p.ctx, 0, 1, 1, 64 * 32 * 32)
    assert rel(act, ref.get_buffer("act", 1, 1)[0]) < CONV_TOL
    p.close()


def test_config3_full_size_conv():
    """8 conv3x3(64) stages at 128 x 128 + pooled head, depth 9, at full size, from a synthetic full pipeline (a tick of
    the plain-loop oracle is 25 GFLOP): forward, backward-data, weight gradient and update of every stage."""
    wl = ps.workload(3)
    full_size_forced(wl, wl.depth + 1, tol=CONV_TOL, synthetic=True, rel_step=0.05)


# ----------------------------------------------------------------------------- several layers per stage (Eq. 3-5)

@pytest.mark.parametrize("balance", [[3], [2, 1], [1, 3, 2], [2, 2, 2, 1]])
@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_several_layers_per_stage_fp32(balance, loss):
    """Exact back-propagation inside a stage, delayed errors between stages; balance [n] is plain online SGD."""
    n = sum(balance)
    widths = [97, 131, 70, 257, 64, 33, 150, 11][:n] + [13]
    w = ps.small_mlp(widths, ps.ACT_GELU, loss, lr=0.02, drift=0.05, seed=11, balance=balance)
    assert w.depth == len(balance)
    run_pair(w, 40, min_move=5e-4, negative=balance == [1, 3, 2])
    run_pair(w, 40, chunks=[(0, 1), (1, 2), (2, 17), (17, 40)], k=0)


def test_several_layers_per_stage_relu_bf16_and_infer():
    w = ps.small_mlp([200, 300, 100, 260, 50, 7], ps.ACT_RELU, ps.LOSS_CE, lr=0.02, drift=0.05, seed=12, balance=[2, 3])
    run_pair(w, 30)
    run_pair(w, 30, bf16=True)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 10)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(w.depth - 1, 10)) < F32_TOL
    assert B.partime_last_launch_count(p.ctx) == 10 * 3          # cmax = 3 forward launches per inference tick
    # what the first stage published is its second layer's output
    assert rel(B.partime_get_buffer(p.ctx, 0, 0, 1, w.layers[1].out_dim), ref.get_buffer("act", 0, 1)[0]) < F32_TOL
    p.close()


def test_several_layers_per_stage_stage_buffers_and_launch_count():
    w = ps.small_mlp([64, 96, 80, 48, 5], ps.ACT_GELU, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=13, balance=[2, 2])
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 9)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, balance=w.balance)
    ref.step(x, tg)
    p.step(torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda())
    assert B.partime_last_launch_count(p.ctx) == 9 * 3 + 1       # 2 cmax - 1 launches per tick + the loss sum
    half = 8 & 1                                                  # the half written at the last tick
    assert rel(B.partime_get_buffer(p.ctx, 0, 0, half, w.layers[1].out_dim), ref.get_buffer("act", 0, half)[0]) < F32_TOL
    assert rel(B.partime_get_buffer(p.ctx, 1, 1, half, w.layers[2].in_dim), ref.get_buffer("err", 1, half)[0]) < 10 * F32_TOL
    for i in range(4):
        assert rel(p.weights(i)[0], ref.get_weights(i)[0]) < F32_TOL
    with pytest.raises(B.PartimeError):
        Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance, exec_mode=B.PT_EXEC_PERSISTENT)
    p.close()


def test_two_layers_per_stage_full_size():
    """The 8 x 4096 fp32 network in 4 stages of two layers: full-size shapes in the launch configuration of the bench."""
    w = ps.workload(5)
    full_size_forced(w, 2 * w.depth + 2)


def test_persistent_barrier_timeout_is_reported_not_hung(monkeypatch):
    """A grid barrier whose bounded wait runs out (forced from the host with a spin limit of zero) makes every
    work-group leave the kernel; the failure is reported by partime_sync and the context can still be destroyed."""
    w = ps.small_mlp([300, 500, 400, 300, 20], ps.ACT_RELU, ps.LOSS_MSE, lr=0.01, drift=0.05, seed=5)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 64)
    monkeypatch.setenv("PARTIME_SPIN_LIMIT", "0")
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, exec_mode=B.PT_EXEC_PERSISTENT)
    monkeypatch.delenv("PARTIME_SPIN_LIMIT")
    p.step(torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda())
    with pytest.raises(B.PartimeError) as e:
        B.partime_sync(p.ctx)
    assert e.value.code == B.PT_EHIP
    p.close()
    # a fresh context with the default limit works
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, exec_mode=B.PT_EXEC_PERSISTENT)
    p.step(torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda())
    B.partime_sync(p.ctx)
    p.close()


# ----------------------------------------------------------------------------- Adam (Sec. V-D)

ADAM = (0.9, 0.999, 1e-8)


@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
@pytest.mark.parametrize("balance", [None, [2, 2]])
def test_adam_small_ragged_fp32(loss, balance):
    # GELU keeps the comparison free of kink decisions
    w = ps.small_mlp([97, 131, 70, 257, 11], ps.ACT_GELU, loss, lr=1e-3, drift=0.05, seed=21, balance=balance)
    run_pair(w, 40, adam=ADAM, pipes=[{}, {"chunks": [(0, 3), (3, 4), (4, 40)]}], return_weights=True, min_move=1e-3,
             negative=balance is None)


def test_adam_wide_rows_bf16_and_single_tick():
    for d in (1000, 2048, 4096):
        w = ps.small_mlp([d, 150, d, 20], ps.ACT_GELU, ps.LOSS_MSE, lr=1e-3, drift=0.02, seed=d)
        run_pair(w, 12, adam=ADAM)
    w = ps.small_mlp([300, 500, 260, 9], ps.ACT_RELU, ps.LOSS_CE, lr=1e-3, drift=0.05, seed=22)
    run_pair(w, 30, adam=ADAM, bf16=True)
    # ticks from the oracle's state (weights, moments, buffers, target history after 20 ticks)
    pair = Pair(w, adam=ADAM, T=23)
    pair.warm(0, 20)
    pair.forced_tick(20)
    pair.forced_tick(21, lr=pair.pick_lr(0.05), negative=True)
    pair.run(22, 23)
    pair.assert_ok()
    pair.close()
    Ws, bs = ps.init_weights(w.layers, w.seed)
    with pytest.raises(B.PartimeError):
        Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, adam=ADAM, exec_mode=B.PT_EXEC_PERSISTENT)


def test_adam_full_size():
    """The 8 x 4096 fp32 network under Adam: full-size shapes in the launch configuration of the bench."""
    w = ps.workload(6)
    full_size_forced(w, 2 * w.depth + 2, adam=w.adam)


# ----------------------------------------------------------------------------- several conv layers per stage

@pytest.mark.parametrize("balance", [[2, 2, 1], [4, 1], [1, 3, 1], [3, 2, 1]])
@pytest.mark.parametrize("act", [ps.ACT_RELU, ps.ACT_GELU])
def test_conv_several_layers_per_stage(balance, act):
    n_conv = sum(balance) - 1
    wl = conv_workload(3, 32, 32, n_conv, 6, lr=0.05, seed=6)
    for l in wl.layers[:-1]:
        l.act = act
    wl.balance = balance
    assert wl.depth == len(balance)
    run_pair(wl, 14, tol=CONV_TOL, min_move=2e-4)
    if balance == [2, 2, 1]:
        run_pair(wl, 12, tol=CONV_TOL, chunks=[(0, 1), (1, 5), (5, 12)], k=0, negative=True)
        # forward-only ticks on the same pipeline shape
        Ws, bs = ps.init_weights(wl.layers, wl.seed)
        x, _ = ps.make_inputs(wl, 8)
        ref = orc.Oracle(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=balance)
        p = Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=balance)
        ro = ref.infer(x)
        out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
        assert max(rel(out[t], ro[t]) for t in range(wl.depth - 1, 8)) < CONV_TOL
        assert B.partime_last_launch_count(p.ctx) == 8 * 3      # two forward launches + the head per tick
        assert rel(B.partime_get_buffer(p.ctx, 0, 0, 1, 64 * 32 * 32), ref.get_buffer("act", 0, 1)[0]) < CONV_TOL
        p.close()


def test_conv_deep_stages_medium():
    """Twelve conv layers at 32 x 64 in three stages of four, plus the head: long in-stage chains."""
    wl = conv_workload(3, 32, 64, 12, 10, lr=0.01, seed=8)
    wl.balance = [4, 4, 4, 1]
    run_pair(wl, 9, tol=CONV_TOL)


@pytest.mark.parametrize("feat", [1, 10, 37, 100, 130])
def test_conv_other_feature_map_counts(feat):
    """Conv stages with other feature-map counts than 64 (the paper's F = 1, 10, 100): blocks of 64 channels,
    padded inside the library."""
    ls = ps.conv_net(3, 32, 32, 3, 5, act=ps.ACT_GELU, feat=feat)
    wl = ps.Workload(f"cnn_f{feat}", ls, loss=ps.LOSS_CE, n_classes=5, lr=0.05, seed=9, balance=[2, 1, 1])
    run_pair(wl, 12, tol=CONV_TOL)
    Ws, bs = ps.init_weights(wl.layers, wl.seed)
    p = Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance)
    for i in range(len(ls)):                       # weights come back in the caller's shapes, unpadded
        W, b = p.weights(i)
        assert W.shape == Ws[i].shape and np.array_equal(W, Ws[i]) and np.array_equal(b, bs[i])
    p.close()


@pytest.mark.parametrize("feat,h,act,adam", [(64, 8, ps.ACT_RELU, None), (64, 4, ps.ACT_GELU, (0.9, 0.999, 1e-8)), (1, 16, ps.ACT_GELU, None),
                                             (10, 8, ps.ACT_RELU, (0.9, 0.999, 1e-8)), (100, 4, ps.ACT_GELU, None)])
def test_conv_frames_256_wide(feat, h, act, adam):
    """The kernel instantiation the 150-layer stack of Sec. V-A runs on (256-wide frames: one row of 256 pixels per tile,
    the 64-column weight-gradient variant), with the feature-map counts of Table 1 and three layers per stage: a free run
    past the fill, a forced tick with the negative control, and forward-only ticks."""
    ls = ps.conv_net(3, h, 256, 6, 5, act=act, feat=feat)
    wl = ps.Workload(f"cnn6_f{feat}_{h}x256", ls, loss=ps.LOSS_CE, n_classes=5, lr=1e-3 if adam else 0.05, seed=21, balance=[3, 3, 1])
    run_pair(wl, 2 * wl.depth + 3, tol=CONV_TOL, adam=adam, negative=True)
    Ws, bs = ps.init_weights(wl.layers, wl.seed)
    x, _ = ps.make_inputs(wl, 6)
    ref = orc.Oracle(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance)
    p = Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(wl.depth - 1, 6)) < CONV_TOL
    assert rel(B.partime_get_buffer(p.ctx, 0, 1, 1, feat * h * 256), ref.get_buffer("act", 1, 1)[0]) < CONV_TOL
    p.close()


def test_bandwidth_probe_returns_a_plausible_rate():
    for mode in (0, 1, 2):
        g = B.partime_bandwidth_probe(512 << 20, mode, 5)   # twice the memory-side cache: the rate is HBM's
        assert 2000.0 < g < 8000.0, (mode, g)               # GB/s: under the published peak, not a stall
    with pytest.raises(B.PartimeError):
        B.partime_bandwidth_probe(1024, 0, 5)          # below the minimum size


# ----------------------------------------------------------------------------- skip connections (Sec. V-C)

def skip_workload(widths, skips, act, loss, **kw):
    w = ps.small_mlp(widths, act, loss, **kw)
    for dst, src in skips.items():
        w.layers[dst].skip_from = src
    return w


@pytest.mark.parametrize("balance", [None, [6], [2, 2, 2], [1, 3, 2], [3, 1, 1, 1]])
@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_skip_connections_fp32(balance, loss):
    """Residual connections inside a stage, to the next stage and across several stages; the skipped tensor and its
    gradient wait in delay lines as long as the stages they cross."""
    w = skip_workload([97, 131, 131, 131, 131, 131, 11], {2: 0, 4: 1, 3: 2}, ps.ACT_GELU, loss, lr=0.02, drift=0.05,
                      seed=41, balance=balance)
    run_pair(w, 40, min_move=1e-3, negative=True)
    run_pair(w, 40, chunks=[(0, 1), (1, 2), (2, 3), (3, 21), (21, 40)], k=0)
    if balance == [1, 3, 2] and loss == ps.LOSS_MSE:
        assert_sees_updates(w, 16)


def test_skip_connections_relu_bf16_adam_and_infer():
    w = skip_workload([200, 300, 300, 300, 260, 260, 7], {2: 0, 4: 3}, ps.ACT_RELU, ps.LOSS_CE, lr=0.02, drift=0.05,
                      seed=42, balance=[2, 2, 2])
    run_pair(w, 30, bf16=True)
    # at the fp32 bar the trajectory has to be unique: an undecided ReLU unit inside a stage changes the gradient that the
    # target of a skip sends back through its delay line, which cannot be handed over through the C ABI
    for l in w.layers[:-1]:
        l.act = ps.ACT_GELU
    run_pair(w, 30)
    w.lr = 1e-3
    run_pair(w, 30, adam=ADAM)
    for l in w.layers[:-1]:
        l.act = ps.ACT_RELU
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, _ = ps.make_inputs(w, 10)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(w.depth - 1, 10)) < F32_TOL
    with pytest.raises(B.PartimeError):
        Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, balance=w.balance, exec_mode=B.PT_EXEC_PERSISTENT)
    p.close()


def test_inference_bf16_between_learning_calls():
    """bf16 pipelines run inference on a tile list of their own (half-size tiles); learning before and after it must not
    notice, and the softmax head stage (split over two tiles here) must come out the same."""
    w = ps.small_mlp([300, 2048, 700, 2048, 100], ps.ACT_GELU, ps.LOSS_CE, lr=0.02, drift=0.05, seed=44)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 30)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_bf16=True)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_dtype=B.PT_BF16)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    D = w.depth
    ro, _ = ref.step(x[:12], tg[:12])
    o, _ = p.step(xd[:12], td[:12])
    assert max(rel(o[t].cpu().numpy(), ro[t]) for t in range(D - 1, 12)) < BF16_TOL
    ri = ref.infer(x[12:22])
    oi = p.infer(xd[12:22]).cpu().numpy()
    assert max(rel(oi[t], ri[t]) for t in range(10)) < BF16_TOL
    ro, rl = ref.step(x[22:30], tg[22:30])
    o, l = p.step(xd[22:30], td[22:30])
    assert max(rel(o[t].cpu().numpy(), ro[t]) for t in range(8)) < BF16_TOL
    assert max(abs(float(l[t]) - rl[t]) / max(abs(rl[t]), 1e-3) for t in range(8)) < 10 * BF16_TOL
    for i in range(len(w.layers)):
        W, b = p.weights(i)
        W0, b0 = ref.get_weights(i)
        assert rel(W, W0) < BF16_TOL and rel(b, b0) < BF16_TOL
    p.close()


def test_calls_of_zero_ticks_change_nothing():
    """Empty input: a learning or inference call of zero ticks is accepted and leaves every kernel family's pipeline where
    it was; the run around it is bit for bit the uninterrupted one."""
    cases = [
        (ps.small_mlp([40, 48, 32, 6], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=51), {}),
        (ms_workload([40, 48, 32, 6], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=52), dict(n_streams=32, w_dtype=B.PT_BF16)),
        (batched_workload([40, 48, 32, 6], ps.ACT_RELU, ps.LOSS_CE, 64, lr=0.05, drift=0.05, seed=53), dict(n_streams=64, w_dtype=B.PT_BF16)),
        (conv_workload(3, 32, 32, 2, 5, lr=0.05, seed=54), {}),
    ]
    for w, kw in cases:
        Ws, bs = ps.init_weights(w.layers, w.seed)
        x, tg = ps.make_inputs(w, 10)
        xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
        outs = []
        for split in (False, True):
            p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, **kw)
            if split:
                o1, l1 = p.step(xd[:4], td[:4])
                o0, l0 = p.step(xd[4:4], td[4:4])
                assert o0.shape[0] == 0 and l0.shape[0] == 0 and p.infer(xd[:0]).shape[0] == 0
                o2, l2 = p.step(xd[4:], td[4:])
                o, l = torch.cat([o1, o2]), torch.cat([l1, l2])
            else:
                o, l = p.step(xd, td)
            outs.append((o.cpu().numpy(), l.cpu().numpy(), [p.weights(i)[0] for i in range(len(w.layers))]))
            B.partime_sync(p.ctx)
            p.close()
        assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), w.name
        for W0, W1 in zip(outs[0][2], outs[1][2]):
            assert np.array_equal(W0, W1), w.name


def test_skip_delay_lines_through_get_and_set_buffer():
    """The delay lines of a skip that crosses stage boundaries are part of what a pipeline carries from tick to tick:
    read by age, written back, refused for layers without a skip and for ages that are not in flight."""
    w = ps.small_mlp([40, 48, 48, 48, 48, 6], ps.ACT_GELU, ps.LOSS_MSE, lr=0.05, drift=0.05, seed=33)
    w.layers[3].skip_from = 0                                  # three boundaries
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 12)
    ref = orc.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k)
    ref.step(x[:9], tg[:9])
    p.step(torch.from_numpy(x[:9]).cuda(), torch.from_numpy(tg[:9]).cuda())
    for age in range(3):
        for which in (3, 4):
            want = ref.get_lane(which - 3, 3, age)
            got = B.partime_get_buffer(p.ctx, which, 3, age, want.size)
            assert rel(got, want) < 1e-4, (which, age, rel(got, want))
            B.partime_set_buffer(p.ctx, which, 3, age, want)
            assert np.array_equal(B.partime_get_buffer(p.ctx, which, 3, age, want.size), want.ravel())
    for layer, age in ((2, 0), (3, 3), (3, -1)):
        with pytest.raises(B.PartimeError) as e:
            B.partime_get_buffer(p.ctx, 3, layer, age, 48)
        assert e.value.code == B.PT_EINVAL
    p.close()


def test_skip_connections_wide_full_rows():
    w = skip_workload([4096, 4096, 4096, 4096, 64], {2: 0}, ps.ACT_GELU, ps.LOSS_MSE, lr=0.02, drift=0.01, seed=43)
    run_pair(w, 12, min_move=1e-3)


# ----------------------------------------------------------------------------- residual connections between conv layers (Sec. V-C)

def conv_skip_workload(h, w, n_conv, feat, skips, act=ps.ACT_GELU, loss=ps.LOSS_CE, n_classes=6, **kw):
    layers = ps.conv_net(3, h, w, n_conv, n_classes, act=act, feat=feat)
    for dst, src in skips.items():
        layers[dst].skip_from = src
    return ps.Workload(f"cnn{n_conv}_{h}x{w}_skip", layers, loss=loss, n_classes=n_classes if loss == ps.LOSS_CE else 0, **kw)


@pytest.mark.parametrize("balance", [None, [6, 1], [2, 2, 2, 1], [1, 3, 2, 1], [3, 1, 1, 1, 1]])
@pytest.mark.parametrize("loss", [ps.LOSS_MSE, ps.LOSS_CE])
def test_conv_skip_connections(balance, loss):
    """Residual connections between feature maps: inside a stage, to the next stage and across several stages (a
    two-conv block that crosses a stage boundary among them); layer 2 is target of one skip and source of another.
    The skipped map and its gradient wait in rings of frames as long as the stages they cross.  37 channels: the last
    channel block is ragged."""
    wl = conv_skip_workload(16, 32, 6, 37, {2: 0, 4: 1, 3: 2}, loss=loss, lr=0.05, seed=71, balance=balance)
    run_pair(wl, 24, tol=CONV_TOL, min_move=1e-4, negative=True)
    if loss == ps.LOSS_CE:
        run_pair(wl, 24, tol=CONV_TOL, chunks=[(0, 1), (1, 2), (2, 3), (3, 13), (13, 24)], k=0)
    if balance == [1, 3, 2, 1] and loss == ps.LOSS_MSE:
        assert_sees_updates(wl, 20, tol=CONV_TOL)


@pytest.mark.parametrize("feat,h,w", [(64, 8, 64), (130, 2, 128), (64, 2, 256)])
def test_conv_skip_connections_full_blocks_adam_and_infer(feat, h, w):
    """Whole blocks of 64 channels (and three of them), the wider frame kernels, Adam, and inference with ReLU."""
    wl = conv_skip_workload(h, w, 4, feat, {2: 0, 3: 1}, loss=ps.LOSS_CE, lr=1e-3, seed=72, balance=[1, 2, 1, 1])
    run_pair(wl, 16, tol=CONV_TOL, adam=ADAM, min_move=2e-4)
    for l in wl.layers[:-1]:
        l.act = ps.ACT_RELU
    Ws, bs = ps.init_weights(wl.layers, wl.seed)
    x, _ = ps.make_inputs(wl, 8)
    ref = orc.Oracle(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance)
    p = Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance)
    ro = ref.infer(x)
    out = p.infer(torch.from_numpy(x).cuda()).cpu().numpy()
    assert max(rel(out[t], ro[t]) for t in range(wl.depth - 1, 8)) < CONV_TOL
    # without the residual adds the output is another one: the comparison above sees them
    plain = [ps.LayerSpec(l.kind, l.act, l.in_dim, l.out_dim, l.c_in, l.c_out, l.h, l.w) for l in wl.layers]
    r0 = orc.Oracle(plain, Ws, bs, loss=wl.loss, lr=wl.lr, balance=wl.balance).infer(x)
    assert rel(r0[7], ro[7]) > 100 * CONV_TOL
    p.close()


def test_conv_skip_refusals():
    wl = conv_skip_workload(8, 32, 3, 16, {2: 0})
    wl.layers[2].c_out = 24
    wl.layers[3].c_in = 24                       # the head takes what layer 2 gives; layer 2 cannot add 16 channels to its 24
    Ws, bs = ps.init_weights(wl.layers, 1)
    with pytest.raises(B.PartimeError):
        Pipeline(wl.layers, Ws, bs, loss=wl.loss, lr=wl.lr)
