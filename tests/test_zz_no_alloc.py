"""partime_step_noalloc (the entry point for callers that cannot allocate) against partime_step: same kernels, the
loss partials in the library's static device array instead of the context's buffer, so every output, loss, weight and
published buffer must be bit-identical.  Two calls in a row, the second on a smaller network (fewer tiles in the last
stage, fewer ticks): what the first call left in the array must not be seen."""
import numpy as np
import pytest
import torch

import partime_streams as ps
from paper_2210_09147_amd import Pipeline, binding as B

pytestmark = pytest.mark.gpu


def both_ways(w, T, chunks, adam=None):
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, T)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    res = []
    for entry in (B.partime_step, B.partime_step_noalloc):
        p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, balance=w.balance, adam=adam)
        out = torch.zeros((T, 1, w.out_size), dtype=torch.float32, device="cuda")
        loss = torch.full((T,), -1.0, dtype=torch.float32, device="cuda")
        for i, j in chunks:
            entry(p.ctx, xd[i:j].data_ptr(), td[i:j].data_ptr(), j - i, out[i:j].data_ptr(), loss[i:j].data_ptr())
        torch.cuda.synchronize()
        state = [p.weights(i) for i in range(len(w.layers))]
        bufs = [B.partime_get_buffer(p.ctx, 1, h, (T - 1) & 1, w.layers[p_first(w, h)].in_dim) for h in range(1, w.depth)]
        res.append((out.cpu().numpy(), loss.cpu().numpy(), state, bufs))
        assert p.tick == T
        p.close()
    (o1, l1, s1, e1), (o2, l2, s2, e2) = res
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    assert np.isfinite(l2).all() and (l2[max(w.depth - 1, w.k):] > 0).all()      # real losses came through the scratch array
    for (W1, b1), (W2, b2) in zip(s1, s2):
        assert np.array_equal(W1, W2) and np.array_equal(b1, b2)
    for a, b in zip(e1, e2):
        assert np.array_equal(a, b)


def p_first(w, h):
    return int(np.sum(w.balance[:h])) if w.balance else h


def test_noalloc_entry_point_matches_partime_step_twice_in_a_row():
    # first call: wide last stage (many tiles, so many loss partials per tick), more than one block of 1024 ticks is not
    # needed to fill the array; MSE is the loss whose partials go through the scratch array
    big = ps.small_mlp([300, 1500, 1200, 3000], ps.ACT_RELU, ps.LOSS_MSE, lr=0.01, drift=0.05, seed=51)
    both_ways(big, 40, [(0, 1), (1, 25), (25, 40)])
    # second call, right after it on the same GPU: a smaller network with fewer tiles and fewer ticks, Adam, two layers
    # in the last stage
    small = ps.small_mlp([64, 96, 80, 24], ps.ACT_GELU, ps.LOSS_MSE, lr=1e-3, drift=0.05, seed=52, balance=[1, 2])
    both_ways(small, 12, [(0, 12)], adam=(0.9, 0.999, 1e-8))
    # and the softmax head, whose loss does not go through the partials at all
    ce = ps.small_mlp([64, 96, 10], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=53)
    both_ways(ce, 9, [(0, 4), (4, 9)])


def test_noalloc_entry_point_refuses_what_it_was_not_built_for():
    w = ps.small_mlp([64, 96, 10], ps.ACT_RELU, ps.LOSS_CE, lr=0.05, drift=0.05, seed=53)
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, 4)
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    out = torch.zeros((4, 1, 10), dtype=torch.float32, device="cuda")
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, exec_mode=B.PT_EXEC_PERSISTENT)
    with pytest.raises(B.PartimeError) as e:
        B.partime_step_noalloc(p.ctx, xd.data_ptr(), td.data_ptr(), 4, out.data_ptr(), 0)
    assert e.value.code == B.PT_EUNSUPPORTED and p.tick == 0
    p.close()
    w.n_streams, w.w_dtype = 32, ps.W_BF16
    x, tg = ps.make_inputs(w, 2)
    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, n_streams=32, w_dtype=B.PT_BF16)
    with pytest.raises(B.PartimeError) as e:
        B.partime_step_noalloc(p.ctx, torch.from_numpy(x).cuda().data_ptr(), torch.from_numpy(tg).cuda().data_ptr(), 2,
                               torch.zeros((2, 32, 10), device="cuda").data_ptr(), 0)
    assert e.value.code == B.PT_EUNSUPPORTED
    p.close()
