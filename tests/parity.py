"""Comparison machinery of the GPU parity tests (a helper module, not a test file).

The HIP path, called through the C ABI, is compared with the CPU oracle on the same seeded inputs:

* element by element, not through one norm per array: an array passes when every element is within
  tol * max|reference| of the reference (plus, for stored weights, one unit in the last place of the storage
  type: both sides round their own exact result to it), and its 2-norm error is within tol as well;
* on the UPDATE, not on the weights: what is compared is W - W_sync, where W_sync is the last state both sides
  had in common (the initial weights, or the oracle's state at the last re-synchronisation), so a missing or wrong
  update cannot hide behind weights that are 10^3 .. 10^7 times larger than what one tick changes;
* on everything a tick publishes: the output row, the loss, the activation and error buffers of every stage
  boundary (through partime_get_buffer), the Adam moments.

ReLU.  Eq. 9 takes phi' at this tick's z and ReLU' jumps at 0.  The oracle sums z in fp64, the kernels in fp32 in
another order, so a unit whose |z| is below the rounding error of such a sum can come out on either side, and both
one-sided derivatives are derivatives of what the respective side evaluated: for such a unit the result is not
unique.  The oracle therefore records every ReLU unit with |z| < BAND and a non-zero error signal (a diagnostic
pinned on the CPU).  A tick without such a unit is compared as it is.  For a tick with such units two more oracle
ticks are run from the same state, one taking derivative 1 and one taking 0 for exactly those units; the elements
in which these two differ are the ones that depend on the undecided units (one weight row per unit, the error
vector of that stage), every other element is unique and is compared at the full bar, and an element of the first
kind must agree with one of the oracle's variants.  After such a tick the library is handed the oracle's state
(weights, moments, both halves of every buffer), so that one undecided unit cannot leak into later ticks.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle as orc
import partime_streams as ps
from paper_2210_09147_amd import Pipeline, binding as B

F32_TOL, BF16_TOL = 1e-5, 2e-2
# Half-width of the band around z = 0 inside which a ReLU decision counts as undecided, relative to the size of the
# unit's terms (sum_i |w_i u_i| + |b|), which is what the rounding error of any summation order is proportional to.
# It depends on how a kernel family sums: per-lane partial sums and a tree (dense, one stream), fp32 matrix-core
# accumulation of bf16 products (32 streams and more), one long fp32 matrix-core accumulation chain (conv).  The
# full-size tests print the largest |z - z_oracle| they see (where a ReLU unit is active its published output is z):
# 3.6e-7 at terms of size ~16 (dense), 2.2e-6 at ~25 (32 streams), 3.6e-6 at ~10 (conv), i.e. 2e-8, 9e-8 and 4e-7 of
# the terms; each band is about five times that.
BAND_DENSE, BAND_MFMA, BAND_CONV = 2.0 ** -23, 2.0 ** -21, 2.0 ** -19
ULP_F32, ULP_BF16 = 2.0 ** -23, 2.0 ** -7     # one unit in the last place relative to the value (upper bound)
# State after n > 1 free ticks (no common state in between): learning amplifies rounding differences from tick to tick,
# and the error signals are differences of nearly equal numbers, so the end-of-run state is compared at FREE_FACTOR
# times the bar (outputs and losses of every tick stay at the bar itself, and so does every single tick taken from
# a common state).  Stored weights: both sides round every tick, the two rounding errors walk apart like sqrt(n).
FREE_FACTOR = 10.0


class Report:
    """Collects what was compared, so that a test can assert it was not blind and print its margins."""

    def __init__(self):
        self.rows = []          # (name, worst element error / (tol * scale), norm error / tol, masked fraction)
        self.failures = []
        self.event_ticks = 0
        self.events = 0
        self.z_err = 0.0        # largest absolute difference of a published ReLU activation (= of z where z > 0)

    def add(self, name, elem, norm, masked, ok, detail=""):
        self.rows.append((name, elem, norm, masked))
        if not ok:
            self.failures.append(f"{name}: element error {elem:.3g} x tol, norm error {norm:.3g} x tol, masked {masked:.2%} {detail}")

    def worst(self):
        return max([max(r[1], r[2]) for r in self.rows], default=0.0)

    def failed(self, prefix=""):
        return [f for f in self.failures if f.startswith(prefix)]


def compare(rep, name, got, ref, tol, *, scale=None, floor=None, P=None, N=None, elem_factor=1.0):
    """got vs ref element by element and in the 2-norm.  scale: what tol is relative to (default max|ref|);
    floor: per-element absolute slack (storage rounding); P, N: the oracle's two variants of a tick with undecided
    ReLU units; elem_factor: multiple of tol allowed to single elements (the norm stays at tol)."""
    got = np.asarray(got, np.float64).ravel()
    ref = np.asarray(ref, np.float64).ravel()
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if got.size == 0:
        return
    if scale is None:
        scale = float(np.max(np.abs(ref)))
    fl = np.zeros_like(ref) if floor is None else np.broadcast_to(np.asarray(floor, np.float64).ravel(), ref.shape)
    lim = elem_factor * tol * scale + fl
    err = np.abs(got - ref)
    finite = np.isfinite(got).all()
    masked = np.zeros(ref.shape, bool)
    if P is not None:
        # Elements that depend on undecided units are not unique: the library may have decided each unit either way
        # (2^n valid results for n units; inside a stage of several layers the units of different layers interact).
        # They get a sanity range only: no further from the reference than twice the largest distance of the oracle's
        # all-active and all-inactive variants over all such elements of the array (element by element the two
        # extremes say little: the contributions of several units can cancel in them and not in a mix).
        Pv, Nv = np.asarray(P, np.float64).ravel(), np.asarray(N, np.float64).ravel()
        masked = Pv != Nv
        reach = 2.0 * float((np.abs(Pv - ref) + np.abs(Nv - ref)).max()) if masked.any() else 0.0
        out = np.maximum(np.abs(got - ref) - reach, 0.0)
        err = np.where(masked, out, err)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(lim > 0, err / np.where(lim > 0, lim, 1.0), np.where(err > 0, np.inf, 0.0))
    elem = float(ratio.max())
    u = ~masked
    nlim = tol * float(np.linalg.norm(ref[u])) + float(np.linalg.norm(fl[u]))
    nerr = float(np.linalg.norm((got - ref)[u]))
    norm = nerr / nlim if nlim > 0 else (np.inf if nerr > 0 else 0.0)
    rep.add(name, elem, norm, float(masked.mean()), finite and elem <= 1.0 and norm <= 1.0)


def compare_bf16_weights(rep, name, got, ref, base, tol, P=None, N=None, min_exact=0.97):
    """Stored bf16 weights one tick after a common state: both sides round their own exact result to bf16, so all but a
    few per cent must be bit-identical, and the rest at most one bf16 step apart, plus the bar on the update itself:
    where a large update nearly cancels the weight, a step of the small result is below the arithmetic error of the
    update.  The scale of that bar is the largest update in the element's row, not the element's own: an update element
    is a sum over the streams of delta[r][s] * x[c][s], and where those terms nearly cancel, one delta[r][s] that the
    two sides rounded to neighbouring bf16 values (its fp32 and fp64 sums straddle a rounding boundary) moves the
    element by a fraction of the terms, not of their sum."""
    shape = np.asarray(ref).shape
    got = np.asarray(got, np.float32).ravel()
    ref = np.asarray(ref, np.float32).ravel()
    base = np.asarray(base, np.float32).ravel()
    u = np.ones(ref.shape, bool)
    if P is not None:
        u = np.asarray(P, np.float32).ravel() == np.asarray(N, np.float32).ravel()
    same = got == ref
    upd = np.abs(ref.astype(np.float64) - base)
    scale = np.broadcast_to(upd.reshape(shape).max(axis=-1, keepdims=True), shape).ravel() if len(shape) == 2 else upd
    step = ULP_BF16 * np.maximum(np.abs(got), np.abs(ref)) + tol * scale
    dist = np.abs(got.astype(np.float64) - ref) / np.maximum(step, 1e-300)
    near = dist <= 1.0
    frac = float(same[u].mean()) if u.any() else 1.0
    ok = bool(near[u].all()) and frac >= min_exact and bool(np.isfinite(got).all())
    rep.add(name + " (bit-identical fraction)", 0.0 if ok else np.inf, (1.0 - frac) / (1.0 - min_exact), float((~u).mean()), ok,
            f"bit-identical {frac:.4f}, all within one step: {bool(near[u].all())}, worst {float(dist[u].max()) if u.any() else 0.0:.2f} steps")


class Pair:
    """One oracle and one or more library pipelines (differing in execution mode or call chunking) over one workload."""

    def __init__(self, w, *, bf16=None, k=None, adam=None, tol=None, pipes=({},), band=None, x=None, tg=None, T=None):
        self.w = w
        self.bf16 = (w.w_dtype == ps.W_BF16) if bf16 is None else bf16
        self.S = w.n_streams
        self.mfma_bf16 = self.S > 1                      # operands of every product rounded to bf16
        self.k = w.k if k is None else k
        self.adam = adam
        self.tol = tol or (BF16_TOL if (self.bf16 or self.mfma_bf16) else F32_TOL)
        self.D = w.depth
        self.layers = w.layers
        self.Ws, self.bs = ps.init_weights(w.layers, w.seed)
        if x is None:
            x, tg = ps.make_inputs(w, T)
        self.x, self.tg = x, tg
        self.ref = orc.Oracle(w.layers, self.Ws, self.bs, loss=w.loss, lr=w.lr, target_delay=self.k, w_bf16=self.bf16,
                              n_streams=self.S, operands_bf16=self.mfma_bf16, balance=w.balance, adam=adam)
        self.relu = any(l.act == ps.ACT_RELU for l in w.layers)
        if band is None:
            band = BAND_CONV if w.layers[0].kind == ps.CONV3X3 else (BAND_MFMA if self.S > 1 else BAND_DENSE)
        self.band = band
        if self.relu:
            self.ref.set_kink_band(band, 0)
        self.pipes, self.chunks = [], []
        for kw in pipes:
            kw = dict(kw)
            self.chunks.append(kw.pop("chunks", None))
            gpu_lr = kw.pop("gpu_lr", None)     # a library that runs with another step size than the oracle (negative controls)
            self.pipes.append(Pipeline(w.layers, self.Ws, self.bs, loss=w.loss, lr=w.lr, target_delay=self.k,
                                       w_dtype=B.PT_BF16 if self.bf16 else B.PT_F32, n_streams=self.S, balance=w.balance,
                                       adam=adam, **kw))
            if gpu_lr is not None:
                B.partime_set_lr(self.pipes[-1].ctx, gpu_lr)
        self.xd, self.td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
        self.rep = Report()
        self.lr = w.lr
        self._take_sync(self.ref)

    # ------------------------------------------------------------------ state
    def close(self):
        for p in self.pipes:
            B.partime_sync(p.ctx)
            p.close()

    def _state_of(self, o):
        st = {"W": [o.get_weights(i) for i in range(len(self.layers))]}
        if self.adam is not None:
            st["M"] = [o.get_moments(i) for i in range(len(self.layers))]
        return st

    def _take_sync(self, o):
        """Remember the state both sides have in common: the base the updates are measured from."""
        self.sync = self._state_of(o)
        self.sync_tick = o.tick

    def _load(self, src):
        """Hand the library the oracle's whole state: weights, moments, both halves of every buffer, tick."""
        st = self._state_of(src)
        for p in self.pipes:
            for i in range(len(self.layers)):
                B.partime_set_state(p.ctx, i, *st["W"][i])
                if self.adam is not None:
                    B.partime_set_opt_state(p.ctx, i, *st["M"][i])
            for h in range(self.D):
                for half in (0, 1):
                    if h < self.D - 1:
                        B.partime_set_buffer(p.ctx, 0, h, half, src.get_buffer("act", h, half))
                    if h > 0:
                        B.partime_set_buffer(p.ctx, 1, h, half, src.get_buffer("err", h, half))
            if self.k > 0:
                B.partime_set_buffer(p.ctx, 2, 0, 0, src.get_history())
            B.partime_set_tick(p.ctx, src.tick)
            # the delay lines of skip connections, by age (the library keeps them in rings indexed by the tick: after set_tick)
            for i in range(len(self.layers)):
                for age in range(src.skip_delay(i)):
                    B.partime_set_buffer(p.ctx, 3, i, age, src.get_lane(0, i, age))
                    B.partime_set_buffer(p.ctx, 4, i, age, src.get_lane(1, i, age))
        self.sync = st
        self.sync_tick = src.tick

    def set_lr(self, lr):
        self.lr = lr
        self.ref.set_lr(lr)
        for p in self.pipes:
            B.partime_set_lr(p.ctx, lr)

    # ------------------------------------------------------------------ comparisons
    def check_state(self, tag, P=None, N=None, rep=None, pipes=None):
        """Updates since the last common state, moments, and the buffers written by the last tick."""
        rep = rep or self.rep
        ref = self.ref
        cur = self._state_of(ref)
        half = (ref.tick - 1) & 1
        n_free = ref.tick - self.sync_tick                   # ticks since both sides had a common state
        strict = n_free <= 1
        tol = self.tol if strict else FREE_FACTOR * self.tol
        steps = 1.0 if strict else 2.5 * np.sqrt(n_free)     # storage rounding of the weights, both sides, n ticks
        var = None
        if P is not None:
            var = (self._state_of(P), self._state_of(N))
        for pi, p in enumerate(pipes or self.pipes):
            nm = f"{tag} pipe{pi}"
            for i in range(len(self.layers)):
                for j, what in enumerate(("W", "b")):
                    got, want, base = p.weights(i)[j], cur["W"][i][j], self.sync["W"][i][j]
                    base64 = base.astype(np.float64)
                    Pd = Nd = None
                    if var:
                        Pd, Nd = var[0]["W"][i][j] - base64, var[1]["W"][i][j] - base64
                    stored_bf16 = self.bf16 and what == "W"
                    floor = steps * (ULP_BF16 if stored_bf16 else ULP_F32) * np.maximum(np.abs(want), np.abs(got))
                    # An Adam step divides by sqrt(v): for a weight whose gradient is near zero that quotient amplifies
                    # the rounding differences of the gradient sum, so single elements get ten times the bar there
                    # So does a conv weight gradient: each element is a sum over all H x W pixels of products of mixed
                    # sign, whose fp32 accumulation error is proportional to the sum of the |terms|, 30 .. 250 times
                    # the sum itself at 10^3 .. 6 10^4 pixels.
                    loose = self.adam is not None or self.layers[i].kind == ps.CONV3X3
                    compare(rep, f"{nm} update of {what}{i}", got - base64, want - base64, tol, floor=floor, P=Pd, N=Nd,
                            elem_factor=10.0 if loose else 1.0)
                    if stored_bf16 and strict:
                        compare_bf16_weights(rep, f"{nm} W{i}", got, want, base, tol,
                                             *((var[0]["W"][i][j], var[1]["W"][i][j]) if var else (None, None)))
                if self.adam is not None:
                    for j, what in enumerate(("mW", "vW", "mb", "vb")):
                        Pm = Nm = None
                        if var:
                            Pm, Nm = var[0]["M"][i][j], var[1]["M"][i][j]
                        compare(rep, f"{nm} {what}{i}", p.moments(i)[j], cur["M"][i][j], tol, P=Pm, N=Nm)
            for h in range(self.D):
                if h < self.D - 1:
                    want = ref.get_buffer("act", h, half)
                    got = B.partime_get_buffer(p.ctx, 0, h, half, want.size)
                    if self.S >= 64:      # these pipelines keep the published activations as bf16
                        want = _round_bf16(want)
                    compare(rep, f"{nm} act{h}", got, want, tol)      # forward: does not depend on the derivative
                    if self.relu and self.S < 64:
                        # where a ReLU unit is active its output IS z: the largest absolute difference is a direct
                        # measurement of how far the library's z is from the oracle's (what BAND must cover)
                        rep.z_err = max(rep.z_err, float(np.abs(np.asarray(got, np.float64) - want.ravel()).max()))
                if h > 0:
                    want = ref.get_buffer("err", h, half)
                    got = B.partime_get_buffer(p.ctx, 1, h, half, want.size)
                    Pe = Ne = None
                    if P is not None:
                        Pe, Ne = P.get_buffer("err", h, half), N.get_buffer("err", h, half)
                    # an error signal at the rounding level of its own sums (a loss head that has nothing left to
                    # learn: softmax - onehot of order 1e-7) has no digits to compare: the test must not end up there
                    assert h < self.D - 1 or float(np.abs(want).max()) > 1e-6 or ref.tick <= max(self.D - 1, self.k), \
                        f"the loss gradient has collapsed (error of the last stage {float(np.abs(want).max()):.1e}): choose inputs that keep the loss up"
                    compare(rep, f"{nm} err{h}", got, want, tol, P=Pe, N=Ne)
            # what the last tick put into the delay lines of skip connections that cross stage boundaries
            for i in range(len(self.layers)):
                if ref.skip_delay(i) < 1:
                    continue
                want = ref.get_lane(0, i, 0)
                compare(rep, f"{nm} skipped tensor into layer {i}", B.partime_get_buffer(p.ctx, 3, i, 0, want.size), want, tol)
                want = ref.get_lane(1, i, 0)
                Pe = Ne = None
                if P is not None:
                    Pe, Ne = P.get_lane(1, i, 0), N.get_lane(1, i, 0)
                compare(rep, f"{nm} skip gradient of layer {i}", B.partime_get_buffer(p.ctx, 4, i, 0, want.size), want, tol, P=Pe, N=Ne)

    def _check_outputs(self, outs, losses, a, b):
        for pi in range(len(self.pipes)):
            for t in range(a, b):
                if t >= self.D - 1:
                    compare(self.rep, f"pipe{pi} out[{t}]", outs[pi][t], self.ro[t], self.tol)
                lt, rt = float(losses[pi][t]), float(self.rl[t])
                ok = abs(lt - rt) <= 10 * self.tol * max(abs(rt), 1e-3)
                self.rep.add(f"pipe{pi} loss[{t}]", abs(lt - rt) / (10 * self.tol * max(abs(rt), 1e-3)), 0.0, 0.0, ok)

    # ------------------------------------------------------------------ running
    def _gpu_run(self, outs, losses, a, b):
        for pi, p in enumerate(self.pipes):
            cuts = sorted({a, b} | {j for (_, j) in (self.chunks[pi] or []) if a < j < b})
            for i, j in zip(cuts[:-1], cuts[1:]):
                o, l = p.step(self.xd[i:j], self.td[i:j])
                outs[pi][i:j] = o.cpu().numpy()
                losses[pi][i:j] = l.cpu().numpy()

    def run(self, T0, T1):
        """Learning ticks T0 .. T1-1 of the stream on both sides.  The library runs freely (its own state from tick to
        tick) except after a tick with undecided ReLU units, where it is handed the oracle's state."""
        n_out = self.w.out_size
        S = self.S
        outs = [np.zeros((T1, S, n_out), np.float32) for _ in self.pipes]
        losses = [np.zeros((T1,), np.float32) for _ in self.pipes]
        if not hasattr(self, "ro"):
            self.ro, self.rl = {}, {}
        pending = T0
        for t in range(T0, T1):
            snap = self.ref.clone() if self.relu else None
            o, l = self.ref.step(self.x[t:t + 1], self.tg[t:t + 1])
            self.ro[t], self.rl[t] = o[0], l[0]
            cnt = self.ref.take_kink_events()[0] if self.relu else 0
            if cnt == 0:
                continue
            self.rep.event_ticks += 1
            self.rep.events += cnt
            P, N = snap, snap.clone()
            P.set_kink_band(self.band, +1)
            N.set_kink_band(self.band, -1)
            P.step(self.x[t:t + 1], self.tg[t:t + 1])
            N.step(self.x[t:t + 1], self.tg[t:t + 1])
            self._gpu_run(outs, losses, pending, t + 1)
            self._check_outputs(outs, losses, pending, t + 1)
            self.check_state(f"tick {t}", P, N)
            self._load(self.ref)
            pending = t + 1
        if pending < T1:
            self._gpu_run(outs, losses, pending, T1)
            self._check_outputs(outs, losses, pending, T1)
        self.check_state(f"tick {T1 - 1}")
        for p in self.pipes:
            assert p.tick == T1
        return outs, losses

    def warm(self, T0, T1):
        """Ticks T0 .. T1-1 on the oracle alone (the library is handed the resulting state by the next forced tick)."""
        self.ref.step(self.x[T0:T1], self.tg[T0:T1])
        if self.relu:
            self.ref.take_kink_events()

    def synthetic_state(self, tick, seed=0, act_scale=1.0, err_scale=1e-3):
        """A full pipeline without the ticks that fill it: every activation buffer gets seeded half-normal values (what a
        ReLU layer publishes), every error buffer seeded normal values, the tick counter moves past the fill.  A single
        tick from such a state exercises every step of every stage; the state need not be one the net can reach."""
        rng = np.random.Generator(np.random.PCG64(seed + 5000))
        for h in range(self.D):
            for half in (0, 1):
                if h < self.D - 1:
                    n = self.ref.stage_out[h]
                    self.ref.set_buffer("act", h, half, np.abs(rng.standard_normal((self.S, n))) * act_scale)
                if h > 0:
                    n = self.ref.stage_in[h]
                    e = rng.standard_normal((self.S, n)) * err_scale
                    first = self.layers[int(np.sum(self.ref.balance[:h]))]
                    if first.kind == ps.GAP_DENSE:      # a pooled layer hands every pixel of a channel the same error
                        e = np.repeat(e.reshape(self.S, first.c_in, -1)[:, :, :1], first.h * first.w, axis=2).reshape(self.S, n)
                    self.ref.set_buffer("err", h, half, e)
        self.ref.tick = tick

    def forced_tick(self, t, lr=None, negative=False):
        """Tick t from the oracle's state on both sides (the library is handed that state first), optionally with a step
        size of its own for this tick (a tick is linear in it: a large one makes the update of every layer stand out of
        the storage rounding of the weights).  negative: first show that the comparison would catch a library that
        does not update, by running the library's tick with step size 0 against the oracle's real tick."""
        assert self.ref.tick == t
        old_lr = self.lr
        self._load(self.ref)
        snap = self.ref.clone()
        if lr is not None:
            self.set_lr(lr)
        o, l = self.ref.step(self.x[t:t + 1], self.tg[t:t + 1])
        if not hasattr(self, "ro"):
            self.ro, self.rl = {}, {}
        self.ro[t], self.rl[t] = o[0], l[0]
        cnt = self.ref.take_kink_events()[0] if self.relu else 0
        P = N = None
        if cnt:
            self.rep.event_ticks += 1
            self.rep.events += cnt
            P, N = snap.clone(), snap.clone()
            for v, side in ((P, +1), (N, -1)):
                v.set_lr(self.lr)
                v.set_kink_band(self.band, side)
                v.step(self.x[t:t + 1], self.tg[t:t + 1])
        S, n_out = self.S, self.w.out_size
        outs = [np.zeros((t + 1, S, n_out), np.float32) for _ in self.pipes]
        losses = [np.zeros((t + 1,), np.float32) for _ in self.pipes]
        if negative:
            for p in self.pipes:
                B.partime_set_lr(p.ctx, 0.0)
            self._gpu_run(outs, losses, t, t + 1)
            neg = Report()
            self.check_state(f"tick {t} (library step size 0)", P, N, rep=neg)
            for pi in range(len(self.pipes)):
                for i in range(len(self.layers)):
                    assert neg.failed(f"tick {t} (library step size 0) pipe{pi} update of W{i}"), \
                        f"the comparison does not see the update of layer {i}: a library that leaves W{i} alone passes"
            self._load(snap)          # back to the state before the tick
            for p in self.pipes:
                B.partime_set_lr(p.ctx, self.lr)
        self._gpu_run(outs, losses, t, t + 1)
        self._check_outputs(outs, losses, t, t + 1)
        self.check_state(f"forced tick {t}", P, N)
        if lr is not None:
            # the tick was taken with a step size of its own: take it again, on the oracle alone, with the real one, so
            # that what follows is the trajectory of the workload (an inflated step can saturate everything after it)
            self.set_lr(old_lr)
            snap.set_lr(old_lr)
            snap.step(self.x[t:t + 1], self.tg[t:t + 1])
            if self.relu:
                snap.take_kink_events()
            self.ref = snap
        # what follows starts from the oracle's state
        self._load(self.ref)
        return cnt

    def pick_lr(self, rel=0.02):
        """A step size for one forced tick under which the update of EVERY layer is at least `rel` of its largest
        weight, from the oracle's gradients of the last tick."""
        need = []
        for i in range(len(self.layers)):
            W = self.ref.get_weights(i)[0]
            if self.adam is not None:
                need.append(rel * float(np.abs(W).max()))       # an Adam step is about the step size itself
                continue
            dW = self.ref.get_grads(i)[0]
            g = float(np.abs(dW).max())
            assert g > 0, f"layer {i} has no gradient yet: run more ticks before forcing one"
            need.append(rel * float(np.abs(W).max()) / g)
        return float(np.float32(max(need)))

    def assert_ok(self, min_rows=1):
        assert len(self.rep.rows) >= min_rows
        assert not self.rep.failures, "\n".join(self.rep.failures[:12] + [f"... {len(self.rep.failures)} failures"])


def _round_bf16(a):
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7fff + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)
