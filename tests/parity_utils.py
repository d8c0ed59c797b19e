"""Shared helpers of the GPU parity tests: run a workload through the HIP
library, run the CPU oracle on the same seeded inputs (all elements, or an
index subset -- every element evolves independently of the others, so a subset
is exact), and compare within the stated tolerances."""
from __future__ import annotations

import numpy as np

from oracle import slowmo_oracle as O
from slowmo_inputs import generator as G
from slowmo_inputs import workloads as W


# ---- tolerances ---------------------------------------------------------------
# Parameters (replicas, x0): the bound the task states, |d| <= 1e-5 (1 + |x|).
# u is (x0 - xbar)/gamma accumulated (Eq. (2)): it carries x's rounding error
# divided by gamma, so the same bound is applied to gamma*u, which has x's units.
# h and v are sums of gradient-sized (sigma) resp. sigma^2-sized terms: the same
# relative bound with sigma resp. sigma^2 as the unit.
def _worst(got, want, scale, unit):
    """max over all elements of scale*|got - want| / (unit + scale*|want|),
    one row (worker) at a time so that whole-model arrays need no huge
    temporaries."""
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (got.shape, want.shape)
    if got.ndim == 2 and got.size > (1 << 24):
        return max((_worst(g, w_, scale, unit) for g, w_ in zip(got, want)), default=0.0)
    want = want.astype(np.float64, copy=False)
    err = scale * np.abs(got.astype(np.float64) - want) / (unit + scale * np.abs(want))
    return float(err.max(initial=0.0))


def assert_params_close(got, want, what):
    worst = _worst(got, want, 1.0, 1.0)
    assert worst <= 1e-5, f"{what}: max |d|/(1+|x|) = {worst:.3e}"
    return worst


def assert_u_close(got, want, lr, what):
    worst = _worst(got, want, lr, 1.0)
    assert worst <= 1e-5, f"{what}: max = {worst:.3e}"
    return worst


def assert_buffer_close(got, want, what, unit):
    worst = _worst(got, want, 1.0, unit)
    assert worst <= 1e-5, f"{what}: max |d|/({unit:g}+|.|) = {worst:.3e}"


def buffer_snapshot_step(w):
    """Inner step k (of the last round) after which h and v are compared.
    Under "reset" the buffers written by the last step of an outer iteration
    are never read again (line 2 of the next iteration zeroes them), and the
    library does not store them: compare after step tau-2 instead (-1: no
    such step when tau = 1)."""
    return w.tau - 2 if w.policy == "reset" else w.tau - 1


# ---- oracle side ----------------------------------------------------------------
def make_oracle(w, index, prec="f64", x_init=None):
    """index: the global element indices the oracle runs on (None: all of
    them, which needs x_init).  x_init: the starting point at those indices if
    it was read back from the device generator instead of computed on the host."""
    if x_init is None:
        x_init = G.initial_params(w.seed, index)
    return O.SlowMoOracle(x_init, m=w.m, tau=w.tau,
                          alpha=w.f32("alpha"), beta=w.f32("beta"), base=w.base,
                          policy=w.policy, momentum=w.f32("momentum"),
                          weight_decay=w.f32("weight_decay"), beta1=w.f32("beta1"),
                          beta2=w.f32("beta2"), eps=w.f32("eps"), prec=prec,
                          exact_average=w.exact_average, **_oracle_groups(w, index))


def _oracle_groups(w, index):
    """Per-tensor hyper-parameters for an oracle that runs on the element
    subset `index`: group sizes are the number of sampled elements per tensor;
    values are the fp32 numbers the library receives."""
    if w.tensor_wd is None and w.tensor_lr_scale is None:
        return {}
    if index is None:
        sizes = np.asarray(w.numel, dtype=np.int64)
    else:
        ends = w.tensor_starts + np.asarray(w.numel, dtype=np.int64)
        tensor = np.searchsorted(ends, np.asarray(index, dtype=np.int64), side="right")
        sizes = np.bincount(tensor, minlength=len(w.numel))
    f32 = lambda vals: None if vals is None else [float(np.float32(v)) for v in vals]  # noqa: E731
    return dict(tensor_sizes=sizes.tolist(), tensor_weight_decay=f32(w.tensor_wd),
                tensor_lr_scale=f32(w.tensor_lr_scale))


def oracle_grads(w, index, step):
    return np.stack([G.gradient(w.seed, i, step, index, w.sigma, bf16=(w.grad_dtype == "bf16"))
                     for i in range(w.m)])


def device_grads(w, prob, index, step):
    """The gradients of global step `step` at `index` (None: everywhere) as the
    DEVICE generator writes them into ring slot 0 -- the same bits as the host
    generator's (a test of its own), without NumPy's generation time."""
    prob.fill_grads(0, step)
    return np.stack([gather(prob, prob.grads[0][i], index) for i in range(w.m)])


_plans = {}


def gather(prob, tensors, index):
    """Values at `index` (None: everywhere).  The grouping of an index array
    by tensor is worked out once and kept while that array is alive."""
    if index is None:
        return prob.gather_all(tensors)
    key = (id(prob), id(index))
    if key not in _plans or _plans[key][0] is not index:
        if len(_plans) > 8:
            _plans.clear()
        _plans[key] = (index, prob.plan(index))
    return prob.gather(tensors, _plans[key][1])


def run_oracles(w, index, rounds, precs=("f64",), x_init=None, grad_fn=None):
    """Runs the oracle builds named in `precs` side by side on the same
    gradients (grad_fn(step) -> (m, n) float32, default: the host generator).
    Returns {prec: (oracle after the last outer step, snapshot taken after the
    local steps of the last round: dict with x, h, v)}."""
    os_ = {p: make_oracle(w, index, p, x_init) for p in precs}
    lr = w.f32("lr")
    snaps = {p: {} for p in precs}
    kb = buffer_snapshot_step(w)
    for t in range(rounds):
        for k in range(w.tau):
            g = grad_fn(t * w.tau + k) if grad_fn else oracle_grads(w, index, t * w.tau + k)
            for p, o in os_.items():
                o.local_step(g, lr)
                if w.mix == "expgraph":     # stochastic gradient push: step, then gossip
                    o.mix_step(O.exponential_graph_in_peers(w.m, t * w.tau + k))
                elif w.mix == "random":
                    o.mix_step(W.in_peers(w, t * w.tau + k))
                if t == rounds - 1 and k == kb:
                    snaps[p].update(h=o.h.copy(), v=None if o.v is None else o.v.copy())
        for p, o in os_.items():
            if t == rounds - 1:
                snaps[p].update(x=o.x.copy())
            o.outer_step(lr)
    return {p: (os_[p], snaps[p]) for p in precs}


def run_oracle(w, index, rounds, prec="f64"):
    return run_oracles(w, index, rounds, (prec,))[prec]


# ---- GPU side -------------------------------------------------------------------
def make_gpu(w, prob):
    from paper_1910_00643_amd.optimizer import SlowMo, make_config
    cfg = make_config(m=w.m, tau=w.tau, alpha=w.alpha, beta=w.beta, base=w.base,
                      policy=w.policy, grad_dtype=w.grad_dtype, momentum=w.momentum,
                      weight_decay=w.weight_decay, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                      no_average=not w.exact_average)
    opt = SlowMo(prob.params, cfg)
    if w.tensor_wd is not None or w.tensor_lr_scale is not None:
        opt.set_tensor_hparams(w.tensor_wd, w.tensor_lr_scale)
    return opt


def _gpu_in_peers(w, step):
    import paper_1910_00643_amd as P
    if w.mix == "expgraph":
        return P.slowmo_expgraph_in_peers(w.m, step)
    return W.in_peers(w, step).tolist()


def run_gpu(w, prob, opt, rounds, index, fused_last=False, fused_mix=False):
    """Runs `rounds` outer iterations; gradients are regenerated before every
    local step (ring slots in turn).  Returns the snapshot (x, h, v at the
    sampled indices) taken after the local steps of the last round."""
    lr = w.lr
    arrays = [opt.grad_pointer_array(prob.grads[s]) for s in range(prob.ring)]
    snap = {}
    step = 0
    kb = buffer_snapshot_step(w)
    for t in range(rounds):
        for k in range(w.tau):
            s = step % prob.ring
            prob.fill_grads(s, step)
            if fused_last and k == w.tau - 1 and not (t == rounds - 1):
                opt.local_outer_step(arrays[s], lr)     # last local step + outer step
                step += 1
                continue
            if w.mix != "none" and fused_mix:       # local step + gossip step as one call
                opt.local_mix_step(arrays[s], lr, _gpu_in_peers(w, step))
            else:
                opt.local_step(arrays[s], lr)
                if w.mix != "none":
                    opt.mix_step(_gpu_in_peers(w, step))
            step += 1
            if t == rounds - 1 and k == kb:
                st = gpu_state(w, prob, opt, index, with_outer=False)
                snap.update(h=st["h"], v=st["v"])
        if t == rounds - 1:
            snap.update(x=gpu_state(w, prob, opt, index, with_outer=False)["x"])
            opt.outer_step(lr)
        elif not fused_last:
            opt.outer_step(lr)
    return snap


def gpu_state(w, prob, opt, index, with_outer=True):
    nt = len(prob.numel)
    out = dict(
        x=np.stack([gather(prob, prob.params[i], index) for i in range(w.m)]),
        h=np.stack([gather(prob, [opt.buffer("h", j, i) for j in range(nt)], index)
                    for i in range(w.m)]))
    out["v"] = None
    if w.base == "adam":
        out["v"] = np.stack([gather(prob, [opt.buffer("v", j, i) for j in range(nt)], index)
                             for i in range(w.m)])
    if with_outer and w.exact_average:
        out["x0"] = gather(prob, [opt.buffer("x0", j) for j in range(nt)], index)
        out["u"] = gather(prob, [opt.buffer("u", j) for j in range(nt)], index)
    elif with_outer:            # every worker has its own x0 and u
        for key in ("x0", "u"):
            out[key] = np.stack([gather(prob, [opt.buffer(key, j, i) for j in range(nt)], index)
                                 for i in range(w.m)])
    return out


def compare_run(w, prob, opt, index, rounds, bitwise_f32=False, fused_last=False,
                fused_mix=False, device_inputs=False):
    """Full comparison of a finished GPU run against the oracle on `index`
    (None: every element).  With fused_last, every outer iteration but the
    final one (whose replicas are inspected before the outer step) ends with
    slowmo_local_outer_step.  device_inputs: the oracle's starting point and
    gradients are read back from the device generator (for index sets too
    large to generate with NumPy in reasonable time)."""
    lr = w.f32("lr")
    x_init = gather(prob, prob.params[0], index) if device_inputs else None   # before any step
    snap = run_gpu(w, prob, opt, rounds, index, fused_last=fused_last, fused_mix=fused_mix)
    final = gpu_state(w, prob, opt, index)
    grad_fn = (lambda step: device_grads(w, prob, index, step)) if device_inputs else None
    res = run_oracles(w, index, rounds, ("f64", "f32") if bitwise_f32 else ("f64",),
                      x_init=x_init, grad_fn=grad_fn)
    o64, s64 = res["f64"]
    worst = {}
    worst["x_local"] = assert_params_close(snap["x"], s64["x"], "replicas after the local steps")
    if "h" in snap:
        assert_buffer_close(snap["h"], s64["h"], "h after the local steps", unit=w.sigma)
        if w.base == "adam":
            assert_buffer_close(snap["v"], s64["v"], "v after the local steps", unit=w.sigma ** 2)
    worst["x0"] = assert_params_close(final["x0"], o64.x0, "x0 after the run")
    worst["u"] = assert_u_close(final["u"], o64.u, lr, "u after the run")
    for i in range(w.m):                 # Section 2: identical on all workers
        own = final["x0"] if w.exact_average else final["x0"][i]
        assert np.array_equal(final["x"][i], own), f"replica {i} differs from x0"
    if bitwise_f32:
        # The SGD and outer kernels round every product and sum separately in
        # the order of the formulas, as the fp32 build of the oracle does.
        o32, s32 = res["f32"]
        assert np.array_equal(snap["x"], s32["x"]), "replicas differ from the fp32 oracle"
        if "h" in snap:
            assert np.array_equal(snap["h"], s32["h"])
        assert np.array_equal(final["x0"], o32.x0), "x0 differs from the fp32 oracle"
        assert np.array_equal(final["u"], o32.u), "u differs from the fp32 oracle"
    return worst
