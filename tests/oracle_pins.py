"""Pins for the CPU oracle: facts fixed by the paper or by mathematics, none of
which re-types the oracle's own formulas.

Each pin is a function pin_*(make) where make(x_init, **kw) builds an oracle
instance (fp64).  test_oracle_pins.py runs them on the real oracle;
test_oracle_mutants.py runs them on deliberately broken copies of the oracle
and requires every planted mistake to be caught by at least one pin.
"""
from __future__ import annotations

import numpy as np
import torch

RT = 1e-12   # fp64 identities hold to a few ulp over the short runs used here


def _rng(seed=0):
    return np.random.default_rng(seed)


def _close(a, b, rtol=RT, atol=1e-13, what=""):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    err = np.abs(a - b)
    bound = atol + rtol * np.maximum(np.abs(a), np.abs(b))
    assert np.all(err <= bound), f"{what}: max err {err.max():.3e} (bound {bound.min():.3e})"


def _grads(rng, T, tau, m, d, scale=1.0):
    return (scale * rng.standard_normal((T, tau, m, d))).astype(np.float32)


# ---------------------------------------------------------------- Section 2

def pin_mean_of_updates(make):
    """Section 2, sentence after Algorithm 1: with plain SGD as base,
    xbar_{t,tau} = x_{t,0} - (gamma/m) sum_i sum_k g^{(i)}_{t,k}."""
    rng = _rng(1)
    T, tau, m, d, lr = 3, 4, 3, 17, 0.05
    g = _grads(rng, T, tau, m, d)
    o = make(rng.standard_normal(d), m=m, tau=tau, alpha=0.8, beta=0.5)
    for t in range(T):
        x_t0 = o.x0.copy()
        for k in range(tau):
            o.local_step(g[t, k], lr)
        xbar = o.x.mean(axis=0)
        _close(xbar, x_t0 - lr / m * g[t].astype(np.float64).sum(axis=(0, 1)),
               what="mean of updates")
        o.outer_step(lr)


def pin_heavy_ball_form(make):
    """Appendix D.1 ("Equivalent Updates"): x_{t+1,0} = x_{t,0} - alpha*gamma*
    sum_k dbar_{t,k} + beta*(x_{t,0} - x_{t-1,0}); with plain SGD dbar is the
    worker-mean gradient, so the right-hand side needs the inputs only."""
    rng = _rng(2)
    T, tau, m, d, lr, alpha, beta = 5, 4, 3, 11, 0.05, 0.75, 0.6
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=alpha, beta=beta)
    prev, cur = x_init.copy(), x_init.copy()
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
        o.outer_step(lr)
        dsum = g[t].astype(np.float64).mean(axis=1).sum(axis=0)
        nxt = cur - alpha * lr * dsum + beta * (cur - prev)
        _close(o.x0, nxt, what=f"heavy-ball form, t={t}")
        prev, cur = cur, nxt


def pin_auxiliary_sequence(make):
    """Appendix D.1: y_t = x_t + beta/(1-beta)*(x_t - x_{t-1}) obeys
    y_{t+1} = y_t - alpha*gamma/(1-beta) * sum_k dbar_{t,k}, y_0 = x_0."""
    rng = _rng(3)
    T, tau, m, d, lr, alpha, beta = 4, 3, 2, 9, 0.1, 1.0, 0.7
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=alpha, beta=beta)
    y = x_init.copy()
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
        x_t = o.x0.copy()
        o.outer_step(lr)
        y = y - alpha * lr / (1 - beta) * g[t].astype(np.float64).mean(axis=1).sum(axis=0)
        y_oracle = o.x0 + beta / (1 - beta) * (o.x0 - x_t)
        _close(y_oracle, y, rtol=1e-11, what=f"auxiliary sequence, t={t}")


def pin_u_closed_form_and_lr_invariance(make):
    """Appendix D.3.3 (unrolled momentum): u_T = sum_s beta^{T-1-s} sum_k
    dbar_{s,k}.  Section 2: dividing by gamma_t makes u independent of the
    fast learning rate, so the same u results under any schedule gamma_t."""
    rng = _rng(4)
    T, tau, m, d, beta = 5, 3, 4, 13, 0.65
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    want = np.zeros(d)
    for s in range(T):
        want += beta ** (T - 1 - s) * g[s].astype(np.float64).mean(axis=1).sum(axis=0)
    for sched in (lambda t: 0.1, lambda t: 0.1 / (1 + t), lambda t: 0.02 * 3 ** t):
        o = make(x_init, m=m, tau=tau, alpha=0.9, beta=beta)
        o.run(lambda t, k: g[t, k], sched, T)
        # (x0 - xbar)/gamma loses digits to cancellation when gamma is small
        _close(o.u, want, rtol=1e-9, atol=1e-9, what="u closed form")


def pin_local_sgd_reduction(make):
    """Section 2: alpha = 1, beta = 0 gives Local SGD, i.e. the new outer
    iterate is the plain average of the replicas (here with the Nesterov base
    of the experiments)."""
    rng = _rng(5)
    T, tau, m, d, lr = 3, 4, 5, 10, 0.1
    g = _grads(rng, T, tau, m, d)
    o = make(rng.standard_normal(d), m=m, tau=tau, alpha=1.0, beta=0.0,
             momentum=0.9, weight_decay=1e-4)
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
        xbar = o.x.mean(axis=0)
        o.outer_step(lr)
        _close(o.x0, xbar, rtol=1e-13, atol=1e-14, what="Local SGD reduction")


def pin_lookahead_reduction(make):
    """Section 2: m = 1, beta = 0 is Lookahead:
    x_{t+1,0} = x_{t,0} + alpha*(x_{t,tau} - x_{t,0})."""
    rng = _rng(6)
    T, tau, d, lr, alpha = 3, 5, 8, 0.05, 0.5
    g = _grads(rng, T, tau, 1, d)
    for base in ("sgd_nesterov", "adam"):
        kw = dict(momentum=0.9) if base == "sgd_nesterov" else dict(beta2=0.98)
        o = make(rng.standard_normal(d), m=1, tau=tau, alpha=alpha, beta=0.0,
                 base=base, **kw)
        for t in range(T):
            x_t0 = o.x0.copy()
            for k in range(tau):
                o.local_step(g[t, k], lr)
            fast = o.x[0].copy()
            o.outer_step(lr)
            _close(o.x0, x_t0 + alpha * (fast - x_t0), rtol=1e-13, atol=1e-14,
                   what="Lookahead reduction")


def pin_replica_consensus(make):
    """Section 2: after lines 6-8 the iterate is identical on all workers."""
    rng = _rng(7)
    T, tau, m, d, lr = 2, 3, 4, 6, 0.1
    g = _grads(rng, T, tau, m, d)
    o = make(rng.standard_normal(d), m=m, tau=tau, alpha=0.7, beta=0.4, momentum=0.9)
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
        assert not np.array_equal(o.x[0], o.x[1])
        o.outer_step(lr)
        for i in range(m):
            assert np.array_equal(o.x[i], o.x0), "replicas differ after the outer step"


def pin_large_minibatch_momentum_sgd(make):
    """Section 2: base SGD, tau = 1, alpha = 1 is large-minibatch SGD with
    learning rate gamma and momentum beta -- checked against the library's
    heavy-ball SGD on the worker-mean gradient."""
    rng = _rng(8)
    T, m, d, lr, beta = 12, 4, 10, 0.05, 0.8
    g = _grads(rng, T, 1, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=1, alpha=1.0, beta=beta)
    p = torch.tensor(x_init, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=beta, dampening=0.0)
    for t in range(T):
        o.local_step(g[t, 0], lr)
        o.outer_step(lr)
        p.grad = torch.tensor(g[t, 0].astype(np.float64).mean(axis=0))
        opt.step()
        _close(o.x0, p.detach().numpy(), rtol=1e-11, atol=1e-12,
               what=f"momentum SGD reduction, t={t}")


# ------------------------------------------------- Table C.1, SGD (Nesterov)

def _torch_sgd_per_worker(x_init, g, lr, mu, wd, reset_every=None):
    """Library Nesterov SGD on one worker's gradient sequence g[step, d]."""
    p = torch.tensor(np.asarray(x_init, dtype=np.float64), requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True, weight_decay=wd)
    for s in range(g.shape[0]):
        if reset_every and s % reset_every == 0:
            opt.state.clear()
        p.grad = torch.tensor(g[s].astype(np.float64))
        opt.step()
    return p.detach().numpy()


def pin_nesterov_base_vs_library(make):
    """Section 2: m = 1, alpha = 1, beta = 0 leaves the bare base optimizer.
    Table C.1's SGD row is the library's Nesterov SGD (no dampening, coupled
    weight decay); under "reset" the library's momentum buffer is dropped
    every tau steps, under "maintain" it is kept."""
    rng = _rng(9)
    T, tau, d, lr, mu, wd = 3, 4, 12, 0.1, 0.9, 1e-2
    g = _grads(rng, T, tau, 1, d)
    x_init = rng.standard_normal(d)
    seq = g.reshape(T * tau, d)
    for policy in ("reset", "maintain"):
        o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, momentum=mu,
                 weight_decay=wd, policy=policy)
        o.run(lambda t, k: g[t, k], lr, T)
        want = _torch_sgd_per_worker(x_init, seq, lr, mu, wd,
                                     reset_every=tau if policy == "reset" else None)
        _close(o.x0, want, rtol=1e-11, atol=1e-12, what=f"Nesterov base ({policy})")


def pin_per_worker_replicas_vs_library(make):
    """Algorithm 1 lines 3-5: within an outer iteration every worker runs the
    base optimizer on ITS OWN gradients from the common start x_{t,0}."""
    rng = _rng(10)
    tau, m, d, lr, mu, wd = 5, 3, 9, 0.1, 0.9, 1e-3
    g = _grads(rng, 2, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=0.6, beta=0.5, momentum=mu, weight_decay=wd)
    for t in range(2):
        start = o.x0.copy()
        for k in range(tau):
            o.local_step(g[t, k], lr)
        for i in range(m):
            want = _torch_sgd_per_worker(start, g[t, :, i, :], lr, mu, wd)
            _close(o.x[i], want, rtol=1e-11, atol=1e-12, what=f"worker {i} replica")
        o.outer_step(lr)


def pin_nesterov_constant_gradient(make):
    """Table C.1 SGD row with a constant gradient c and h_0 = 0:
    h_k = c(1-mu^k)/(1-mu) and sum_{k<tau} d_k =
    c[tau + mu/(1-mu) * (tau - mu(1-mu^tau)/(1-mu))]."""
    tau, d, lr, mu = 7, 5, 0.1, 0.9
    c = np.linspace(-2, 2, d)
    x_init = np.linspace(1, 3, d)
    g = np.broadcast_to(c.astype(np.float32), (1, d))
    cf = g[0].astype(np.float64)
    o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, momentum=mu, policy="maintain")
    for k in range(tau):
        o.local_step(g, lr)
    sum_d = cf * (tau + mu / (1 - mu) * (tau - mu * (1 - mu ** tau) / (1 - mu)))
    _close(o.h[0], cf * (1 - mu ** tau) / (1 - mu), what="h closed form")
    _close(o.x[0], x_init - lr * sum_d, what="sum of Nesterov directions")
    o.outer_step(lr)
    for k in range(tau):
        o.local_step(g, lr)
    _close(o.h[0], cf * (1 - mu ** (2 * tau)) / (1 - mu), what="maintained h after 2 tau")


def pin_reset_restarts_momentum(make):
    """Appendix B.4 / Table C.1 caption: under "reset" h_{t,0} = 0, so with a
    constant gradient every outer iteration repeats the same displacement;
    under "maintain" the second one is larger."""
    tau, d, lr, mu = 4, 3, 0.1, 0.9
    g = np.ones((1, d), np.float32)
    disp = {}
    for policy in ("reset", "maintain"):
        o = make(np.zeros(d), m=1, tau=tau, alpha=1.0, beta=0.0, momentum=mu, policy=policy)
        steps = []
        for t in range(3):
            before = o.x0.copy()
            for k in range(tau):
                o.local_step(g, lr)
            o.outer_step(lr)
            steps.append(o.x0 - before)
        disp[policy] = steps
    _close(disp["reset"][1], disp["reset"][0], what="reset repeats")
    _close(disp["reset"][2], disp["reset"][0], what="reset repeats")
    _close(disp["maintain"][0], disp["reset"][0], what="first iteration equal")
    assert np.all(np.abs(disp["maintain"][1]) > 1.5 * np.abs(disp["reset"][1]))


def pin_weight_decay_geometric(make):
    """Coupled L2 decay with zero gradient and no momentum:
    x_k = (1 - gamma*wd)^k x_0; and wd = 0 leaves x unchanged."""
    tau, d, lr, wd = 9, 6, 0.1, 0.05
    x_init = np.linspace(-3, 3, d)
    g = np.zeros((1, d), np.float32)
    o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, weight_decay=wd)
    for k in range(tau):
        o.local_step(g, lr)
        _close(o.x[0], (1 - lr * wd) ** (k + 1) * x_init, what="geometric decay")
    o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, weight_decay=0.0)
    o.local_step(g, lr)
    assert np.array_equal(o.x[0], x_init)


# ------------------------------------------------------- Table C.1, Adam

def _torch_adam(x_init, g, lr, b1, b2, eps, reset_every=None):
    p = torch.tensor(np.asarray(x_init, dtype=np.float64), requires_grad=True)
    mk = lambda: torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps)  # noqa: E731
    opt = mk()
    for s in range(g.shape[0]):
        if reset_every and s % reset_every == 0:
            opt = mk()
        p.grad = torch.tensor(g[s].astype(np.float64))
        opt.step()
    return p.detach().numpy()


def pin_adam_base_vs_library(make):
    """Table C.1's Adam row (eps added after the root of the bias-corrected
    second moment) is algebraically the library's Adam; "maintain" keeps
    moments and step count across outer iterations, "reset" restarts them."""
    rng = _rng(11)
    T, tau, d, lr, b1, b2, eps = 3, 4, 10, 1e-2, 0.9, 0.98, 1e-8
    g = _grads(rng, T, tau, 1, d)
    x_init = rng.standard_normal(d)
    for policy in ("maintain", "reset"):
        o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, base="adam",
                 beta1=b1, beta2=b2, eps=eps, policy=policy)
        o.run(lambda t, k: g[t, k], lr, T)
        want = _torch_adam(x_init, g.reshape(T * tau, d), lr, b1, b2, eps,
                           reset_every=tau if policy == "reset" else None)
        _close(o.x0, want, rtol=1e-10, atol=1e-12, what=f"Adam base ({policy})")


def pin_adam_per_worker_vs_library(make):
    rng = _rng(12)
    tau, m, d, lr, b1, b2, eps = 6, 3, 7, 1e-2, 0.9, 0.98, 1e-8
    g = _grads(rng, 1, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.5, base="adam",
             beta1=b1, beta2=b2, eps=eps)
    for k in range(tau):
        o.local_step(g[0, k], lr)
    for i in range(m):
        _close(o.x[i], _torch_adam(x_init, g[0, :, i, :], lr, b1, b2, eps),
               rtol=1e-10, atol=1e-12, what=f"Adam worker {i}")


def pin_adam_constant_gradient(make):
    """With a constant gradient c the bias-corrected moments are exactly c and
    c^2 at every step, so x_k = x_0 - k*gamma*c/(|c| + eps) -- from step 1 on,
    which only holds if the bias-correction exponent counts the current
    update.  c = 0 gives a zero direction, not 0/0."""
    tau, d, lr, eps = 5, 6, 1e-2, 1e-3
    c = np.array([-2.0, -0.5, 0.0, 0.25, 1.0, 3.0])
    g = c.astype(np.float32)[None, :]
    x_init = np.linspace(-1, 1, d)
    o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, base="adam",
             beta1=0.9, beta2=0.98, eps=eps, policy="maintain")
    n = 0
    for t in range(2):
        for k in range(tau):
            o.local_step(g, lr)
            n += 1
            _close(o.x[0], x_init - n * lr * c / (np.abs(c) + eps), rtol=1e-11,
                   what=f"Adam constant gradient, step {n}")
        o.outer_step(lr)
    assert np.all(np.isfinite(o.x0))


# ------------------------------------------- Algorithm 1, lines 6-8 together

def pin_constant_gradient_slowmo(make):
    """Eq. (2)-(3) with plain SGD and constant per-worker gradients c_i (mean
    cbar): u_t = tau*cbar*(1-beta^t)/(1-beta) and
    x_{T,0} = x_{0,0} - alpha*gamma*tau*cbar*sum_{t=1..T}(1-beta^t)/(1-beta)."""
    T, tau, m, d, lr, alpha, beta = 6, 3, 4, 5, 0.1, 0.8, 0.6
    rng = _rng(13)
    c = rng.standard_normal((m, d)).astype(np.float32)
    cbar = c.astype(np.float64).mean(axis=0)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=alpha, beta=beta)
    acc = 0.0
    for t in range(1, T + 1):
        for k in range(tau):
            o.local_step(c, lr)
        o.outer_step(lr)
        geo = (1 - beta ** t) / (1 - beta)
        acc += geo
        _close(o.u, tau * cbar * geo, rtol=1e-10, atol=1e-12, what=f"u_t closed form t={t}")
        _close(o.x0, x_init - alpha * lr * tau * cbar * acc, rtol=1e-11, atol=1e-12,
               what=f"x_T closed form t={t}")


def pin_mean_is_symmetric_and_m1_identity(make):
    """Line 6 is a plain mean: permuting the workers changes nothing beyond
    rounding; with m = 1 (alpha = 1, beta = 0) the outer step is the identity."""
    rng = _rng(14)
    tau, m, d, lr = 3, 5, 8, 0.1
    g = _grads(rng, 1, tau, m, d)
    x_init = rng.standard_normal(d)
    res = []
    for perm in (np.arange(m), np.array([3, 0, 4, 1, 2])):
        o = make(x_init, m=m, tau=tau, alpha=0.9, beta=0.3, momentum=0.9)
        for k in range(tau):
            o.local_step(g[0, k][perm], lr)
        o.outer_step(lr)
        res.append(o.x0.copy())
    _close(res[0], res[1], rtol=1e-14, atol=1e-15, what="worker permutation")
    o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, momentum=0.9)
    for k in range(tau):
        o.local_step(g[0, k][:1], lr)
    fast = o.x[0].copy()
    o.outer_step(lr)
    _close(o.x0, fast, rtol=1e-14, atol=1e-15, what="m=1 identity")


def pin_outer_uses_lr_of_outer_call(make):
    """Eq. (2)-(3): gamma_t appears as 1/gamma_t in u and as alpha*gamma_t in
    the iterate; with beta = 0 they cancel, so x_{t+1,0} must not depend on the
    value handed to the outer step, while u scales with its inverse."""
    rng = _rng(15)
    tau, m, d = 3, 2, 6
    g = _grads(rng, 1, tau, m, d)
    x_init = rng.standard_normal(d)
    outs = []
    for lr_outer in (0.1, 0.4):
        o = make(x_init, m=m, tau=tau, alpha=0.5, beta=0.0)
        for k in range(tau):
            o.local_step(g[0, k], 0.1)
        o.outer_step(lr_outer)
        outs.append((o.x0.copy(), o.u.copy()))
    _close(outs[0][0], outs[1][0], rtol=1e-12, what="x0 independent of outer lr at beta=0")
    _close(outs[0][1], 4.0 * outs[1][1], rtol=1e-12, what="u scales with 1/gamma")


# --------------------------- buffer strategy "average" (Appendix B.4, Alg. C.4)

def pin_average_policy_degenerate_cases(make):
    """Averaging over one worker, or over workers that all see the same
    gradients, changes nothing: the run equals the "maintain" run."""
    rng = _rng(20)
    T, tau, d, lr = 3, 3, 7, 0.05
    x_init = rng.standard_normal(d)
    for base, kw in (("sgd_nesterov", dict(momentum=0.9, weight_decay=1e-3)),
                     ("adam", dict(beta2=0.98))):
        g1 = _grads(rng, T, tau, 1, d)
        same = np.repeat(g1, 3, axis=2)
        for m, g in ((1, g1), (3, same)):
            res = []
            for policy in ("maintain", "average"):
                o = make(x_init, m=m, tau=tau, alpha=0.8, beta=0.5, base=base, policy=policy, **kw)
                o.run(lambda t, k: g[t, k], lr, T)
                res.append((o.x0.copy(), o.h.copy()))
            _close(res[0][0], res[1][0], rtol=1e-13, what=f"average == maintain ({base}, m={m})")
            _close(res[0][1], res[1][1], rtol=1e-13, what="buffers")


def pin_average_policy_mean_iterate_is_single_worker_nesterov(make):
    """The Nesterov base is linear in (x, h, g), and averaging parameters and
    buffers leaves their worker-means unchanged; so with alpha = 1, beta = 0
    the outer iterate follows the library's Nesterov SGD driven by the
    worker-mean gradient, momentum running across the outer iterations
    (Algorithm C.4 with its two AllReduces)."""
    rng = _rng(21)
    T, tau, m, d, lr, mu, wd = 4, 3, 4, 9, 0.05, 0.9, 1e-2
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.0, momentum=mu, weight_decay=wd,
             policy="average")
    p = torch.tensor(x_init, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True, weight_decay=wd)
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
            p.grad = torch.tensor(g[t, k].astype(np.float64).mean(axis=0))
            opt.step()
        o.outer_step(lr)
        _close(o.x0, p.detach().numpy(), rtol=1e-11, atol=1e-12, what=f"mean iterate, t={t}")
    hbar = opt.state[p]["momentum_buffer"].numpy()
    _close(o.h.mean(axis=0), hbar, rtol=1e-11, atol=1e-12, what="mean momentum buffer")


def pin_average_policy_makes_buffers_common(make):
    """At the start of outer iteration t >= 1 every worker holds the same
    buffers, the mean of the previous ones: after one more step,
    h_i - g_i = mu * mean(h_prev) for all i (SGD, wd = 0), and for Adam
    h_i - (1-b1) g_i = b1 * mean(h_prev), v_i - (1-b2) g_i^2 = b2 * mean(v_prev)."""
    rng = _rng(22)
    tau, m, d, lr, mu, b1, b2 = 3, 4, 6, 0.05, 0.9, 0.9, 0.98
    g = _grads(rng, 2, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.3, momentum=mu, policy="average")
    for k in range(tau):
        o.local_step(g[0, k], lr)
    h_prev = o.h.mean(axis=0)
    assert np.abs(o.h - h_prev).max() > 1e-3
    o.outer_step(lr)
    o.local_step(g[1, 0], lr)
    for i in range(m):
        _close(o.h[i] - g[1, 0, i].astype(np.float64), mu * h_prev, rtol=1e-11, atol=1e-12,
               what=f"SGD buffer of worker {i}")
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.3, base="adam", beta1=b1, beta2=b2,
             policy="average")
    for k in range(tau):
        o.local_step(g[0, k], lr)
    h_prev, v_prev, l_prev = o.h.mean(axis=0), o.v.mean(axis=0), o.l
    o.outer_step(lr)
    o.local_step(g[1, 0], lr)
    assert o.l == l_prev + 1            # the step count runs on
    gi = g[1, 0].astype(np.float64)
    for i in range(m):
        _close(o.h[i] - (1 - b1) * gi[i], b1 * h_prev, rtol=1e-10, atol=1e-12, what="Adam h")
        _close(o.v[i] - (1 - b2) * gi[i] ** 2, b2 * v_prev, rtol=1e-10, atol=1e-12, what="Adam v")


# ------------------------------------ Section 6: SlowMo without the exact average

def pin_noaverage_is_m_independent_single_worker_runs(make):
    """Section 6 (SlowMo-noaverage): without line 6 each worker applies lines
    7-8 to its own replica, so the m workers never interact: the run equals m
    separate single-worker runs on each worker's gradients."""
    rng = _rng(30)
    T, tau, m, d, lr = 3, 4, 3, 8, 0.05
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    for base, kw in (("sgd_nesterov", dict(momentum=0.9, weight_decay=1e-3, policy="reset")),
                     ("adam", dict(beta2=0.98, policy="maintain"))):
        o = make(x_init, m=m, tau=tau, alpha=0.9, beta=0.6, base=base, exact_average=False, **kw)
        o.run(lambda t, k: g[t, k], lr, T)
        assert o.x0.shape == (m, d) and o.u.shape == (m, d)
        for i in range(m):
            s = make(x_init, m=1, tau=tau, alpha=0.9, beta=0.6, base=base, **kw)
            s.run(lambda t, k: g[t, k, i:i + 1], lr, T)
            _close(o.x0[i], s.x0, rtol=1e-13, what=f"x0 of worker {i} ({base})")
            _close(o.u[i], s.u, rtol=1e-13, what=f"u of worker {i}")
            _close(o.x[i], s.x[0], rtol=1e-13, what=f"replica of worker {i}")
        assert np.abs(o.x0[0] - o.x0[1]).max() > 1e-3      # no consensus without line 6


def pin_noaverage_with_common_gradients_equals_slowmo(make):
    """If all workers see the same gradients their replicas coincide, the
    average changes nothing, and both variants give the same iterates."""
    rng = _rng(31)
    T, tau, m, d, lr = 3, 3, 4, 6, 0.05
    g = np.repeat(_grads(rng, T, tau, 1, d), m, axis=2)
    x_init = rng.standard_normal(d)
    a = make(x_init, m=m, tau=tau, alpha=0.8, beta=0.5, momentum=0.9)
    b = make(x_init, m=m, tau=tau, alpha=0.8, beta=0.5, momentum=0.9, exact_average=False)
    a.run(lambda t, k: g[t, k], lr, T)
    b.run(lambda t, k: g[t, k], lr, T)
    for i in range(m):
        _close(b.x0[i], a.x0, rtol=1e-13, what="x0")
        _close(b.u[i], a.u, rtol=1e-13, what="u")


# ------------------------------ Appendix C.1: the mixing step of gradient push

def _mixing_matrix(in_peer):
    m = len(in_peer)
    P = np.zeros((m, m))
    for j in range(m):
        receivers = [i for i in range(m) if i != j and in_peer[i] == j]
        for i in [j] + receivers:
            P[i, j] = 1.0 / (1 + len(receivers))
    return P


def pin_mixing_is_the_matrix_product(make):
    """Appendix C.1, matrix form: X_{k+1} = X P^T with a column-stochastic P;
    checked against a library matrix product for a permutation (every node
    one sender, one receiver), a star-like map and a map with idle nodes."""
    rng = _rng(40)
    m, d = 6, 11
    for in_peer in ([5, 0, 1, 2, 3, 4], [2, 0, 3, 1, 5, 4], [0, 0, 0, 1, 1, 5], [0, 1, 2, 3, 4, 5]):
        o = make(rng.standard_normal(d), m=m, tau=3, alpha=1.0, beta=0.5)
        o.x[...] = rng.standard_normal((m, d))
        o.w[...] = rng.uniform(0.5, 1.5, m)
        X, w = o.x.copy(), o.w.copy()
        P = _mixing_matrix(in_peer)
        _close(P.sum(axis=0), np.ones(m), what="P is column-stochastic")
        o.mix_step(in_peer)
        _close(o.x, P @ X, rtol=1e-13, what=f"mixing {in_peer}")
        _close(o.w, P @ w, rtol=1e-13, what="push-sum weights")
        _close(o.x.sum(axis=0), X.sum(axis=0), rtol=1e-12, atol=1e-13, what="mass is conserved")


def pin_exponential_graph_averages_exactly_in_log2_m_steps(make):
    """On m = 2^p nodes the one-peer exponential graph (hops 1, 2, ..., 2^(p-1))
    is a butterfly: after p mixing steps every node holds the exact average,
    the push-sum weights stay 1 and z = x."""
    rng = _rng(41)
    for m in (2, 4, 8, 16):
        d = 7
        o = make(rng.standard_normal(d), m=m, tau=3, alpha=1.0, beta=0.5)
        O = type(o)
        o.x[...] = rng.standard_normal((m, d))
        mean = o.x.mean(axis=0)
        p = int(np.log2(m))
        seen = set()
        for step in range(p):
            peers = O.exponential_graph_in_peers(m, step)
            assert sorted(peers.tolist()) == list(range(m))      # a permutation
            seen.add(int((0 - peers[0]) % m))
            o.mix_step(peers)
        assert seen == {1 << k for k in range(p)}
        for i in range(m):
            _close(o.x[i], mean, rtol=1e-13, atol=1e-14, what=f"consensus on {m} nodes")
        _close(o.w, np.ones(m), what="weights")
        _close(o.debiased(), o.x, what="z = x")
    peers = O.exponential_graph_in_peers(6, 2)          # m = 6: hops 1, 2, 4
    assert peers.tolist() == [(i - 4) % 6 for i in range(6)]
    assert O.exponential_graph_in_peers(6, 3).tolist() == [(i - 1) % 6 for i in range(6)]


def pin_mixing_debiased_iterates_reach_consensus(make):
    """Push-sum: with column- but not row-stochastic mixing matrices whose
    union over time is strongly connected, x_i / w_i converges to the average
    of the initial values although x_i itself does not (the reason the
    algorithm keeps w)."""
    rng = _rng(42)
    m, d = 5, 4
    o = make(rng.standard_normal(d), m=m, tau=3, alpha=1.0, beta=0.5)
    o.x[...] = rng.standard_normal((m, d))
    mean = o.x.mean(axis=0)
    for _ in range(300):
        o.mix_step([4, 0, 0, 2, 3])      # node 0 has two receivers, node 1 none
        o.mix_step([1, 2, 3, 4, 0])      # a ring in the other direction
    assert abs(o.w.sum() - m) < 1e-12 and np.abs(o.w - 1).max() > 1e-2
    assert np.abs(o.x - mean).max() > 1e-2
    for i in range(m):
        _close(o.debiased()[i], mean, rtol=1e-9, atol=1e-10, what="push-sum consensus")


# Appendix C.1: "each node cycles through the peers 2^0, 2^1, ..., 2^floor(log2(m-1))
# hops away".  The hop lists are written out by hand, one period each.
EXPGRAPH_HOPS = {2: [1], 3: [1, 2], 4: [1, 2], 5: [1, 2, 4], 6: [1, 2, 4], 8: [1, 2, 4],
                 9: [1, 2, 4, 8], 16: [1, 2, 4, 8], 17: [1, 2, 4, 8, 16], 19: [1, 2, 4, 8, 16],
                 32: [1, 2, 4, 8, 16], 33: [1, 2, 4, 8, 16, 32]}


def pin_exponential_graph_hop_list_over_two_periods(make):
    """Appendix C.1: the hops are 2^0 .. 2^floor(log2(m-1)) in turn, then the
    list starts over; worker i receives from the worker `hop` ranks below it.
    No hop is a multiple of m (nobody "receives from itself"), also for
    m = 2^p, where a period of floor(log2 m) + 1 would add the hop m."""
    O = type(make(np.zeros(1), m=1, tau=1, alpha=1.0, beta=0.0))
    for m, hops in EXPGRAPH_HOPS.items():
        for step in range(2 * len(hops) + 1):
            hop = hops[step % len(hops)]
            peers = np.asarray(O.exponential_graph_in_peers(m, step)).tolist()
            assert peers == [(i - hop) % m for i in range(m)], (m, step, peers)
            assert all(p != i for i, p in enumerate(peers)), (m, step)


def pin_exact_average_after_push_sum_restores_the_unbiased_state(make):
    """Algorithm C.1 + Algorithm 1 line 6.  Mixing with a column-stochastic P
    that is not doubly stochastic moves mass between the workers but conserves
    its total (and the total weight m), so with the plain SGD base the sum of
    the replicas after tau steps is m*x_{t,0} - gamma*sum_i sum_k g_i,k
    whatever the maps were: the exact average is x_{t,0} minus gamma times the
    mean gradient sum, and with alpha = 1, beta = 0 it is the new iterate.
    After line 6 every worker holds that one point, which is unbiased: its
    de-biased value z = x / w must be the point itself, i.e. w = 1 again, and
    the next outer iteration starts like the first one."""
    rng = _rng(43)
    T, tau, m, d, lr = 3, 4, 5, 9, 0.05
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    maps = ([0, 0, 0, 2, 3], [1, 2, 3, 4, 0], [4, 4, 1, 1, 2], [0, 1, 0, 0, 0])   # no permutations but one
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.0)
    x_t0 = x_init.copy()
    for t in range(T):
        for k in range(tau):
            o.local_step(g[t, k], lr)
            o.mix_step(maps[(t * tau + k) % len(maps)])
        assert abs(o.w.sum() - m) < 1e-12, "total push-sum weight"
        assert np.abs(o.w - 1).max() > 1e-2, "the maps must unbalance the weights"
        assert np.abs(o.debiased() - o.x).max() > 1e-3
        want = x_t0 - lr / m * g[t].astype(np.float64).sum(axis=(0, 1))
        o.outer_step(lr)
        _close(o.x0, want, rtol=1e-12, atol=1e-13, what=f"average of the mass, t={t}")
        for i in range(m):
            assert np.array_equal(o.x[i], o.x0)
            _close(o.debiased()[i], o.x0, rtol=1e-15, atol=0.0,
                   what="z = x after the exact average (w back to 1)")
        x_t0 = want


def pin_no_average_keeps_the_push_sum_weights(make):
    """Section 6 with gossip as the only exchange: without line 6 nothing but
    the mixing steps touches the push-sum weights.  With alpha = 1, beta = 0
    lines 7-8 return each worker's own replica, so across the outer step the
    replicas, the weights and hence the de-biased points z = x / w stay what
    they were, and the total weight stays m."""
    rng = _rng(44)
    tau, m, d, lr = 3, 4, 6, 0.05
    g = _grads(rng, 2, tau, m, d)
    o = make(rng.standard_normal(d), m=m, tau=tau, alpha=1.0, beta=0.0, exact_average=False)
    for t in range(2):
        for k in range(tau):
            o.local_step(g[t, k], lr)
            o.mix_step([[0, 0, 1, 1], [3, 0, 0, 2]][k % 2])
        x, w, z = o.x.copy(), o.w.copy(), o.debiased().copy()
        assert np.abs(w - 1).max() > 1e-2 and abs(w.sum() - m) < 1e-12
        o.outer_step(lr)
        _close(o.x, x, rtol=1e-13, atol=1e-14, what="replicas across the outer step")
        _close(o.debiased(), z, rtol=1e-13, atol=1e-14, what="de-biased points across the outer step")
        assert abs(o.w.sum() - m) < 1e-12


def pin_weight_decay_under_push_sum_acts_on_the_numerator(make):
    """Reading: with gossip between the steps the coupled L2 term is wd * x
    with x the push-sum numerator (the replica itself), not wd * x / w.  The
    base step is then linear in (x, h, g) and mixing conserves sums, so the
    worker-mean of the replicas follows the library's Nesterov SGD with weight
    decay on the worker-mean gradient for ANY column-stochastic maps -- the
    mass bookkeeping push-sum rests on.  (With wd * x / w the mean would pick
    up sum_i x_i / w_i instead of sum_i x_i and this fails.)"""
    rng = _rng(45)
    tau, m, d, lr, mu, wd = 6, 4, 7, 0.05, 0.9, 0.05
    g = _grads(rng, 1, tau, m, d)
    x_init = rng.standard_normal(d)
    o = make(x_init, m=m, tau=tau, alpha=1.0, beta=0.0, momentum=mu, weight_decay=wd,
             policy="maintain")
    p = torch.tensor(x_init, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True, weight_decay=wd)
    for k in range(tau):
        o.local_step(g[0, k], lr)
        o.mix_step([[0, 0, 1, 1], [3, 0, 0, 2], [1, 2, 3, 0]][k % 3])
        p.grad = torch.tensor(g[0, k].astype(np.float64).mean(axis=0))
        opt.step()
    assert np.abs(o.w - 1).max() > 1e-2
    # only x is mixed, h is not: mean(x) sees the buffers through mean(d_i)
    # alone, which is what one worker driven by the mean gradient computes
    _close(o.x.mean(axis=0), p.detach().numpy(), rtol=1e-11, atol=1e-12,
           what="mean replica under push-sum with weight decay")


# ------------------------------------------- per-tensor hyper-parameters

def pin_step_decay_schedule_of_the_image_experiments(make):
    """Section 4: linear warm-up over the first 5 epochs, then a factor 10 down
    at epochs 30, 60, 80 (ImageNet, 90 epochs) or 100, 150, 175 (CIFAR-10, 200
    epochs).  Values written out by hand for 100 steps per epoch."""
    O = type(make(np.zeros(1), m=1, tau=1, alpha=1.0, beta=0.0))
    f = O.lr_warmup_step_decay
    S, base, start = 100, 3.2, 0.1                      # 0.1 x 32 workers (Appendix A.2)
    imagenet = [30 * S, 60 * S, 80 * S]
    expect = {0: 0.1, 1: 0.1 + 3.1 / 500, 250: 1.65, 499: 3.2 - 3.1 / 500, 500: 3.2, 501: 3.2,
              2999: 3.2, 3000: 0.32, 3001: 0.32, 5999: 0.32, 6000: 0.032, 7999: 0.032,
              8000: 0.0032, 8999: 0.0032}
    for step, lr in expect.items():
        assert abs(f(base, start, 5 * S, imagenet, 0.1, step) - lr) <= 1e-12 * max(1.0, lr), step
    cifar = [100 * S, 150 * S, 175 * S]
    for step, lr in {9999: 3.2, 10000: 0.32, 15000: 0.032, 17499: 0.032, 17500: 0.0032,
                     19999: 0.0032}.items():
        assert abs(f(base, start, 5 * S, cifar, 0.1, step) - lr) <= 1e-12, step
    # no warm-up, no milestone: constant
    assert f(0.05, 0.0, 0, [], 0.1, 0) == 0.05 and f(0.05, 0.0, 0, [], 0.1, 10 ** 6) == 0.05
    # the warm-up is a straight line: equal increments
    inc = [f(base, start, 500, imagenet, 0.1, s + 1) - f(base, start, 500, imagenet, 0.1, s)
           for s in range(499)]
    assert max(inc) - min(inc) < 1e-12 and abs(inc[0] - 3.1 / 500) < 1e-12


def pin_inverse_square_root_schedule_of_the_translation_experiment(make):
    """Appendix A.3: the rate rises linearly for 4000 steps to 1e-3 and then
    decays in proportion to 1 / sqrt(step): four times the steps, half the rate."""
    O = type(make(np.zeros(1), m=1, tau=1, alpha=1.0, beta=0.0))
    f = O.lr_warmup_inverse_sqrt
    assert f(1e-3, 0.0, 4000, 0) == 0.0
    assert abs(f(1e-3, 0.0, 4000, 1000) - 0.25e-3) < 1e-18
    assert abs(f(1e-3, 0.0, 4000, 3999) - 1e-3 * 3999 / 4000) < 1e-18
    assert f(1e-3, 0.0, 4000, 4000) == 1e-3
    assert abs(f(1e-3, 0.0, 4000, 16000) - 0.5e-3) < 1e-18
    assert abs(f(1e-3, 0.0, 4000, 64000) - 0.25e-3) < 1e-18
    assert abs(f(1e-3, 0.0, 4000, 4001) - 1e-3 * (4000 / 4001) ** 0.5) < 1e-18
    # a warm-up that starts above zero
    assert f(1e-3, 1e-7, 4000, 0) == 1e-7 and abs(f(1e-3, 1e-7, 4000, 2000) - (1e-7 + (1e-3 - 1e-7) / 2)) < 1e-18
    # after the warm-up, rate x sqrt(step) is constant
    c = [f(7e-4, 0.0, 100, s) * s ** 0.5 for s in (100, 101, 1000, 12345)]
    assert max(c) - min(c) < 1e-15


def pin_parameter_groups_vs_library(make):
    """Per-tensor weight decay and learning-rate scale are the library
    optimizers' parameter groups: m = 1, alpha = 1, beta = 0 leaves the bare
    base optimizer, compared with torch.optim.SGD / Adam with one group per
    tensor."""
    rng = _rng(50)
    T, tau, lr, mu = 2, 4, 0.05, 0.9
    sizes = [5, 1, 7, 3]
    wds = [1e-2, 0.0, 5e-3, 0.0]
    scales = [1.0, 0.5, 2.0, 0.25]
    d = sum(sizes)
    g = _grads(rng, T, tau, 1, d)
    x_init = rng.standard_normal(d)
    bounds = np.cumsum([0] + sizes)
    for base in ("sgd_nesterov", "adam"):
        kw = dict(momentum=mu) if base == "sgd_nesterov" else dict(beta2=0.98)
        o = make(x_init, m=1, tau=tau, alpha=1.0, beta=0.0, base=base, policy="maintain",
                 tensor_sizes=sizes, tensor_weight_decay=wds, tensor_lr_scale=scales, **kw)
        ps = [torch.tensor(x_init[a:b], dtype=torch.float64, requires_grad=True)
              for a, b in zip(bounds[:-1], bounds[1:])]
        # the oracle rounds lr * scale to fp32, as the kernels receive it
        groups = [dict(params=[p], lr=float(np.float32(np.float32(lr) * np.float32(s))),
                       weight_decay=w) for p, s, w in zip(ps, scales, wds)]
        opt = torch.optim.SGD(groups, lr=lr, momentum=mu, nesterov=True) \
            if base == "sgd_nesterov" else torch.optim.Adam(groups, lr=lr, betas=(0.9, 0.98))
        for t in range(T):
            for k in range(tau):
                o.local_step(g[t, k], lr)
                for p, a, b in zip(ps, bounds[:-1], bounds[1:]):
                    p.grad = torch.tensor(g[t, k, 0, a:b].astype(np.float64))
                opt.step()
            o.outer_step(lr)
        want = np.concatenate([p.detach().numpy() for p in ps])
        _close(o.x0, want, rtol=1e-10, atol=1e-12, what=f"parameter groups ({base})")


def pin_per_tensor_learning_rate_keeps_u_in_gradient_units(make):
    """Section 2: dividing by gamma_t keeps u free of the fast learning rate.
    With per-tensor gamma_t (plain SGD base) u must therefore not depend on
    the scales at all, and each tensor's iterate moves as if it were alone."""
    rng = _rng(51)
    T, tau, m, lr = 3, 3, 3, float(np.float32(0.1))    # scaled rates are rounded to fp32
    sizes = [4, 6]
    d = sum(sizes)
    g = _grads(rng, T, tau, m, d)
    x_init = rng.standard_normal(d)
    ref = make(x_init, m=m, tau=tau, alpha=0.9, beta=0.6)
    ref.run(lambda t, k: g[t, k], lr, T)
    o = make(x_init, m=m, tau=tau, alpha=0.9, beta=0.6, tensor_sizes=sizes,
             tensor_lr_scale=[1.0, 0.5])
    o.run(lambda t, k: g[t, k], lr, T)
    _close(o.u, ref.u, rtol=1e-10, atol=1e-11, what="u does not see the scales")
    _close(o.x0[:4], ref.x0[:4], rtol=1e-12, what="tensor with scale 1")
    half = make(x_init, m=m, tau=tau, alpha=0.9, beta=0.6)
    half.run(lambda t, k: g[t, k], 0.5 * lr, T)
    _close(o.x0[4:], half.x0[4:], rtol=1e-12, what="tensor with scale 1/2")


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
