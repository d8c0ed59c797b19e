"""HIP path vs CPU oracle on the same seeded inputs, through the C ABI."""
import dataclasses
import os
import gc

import numpy as np
import pytest

from slowmo_inputs import generator as G
from slowmo_inputs import workloads as W

import parity_utils as PU

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _free_gpu_memory():
    yield
    import torch
    gc.collect()
    torch.cuda.empty_cache()


def _problem(w, **kw):
    from slowmo_inputs.gpu_problem import GpuProblem
    return GpuProblem(w, "cuda:0", **kw)


def _tile_edges(w, count=256):
    """Global element indices where local-step / outer-step tiles begin (a
    seeded sample of them).  Tiles are fixed-size pieces of a tensor; the size
    is read off the library's own plan."""
    import paper_1910_00643_amd as P
    t_local = max(r[3] for r in P.slowmo_plan_local(1, [100_000]))
    t_outer = max(r[3] for r in P.slowmo_plan_outer(1, [100_000]))
    rng = np.random.default_rng(w.seed)
    starts, numel = w.tensor_starts, np.asarray(w.numel, dtype=np.int64)
    edges = set()
    big = np.nonzero(numel > 0)[0]
    for j in rng.choice(big, size=count, p=numel[big] / numel[big].sum()):
        for t in (t_local, t_outer):
            k = int(rng.integers(0, -(-numel[j] // t)))
            edges.add(int(starts[j] + k * t))
    return sorted(edges)


# ---- input generator: device == host, bit for bit -------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_device_generator_matches_host(dtype):
    import torch
    from slowmo_inputs import device
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    n, first, seed, step, scale, m = 70_001, 2 ** 33 + 12345, 987654321, 17, 0.1, 3
    out = torch.zeros((m, n), dtype=td, device="cuda:0")
    device.fill(out, first, seed, 2, step, scale, n_workers=m)
    idx = first + np.arange(n, dtype=np.int64)
    for wk in range(m):
        want = G.gradient(seed, 2 + wk, step, idx, scale, bf16=(dtype == "bf16"))
        got = out[wk].to(torch.float32).cpu().numpy()
        assert np.array_equal(got, want), f"worker {wk}"


# ---- element-by-element parity at small sizes --------------------------------------
def test_tiny_config_every_element():
    """The tiny configuration in full: m=4, d=65536, tau=12, 10 outer rounds."""
    w = W.tiny()
    prob = _problem(w)
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    worst = PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=True)
    print("tiny worst errors", worst)
    # second route to the expected values: the stored fp64 oracle output
    from test_oracle_pins import _read_golden
    rows, _ = _read_golden()
    final = PU.gpu_state(w, prob, opt, np.array([r[0] for r in rows], dtype=np.int64))
    PU.assert_params_close(final["x0"], [r[1] for r in rows], "x0 vs stored oracle values")
    opt.close()


@pytest.mark.parametrize("base,grad_dtype,policy,param_layout,grad_layout", [
    ("sgd_nesterov", "f32", "reset", "separate", "separate"),
    ("sgd_nesterov", "f32", "maintain", "flat", "flat"),        # unaligned pointers
    ("sgd_nesterov", "bf16", "reset", "separate", "flat"),
    ("adam", "bf16", "maintain", "separate", "separate"),
    ("adam", "f32", "reset", "flat", "separate"),
    ("adam", "bf16", "maintain", "flat", "flat"),
    ("sgd_nesterov", "f32", "average", "separate", "separate"),   # Alg. C.4-style buffers
    ("sgd_nesterov", "bf16", "average", "flat", "flat"),
    ("adam", "bf16", "average", "separate", "padded"),
    ("adam", "f32", "average", "flat", "flat"),
    ("sgd_nesterov", "f32", "reset", "separate", "padded"),
    ("adam", "bf16", "maintain", "separate", "padded"),
])
def test_ragged_tensor_list_every_element(base, grad_dtype, policy, param_layout, grad_layout):
    """26 tensors with lengths 0, 1, 2, 3, 5, ... 131077: ragged tails, empty
    tensors, runs that share a tile and tensors that span several tiles, with
    aligned (separate allocations) and unaligned (packed) pointers."""
    w = W.ragged_mini(base=base, grad_dtype=grad_dtype, policy=policy)
    prob = _problem(w, ring=3, param_layout=param_layout, grad_layout=grad_layout)
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    worst = PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"))
    print(base, grad_dtype, policy, "worst errors", worst)
    opt.close()


@pytest.mark.parametrize("base,grad_dtype,policy,param_layout", [
    ("sgd_nesterov", "f32", "reset", "separate"),
    ("sgd_nesterov", "bf16", "maintain", "flat"),
    ("adam", "bf16", "maintain", "separate"),
])
def test_noaverage_variant_every_element(base, grad_dtype, policy, param_layout):
    """Section 6: no exact average; per-worker x0 and u."""
    w = dataclasses.replace(W.ragged_mini(base=base, grad_dtype=grad_dtype, policy=policy),
                            exact_average=False)
    prob = _problem(w, ring=2, param_layout=param_layout, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"))
    opt.close()


@pytest.mark.parametrize("fused_mix", [False, True])
@pytest.mark.parametrize("m,base,param_layout", [(4, "sgd_nesterov", "separate"),
                                                 (8, "sgd_nesterov", "flat"),
                                                 (6, "sgd_nesterov", "separate"),
                                                 (19, "adam", "separate"), (1, "sgd_nesterov", "flat")])
def test_gradient_push_mixing_every_element(m, base, param_layout, fused_mix):
    """SGP as base optimizer (Algorithm C.1): every local step is followed by
    a gossip step on the one-peer exponential graph; m = 6 and 19 give
    permutations with several cycles, m = 1 an idle step.  With fused_mix the
    pair is one call (one kernel for the 16-byte aligned "separate" layout,
    the two kernels for "flat")."""
    w = dataclasses.replace(W.ragged_mini(base=base, m=m, policy="maintain"), mix="expgraph",
                            tau=7, rounds=2)
    prob = _problem(w, ring=2, param_layout=param_layout, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"),
                   fused_mix=fused_mix)
    opt.close()


@pytest.mark.parametrize("base,grad_dtype,policy,mix", [
    ("sgd_nesterov", "f32", "reset", "random"), ("adam", "bf16", "maintain", "random"),
    ("adam", "f32", "reset", "expgraph"), ("sgd_nesterov", "bf16", "average", "random")])
def test_fused_local_and_mixing_step_equals_the_two_calls_bitwise(base, grad_dtype, policy, mix):
    """slowmo_local_mix_step against slowmo_local_step + slowmo_mix_step on
    the same inputs: replicas, buffers, x0, u and push-sum weights bit for bit
    (also for Adam, whose arithmetic is the same code in both kernels)."""
    w = dataclasses.replace(W.ragged_mini(base=base, grad_dtype=grad_dtype, m=11, policy=policy),
                            mix=mix, tau=3, rounds=2)
    idx = np.arange(w.d, dtype=np.int64)
    states = []
    for fused in (False, True):
        prob = _problem(w, ring=2, param_layout="separate", grad_layout="separate")
        opt = PU.make_gpu(w, prob)
        snap = PU.run_gpu(w, prob, opt, w.rounds, idx, fused_mix=fused)
        final = PU.gpu_state(w, prob, opt, idx)
        states.append((snap, final, opt.pushsum_weights()))
        opt.close()
    (s0, f0, w0), (s1, f1, w1) = states
    assert w0 == w1
    if policy == "reset":       # h, v after the last local step are dead and need not be stored
        f0.pop("h"), f0.pop("v")
    for a, b in ((s0, s1), (f0, f1)):
        for key in a:
            if a[key] is not None:
                assert np.array_equal(a[key], b[key], equal_nan=False), key


def test_mixing_accepts_any_map_and_rejects_bad_indices():
    import paper_1910_00643_amd as P
    w = dataclasses.replace(W.ragged_mini(m=5), tau=1, rounds=1)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    o = PU.make_oracle(w, idx, "f32")
    prob.fill_grads(0, 0)
    opt.local_step(prob.grads[0], w.lr)
    o.local_step(PU.oracle_grads(w, idx, 0), w.f32("lr"))
    for peers in ([1, 0, 2, 4, 3], [2, 3, 4, 0, 1], [0, 1, 2, 3, 4], [4, 0, 1, 2, 3],
                  [0, 0, 1, 2, 3], [0, 0, 0, 0, 0], [1, 0, 0, 4, 4], [1, 2, 0, 0, 3],
                  [1, 0, 3, 4, 2]):      # the last: a permutation met with unequal weights
        opt.mix_step(peers)
        o.mix_step(peers)
        got = np.stack([prob.gather(prob.params[i], idx) for i in range(w.m)])
        assert np.array_equal(got, o.x), peers
        assert np.array_equal(np.asarray(opt.pushsum_weights(), np.float32), o.w), peers
    for bad in ([1, 2, 3, 4, 5], [-1, 0, 1, 2, 3]):
        with pytest.raises(P.SlowMoError) as e:
            opt.mix_step(bad)
        assert e.value.status == P.binding.SLOWMO_ERR_ARG
    opt.close()


@pytest.mark.parametrize("m,base,param_layout,exact", [
    (5, "sgd_nesterov", "separate", True), (8, "sgd_nesterov", "flat", True),
    (19, "adam", "separate", True), (33, "sgd_nesterov", "separate", True),
    (6, "sgd_nesterov", "flat", False), (2, "sgd_nesterov", "separate", True)])
def test_push_sum_with_any_in_neighbour_map_every_element(m, base, param_layout, exact):
    """Stochastic gradient push with a column-stochastic P that is not doubly
    stochastic (Algorithm C.1): a seeded random in-neighbour map after every
    local step.  Replicas, push-sum weights and de-biased parameters against
    the oracle; the weights return to 1 at an exact average and keep moving
    without one (Section 6)."""
    import torch
    w = dataclasses.replace(W.ragged_mini(base=base, m=m, policy="maintain"), mix="random",
                            tau=4, rounds=2, exact_average=exact)
    prob = _problem(w, ring=2, param_layout=param_layout, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    precs = ("f64", "f32")
    os_ = {p: PU.make_oracle(w, idx, p) for p in precs}
    z = [[torch.full_like(t, float("nan")) for t in prob.params[i]] for i in range(m)]
    step = 0
    moved = False
    for t in range(w.rounds):
        for k in range(w.tau):
            prob.fill_grads(step % 2, step)
            peers = W.in_peers(w, step)
            if step % 2:                     # the pair as one call on every other step
                opt.local_mix_step(prob.grads[step % 2], w.lr, peers.tolist())
            else:
                opt.local_step(prob.grads[step % 2], w.lr)
                opt.mix_step(peers.tolist())
            g = PU.oracle_grads(w, idx, step)
            for o in os_.values():
                o.local_step(g, w.f32("lr"))
                o.mix_step(peers)
            step += 1
            wg = np.asarray(opt.pushsum_weights(), np.float32)
            assert np.array_equal(wg, os_["f32"].w), (t, k)
            np.testing.assert_allclose(wg.sum(), m, rtol=1e-6)      # P is column-stochastic
            moved = moved or bool(np.any(wg != 1))
            opt.debias(z)
            got_x = np.stack([prob.gather(prob.params[i], idx) for i in range(m)])
            got_z = np.stack([prob.gather(z[i], idx) for i in range(m)])
            PU.assert_params_close(got_x, os_["f64"].x, f"replicas after gossip step {step}")
            PU.assert_params_close(got_z, os_["f64"].debiased(), f"de-biased parameters, step {step}")
            if base == "sgd_nesterov":
                assert np.array_equal(got_x, os_["f32"].x), (t, k)
                assert np.array_equal(got_z, os_["f32"].debiased()), (t, k)
        opt.outer_step(w.lr)
        for o in os_.values():
            o.outer_step(w.f32("lr"))
        wg = np.asarray(opt.pushsum_weights(), np.float32)
        assert np.array_equal(wg, os_["f32"].w)
        assert exact == bool(np.all(wg == 1)) or m == 1
    assert moved or m == 1
    final = PU.gpu_state(w, prob, opt, idx)
    PU.assert_params_close(final["x"], os_["f64"].x, "replicas after the run")
    PU.assert_u_close(final["u"], os_["f64"].u, w.f32("lr"), "u after the run")
    if base == "sgd_nesterov":
        assert np.array_equal(final["x"], os_["f32"].x)
        assert np.array_equal(final["u"], os_["f32"].u)
    opt.close()


def test_push_sum_weights_survive_export_and_import():
    w = dataclasses.replace(W.ragged_mini(m=7, policy="maintain"), mix="random", tau=3, rounds=1)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    prob.fill_grads(0, 0)
    opt.local_step(prob.grads[0], w.lr)
    opt.mix_step(W.in_peers(w, 0).tolist())
    opt.mix_step(W.in_peers(w, 1).tolist())
    want = opt.pushsum_weights()
    assert any(v != 1 for v in want)
    blob = opt.export_state()
    opt.mix_step(W.in_peers(w, 2).tolist())
    assert opt.pushsum_weights() != want
    opt.import_state(blob)
    assert opt.pushsum_weights() == want
    opt.close()


@pytest.mark.parametrize("base,exact_average", [("sgd_nesterov", True), ("adam", True),
                                                ("sgd_nesterov", False)])
def test_per_tensor_hyperparameters_every_element(base, exact_average):
    """Parameter groups: every tensor its own weight decay and learning-rate
    scale (e.g. no decay on the small vectors, smaller steps on some)."""
    w0 = W.ragged_mini(base=base)
    nt = len(w0.numel)
    wd = tuple(0.0 if n < 300 else 1e-4 * (1 + j % 3) for j, n in enumerate(w0.numel))
    sc = tuple((1.0, 0.5, 0.1, 2.0, 0.3)[j % 5] for j in range(nt))
    w = dataclasses.replace(w0, tensor_wd=wd, tensor_lr_scale=sc, exact_average=exact_average)
    prob = _problem(w, ring=2, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"))
    import paper_1910_00643_amd as P
    for bad in (dict(weight_decay=[-1.0] * nt), dict(lr_scale=[0.0] * nt),
                dict(lr_scale=[float("nan")] * nt)):
        with pytest.raises(P.SlowMoError):
            opt.set_tensor_hparams(**bad)
    opt.close()


@pytest.mark.parametrize("base,policy,exact_average", [("sgd_nesterov", "reset", True),
                                                       ("adam", "maintain", True),
                                                       ("sgd_nesterov", "maintain", False)])
def test_export_import_resumes_bit_for_bit(base, policy, exact_average):
    """Stop inside an outer iteration, export the state, rebuild everything
    from the saved bytes in a new context, continue: same bits as the
    uninterrupted run (and within tolerance of the oracle)."""
    import torch
    import paper_1910_00643_amd as P
    w = dataclasses.replace(W.ragged_mini(base=base, policy=policy), exact_average=exact_average)
    idx = np.arange(w.d, dtype=np.int64)
    stop = 2 * w.tau + 2                    # two rounds and two local steps
    total = w.rounds * w.tau

    def advance(prob, opt, first, last):
        for step in range(first, last):
            prob.fill_grads(0, step)
            opt.local_step(prob.grads[0], w.lr)
            if (step + 1) % w.tau == 0:
                opt.outer_step(w.lr)

    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    advance(prob, opt, 0, stop)
    blob = opt.export_state().cpu()         # as a checkpoint file would hold it
    saved = [[t.clone() for t in p] for p in prob.params]
    assert opt.counters()[:2] == (2, 2)
    advance(prob, opt, stop, total)
    want = PU.gpu_state(w, prob, opt, idx)
    opt.close()

    prob2 = _problem(w, grad_layout="separate")
    opt2 = PU.make_gpu(w, prob2)
    for p, q in zip(prob2.params, saved):   # replicas are restored after create
        for a, b in zip(p, q):
            a.copy_(b)
    opt2.import_state(blob.cuda())
    assert opt2.counters() == (2, 2, 2 * w.tau + 2 if base == "adam" else opt2.counters()[2])
    advance(prob2, opt2, stop, total)
    got = PU.gpu_state(w, prob2, opt2, idx)
    for key in ("x", "x0", "u", "h"):
        assert np.array_equal(got[key], want[key]), key
    o64, _ = PU.run_oracle(w, idx, w.rounds)
    PU.assert_params_close(got["x0"], o64.x0, "x0 after resume")
    # a blob from another configuration is refused
    w3 = dataclasses.replace(w, m=w.m + 1)
    prob3 = _problem(w3, grad_layout="separate")
    opt3 = PU.make_gpu(w3, prob3)
    with pytest.raises(P.SlowMoError):
        opt3.import_state(torch.zeros(P.slowmo_export_bytes(opt3.ctx), dtype=torch.uint8, device="cuda:0"))
    with pytest.raises(P.SlowMoError):
        opt3.import_state(blob.cuda())
    opt2.close()
    opt3.close()


@pytest.mark.parametrize("base,grad_dtype,policy,tau,layouts", [
    ("sgd_nesterov", "f32", "reset", 5, ("separate", "padded")),
    ("sgd_nesterov", "bf16", "maintain", 5, ("separate", "separate")),
    ("sgd_nesterov", "f32", "average", 5, ("separate", "padded")),
    ("sgd_nesterov", "f32", "reset", 1, ("separate", "separate")),     # first step is also the last
    ("adam", "bf16", "maintain", 5, ("separate", "padded")),
    ("adam", "f32", "reset", 3, ("separate", "separate")),
    ("adam", "bf16", "average", 4, ("separate", "padded")),
    ("sgd_nesterov", "f32", "reset", 5, ("flat", "flat")),             # unaligned: two kernels
])
def test_fused_last_local_and_outer_step(base, grad_dtype, policy, tau, layouts):
    """slowmo_local_outer_step == slowmo_local_step + slowmo_outer_step, bit
    for bit, and within tolerance of the oracle."""
    w = dataclasses.replace(W.ragged_mini(base=base, grad_dtype=grad_dtype, policy=policy), tau=tau,
                            tensor_wd=tuple(1e-4 * (j % 3) for j in range(26)),
                            tensor_lr_scale=tuple((1.0, 0.5, 2.0)[j % 3] for j in range(26)))
    idx = np.arange(w.d, dtype=np.int64)
    res = []
    for fused in (False, True):
        prob = _problem(w, ring=2, param_layout=layouts[0], grad_layout=layouts[1])
        opt = PU.make_gpu(w, prob)
        PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"),
                       fused_last=fused)
        res.append(PU.gpu_state(w, prob, opt, idx))
        if fused:
            import paper_1910_00643_amd as P
            prob.fill_grads(0, 0)
            if tau > 1:
                with pytest.raises(P.SlowMoError) as e:     # not the last local step
                    opt.local_outer_step(prob.grads[0], w.lr)
                assert e.value.status == P.binding.SLOWMO_ERR_STATE
        opt.close()
    for key in ("x", "x0", "u"):
        assert np.array_equal(res[0][key], res[1][key]), key
    if policy != "reset":
        assert np.array_equal(res[0]["h"], res[1]["h"])
        if base == "adam":
            assert np.array_equal(res[0]["v"], res[1]["v"])


def _with_env(name, value, make):
    """make() with the environment variable set (the library reads its knobs at
    slowmo_create)."""
    import os
    old = os.environ.get(name)
    os.environ[name] = value
    try:
        return make()
    finally:
        if old is None:
            os.environ.pop(name, None)
        else:
            os.environ[name] = old


@pytest.mark.parametrize("base,grad_dtype,policy,m,layouts", [
    ("sgd_nesterov", "f32", "reset", 3, ("separate", "padded")),
    ("sgd_nesterov", "bf16", "maintain", 3, ("separate", "separate")),
    ("sgd_nesterov", "f32", "average", 3, ("separate", "padded")),     # buffers averaged: ordinary tiles
    ("adam", "bf16", "maintain", 3, ("separate", "padded")),
    ("adam", "f32", "reset", 3, ("separate", "separate")),
    ("sgd_nesterov", "f32", "reset", 3, ("flat", "padded")),           # unaligned replicas: no big tile
    ("sgd_nesterov", "f32", "reset", 17, ("separate", "separate")),
])
@pytest.mark.parametrize("fused", [False, True])
def test_big_tiles_equal_the_ordinary_tiles_bitwise(base, grad_dtype, policy, m, layouts, fused):
    """The outer step and the fused last step on 65 536-element pieces (one
    1024-thread workgroup each; the tensors of 70 001 and 131 077 elements have
    one and two of them, plus a rest) against the same run on ordinary tiles,
    bit for bit, and against the oracle."""
    w = dataclasses.replace(W.ragged_mini(base=base, grad_dtype=grad_dtype, policy=policy, m=m),
                            tau=3, rounds=3,
                            tensor_wd=tuple(1e-4 * (j % 3) for j in range(26)),
                            tensor_lr_scale=tuple((1.0, 0.5, 2.0)[j % 3] for j in range(26)))
    idx = np.arange(w.d, dtype=np.int64)
    res = []
    for big in ("0", "1"):        # by itself the library takes big tiles only for large lists
        prob = _problem(w, ring=2, param_layout=layouts[0], grad_layout=layouts[1])
        opt = _with_env("SLOWMO_BIG_TILES", big, lambda: PU.make_gpu(w, prob))
        PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"),
                       fused_last=fused)
        res.append(PU.gpu_state(w, prob, opt, idx))
        opt.close()
    for key in ("x", "x0", "u", "h") + (("v",) if base == "adam" else ()):
        assert np.array_equal(res[0][key], res[1][key]), key


@pytest.mark.parametrize("m", [1, 2, 7, 33, 300])
def test_worker_counts(m):
    """m = 1 (Lookahead-like), odd m (true division by m), m above the
    unrolled group, m above the workgroup size."""
    w = dataclasses.replace(W.ragged_mini(m=m), shapes=tuple([("a", (5000,)), ("b", (37,)), ("c", (4099,))]),
                            rounds=2, tau=3)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    PU.compare_run(w, prob, opt, np.arange(w.d, dtype=np.int64), w.rounds, bitwise_f32=True)
    opt.close()


@pytest.mark.parametrize("base,grad_dtype,policy", [
    ("sgd_nesterov", "f32", "reset"), ("sgd_nesterov", "bf16", "reset"), ("adam", "bf16", "reset"),
    ("adam", "f32", "maintain"), ("sgd_nesterov", "f32", "maintain")])
def test_big_tiles_when_the_first_step_is_also_the_last(base, grad_dtype, policy):
    """tau = 1: every call is the fused step; under "reset" always with the
    buffers read as zero and not stored, under "maintain" the very first one
    reads them as zero."""
    w = dataclasses.replace(W.ragged_mini(base=base, grad_dtype=grad_dtype, policy=policy, m=5),
                            tau=1, rounds=4)
    idx = np.arange(w.d, dtype=np.int64)
    res = []
    for big in ("0", "1"):
        prob = _problem(w, ring=2, grad_layout="padded")
        opt = _with_env("SLOWMO_BIG_TILES", big, lambda: PU.make_gpu(w, prob))
        PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"),
                       fused_last=True)
        res.append(PU.gpu_state(w, prob, opt, idx))
        opt.close()
    for key in ("x", "x0", "u") + (("h",) if policy == "maintain" else ()):
        assert np.array_equal(res[0][key], res[1][key]), key


@pytest.mark.parametrize("m,fused", [(8, True), (9, True), (16, False), (33, True), (33, False),
                                     (150, True), (1024, True)])
def test_worker_counts_on_big_tiles(m, fused):
    """Tensors of exactly one big tile (no rest), one big tile and five
    elements, two big tiles, and one too small for any, at several worker
    counts (big tiles forced: by itself the library takes them only when there
    are enough to occupy the chip)."""
    w = dataclasses.replace(W.ragged_mini(m=m),
                            shapes=tuple([("a", (65536,)), ("b", (65541,)), ("c", (3,)),
                                          ("d", (131072,)), ("e", (65535,))]),
                            rounds=2, tau=2)
    prob = _problem(w, grad_layout="separate")
    opt = _with_env("SLOWMO_BIG_TILES", "1", lambda: PU.make_gpu(w, prob))
    PU.compare_run(w, prob, opt, np.arange(w.d, dtype=np.int64), w.rounds, bitwise_f32=True,
                   fused_last=fused)
    opt.close()


@pytest.mark.parametrize("mix,exact", [("random", True), ("expgraph", True), ("random", False)])
def test_largest_worker_count_with_gossip(mix, exact):
    """m = SLOWMO_MAX_WORKERS = 1024 replicas: pointer tables, mixing order
    (up to 1024 entries, many groups) and the ordered mean at their largest."""
    w = dataclasses.replace(W.ragged_mini(m=1024, policy="maintain"), mix=mix, exact_average=exact,
                            shapes=(("a", (300,)), ("b", (5,)), ("c", (1030,))), rounds=2, tau=3)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    PU.compare_run(w, prob, opt, np.arange(w.d, dtype=np.int64), w.rounds, bitwise_f32=True,
                   fused_mix=True)
    opt.close()


def test_empty_tensor_list_and_tau_one():
    w = dataclasses.replace(W.ragged_mini(), shapes=(("e0", (0,)), ("e1", (0,))), rounds=2, tau=1)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    for _ in range(2):
        opt.local_step(prob.grads[0], w.lr)
        opt.outer_step(w.lr)
    assert opt.counters()[0] == 2
    opt.close()


def test_run_to_run_bitwise_determinism():
    w = W.ragged_mini()
    idx = np.arange(w.d, dtype=np.int64)
    res = []
    for _ in range(2):
        prob = _problem(w, ring=2)
        opt = PU.make_gpu(w, prob)
        PU.run_gpu(w, prob, opt, w.rounds, idx)
        res.append(PU.gpu_state(w, prob, opt, idx))
        opt.close()
    for key in ("x", "h", "x0", "u"):
        assert np.array_equal(res[0][key], res[1][key]), key


def test_gradient_pointer_table_follows_changing_pointers():
    """More distinct gradient buffers than table slots, used in turn, then the
    same buffer twice in a row (table reuse)."""
    w = dataclasses.replace(W.ragged_mini(), tau=7, rounds=2)
    prob = _problem(w, ring=6, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=True)
    opt.close()


def test_learning_rate_schedule_and_side_stream():
    """gamma is a per-call scalar (it may follow a schedule inside and across
    outer iterations, Section 2), and all work goes to the stream handed in:
    here a non-default stream of default priority."""
    import torch
    w = W.ragged_mini()
    idx = np.arange(w.d, dtype=np.int64)
    lr_local = lambda step: float(np.float32(0.02 * (1 + step % 4)))        # noqa: E731
    lr_outer = lambda t: float(np.float32(0.05 / (1 + t)))                  # noqa: E731
    o = PU.make_oracle(w, idx)
    o32 = PU.make_oracle(w, idx, "f32")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        prob = _problem(w, grad_layout="separate")
        opt = PU.make_gpu(w, prob)
        step = 0
        for t in range(w.rounds):
            for k in range(w.tau):
                prob.fill_grads(0, step)
                opt.local_step(prob.grads[0], lr_local(step))
                g = PU.oracle_grads(w, idx, step)
                o.local_step(g, lr_local(step))
                o32.local_step(g, lr_local(step))
                step += 1
            opt.outer_step(lr_outer(t))
            o.outer_step(lr_outer(t))
            o32.outer_step(lr_outer(t))
        side.synchronize()
        final = PU.gpu_state(w, prob, opt, idx)
    PU.assert_params_close(final["x0"], o.x0, "x0 under a schedule")
    assert np.array_equal(final["x0"], o32.x0) and np.array_equal(final["u"], o32.u)
    opt.close()


@pytest.mark.parametrize("base", ["sgd_nesterov", "adam"])
def test_run_under_the_papers_schedules(base):
    """A short run whose learning rate follows the schedules of the paper's
    experiments: warm-up and step decay for SGD (Section 4), warm-up and
    inverse square root for Adam (Appendix A.3).  The GPU side takes the rate
    from the library's helper, the oracle from its own function; the constants
    are exact in fp32, so both get the same float."""
    import paper_1910_00643_amd as P
    from oracle import slowmo_oracle as O
    w = dataclasses.replace(W.ragged_mini(base=base), tau=4, rounds=5)
    idx = np.arange(w.d, dtype=np.int64)
    if base == "sgd_nesterov":
        gpu_lr = lambda s: P.slowmo_lr_step_decay(0.125, 0.0078125, 6, [10, 14, 17], 0.5, s)    # noqa: E731
        ref_lr = lambda s: O.lr_warmup_step_decay(0.125, 0.0078125, 6, [10, 14, 17], 0.5, s)    # noqa: E731
    else:
        gpu_lr = lambda s: P.slowmo_lr_inverse_sqrt(0.0009765625, 0.0, 8, s)                    # noqa: E731
        ref_lr = lambda s: O.lr_warmup_inverse_sqrt(0.0009765625, 0.0, 8, s)                    # noqa: E731
    o = PU.make_oracle(w, idx)
    o32 = PU.make_oracle(w, idx, "f32")
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    step = 0
    for t in range(w.rounds):
        for k in range(w.tau):
            lr = gpu_lr(step + 1)                   # step 0 of a warm-up from zero has rate 0
            assert lr == float(np.float32(ref_lr(step + 1))), (step, lr)
            prob.fill_grads(0, step)
            opt.local_step(prob.grads[0], lr)
            g = PU.oracle_grads(w, idx, step)
            o.local_step(g, lr)
            o32.local_step(g, lr)
            step += 1
        opt.outer_step(lr)                          # gamma_t of Eq. (2)-(3): the current rate
        o.outer_step(lr)
        o32.outer_step(lr)
    final = PU.gpu_state(w, prob, opt, idx)
    PU.assert_params_close(final["x0"], o.x0, "x0 under the paper's schedule")
    if base == "sgd_nesterov":
        assert np.array_equal(final["x0"], o32.x0) and np.array_equal(final["u"], o32.u)
    opt.close()


def test_two_contexts_side_by_side():
    """Contexts share nothing: two optimizers over different tensor lists,
    stepped alternately, give the results each gives alone."""
    wa = W.ragged_mini()
    wb = dataclasses.replace(W.ragged_mini(base="adam", grad_dtype="bf16"), m=2)
    probs = [_problem(wa, grad_layout="separate"), _problem(wb, grad_layout="separate")]
    opts = [PU.make_gpu(wa, probs[0]), PU.make_gpu(wb, probs[1])]
    for t in range(2):
        for k in range(wa.tau):
            for w, prob, opt in zip((wa, wb), probs, opts):
                prob.fill_grads(0, t * w.tau + k)
                opt.local_step(prob.grads[0], w.lr)
        for w, opt in zip((wa, wb), opts):
            opt.outer_step(w.lr)
    for w, prob, opt in zip((wa, wb), probs, opts):
        idx = np.arange(w.d, dtype=np.int64)
        o64, _ = PU.run_oracle(w, idx, 2)
        PU.assert_params_close(PU.gpu_state(w, prob, opt, idx)["x0"], o64.x0, w.name)
        opt.close()


def test_outer_iteration_replayed_from_a_hip_graph():
    """One whole outer iteration (tau-1 local steps and the fused last step)
    captured into a HIP graph and replayed.  With unchanged gradient pointers
    the library only launches kernels (the pointer table is already on the
    device), and for the SGD base with the reset policy every outer iteration
    is the same sequence of launches with the same arguments, so each replay
    must equal one more eager outer iteration, bit for bit.  Replays are
    separated by eager work and synchronizations."""
    import torch
    w = W.ragged_mini()
    idx = np.arange(w.d, dtype=np.int64)

    def build():
        prob = _problem(w, ring=1, grad_layout="separate")
        opt = PU.make_gpu(w, prob)
        prob.fill_grads(0, 0)                   # one gradient set, used by every step
        return prob, opt, opt.grad_pointer_array(prob.grads[0])

    def one_round(opt, arr):
        for k in range(w.tau - 1):
            opt.local_step(arr, w.lr)
        opt.local_outer_step(arr, w.lr)

    ref_prob, ref_opt, ref_arr = build()
    prob, opt, arr = build()
    one_round(ref_opt, ref_arr)
    one_round(opt, arr)                         # eager: uploads the pointer table
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=cap):
        one_round(opt, arr)                     # recorded, not executed
    torch.cuda.synchronize()
    assert np.array_equal(PU.gpu_state(w, prob, opt, idx)["x0"],
                          PU.gpu_state(w, ref_prob, ref_opt, idx)["x0"])
    for rep in range(4):
        graph.replay()
        torch.cuda.synchronize()
        one_round(ref_opt, ref_arr)
        assert np.isfinite(torch.randn(1 << 16, device="cuda:0").sum().item())   # eager work
        got = PU.gpu_state(w, prob, opt, idx)
        ref = PU.gpu_state(w, ref_prob, ref_opt, idx)
        for key in ("x", "x0", "u"):
            assert np.array_equal(got[key], ref[key]), (rep, key)
    opt.close()
    ref_opt.close()


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_configurations(seed):
    """Seeded random draws over everything the library accepts: tensor lists
    with empty, tiny and multi-tile tensors, worker counts, tau, both base
    optimizers, gradient dtypes, the three buffer strategies, the variant
    without the exact average, gossip steps, parameter groups, aligned and
    packed (unaligned) layouts, separate or fused end of the outer iteration."""
    rng = np.random.default_rng(1000 + seed)
    n_t = int(rng.integers(1, 10))
    sizes = [int(rng.choice([0, 1, 3, 4, 7, 64, 255, 256, 257, 1000, 2049, 5000, 40_001]))
             for _ in range(n_t)]
    if sum(sizes) == 0:
        sizes[0] = 17
    base = str(rng.choice(["sgd_nesterov", "adam"]))
    policy = str(rng.choice(["reset", "maintain", "average"]))
    exact = seed % 4 != 3                   # every fourth draw: no exact average (Section 6)
    if not exact and policy == "average":
        policy = "maintain"
    # gossip (one-peer exponential graph, or any in-neighbour map) also without the exact
    # average: as the only exchange it is the SGP-SlowMo-noaverage variant of Section 6
    mix = ("expgraph", "random", "none", "none", "none", "none")[int(rng.integers(0, 6))]
    groups = bool(rng.integers(0, 2))
    w = Workload = dataclasses.replace(
        W.ragged_mini(base=base, grad_dtype=str(rng.choice(["f32", "bf16"])), policy=policy,
                      m=int(rng.integers(1, 7))),
        shapes=tuple((f"t{j}", (n,)) for j, n in enumerate(sizes)),
        tau=int(rng.integers(1, 5)), rounds=3, exact_average=exact, mix=mix,
        alpha=float(rng.choice([0.5, 1.0])), beta=float(rng.choice([0.0, 0.4, 0.8])),
        tensor_wd=tuple(float(rng.choice([0.0, 1e-4, 1e-3])) for _ in sizes) if groups else None,
        tensor_lr_scale=tuple(float(rng.choice([1.0, 0.5, 2.0])) for _ in sizes) if groups else None)
    del Workload
    layouts = (str(rng.choice(["separate", "flat", "arena"])),
               str(rng.choice(["separate", "flat", "padded"])))
    fused = bool(rng.integers(0, 2)) and exact and mix == "none"
    fused_mix = mix != "none" and seed % 2 == 0
    print("config", seed, dict(sizes=sizes, m=w.m, tau=w.tau, base=base, grads=w.grad_dtype,
                               policy=policy, exact=exact, mix=mix, groups=groups,
                               layouts=layouts, fused=fused, fused_mix=fused_mix), flush=True)
    prob = _problem(w, ring=2, param_layout=layouts[0], grad_layout=layouts[1])
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=(base == "sgd_nesterov"),
                   fused_last=fused, fused_mix=fused_mix)
    opt.close()


def test_c_abi_from_plain_c_matches_the_closed_form():
    """tests/abi_c_check (plain C, built by __graft_entry__.build()) drives the
    library through include/slowmo.h alone and checks Eq. (2)-(3)'s closed form
    for constant gradients on the GPU."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_c_check")
    assert os.path.exists(exe), "tests/abi_c_check is not built: run __graft_entry__.build()"
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.startswith("OK"), run.stdout + run.stderr


def test_denormal_values_are_not_flushed():
    """fp32 subnormals take part in the arithmetic as IEEE values (no
    flush-to-zero): gradients around 1e-38 give momentum buffers full of
    subnormal numbers, which must equal the fp32 oracle's bit for bit."""
    w = dataclasses.replace(W.ragged_mini(policy="maintain"), sigma=1e-38, weight_decay=0.0,
                            rounds=2)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    snap = PU.run_gpu(w, prob, opt, w.rounds, idx)
    _, s32 = PU.run_oracle(w, idx, w.rounds, "f32")
    tiny = np.abs(s32["h"]) < np.finfo(np.float32).tiny
    assert np.count_nonzero(tiny & (s32["h"] != 0)) > 1000        # the case is really exercised
    assert np.array_equal(snap["h"], s32["h"])
    assert np.array_equal(snap["x"], s32["x"])
    opt.close()


def test_call_sequence_errors_leave_state_unchanged():
    import paper_1910_00643_amd as P
    w = dataclasses.replace(W.ragged_mini(), tau=2, rounds=1)
    prob = _problem(w)
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    with pytest.raises(P.SlowMoError) as e:
        opt.outer_step(w.lr)                       # no local step yet
    assert e.value.status == P.binding.SLOWMO_ERR_STATE
    prob.fill_grads(0, 0)
    opt.local_step(prob.grads[0], w.lr)
    with pytest.raises(P.SlowMoError):
        opt.local_step(prob.grads[0], float("nan"))
    with pytest.raises(P.SlowMoError):
        opt.local_step(prob.grads[0], 0.0)
    prob.fill_grads(0, 1)
    opt.local_step(prob.grads[0], w.lr)
    with pytest.raises(P.SlowMoError) as e:
        opt.local_step(prob.grads[0], w.lr)        # tau steps already taken
    assert e.value.status == P.binding.SLOWMO_ERR_STATE
    assert opt.counters()[:2] == (0, 2)
    snap = PU.gpu_state(w, prob, opt, idx, with_outer=False)
    opt.outer_step(w.lr)
    final = PU.gpu_state(w, prob, opt, idx)
    o64, s64 = PU.run_oracle(w, idx, 1)
    PU.assert_params_close(snap["x"], s64["x"], "replicas")
    PU.assert_params_close(final["x0"], o64.x0, "x0")
    opt.close()


@pytest.mark.parametrize("ring", [3, 20])
def test_gradient_pointer_tables_are_cached_and_evicted_correctly(ring):
    """The library keeps the most recent 16 distinct gradient-pointer tables
    on the device.  3 gradient sets in turn: every table is found again; 20
    sets in turn: every call evicts the oldest table and uploads anew.  The
    results must not depend on it."""
    w = dataclasses.replace(W.ragged_mini(), tau=7, rounds=6)
    prob = _problem(w, ring=ring, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    PU.compare_run(w, prob, opt, idx, w.rounds, bitwise_f32=True)
    opt.close()


def test_host_pointers_are_rejected_before_any_kernel_runs():
    """A host array passed where a device tensor belongs must come back as an
    argument error from the host-side range check, not reach a kernel."""
    import torch
    import paper_1910_00643_amd as P
    from paper_1910_00643_amd.optimizer import make_config
    B = P.binding
    dev = torch.zeros(1000, dtype=torch.float32, device="cuda:0")
    host = np.zeros(1000, dtype=np.float32)
    pinned = torch.zeros(1000, dtype=torch.float32).pin_memory()
    # the check itself, first: it launches nothing
    P.slowmo_check_device_range(dev.data_ptr(), 4000)
    P.slowmo_check_device_range(dev.data_ptr() + 400, 3600)
    P.slowmo_check_device_range(pinned.data_ptr(), 4000)       # pinned host memory is device-accessible
    for ptr, nbytes in ((host.ctypes.data, 4000), (0, 16)):
        with pytest.raises(P.SlowMoError) as e:
            P.slowmo_check_device_range(ptr, nbytes)
        assert e.value.status == B.SLOWMO_ERR_ARG
    whole = torch.empty(1 << 22, dtype=torch.uint8, device="cuda:0")    # an allocation of its own
    with pytest.raises(P.SlowMoError) as e:
        P.slowmo_check_device_range(whole.data_ptr(), (1 << 30) + whole.numel())
    assert e.value.status == B.SLOWMO_ERR_ARG
    # only now through slowmo_create (the check has just been shown to reject this pointer)
    cfg = make_config(m=2, tau=2, alpha=1.0, beta=0.5, base="sgd_nesterov", momentum=0.9)
    x = [torch.zeros(1000, dtype=torch.float32, device="cuda:0") for _ in range(2)]
    nbytes = P.slowmo_state_bytes(cfg, [1000])
    state = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(P.SlowMoError) as e:
        P.slowmo_create(cfg, [1000], [x[0].data_ptr(), host.ctypes.data], state.data_ptr(), nbytes)
    assert e.value.status == B.SLOWMO_ERR_ARG and "parameter tensor" in e.value.message
    ctx = P.slowmo_create(cfg, [1000], [t.data_ptr() for t in x], state.data_ptr(), nbytes)
    P.slowmo_destroy(ctx)
    torch.cuda.synchronize()


def test_failed_mixing_calls_leave_replicas_weights_and_counters_unchanged():
    import torch
    import paper_1910_00643_amd as P
    B = P.binding
    w = dataclasses.replace(W.ragged_mini(m=4), tau=2, rounds=1)
    prob = _problem(w, grad_layout="separate")
    opt = PU.make_gpu(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    prob.fill_grads(0, 0)
    opt.local_mix_step(prob.grads[0], w.lr, [0, 0, 1, 1])
    before = (PU.gpu_state(w, prob, opt, idx, with_outer=False), opt.pushsum_weights(), opt.counters())
    assert before[1] != [1.0] * 4 and before[2][:2] == (0, 1)
    for bad_peers in ([0, 0, 1, 4], [0, -1, 1, 1]):
        for call in (lambda p: opt.mix_step(p), lambda p: opt.local_mix_step(prob.grads[0], w.lr, p)):
            with pytest.raises(P.SlowMoError) as e:
                call(bad_peers)
            assert e.value.status == B.SLOWMO_ERR_ARG
    with pytest.raises(P.SlowMoError) as e:
        opt.local_mix_step(prob.grads[0], -1.0, [0, 0, 1, 1])
    assert e.value.status == B.SLOWMO_ERR_ARG
    # de-bias: a missing destination and a misaligned one
    z = [[torch.empty_like(t) for t in prob.params[i]] for i in range(w.m)]
    ptrs = [t.data_ptr() for zi in z for t in zi]
    big = next(k for k, n in enumerate(prob.numel) if n > 8)
    with pytest.raises(P.SlowMoError) as e:
        B.slowmo_debias(opt.ctx, ptrs[:big] + [0] + ptrs[big + 1:])
    assert e.value.status == B.SLOWMO_ERR_ARG
    with pytest.raises(P.SlowMoError) as e:
        B.slowmo_debias(opt.ctx, ptrs[:big] + [ptrs[big] + 2] + ptrs[big + 1:])
    assert e.value.status == B.SLOWMO_ERR_ALIGN
    after = (PU.gpu_state(w, prob, opt, idx, with_outer=False), opt.pushsum_weights(), opt.counters())
    assert after[1] == before[1] and after[2] == before[2]
    for key in ("x", "h"):
        assert np.array_equal(before[0][key], after[0][key]), key
    # the context still works: finish the outer iteration
    prob.fill_grads(0, 1)
    opt.local_mix_step(prob.grads[0], w.lr, [1, 0, 3, 2])
    with pytest.raises(P.SlowMoError) as e:
        opt.local_mix_step(prob.grads[0], w.lr, [1, 0, 3, 2])      # tau steps already taken
    assert e.value.status == B.SLOWMO_ERR_STATE
    opt.outer_step(w.lr)
    assert opt.pushsum_weights() == [1.0] * 4
    opt.close()


# ---- full sizes, every element ---------------------------------------------------
def _every_element(w, rounds):
    """The whole model, in the launch configuration bench.py times (separate
    parameter allocations, 512-byte aligned gradient tensors, the fused call at
    the end of every outer iteration but the last, which ends with the two
    separate calls): every element of every replica, of h, x0 and u against the
    fp64 oracle within the tolerance and against the fp32 oracle bit for bit.
    The oracle's inputs are read back from the device generator."""
    prob = _problem(w, ring=2, grad_layout="padded")
    opt = PU.make_gpu(w, prob)
    worst = PU.compare_run(w, prob, opt, None, rounds, bitwise_f32=True, fused_last=True,
                           device_inputs=True)
    print(w.name, "every element of", w.d, "x", w.m, "workers,", rounds, "rounds: worst errors",
          worst, flush=True)
    opt.close()


def test_resnet18_shaped_every_element():
    w = W.resnet18()
    _every_element(w, w.rounds)             # all 20 outer iterations


def test_resnet50_shaped_every_element():
    _every_element(W.resnet50(), 2)         # 32 replicas of 25.6M elements, 24 local steps


@pytest.mark.skipif(os.environ.get("SLOWMO_FULL_PARITY") != "1",
                    reason="several minutes and about 100 GB of host memory: set SLOWMO_FULL_PARITY=1")
def test_transformer_big_shaped_every_element_one_round():
    """Every element of the 8 x 209 911 808 replicas, of h, v, x0 and u after one
    outer iteration (48 Adam steps on bf16 gradients + outer step) against the
    fp64 oracle.  Not part of the default run (its size); the default run
    checks this configuration on samples and a dense slab."""
    w = W.transformer_big()
    prob = _problem(w, ring=2, grad_layout="padded")
    opt = PU.make_gpu(w, prob)
    worst = PU.compare_run(w, prob, opt, None, 1, bitwise_f32=False, device_inputs=True)
    print(w.name, "every element of", w.d, "x", w.m, "workers, 1 round: worst errors", worst,
          flush=True)
    opt.close()


# ---- full sizes, sampled elements ------------------------------------------------
def _sampled(w, rounds, n_random, ring=2, halo=4, slab=None):
    """slab = (first, count): a dense run of consecutive global indices checked
    in full in addition to the sample; its inputs for the oracle are read back
    from the device generator."""
    prob = _problem(w, ring=ring, grad_layout="padded")     # the layout bench.py times
    opt = PU.make_gpu(w, prob)
    idx = prob.sample_indices(n_random, edges=_tile_edges(w), halo=halo, seed=w.seed)
    if slab is not None:
        idx = np.union1d(idx, np.arange(slab[0], slab[0] + slab[1], dtype=np.int64))
    # as bench.py runs it: outer iterations end with the fused call where that applies
    worst = PU.compare_run(w, prob, opt, idx, rounds, bitwise_f32=(w.base == "sgd_nesterov"),
                           fused_last=(w.exact_average and w.mix == "none"),
                           fused_mix=(w.mix != "none"), device_inputs=slab is not None)
    print(w.name, "sampled", idx.size, "worst errors", worst)
    opt.close()


def test_resnet18_shaped_sampled():
    w = W.resnet18()
    _sampled(w, w.rounds, 2000)


def test_resnet50_shaped_sampled():
    w = W.resnet50()
    _sampled(w, w.rounds, 1500)


def test_transformer_big_shaped_sampled():
    """Sampled indices plus a dense slab of 3.2M consecutive elements that runs
    from inside the embedding across the first encoder layer's q, k (weights
    and biases) into v: six tensors, two of them 1024 elements long."""
    w = W.transformer_big()
    emb = w.numel[0]
    assert emb == 32768 * 1024 and w.numel[1:5] == [1024 * 1024, 1024, 1024 * 1024, 1024]
    _sampled(w, w.rounds, 3000, slab=(emb - 1_000_000, 3_200_000))


def test_resnet50_shaped_noaverage_sampled():
    w = dataclasses.replace(W.resnet50(), exact_average=False, rounds=4)
    _sampled(w, w.rounds, 1500)


def test_resnet50_shaped_average_policy_sampled():
    """Buffer strategy "average" at full size (the outer kernel also averages
    the m momentum buffers)."""
    w = dataclasses.replace(W.resnet50(), policy="average", rounds=4)
    _sampled(w, w.rounds, 1500)


@pytest.mark.parametrize("mix", ["expgraph", "random"])
def test_resnet50_shaped_gradient_push_sampled(mix):
    """Stochastic gradient push as base optimizer at full size, as bench.py
    --mix runs it: every local step and its gossip step as one fused call."""
    w = dataclasses.replace(W.resnet50(), mix=mix, rounds=3)
    _sampled(w, w.rounds, 1500)


def test_transformer_big_shaped_gradient_push_sampled():
    w = dataclasses.replace(W.transformer_big(), mix="expgraph", rounds=1, tau=12)
    _sampled(w, w.rounds, 2000)


def test_stress_1e9_sampled():
    """d = 1e9, m = 8: 96 GB of replicas, momentum and gradients; element and
    byte offsets beyond 32 bits."""
    w = W.stress()
    # dense slab: 4M elements across the 2 GiB byte offset of the replica (element 2^29)
    _sampled(w, w.rounds, 6000, ring=1, slab=((1 << 29) - 2_000_000, 4_000_000))
