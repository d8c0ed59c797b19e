"""Error behaviour at the C boundary, on the GPU but without provoking any
GPU error: bad arguments are caught on the host before the first launch, and
launch failures are simulated by the library's own host-side hook
(SLOWMO_TEST_FAIL_LAUNCH=n: the n-th launch of a context is not issued and
reports a failure), so every kernel that does run is a normal one."""
import dataclasses
import gc
import os

import numpy as np
import pytest

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


def _make(w, prob, fail_launch_at=0):
    """A context whose n-th kernel launch (1-based, counted after create)
    reports a launch failure without launching anything."""
    if fail_launch_at:
        os.environ["SLOWMO_TEST_FAIL_LAUNCH"] = str(fail_launch_at)
    try:
        return PU.make_gpu(w, prob)
    finally:
        os.environ.pop("SLOWMO_TEST_FAIL_LAUNCH", None)


def _everything(w, prob, opt, idx):
    st = PU.gpu_state(w, prob, opt, idx)
    return st, opt.pushsum_weights(), opt.counters()


def _assert_same(a, b):
    assert a[1] == b[1] and a[2] == b[2]
    for key in ("x", "h", "x0", "u"):
        assert np.array_equal(a[0][key], b[0][key]), key


@pytest.mark.parametrize("layout", ["separate", "flat"])     # one fused kernel / two kernels
def test_bad_arguments_to_the_step_and_gossip_pair_change_nothing(layout):
    import paper_1910_00643_amd as P
    B = P.binding
    w = dataclasses.replace(W.ragged_mini(m=4, policy="maintain"), tau=3, rounds=1)
    prob = _problem(w, param_layout=layout, grad_layout="separate")
    opt = _make(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    prob.fill_grads(0, 0)
    opt.local_mix_step(prob.grads[0], w.lr, [0, 0, 1, 1])
    before = _everything(w, prob, opt, idx)
    assert before[1] != [1.0] * 4 and before[2][:2] == (0, 1)
    for bad in ([0, 0, 1, 4], [0, -1, 1, 1]):
        with pytest.raises(P.SlowMoError) as e:
            opt.local_mix_step(prob.grads[0], w.lr, bad)
        assert e.value.status == B.SLOWMO_ERR_ARG
    ptrs = [t.data_ptr() if t.numel() else 0 for g in prob.grads[0] for t in g]
    big = next(k for k, n in enumerate(prob.numel) if n > 8)
    with pytest.raises(P.SlowMoError) as e:          # a gradient pointer off its element size
        B.slowmo_local_mix_step(opt.ctx, ptrs[:big] + [ptrs[big] + 2] + ptrs[big + 1:], w.lr,
                                [1, 0, 3, 2])
    assert e.value.status == B.SLOWMO_ERR_ALIGN
    _assert_same(before, _everything(w, prob, opt, idx))
    opt.close()


@pytest.mark.parametrize("layout", ["separate", "flat"])
def test_refused_first_launch_changes_nothing_and_the_context_goes_on(layout):
    """The call's tables are uploaded, its first launch is refused: counters,
    weights, replicas and buffers are as before, and the same call then works
    and gives the result of a run that never failed."""
    import paper_1910_00643_amd as P
    w = dataclasses.replace(W.ragged_mini(m=4, policy="maintain"), tau=3, rounds=1)
    idx = np.arange(w.d, dtype=np.int64)
    peers = [[0, 0, 1, 1], [1, 0, 3, 2], [3, 0, 0, 2]]
    runs = []
    # the first call takes one launch (fused) or two (packed replicas: two kernels);
    # the refused launch is the first one of the second call
    for fail_at in (0, 2 if layout == "separate" else 3):
        prob = _problem(w, param_layout=layout, grad_layout="separate")
        opt = _make(w, prob, fail_at)
        for k in range(w.tau):
            prob.fill_grads(0, k)
            if fail_at and k == 1:
                before = _everything(w, prob, opt, idx)
                with pytest.raises(P.SlowMoError) as e:
                    opt.local_mix_step(prob.grads[0], w.lr, peers[k])
                assert e.value.status == P.binding.SLOWMO_ERR_HIP
                _assert_same(before, _everything(w, prob, opt, idx))
            opt.local_mix_step(prob.grads[0], w.lr, peers[k])
        opt.outer_step(w.lr)
        runs.append(_everything(w, prob, opt, idx))
        opt.close()
    _assert_same(runs[0], runs[1])


def test_launch_refused_halfway_is_reported_and_the_context_refuses_further_steps():
    """Two-kernel path (packed, unaligned replicas): the local step is
    launched, the gossip launch after it is refused.  The replicas are stepped
    but not mixed, which cannot be undone: the call says so, counters and
    weights keep their old values, and the context accepts no further step."""
    import paper_1910_00643_amd as P
    B = P.binding
    w = dataclasses.replace(W.ragged_mini(m=4, policy="maintain"), tau=3, rounds=1)
    prob = _problem(w, param_layout="flat", grad_layout="separate")
    opt = _make(w, prob, fail_launch_at=2)
    prob.fill_grads(0, 0)
    with pytest.raises(P.SlowMoError) as e:
        opt.local_mix_step(prob.grads[0], w.lr, [0, 0, 1, 1])
    assert e.value.status == B.SLOWMO_ERR_HIP and "partly" in e.value.message
    assert opt.counters()[:2] == (0, 0) and opt.pushsum_weights() == [1.0] * 4
    for call in (lambda: opt.local_step(prob.grads[0], w.lr), lambda: opt.mix_step([1, 0, 3, 2]),
                 lambda: opt.local_mix_step(prob.grads[0], w.lr, [1, 0, 3, 2]),
                 lambda: opt.outer_step(w.lr), lambda: opt.local_outer_step(prob.grads[0], w.lr),
                 lambda: opt.import_state(opt.export_state())):
        with pytest.raises(P.SlowMoError) as e:
            call()
        assert e.value.status == B.SLOWMO_ERR_STATE and "destroy" in e.value.message
    opt.close()


def test_gossip_launch_refused_for_the_second_group_of_workers():
    """One launch per connected group: pairs (0,1) and (2,3) are two launches."""
    import paper_1910_00643_amd as P
    w = dataclasses.replace(W.ragged_mini(m=4, policy="maintain"), tau=3, rounds=1)
    prob = _problem(w, grad_layout="separate")
    opt = _make(w, prob, fail_launch_at=2)
    with pytest.raises(P.SlowMoError) as e:
        opt.mix_step([1, 0, 3, 2])
    assert e.value.status == P.binding.SLOWMO_ERR_HIP and "partly" in e.value.message
    assert opt.pushsum_weights() == [1.0] * 4
    with pytest.raises(P.SlowMoError) as e:
        opt.mix_step([1, 0, 3, 2])
    assert e.value.status == P.binding.SLOWMO_ERR_STATE
    opt.close()


@pytest.mark.parametrize("fused", [False, True])
def test_outer_step_on_big_tiles_is_two_launches(fused):
    """With big tiles the outer step (alone or fused with the last local step)
    launches one kernel for the whole 65 536-element pieces and one for the
    rest.  The first refused: nothing has changed and the call can be repeated;
    the second refused: the call says that memory is partly updated, and the
    context refuses further steps."""
    import paper_1910_00643_amd as P
    B = P.binding
    w = dataclasses.replace(W.ragged_mini(m=4, policy="reset"), tau=3, rounds=1)
    idx = np.arange(w.d, dtype=np.int64)
    first = 3 if fused else 4           # launches before the call: tau - 1 or tau local steps
    results = []
    for fail_at in (0, first, first + 1):
        prob = _problem(w, grad_layout="separate")
        os.environ["SLOWMO_BIG_TILES"] = "1"
        try:
            opt = _make(w, prob, fail_at)
        finally:
            os.environ.pop("SLOWMO_BIG_TILES", None)
        for k in range(w.tau - (1 if fused else 0)):
            prob.fill_grads(0, k)
            opt.local_step(prob.grads[0], w.lr)
        prob.fill_grads(0, w.tau - 1)
        call = (lambda: opt.local_outer_step(prob.grads[0], w.lr)) if fused else \
            (lambda: opt.outer_step(w.lr))
        if fail_at == first:
            before = _everything(w, prob, opt, idx)
            with pytest.raises(P.SlowMoError) as e:
                call()
            assert e.value.status == B.SLOWMO_ERR_HIP and "partly" not in e.value.message
            _assert_same(before, _everything(w, prob, opt, idx))
        if fail_at == first + 1:
            with pytest.raises(P.SlowMoError) as e:
                call()
            assert e.value.status == B.SLOWMO_ERR_HIP and "partly" in e.value.message
            with pytest.raises(P.SlowMoError) as e:
                call()
            assert e.value.status == B.SLOWMO_ERR_STATE and "destroy" in e.value.message
        else:
            call()
            results.append(_everything(w, prob, opt, idx))
        opt.close()
    _assert_same(results[0], results[1])


def test_import_checks_the_whole_blob_before_it_touches_the_context():
    """A blob with a good header whose later parts are bad (a non-positive
    push-sum weight; counters that do not fit) is refused with the context's
    arrays, counters and weights untouched; a good blob is then accepted and
    the import has completed when the call returns."""
    import torch
    import paper_1910_00643_amd as P
    B = P.binding
    w = dataclasses.replace(W.ragged_mini(m=4, policy="maintain"), tau=3, rounds=1)
    prob = _problem(w, grad_layout="separate")
    opt = _make(w, prob)
    idx = np.arange(w.d, dtype=np.int64)
    prob.fill_grads(0, 0)
    opt.local_mix_step(prob.grads[0], w.lr, [0, 0, 1, 1])
    good = opt.export_state()
    prob.fill_grads(0, 1)
    opt.local_mix_step(prob.grads[0], w.lr, [3, 0, 0, 2])
    before = _everything(w, prob, opt, idx)
    assert before[2][:2] == (0, 2)

    bad_weight = good.clone()
    bad_weight[256:260] = torch.tensor([-1.0], dtype=torch.float32).view(torch.uint8).cuda()
    bad_k = good.clone()            # header: magic 8, version 4, then m, n_tensors, base, no_average, k
    bad_k[28:32] = torch.tensor([w.tau + 1], dtype=torch.int32).view(torch.uint8).cuda()
    for blob in (bad_weight, bad_k, good[:good.numel() - 4]):
        with pytest.raises(P.SlowMoError) as e:
            opt.import_state(blob)
        assert e.value.status == B.SLOWMO_ERR_ARG
        _assert_same(before, _everything(w, prob, opt, idx))
    # no synchronization by the caller between the import and the inspection
    B.slowmo_import_state(opt.ctx, good.data_ptr(), good.numel(),
                          torch.cuda.current_stream().cuda_stream)
    assert opt.counters()[:2] == (0, 1)
    again = opt.export_state()
    assert torch.equal(again, good)
    opt.close()
