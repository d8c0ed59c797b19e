"""The C ABI without a GPU: the library loads, exports every declared symbol,
rejects bad arguments before touching the device, and tiles correctly."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1910_00643_amd as P
from paper_1910_00643_amd import binding as B
from paper_1910_00643_amd.optimizer import make_config
from slowmo_inputs import shapes as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "slowmo.h")).read()
    declared = set(re.findall(r"\b(slowmo_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in P.slowmo_version()


def test_config_struct_matches_header_layout():
    assert C.sizeof(B.slowmo_config) == 52
    assert C.sizeof(B.slowmo_plan_run) == 24


def _cfg(**kw):
    base = dict(m=4, tau=12, alpha=1.0, beta=0.7, momentum=0.9, weight_decay=1e-4)
    base.update(kw)
    return make_config(**base)


@pytest.mark.parametrize("kw", [dict(m=0), dict(m=B.SLOWMO_MAX_WORKERS + 1), dict(tau=0),
                                dict(alpha=0.0), dict(alpha=float("inf")), dict(beta=1.0),
                                dict(beta=-0.1), dict(momentum=1.0), dict(weight_decay=-1.0),
                                dict(base="adam", beta1=1.0), dict(base="adam", eps=-1.0),
                                dict(beta=float("nan")), dict(no_average=True, policy="average")])
def test_bad_hyperparameters_are_rejected(kw):
    cfg = _cfg(**kw)
    assert P.slowmo_state_bytes(cfg, [16]) == 0
    with pytest.raises(P.SlowMoError) as e:
        P.slowmo_create(cfg, [16], [256] * cfg.m, 4096, 1 << 20)
    assert e.value.status == B.SLOWMO_ERR_ARG and e.value.message


def test_bad_enums_and_sizes_are_rejected():
    cfg = _cfg()
    for field in ("base", "policy", "grad_dtype"):
        bad = _cfg()
        setattr(bad, field, 7)
        assert P.slowmo_state_bytes(bad, [16]) == 0
    assert P.slowmo_state_bytes(cfg, [16, -1]) == 0
    assert P.slowmo_state_bytes(cfg, []) == 0
    assert P.slowmo_state_bytes(cfg, [16]) > 0


def test_create_rejects_bad_pointers_before_using_the_device():
    cfg = _cfg(m=2)
    n = P.slowmo_state_bytes(cfg, [64, 8])
    good = [0x10000, 0x20000, 0x30000, 0x40000]
    state = 0x100000

    def create(params=good, st=state, nbytes=n):
        P.slowmo_create(cfg, [64, 8], params, st, nbytes)

    with pytest.raises(P.SlowMoError) as e:
        create(params=[0x10000, 0, 0x30000, 0x40000])
    assert e.value.status == B.SLOWMO_ERR_ARG
    with pytest.raises(P.SlowMoError) as e:
        create(params=[0x10002, 0x20000, 0x30000, 0x40000])
    assert e.value.status == B.SLOWMO_ERR_ALIGN
    with pytest.raises(P.SlowMoError) as e:
        create(st=state + 16)
    assert e.value.status == B.SLOWMO_ERR_ALIGN
    with pytest.raises(P.SlowMoError) as e:
        create(nbytes=n - 1)
    assert e.value.status == B.SLOWMO_ERR_NOMEM
    with pytest.raises(P.SlowMoError) as e:
        create(params=[0x10000, 0x20000, 0x10080, 0x40000])     # replicas overlap
    assert e.value.status == B.SLOWMO_ERR_ARG and "overlap" in e.value.message
    with pytest.raises(P.SlowMoError) as e:
        create(params=[0x10000, 0x20000, 0x30000, state + 64])  # overlaps the workspace
    assert e.value.status == B.SLOWMO_ERR_ARG
    with pytest.raises(P.SlowMoError) as e:
        create(st=0)
    assert e.value.status == B.SLOWMO_ERR_ARG


def test_exponential_graph_peers_match_the_oracles():
    """Appendix C.1: hops 1, 2, 4, ..., 2^floor(log2(m-1)), one per iteration;
    the library's table against the oracle's own implementation."""
    from oracle import slowmo_oracle as O
    for m in (1, 2, 3, 4, 5, 8, 19, 32, 33):
        for step in range(9):
            assert P.slowmo_expgraph_in_peers(m, step) == \
                O.exponential_graph_in_peers(m, step).tolist()[:m], (m, step)
    assert P.slowmo_expgraph_in_peers(32, 4) == [(i - 16) % 32 for i in range(32)]
    with pytest.raises(P.SlowMoError):
        P.slowmo_expgraph_in_peers(0, 0)


def test_exponential_graph_hop_list_over_two_periods():
    """Appendix C.1 names the hops: 2^0 .. 2^floor(log2(m-1)), then again from
    the start.  The library's table against that list written out by hand
    (two full periods and one step more), also for m = 2^p, where no hop may be
    a multiple of m."""
    from oracle_pins import EXPGRAPH_HOPS
    for m, hops in EXPGRAPH_HOPS.items():
        for step in range(2 * len(hops) + 1):
            hop = hops[step % len(hops)]
            got = P.slowmo_expgraph_in_peers(m, step)
            assert got == [(i - hop) % m for i in range(m)], (m, step, got)


def test_null_context_calls_fail_cleanly():
    lib = B.lib()
    assert lib.slowmo_local_step(None, None, 0.1, None) == B.SLOWMO_ERR_ARG
    assert lib.slowmo_outer_step(None, 0.1, None) == B.SLOWMO_ERR_ARG
    assert lib.slowmo_mix_step(None, None, None) == B.SLOWMO_ERR_ARG
    assert lib.slowmo_destroy(None) == B.SLOWMO_OK
    assert lib.slowmo_get_counters(None, None, None, None) == B.SLOWMO_ERR_ARG
    assert "NULL" in P.slowmo_last_error(None)


def _check_cover(runs, m_eff, numel, local):
    """Every (worker, tensor, element) appears in exactly one run."""
    seen = {}
    for tile, worker, tensor, n, off in runs:
        assert n > 0 and off >= 0 and off + n <= numel[tensor]
        key = (worker, tensor)
        seen.setdefault(key, []).append((off, n))
    workers = range(m_eff) if local else [-1]
    for wk in workers:
        for j, total in enumerate(numel):
            pieces = sorted(seen.get((wk, j), []))
            pos = 0
            for off, n in pieces:
                assert off == pos, (wk, j, off, pos)
                pos += n
            assert pos == total, (wk, j)
            for off, n in pieces[1:]:
                assert off % 4 == 0          # a tensor continues 16-byte aligned


@pytest.mark.parametrize("shapes,m", [(S.ragged_mini(), 3), (S.resnet50(), 32),
                                      (S.resnet18(), 8), (S.tiny_flat(), 4)])
def test_tiling_covers_everything_once(shapes, m):
    numel = S.numels(shapes)
    local = P.slowmo_plan_local(m, numel)
    _check_cover(local, m, numel, local=True)
    outer = P.slowmo_plan_outer(m, numel)
    _check_cover(outer, m, numel, local=False)
    # one run per tile, numbered consecutively in launch order (worker-major)
    assert [r[0] for r in local] == list(range(len(local)))
    assert [r[0] for r in outer] == list(range(len(outer)))
    assert [r[1] for r in local] == sorted(r[1] for r in local)
    tile = max(r[3] for r in local)
    assert tile <= 1024 and all(r[4] % tile == 0 for r in local)
    # nearly all tiles are full: small tensors add only a few short ones
    if sum(numel) * m > 1000 * tile:
        assert np.mean([r[3] == tile for r in local]) > 0.95


def test_plan_of_transformer_big_and_1e9():
    numel = S.numels(S.transformer_big())
    assert len(P.slowmo_plan_local(1, numel)) > 0
    lib = B.lib()
    arr = (C.c_int64 * 1)(10 ** 9)
    n_local = lib.slowmo_plan_local(8, 1, arr, None, 0)
    n_outer = lib.slowmo_plan_outer(8, 1, arr, None, 0)
    tile = max(r[3] for r in P.slowmo_plan_local(1, [100_000]))
    assert n_local == 8 * -(-10 ** 9 // tile) and n_outer >= 10 ** 9 // (1 << 20)
    assert lib.slowmo_plan_local(0, 1, arr, None, 0) == -1


def _random_in_peer(rng, m, kind):
    if kind == "any":                       # arbitrary map: trees, cycles, fixed points
        return rng.integers(0, m, size=m)
    if kind == "star":                      # one worker sends to everybody
        return np.zeros(m, dtype=np.int64)
    if kind == "chain":                     # i receives from i+1, the last from nobody
        return np.minimum(np.arange(m) + 1, m - 1)
    perm = rng.permutation(m)               # a permutation, some workers idle
    idle = rng.random(m) < 0.3
    p = np.arange(m)
    act = np.flatnonzero(~idle)
    p[act] = act[rng.permutation(len(act))]
    return p


@pytest.mark.parametrize("kind", ["any", "star", "chain", "perm"])
def test_mix_plan_applied_in_place_equals_the_simultaneous_update(kind):
    """The update order slowmo_plan_mix reports, applied entry by entry to ONE
    array (as the kernel does, fp32, product and sum rounded separately), must
    give what the oracle computes from a saved copy of the old values --
    bit for bit -- for any in-neighbour map (Algorithm C.1, X <- X P^T)."""
    from oracle import slowmo_oracle as O
    lib = O.load("f32")
    rng = np.random.default_rng(7)
    f32 = np.float32
    for m in (1, 2, 3, 5, 8, 17, 64):
        for _ in range(6):
            peers = np.asarray(_random_in_peer(rng, m, kind), dtype=np.int32)
            plan = P.slowmo_plan_mix(peers.tolist())
            assert plan is not None and len(plan) <= m
            d = 5
            x = rng.standard_normal((m, d)).astype(f32)
            want = x.copy()
            w = np.ones(m, f32)
            lib.oracle_mix_step(want.ctypes.data_as(C.c_void_p), w.ctypes.data_as(C.c_void_p),
                                m, d, peers.ctypes.data_as(C.c_void_p))
            got = x.copy()
            seen = set()
            held = first = None          # what the kernel keeps in registers
            saved = [None] * (B.SLOWMO_MIX_SAVED_REGISTERS + 1)      # numbered from 1
            loads = 0
            group_of = {}
            for worker, source, keep, take, flags in plan:
                keep, take = f32(keep), f32(take)
                assert worker not in seen
                if flags & B.SLOWMO_MIX_GROUP_START:    # another launch: registers start empty
                    held = first = None
                    saved = [None] * (B.SLOWMO_MIX_SAVED_REGISTERS + 1)
                    group = len(set(group_of.values()))
                    assert not flags & (B.SLOWMO_MIX_OWN_HELD | B.SLOWMO_MIX_SOURCE_HELD
                                        | B.SLOWMO_MIX_SOURCE_IS_FIRST)
                    assert not (B.SLOWMO_MIX_OWN_SAVED(flags) or B.SLOWMO_MIX_SOURCE_SAVED(flags)
                                or B.SLOWMO_MIX_SAVE(flags))
                group_of[worker] = group
                assert max(B.SLOWMO_MIX_SAVE(flags), B.SLOWMO_MIX_OWN_SAVED(flags),
                           B.SLOWMO_MIX_SOURCE_SAVED(flags)) <= B.SLOWMO_MIX_SAVED_REGISTERS
                if flags & B.SLOWMO_MIX_OWN_HELD:
                    own = held
                elif B.SLOWMO_MIX_OWN_SAVED(flags):
                    own = saved[B.SLOWMO_MIX_OWN_SAVED(flags)]
                    assert own is not None
                else:
                    own = got[worker].copy()
                    loads += 1
                if flags & B.SLOWMO_MIX_OPENS_CYCLE:
                    first = own
                if flags & B.SLOWMO_MIX_NO_SOURCE:
                    assert peers[worker] == worker
                    got[worker] = keep * own
                else:
                    assert source == peers[worker] != worker
                    if B.SLOWMO_MIX_SAVE(flags):
                        assert held is not None
                        saved[B.SLOWMO_MIX_SAVE(flags)] = held
                    if flags & B.SLOWMO_MIX_SOURCE_IS_FIRST:
                        held = first
                    elif B.SLOWMO_MIX_SOURCE_SAVED(flags):
                        held = saved[B.SLOWMO_MIX_SOURCE_SAVED(flags)]
                        assert held is not None
                    elif not flags & B.SLOWMO_MIX_SOURCE_HELD:
                        assert source not in seen       # memory still holds the old value
                        held = got[source].copy()
                        loads += 1
                    got[worker] = keep * own + take * held
                seen.add(worker)
            assert not plan or plan[0][4] & B.SLOWMO_MIX_GROUP_START
            for worker, source, *_ in plan:     # a group is closed under "receives from"
                assert group_of[worker] == group_of.get(source, group_of[worker])
                assert source in group_of
            if kind in ("perm", "chain"):   # nothing is read twice
                assert loads == len(plan)
            if kind == "star" and m > 1:    # the sender is read once for all its receivers
                assert loads == m
            np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
            # workers without an entry are idle: nobody sends to or receives from them
            for i in set(range(m)) - seen:
                assert peers[i] == i and not np.any(np.delete(peers, i) == i)


def test_mix_plan_rejects_bad_maps():
    assert P.slowmo_plan_mix([0, 3]) is None
    assert P.slowmo_plan_mix([-1, 0]) is None
    assert P.slowmo_plan_mix([]) is None


def test_learning_rate_schedules_match_the_oracle_and_reject_bad_arguments():
    """The two schedules of the paper's experiments (Section 4, Appendix A.3):
    the library's value is the oracle's, rounded to float."""
    from oracle import slowmo_oracle as O
    S = 100
    for ms in ([30 * S, 60 * S, 80 * S], [100 * S, 150 * S, 175 * S], []):
        for step in list(range(0, 520, 7)) + [2999, 3000, 3001, 6000, 8000, 8999, 10000, 15000,
                                               17500, 10 ** 7]:
            want = np.float32(O.lr_warmup_step_decay(3.2, 0.1, 5 * S, ms, 0.1, step))
            got = P.slowmo_lr_step_decay(3.2, 0.1, 5 * S, ms, 0.1, step)
            # base_lr and factor reach the library as floats
            assert abs(got - want) <= 2e-7 * want, (ms, step, got, want)
    for step in (0, 1, 1000, 3999, 4000, 4001, 16000, 64000, 10 ** 7):
        want = np.float32(O.lr_warmup_inverse_sqrt(1e-3, 0.0, 4000, step))
        got = P.slowmo_lr_inverse_sqrt(1e-3, 0.0, 4000, step)
        assert abs(got - want) <= 2e-7 * want, (step, got, want)
    assert P.slowmo_lr_inverse_sqrt(1e-3, 0.0, 4000, 16000) == pytest.approx(0.5e-3, rel=1e-6)
    assert P.slowmo_lr_step_decay(3.2, 0.1, 500, [3000, 6000, 8000], 0.1, 6000) == \
        pytest.approx(0.032, rel=1e-6)
    bad = [lambda: P.slowmo_lr_step_decay(0.0, 0.0, 5, [], 0.1, 0),
           lambda: P.slowmo_lr_step_decay(1.0, -0.1, 5, [], 0.1, 0),
           lambda: P.slowmo_lr_step_decay(1.0, 0.0, -1, [], 0.1, 0),
           lambda: P.slowmo_lr_step_decay(1.0, 0.0, 5, [30, 20], 0.1, 0),
           lambda: P.slowmo_lr_step_decay(1.0, 0.0, 5, [10], 0.0, 0),
           lambda: P.slowmo_lr_step_decay(1.0, 0.0, 5, [10], 1.5, 0),
           lambda: P.slowmo_lr_step_decay(1.0, 0.0, 5, [10], 0.1, -1),
           lambda: P.slowmo_lr_step_decay(float("inf"), 0.0, 5, [10], 0.1, 0),
           lambda: P.slowmo_lr_inverse_sqrt(0.0, 0.0, 10, 0),
           lambda: P.slowmo_lr_inverse_sqrt(1e-3, -1.0, 10, 0),
           lambda: P.slowmo_lr_inverse_sqrt(1e-3, 0.0, -1, 0),
           lambda: P.slowmo_lr_inverse_sqrt(1e-3, 0.0, 10, -5)]
    for call in bad:
        with pytest.raises(P.SlowMoError) as e:
            call()
        assert e.value.status == B.SLOWMO_ERR_ARG
