"""Seeded input generators and shape lists (CPU only)."""
import numpy as np
import torch

from slowmo_inputs import generator as G
from slowmo_inputs import shapes as S
from slowmo_inputs import workloads as W


def test_shape_list_totals():
    # (tensors, elements) of the architectures named by the benchmark configs
    for fn, n_t, n_e in ((S.resnet18, 62, 11_689_512), (S.resnet50, 161, 25_557_032),
                         (S.transformer_big, 253, 209_911_808)):
        s = fn()
        assert len(s) == n_t and S.total(s) == n_e
    assert sum(1 for n in S.numels(S.resnet50()) if n <= 2048) == 107
    assert S.total(S.tiny_flat()) == 65536 and S.total(S.stress_flat()) == 10 ** 9
    assert 0 in S.numels(S.ragged_mini()) and 1 in S.numels(S.ragged_mini())


def test_mix64_known_values():
    # SplitMix64 seeded with 0: the first outputs of the published generator
    # are mix64(k * 0x9E3779B97F4A7C15), k = 1, 2, 3.
    g = 0x9E3779B97F4A7C15
    got = [int(G.mix64(np.uint64((k * g) & (2 ** 64 - 1)))) for k in (1, 2, 3)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_unit_normal_moments_and_exactness():
    idx = np.arange(2_000_000, dtype=np.int64)
    n = G.unit_normal(123, 3, 7, idx)
    assert n.dtype == np.float32
    assert abs(float(n.mean())) < 3e-3 and abs(float(n.var()) - 1.0) < 5e-3
    assert float(np.abs(n).max()) < 6.0
    # every value is an integer multiple of 2**-16: exactly representable
    assert np.array_equal(n.astype(np.float64) * 65536.0, np.round(n.astype(np.float64) * 65536.0))
    # excess kurtosis of Irwin-Hall(12) is -0.1
    k = float(((n.astype(np.float64)) ** 4).mean()) - 3.0
    assert abs(k + 0.1) < 0.03


def test_streams_are_distinct_and_reproducible():
    idx = np.arange(4096, dtype=np.int64)
    a = G.unit_normal(1, 0, 0, idx)
    assert np.array_equal(a, G.unit_normal(1, 0, 0, idx))
    for other in (G.unit_normal(2, 0, 0, idx), G.unit_normal(1, 1, 0, idx),
                  G.unit_normal(1, 0, 1, idx)):
        assert abs(float(np.corrcoef(a, other)[0, 1])) < 0.06
    # a value depends on its global index only, not on which slice asked for it
    sub = np.array([5, 77, 4095], dtype=np.int64)
    assert np.array_equal(G.unit_normal(1, 0, 0, sub), a[sub])
    big = np.array([2 ** 33 + 5], dtype=np.int64)       # indices beyond 32 bits
    assert np.isfinite(G.unit_normal(1, 0, 0, big)).all()


def test_bf16_rounding_matches_library_and_widening_is_exact():
    x = (np.float32(0.1) * G.unit_normal(9, 0, 0, np.arange(200_000))).astype(np.float32)
    ties = np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-39], dtype=np.float32)
    x = np.concatenate([x, ties])
    bits = G.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())
    wide = G.bf16_bits_to_f32(bits)
    assert np.array_equal(wide, want.to(torch.float32).numpy())
    g = G.gradient(9, 1, 2, np.arange(1000), 0.1, bf16=True)
    assert np.array_equal(G.bf16_bits_to_f32(G.f32_to_bf16_bits(g)), g)


def test_workloads_follow_the_benchmark_configs():
    t, r18, r50, tb, st = W.tiny(), W.resnet18(), W.resnet50(), W.transformer_big(), W.stress()
    assert (t.m, t.d, t.tau, t.beta, t.rounds) == (4, 65536, 12, 0.7, 10)
    assert (r18.m, r18.d, r18.tau, r18.beta) == (8, 11_689_512, 12, 0.6)
    assert (r50.m, r50.d, r50.tau, r50.beta) == (32, 25_557_032, 12, 0.6)
    assert (tb.m, tb.d, tb.tau, tb.base, tb.grad_dtype) == (8, 209_911_808, 48, "adam", "bf16")
    assert (st.m, st.d, st.tau, st.lr) == (8, 10 ** 9, 48, 0.05)
    assert r50.updates_per_round == 32 * 25_557_032 * 12
    assert len({w.seed for w in (t, r18, r50, tb, st)}) == 5
    assert t.tensor_starts.tolist() == [0]
    assert r18.tensor_starts[1] == 64 * 3 * 7 * 7
