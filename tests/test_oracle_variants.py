"""Pins for the variants of the method that the paper studies next to its main configuration:
average weighted merging and the largest-index pivot (Section 4.2, first experiment), the
random pivot (Section 5.4, "Choice of Pivotal State").  CPU only."""
import json
import os

import numpy as np
import pytest

from oracle import ref
from paper_2407_08454_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64.json")
M64 = (1 << 64) - 1


def _slice(seed, n, dtype="f32", H=2):
    parts = [synth.gen_slice(seed, h, n, 128, 1, None, dtype) for h in range(H)]
    return np.stack([p[1] for p in parts])[None], np.stack([p[2] for p in parts])[None]


def _identify(K, mass, rule, seed=0, budget=0.5):
    return ref.identify_sets(K, mass, "f32", budget, 0.17, 0.12, 0.75, True, None, None, pivot_rule=rule,
                             pivot_seed=seed)


def test_generator_reproduces_the_published_outputs():
    g = json.load(open(GOLDEN))
    gamma = int(g["gamma"], 16)
    for k, want in enumerate(g["seed0_outputs"]):
        assert ref.splitmix64_at((k * gamma) & M64) == int(want, 16)


def test_random_offset_is_the_scaled_upper_half_of_the_draw():
    rng = np.random.default_rng(0)
    for _ in range(200):
        seed, bh, lo, m = int(rng.integers(0, 1 << 62)), int(rng.integers(0, 5000)), int(rng.integers(0, 1 << 20)), \
            int(rng.integers(1, 3000))
        z = (seed + ((bh << 32) | lo)) & M64                 # restated with Python integers
        z = (z + 0x9E3779B97F4A7C15) & M64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        z ^= z >> 31
        assert ref.random_offset(seed, bh, lo, m) == ((z >> 32) * m) >> 32
    counts = np.bincount([ref.random_offset(7, 3, lo, 10) for lo in range(20000)], minlength=10)
    assert counts.min() > 1800 and counts.max() < 2200     # uniform over the set's members


def test_pivot_rules_change_only_the_pivot():
    n = 600
    K, _ = _slice(31, n)
    mass = np.random.default_rng(1).uniform(0.5, 2.0, (1, 2, n))
    base = _identify(K, mass, ref.PIVOT_MAX_SCORE)
    last = _identify(K, mass, ref.PIVOT_LAST)
    rnd = _identify(K, mass, ref.PIVOT_RANDOM, seed=5)
    rnd2 = _identify(K, mass, ref.PIVOT_RANDOM, seed=5)
    rnd3 = _identify(K, mass, ref.PIVOT_RANDOM, seed=6)
    for o in (last, rnd, rnd3):
        for k in ("set_id", "set_start", "n_sets", "status"):
            assert np.array_equal(o[k], base[k])
    assert np.array_equal(rnd["pivot"], rnd2["pivot"]) and not np.array_equal(rnd["pivot"], rnd3["pivot"])
    for h in range(2):
        M = int(base["n_sets"][0, h])
        st = base["set_start"][0, h]
        ends = np.append(st[1:M], n)
        assert np.array_equal(last["pivot"][0, h, :M], ends - 1)          # largest index of every set
        pr = rnd["pivot"][0, h, :M]
        assert ((pr >= st[:M]) & (pr < ends)).all()
        want = [st[s] + ref.random_offset(5, h, int(st[s]), int(ends[s] - st[s])) for s in range(M)]
        assert np.array_equal(pr, want)
        multi = ends - st[:M] > 1
        assert (pr[multi] != base["pivot"][0, h, :M][multi]).any()       # not the arg-max in disguise
        assert np.array_equal(pr[~multi], st[:M][~multi])                 # a singleton's only choice


@pytest.mark.parametrize("scale", [True, False])
def test_average_weights_give_the_mean(scale):
    n = 400
    K, V = _slice(32, n)
    mass = np.random.default_rng(2).uniform(0.5, 2.0, (1, 2, n))
    o = _identify(K, mass, ref.PIVOT_LAST)
    ko, vo, w = ref.merge(K, V, "f32", o["set_start"], o["pivot"], o["n_sets"], weights=ref.WEIGHTS_AVERAGE,
                          value_scale_by_set_size=scale)
    for h in range(2):
        M = int(o["n_sets"][0, h])
        st = np.append(o["set_start"][0, h, :M], n)
        for s in range(M):
            lo, hi = st[s], st[s + 1]
            np.testing.assert_allclose(w[0, h, lo:hi], 1.0 / (hi - lo), rtol=1e-15)
            np.testing.assert_allclose(ko[0, h, s], K[0, h, lo:hi].astype(np.float64).mean(0), rtol=1e-12, atol=1e-14)
            vref = V[0, h, lo:hi].astype(np.float64).sum(0) if scale else V[0, h, lo:hi].astype(np.float64).mean(0)
            np.testing.assert_allclose(vo[0, h, s], vref, rtol=1e-12, atol=1e-14)
    # the pivot does not matter for uniform weights
    o2 = _identify(K, mass, ref.PIVOT_RANDOM, seed=9)
    ko2, vo2, _ = ref.merge(K, V, "f32", o2["set_start"], o2["pivot"], o2["n_sets"], weights=ref.WEIGHTS_AVERAGE,
                            value_scale_by_set_size=scale)
    assert np.array_equal(ko, ko2) and np.array_equal(vo, vo2)


def test_gaussian_weights_follow_the_chosen_pivot():
    # two far-apart clusters in one set: the merged key sits with the pivot's cluster
    K = np.zeros((1, 1, 6, 128), np.float32)
    K[0, 0, :3, 0] = [1.0, 1.1, 0.9]
    K[0, 0, 3:, 1] = [5.0, 5.1, 4.9]
    V = np.ones_like(K)
    st = np.array([[[0, 6]]], np.int32)
    for p, axis in ((0, 0), (5, 1)):
        ko, _, w = ref.merge(K, V, "f32", st, np.array([[[p]]], np.int32), np.array([[1]], np.int32))
        assert w[0, 0, p] == w[0, 0].max() and ko[0, 0, 0, axis] > 0.8 and ko[0, 0, 0, 1 - axis] < 0.5
