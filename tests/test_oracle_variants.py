"""Pins for the variants of the method that the paper studies next to its main configuration:
average weighted merging and the largest-index pivot (Section 4.2, first experiment), the
random pivot (Section 5.4, "Choice of Pivotal State").  CPU only."""
import json
import math
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


# ---------------------------------------------------------------------------------------------
# the anchor reading of Algorithm 1: similarity to the set's own top token
# ---------------------------------------------------------------------------------------------

def _anchor(K, mass, thr=0.75, recent=0.17, heavy=0.12, budget=0.5, enforce=False, lens=None, dtype="f32"):
    return ref.identify_sets(K, mass, dtype, budget, recent, heavy, thr, enforce, None, lens, set_rule=ref.SETS_ANCHOR)


def _restated_anchor_sets(k64, prot, thr):
    """The same rule from the full cosine matrix (numpy): a set's extent is the trailing run of
    admissible columns in its anchor's row."""
    n = len(k64)
    norm = np.sqrt((k64 * k64).sum(1))
    with np.errstate(divide="ignore", invalid="ignore"):
        C = np.where((norm[:, None] > 0) & (norm[None, :] > 0), (k64 @ k64.T) / (norm[:, None] * norm[None, :]), 0.0)
    starts, i = [], n - 1
    while i >= 0:
        s = i
        if not prot[i]:
            ok = (C[i, :i] > thr) & ~prot[:i].astype(bool)
            bad = np.flatnonzero(~ok)
            s = (bad[-1] + 1) if len(bad) else 0
        starts.append(s)
        i = s - 1
    return starts[::-1]


@pytest.mark.parametrize("dtype,seed", [("f32", 0), ("f16", 1), ("bf16", 2)])
def test_anchor_sets_match_the_matrix_restatement_and_invariants(dtype, seed):
    n = 700
    parts = [synth.gen_slice(40 + seed, h, n, 128, 1, None, dtype) for h in range(3)]
    K = np.stack([p[1] for p in parts])[None]
    mass = np.random.default_rng(seed).uniform(0.5, 2.0, (1, 3, n))
    for thr in (0.75, 0.5, 0.9):
        o = _anchor(K, mass, thr, dtype=dtype)
        for h in range(3):
            M = int(o["n_sets"][0, h])
            want = _restated_anchor_sets(synth.to_f64(K[0, h], dtype), o["protected"][0, h], thr)
            if o["anchor_margin"][0, h] > 1e-12:             # otherwise a decision sits on the threshold
                assert o["set_start"][0, h, :M].tolist() == want
            sid = o["set_id"][0, h]
            assert sid[0] == 0 and sid[-1] == M - 1 and set(np.diff(sid)) <= {0, 1}
            prot = np.flatnonzero(o["protected"][0, h])
            assert len(prot) == math.floor(0.17 * n) + math.floor(0.12 * n)
            sizes = np.bincount(sid, minlength=M)
            assert (sizes[sid[prot]] == 1).all()             # conserved tokens are singletons
            assert ((o["pivot"][0, h, :M] >= o["set_start"][0, h, :M])).all()


def test_anchor_sets_on_a_slowly_turning_key():
    # keys on a circle, turning by theta per token: neighbours always pass the threshold, so the
    # adjacent chain gives one set; against the anchor only floor(acos(eps)/theta) tokens do
    n, theta, eps = 100, 0.1, 0.75
    t = np.arange(n)
    K = np.zeros((1, 1, n, 128), np.float32)
    K[0, 0, :, 0], K[0, 0, :, 1] = np.cos(theta * t), np.sin(theta * t)
    mass = np.ones((1, 1, n))
    kw = dict(recent=0.0, heavy=0.0, budget=1.0)
    chain = ref.identify_sets(K, mass, "f32", 1.0, 0.0, 0.0, eps, False, None)
    assert chain["n_sets"][0, 0] == 1
    o = _anchor(K, mass, eps, **kw)
    per_set = math.floor(math.acos(eps) / theta) + 1         # the anchor and the tokens within the angle
    assert per_set == 8
    M = math.ceil(n / per_set)
    assert o["n_sets"][0, 0] == M
    # sets are cut from the last token downwards; the first set takes what is left
    assert o["set_start"][0, 0, :M].tolist() == [0] + list(range(n - per_set * (M - 1), n, per_set))


def test_anchor_special_cases():
    n = 64
    rng = np.random.default_rng(3)
    mass = rng.uniform(1, 2, (1, 1, n))
    K = np.tile(rng.standard_normal(128).astype(np.float32), (1, 1, n, 1))
    o = _anchor(K, mass, 0.75, recent=0.1, heavy=0.1)        # identical keys: one set per free stretch
    free = ~o["protected"][0, 0].astype(bool)
    stretches = int(np.sum(free & ~np.concatenate([[False], free[:-1]])))
    assert o["n_sets"][0, 0] == stretches + int((~free).sum())
    K = np.zeros((1, 1, n, 128), np.float32)
    K[0, 0, np.arange(n), np.arange(n)] = 1.0                # orthogonal keys: all singletons
    assert _anchor(K, mass, 0.75)["n_sets"][0, 0] == n
    K = rng.standard_normal((1, 1, n, 128)).astype(np.float32)
    assert _anchor(K, mass, 1.0, recent=0, heavy=0)["n_sets"][0, 0] == n          # nothing exceeds 1
    assert _anchor(K, mass, -1.5, recent=0, heavy=0)["n_sets"][0, 0] == 1         # everything exceeds -1.5
    # strictness: similarity exactly at the threshold does not join
    K = np.zeros((1, 1, 3, 128), np.float32)
    K[0, 0, :, 0] = [1, 1, 1]
    K[0, 0, 0, 1] = 1.0                                      # cos(k2, k0) = cos(k1, k0) = 1/sqrt(2)
    c = float(np.float64(1.0) / np.sqrt(np.float64(2.0)))
    m3 = np.ones((1, 1, 3))
    assert _anchor(K, m3, c, recent=0, heavy=0)["set_start"][0, 0, :2].tolist() == [0, 1]
    assert _anchor(K, m3, np.nextafter(c, 0), recent=0, heavy=0)["n_sets"][0, 0] == 1


def test_anchor_rule_reports_a_missed_budget_and_truncates():
    n = 300
    parts = synth.gen_slice(50, 0, n, 128, 1, None, "f32")
    K = parts[1][None, None]
    mass = np.random.default_rng(4).uniform(1, 2, (1, 1, n))
    o = ref.identify_sets(K, mass, "f32", 0.2, 0.1, 0.05, 0.95, True, 60, None, set_rule=ref.SETS_ANCHOR)
    M = int(o["n_sets"][0, 0])
    assert M > 60 and o["status"][0, 0] == (ref.SLICE_INFEASIBLE | ref.SLICE_TRUNCATED)
    free = _anchor(K, mass, 0.95, recent=0.1, heavy=0.05)
    assert np.array_equal(free["set_start"][0, 0, :61], o["set_start"][0, 0])     # no fallback: same sets, cut off


# ---------------------------------------------------------------------------------------------
# comparison workload: eviction by aggregated attention score (Section 2.3)
# ---------------------------------------------------------------------------------------------

def test_eviction_keeps_the_recent_window_and_the_largest_scores():
    rng = np.random.default_rng(5)
    n, d = 500, 128
    K = rng.standard_normal((1, 2, n, d)).astype(np.float32)
    V = rng.standard_normal((1, 2, n, d)).astype(np.float32)
    mass = rng.uniform(0, 1, (1, 2, n))
    mass[0, 1, 100:140] = mass[0, 1, 100]                    # a block of ties
    for budget, recent in ((0.5, 0.17), (0.35, 0.08), (0.1, 0.3), (1.0, 0.0)):
        cap_rows = math.floor(budget * n)
        kept, n_kept, ko, vo = ref.evict(K, V, mass, "f32", budget, recent, cap_rows)
        for h in range(2):
            n_recent = min(math.floor(recent * n), cap_rows)
            pre = n - n_recent
            k = min(cap_rows - n_recent, pre)
            # restated with numpy: a stable sort by descending score keeps the lower index first
            order = np.argsort(-mass[0, h, :pre], kind="stable")[:k]
            want = np.sort(np.concatenate([order, np.arange(pre, n)]))
            assert n_kept[0, h] == len(want) == cap_rows
            assert np.array_equal(kept[0, h, :len(want)], want)
            assert np.array_equal(ko[0, h, :len(want)], K[0, h, want].astype(np.float64))
            assert np.array_equal(vo[0, h, :len(want)], V[0, h, want].astype(np.float64))
    kept, n_kept, _, _ = ref.evict(K, V, mass, "f32", 0.5, 0.17, 300, seq_lens=[37])
    assert n_kept[0, 0] == 18 and (kept[0, :, 18:] == -1).all() and kept[0, 0, 17] == 36


# ---------------------------------------------------------------------------------------------
# comparison workload: value-only merging into the nearest kept token (Section 2.3; a reading)
# ---------------------------------------------------------------------------------------------

def _values_by_hand(n, keep_positions, d=128):
    """Scores that make the eviction policy keep exactly keep_positions (no recent window), values
    whose first element is the token index and whose second is 1."""
    K = np.zeros((1, 1, n, d), np.float32)
    V = np.zeros((1, 1, n, d), np.float32)
    V[0, 0, :, 0] = np.arange(n)
    V[0, 0, :, 1] = 1.0
    mass = np.zeros((1, 1, n))
    mass[0, 0, list(keep_positions)] = 1.0
    K[0, 0, :, 2] = np.arange(n)                             # a key tells its position
    return K, V, mass


def test_value_merge_worked_examples():
    # kept 1 and 6 of 8 tokens: tokens 0..3 are nearest to 1 (token 3: distance 2 against 3), 4..7 to 6
    K, V, mass = _values_by_hand(8, (1, 6))
    kept, n_kept, ko, vo, cnt = ref.evict_merge_values(K, V, mass, "f32", 0.25, 0.0, 2)
    assert n_kept[0, 0] == 2 and kept[0, 0].tolist() == [1, 6] and cnt[0, 0].tolist() == [4, 4]
    assert vo[0, 0, :, 0].tolist() == [1.5, 5.5] and vo[0, 0, :, 1].tolist() == [1.0, 1.0]
    assert ko[0, 0, :, 2].tolist() == [1.0, 6.0]             # keys: the kept rows, untouched
    # kept 1 and 5: token 3 is as far from 1 as from 5 and goes to the later one
    K, V, mass = _values_by_hand(8, (1, 5))
    kept, n_kept, ko, vo, cnt = ref.evict_merge_values(K, V, mass, "f32", 0.25, 0.0, 2)
    assert cnt[0, 0].tolist() == [3, 5]
    assert vo[0, 0, :, 0].tolist() == [1.0, (3 + 4 + 5 + 6 + 7) / 5]
    # a single kept token takes everything; tokens after the last kept one go to it
    K, V, mass = _values_by_hand(9, (2,))
    kept, n_kept, ko, vo, cnt = ref.evict_merge_values(K, V, mass, "f32", 0.12, 0.0, 1)
    assert kept[0, 0].tolist() == [2] and cnt[0, 0].tolist() == [9] and vo[0, 0, 0, 0] == 4.0
    # everything kept: the identity
    K, V, mass = _values_by_hand(8, range(8))
    kept, n_kept, ko, vo, cnt = ref.evict_merge_values(K, V, mass, "f32", 1.0, 0.0, 8)
    assert np.array_equal(vo[0, 0], V[0, 0].astype(np.float64)) and (cnt == 1).all()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_value_merge_equals_means_over_midpoint_ranges(dtype):
    """The nearest kept token by position is the same as cutting the sequence half-way between
    neighbouring kept tokens (the token in the middle of an even gap goes to the later one): the
    ranges are rebuilt with numpy from the kept positions and averaged."""
    n, H = 700, 3
    parts = [synth.gen_slice(9, h, n, 128, 1, None, dtype) for h in range(H)]
    K = np.stack([p[1] for p in parts])[None]
    V = np.stack([p[2] for p in parts])[None]
    mass = np.random.default_rng(2).uniform(0, 1, (1, H, n))
    # bf16 travels as its 16 bits; the upper half of an fp32 is the same number
    Vf = (V.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if dtype == "bf16" else V.astype(np.float64)
    for budget, recent, lens in ((0.5, 0.17, None), (0.1, 0.02, None), (0.35, 0.08, [413])):
        cap = math.floor(budget * n)
        kept, n_kept, ko, vo, cnt = ref.evict_merge_values(K, V, mass, dtype, budget, recent, cap, seq_lens=lens)
        k2, n2, ko2, _ = ref.evict(K, V, mass, dtype, budget, recent, cap, seq_lens=lens)
        assert np.array_equal(kept, k2) and np.array_equal(n_kept, n2) and np.array_equal(ko, ko2)
        nn = n if lens is None else lens[0]
        for h in range(H):
            m = int(n_kept[0, h])
            p = kept[0, h, :m].astype(np.int64)
            edges = np.concatenate([[0], -((-(p[:-1] + p[1:])) // 2), [nn]])      # ceil of the midpoints
            assert np.array_equal(cnt[0, h, :m], np.diff(edges))
            for s in range(m):
                want = Vf[0, h, edges[s]:edges[s + 1]].mean(axis=0)
                np.testing.assert_allclose(vo[0, h, s], want, rtol=1e-12, atol=1e-13)
            # nothing is lost: the means weighted by their counts add up to the sum of all values
            np.testing.assert_allclose((vo[0, h, :m] * cnt[0, h, :m, None]).sum(0), Vf[0, h, :nn].sum(0), rtol=1e-10, atol=1e-10)
