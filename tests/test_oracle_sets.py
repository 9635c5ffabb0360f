"""Pins for the oracle's merging-set identification (Section 3.2; Section 4.1 Def. 4.1,
Algorithm 1; conserved top-k / recent states, Sections 4.1 and 5.1; pivot, Eq. (7)).
CPU only: brute-force enumeration of all contiguous partitions, direction invariance,
special cases, invariants, and the printed hyper-parameters."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import ref
from paper_2407_08454_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _cos(K64):
    num = (K64[1:] * K64[:-1]).sum(1)
    den = np.linalg.norm(K64[1:], axis=1) * np.linalg.norm(K64[:-1], axis=1)
    out = np.zeros(len(K64))
    ok = den > 0
    out[1:][ok] = num[ok] / den[ok]
    return out


def _protected(mass, n, recent_ratio, heavy_ratio):
    n_recent = math.floor(recent_ratio * n)
    n_heavy = min(math.floor(heavy_ratio * n), n - n_recent)
    prot = np.zeros(n, bool)
    prot[n - n_recent:] = True
    order = sorted(range(n - n_recent), key=lambda j: (-mass[j], j))
    prot[order[:n_heavy]] = True
    return prot


def _forward_runs(sim, prot, eps):
    """Boundary flags by a forward scan of maximal runs (the other scan direction)."""
    n = len(prot)
    bnd = np.ones(n, bool)
    for j in range(1, n):
        bnd[j] = not (sim[j] > eps and not prot[j - 1] and not prot[j])
    return bnd


def _bnd_from_set_id(set_id, n):
    bnd = np.ones(n, bool)
    bnd[1:] = set_id[1:n] != set_id[:n - 1]
    return bnd


def _run(K, mass, dtype="f32", budget=1.0, recent=0.0, heavy=0.0, eps=0.75, enforce=False, cap_rows=None,
         seq_lens=None):
    return ref.identify_sets(K, mass, dtype, budget, recent, heavy, eps, enforce, cap_rows, seq_lens)


def _check_invariants(o, b, h, n, mass, prot):
    sid = o["set_id"][b, h]
    M = int(o["n_sets"][b, h])
    st = o["set_start"][b, h]
    pv = o["pivot"][b, h]
    assert (sid[n:] == -1).all()
    if n == 0:
        assert M == 0
        return
    # contiguous, disjoint, covering: ids start at 0 and grow by 0 or 1
    assert sid[0] == 0 and sid[n - 1] == M - 1
    assert set(np.diff(sid[:n]).tolist()) <= {0, 1}
    shown = min(M, o["cap_rows"])
    for s in range(shown):
        lo, hi = st[s], st[s + 1]
        assert (sid[lo:hi] == s).all() and lo < hi
        assert lo <= pv[s] < hi                                 # pivot inside its set
        seg = mass[lo:hi]
        assert pv[s] == lo + int(np.argmax(seg))                # first maximum
    if M <= o["cap_rows"]:
        assert st[M] == n and (pv[M:] == -1).all()
    for j in np.flatnonzero(prot):                              # conserved tokens are singletons
        assert (sid[:n] == sid[j]).sum() == 1


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_enumeration_of_partitions(seed):
    rng = np.random.default_rng(seed)
    n, d = int(rng.integers(2, 12)), 6
    q, k, v, _ = synth.gen_slice(100 + seed, 0, n, d, 1, 0.9, "f32")
    mass = rng.random(n)
    recent, heavy, eps = [(0, 0, 0.75), (0.2, 0.1, 0.75), (0.1, 0.3, 0.5)][seed % 3]
    o = _run(k[None, None], mass[None, None], recent=recent, heavy=heavy, eps=eps)
    sim = _cos(k.astype(np.float64))
    prot = _protected(mass, n, recent, heavy)
    np.testing.assert_allclose(o["sim"][0, 0], sim, atol=1e-15)
    assert (o["protected"][0, 0].astype(bool) == prot).all()
    ok = []
    for bits in itertools.product([False, True], repeat=n - 1):
        bnd = (True,) + bits
        good = True
        for j in range(1, n):
            mergeable = (not prot[j - 1]) and (not prot[j]) and sim[j] > eps
            if bnd[j] == mergeable:     # a boundary where merging is due, or a merge where it is not
                good = False
                break
        if good:
            ok.append(np.array(bnd))
    assert len(ok) == 1
    assert (_bnd_from_set_id(o["set_id"][0, 0], n) == ok[0]).all()
    assert o["n_sets"][0, 0] == ok[0].sum()
    _check_invariants(o, 0, 0, n, mass, prot)


@pytest.mark.parametrize("dtype,seed", [("f32", 0), ("f16", 1), ("bf16", 2)])
def test_direction_invariance_and_invariants_on_workload(dtype, seed):
    n = 700
    q, k, v, _ = synth.gen_slice(seed, 3, n, 128, 1, None, dtype)
    mass = np.random.default_rng(seed).random(n) ** 4
    o = _run(k[None, None], mass[None, None], dtype, budget=0.5, recent=0.17, heavy=0.12, enforce=True,
             cap_rows=350)
    sim = _cos(synth.to_f64(k, dtype))
    prot = _protected(mass, n, 0.17, 0.12)
    assert prot.sum() == math.floor(0.17 * n) + math.floor(0.12 * n)
    fwd = _forward_runs(sim, prot, 0.75)
    assert o["status"][0, 0] == ref.SLICE_OK
    assert (_bnd_from_set_id(o["set_id"][0, 0], n) == fwd).all()
    assert o["n_sets"][0, 0] <= 350
    _check_invariants(o, 0, 0, n, mass, prot)


def test_special_cases():
    n, d = 40, 8
    mass = np.linspace(2.0, 1.0, n)
    # identical keys: one set per unprotected stretch
    K = np.tile(np.arange(1, d + 1, dtype=np.float32), (n, 1))
    o = _run(K[None, None], mass[None, None], recent=0.1, heavy=0.05)   # protects 36..39 and 0,1
    assert o["n_sets"][0, 0] == 4 + 2 + 1
    # mutually orthogonal keys: all singletons
    K = np.zeros((8, 8), np.float32)
    K[np.arange(8), np.arange(8)] = np.arange(1, 9)
    o = _run(K[None, None], np.ones((1, 1, 8)), eps=0.0)
    assert o["n_sets"][0, 0] == 8 and (o["sim"] == 0).all()
    # threshold below -1: everything unprotected merges; threshold >= 1: identity pass
    rng = np.random.default_rng(0)
    K = rng.standard_normal((n, d)).astype(np.float32)
    o = _run(K[None, None], mass[None, None], eps=-1.5)
    assert o["n_sets"][0, 0] == 1 and o["pivot"][0, 0, 0] == 0
    o = _run(K[None, None], mass[None, None], eps=1.0)
    assert o["n_sets"][0, 0] == n and (o["pivot"][0, 0] == np.arange(n)).all()
    # zero-norm key: similarity 0 on both sides, so it splits for any threshold >= 0
    K[5] = 0
    o = _run(K[None, None], mass[None, None], eps=-1.5)
    assert o["sim"][0, 0, 5] == 0 and o["sim"][0, 0, 6] == 0 and o["n_sets"][0, 0] == 1
    o = _run(K[None, None], mass[None, None], eps=0.0)
    sid = o["set_id"][0, 0]
    assert sid[5] != sid[4] and sid[6] != sid[5]


def test_threshold_is_strict():
    # cos((1,0),(3,4)) = 3/5 exactly as computed in IEEE double
    K = np.array([[1, 0], [3, 4]], np.float32)
    m = np.ones((1, 1, 2))
    assert _run(K[None, None], m, eps=0.6)["n_sets"][0, 0] == 2
    assert _run(K[None, None], m, eps=np.nextafter(0.6, 0))["n_sets"][0, 0] == 1


def test_ties_topk_lower_index_and_pivot_first_maximum():
    n = 10
    K = np.ones((n, 4), np.float32)
    mass = np.array([1, 3, 3, 3, 1, 1, 2, 2, 1, 1], float)
    o = _run(K[None, None], mass[None, None], heavy=0.2)          # 2 of the three 3's: indices 1, 2
    assert o["protected"][0, 0].tolist() == [0, 1, 1, 0, 0, 0, 0, 0, 0, 0]
    # sets: {0} {1} {2} {3..9}; pivot of the last is index 3 (mass 3)
    assert o["n_sets"][0, 0] == 4 and o["pivot"][0, 0, :4].tolist() == [0, 1, 2, 3]
    o = _run(K[None, None], np.array([1, 1, 2, 2, 1.0, 2, 0, 0, 0, 0])[None, None])
    assert o["n_sets"][0, 0] == 1 and o["pivot"][0, 0, 0] == 2


def test_printed_hyperparameters_give_the_expected_counts():
    g = json.load(open(os.path.join(GOLDEN, "presets.json")))
    assert g["threshold"] == 0.75
    want = {(0.5, 4096): (696, 491, 2048), (0.35, 4096): (327, 81, 1433), (0.5, 512): (87, 61, 256)}
    for sc in g["scenarios"]:
        for n in (4096, 512):
            if (sc["budget"], n) not in want:
                continue
            K = np.ones((1, 1, n, 2), np.float32)
            mass = np.arange(n, 0, -1, dtype=float)[None, None]
            o = _run(K, mass, budget=sc["budget"], recent=sc["recent_ratio"], heavy=sc["heavy_ratio"],
                     eps=g["threshold"], enforce=True, cap_rows=n)
            nr, nh, cap = want[(sc["budget"], n)]
            p = o["protected"][0, 0]
            assert p[n - nr:].all() and p[:nh].all() and p.sum() == nr + nh
            # identical keys: one big set between the heavy prefix and the recent window
            assert o["n_sets"][0, 0] == nr + nh + 1 <= cap
        # the conserved fraction must leave room for merged states inside the budget
        assert sc["recent_ratio"] + sc["heavy_ratio"] < sc["budget"]


@pytest.mark.parametrize("seed", range(10))
def test_budget_fallback_equals_largest_feasible_threshold(seed):
    """With distinct similarities, removing the most similar boundaries until the budget is
    met equals running the plain rule at the largest threshold <= epsilon that meets it."""
    rng = np.random.default_rng(seed)
    n, d = int(rng.integers(6, 40)), 5
    K = rng.standard_normal((n, d)).astype(np.float32)
    mass = rng.random(n)
    recent, heavy, eps, budget = 0.1, 0.1, 0.6, 0.5
    cap = math.floor(budget * n)
    o = _run(K[None, None], mass[None, None], budget=budget, recent=recent, heavy=heavy, eps=eps,
             enforce=True, cap_rows=n)
    sim = _cos(K.astype(np.float64))
    prot = _protected(mass, n, recent, heavy)
    cands = sorted({eps} | {np.nextafter(s, -np.inf) for s in sim[1:] if s <= eps}, reverse=True)
    found = None
    for e in cands:                                   # thresholds from epsilon downwards
        if _forward_runs(sim, prot, e).sum() <= cap:
            found = e
            break
    if found is None:
        assert o["status"][0, 0] & ref.SLICE_INFEASIBLE
        want = _forward_runs(sim, prot, -2.0)         # everything mergeable is merged
    else:
        assert not (o["status"][0, 0] & ref.SLICE_INFEASIBLE)
        want = _forward_runs(sim, prot, found)
        assert bool(o["status"][0, 0] & ref.SLICE_FALLBACK) == (found != eps)
        if found != eps:
            assert o["n_sets"][0, 0] == cap
            assert np.nextafter(o["min_removed_sim"][0, 0], -np.inf) == found
    assert (_bnd_from_set_id(o["set_id"][0, 0], n) == want).all()
    _check_invariants(o, 0, 0, n, mass, prot)


def test_fallback_ties_prefer_the_higher_index():
    # keys alternate between two directions: all boundary similarities are equal (0)
    n = 8
    K = np.zeros((n, 2), np.float32)
    K[0::2, 0] = 1
    K[1::2, 1] = 1
    o = _run(K[None, None], np.ones((1, 1, n)), budget=0.75, eps=0.5, enforce=True, cap_rows=n)
    # 8 singletons, cap 6: remove the boundaries at 7 and 6
    assert o["n_sets"][0, 0] == 6 and o["set_id"][0, 0].tolist() == [0, 1, 2, 3, 4, 5, 5, 5]


def test_truncation_and_ragged():
    N, d = 30, 4
    rng = np.random.default_rng(3)
    K = rng.standard_normal((3, 2, N, d)).astype(np.float32)
    mass = rng.random((3, 2, N))
    lens = np.array([30, 11, 0], np.int32)
    o = _run(K, mass, eps=0.2, cap_rows=5, seq_lens=lens)
    for b in range(3):
        for h in range(2):
            n = lens[b]
            full = _run(K[b:b + 1, h:h + 1, :n].copy(), mass[b:b + 1, h:h + 1, :n].copy(), eps=0.2)
            M = full["n_sets"][0, 0]
            assert o["n_sets"][b, h] == M
            assert (o["set_id"][b, h, :n] == full["set_id"][0, 0]).all() and (o["set_id"][b, h, n:] == -1).all()
            assert bool(o["status"][b, h] & ref.SLICE_TRUNCATED) == (M > 5)
            k = min(M, 5)
            assert (o["pivot"][b, h, :k] == full["pivot"][0, 0, :k]).all()
            assert (o["set_start"][b, h, :k + 1] == full["set_start"][0, 0, :k + 1]).all()
            if M <= 5:
                assert (o["set_start"][b, h, k:] == n).all()
