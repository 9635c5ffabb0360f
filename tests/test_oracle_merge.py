"""Pins for the oracle's Gaussian-kernel weighted merging (Section 4.2: Def. 4.2 Eq. (4),
Eq. (5)-(6), Algorithm 2) and for the whole pass.  CPU only: closed forms that follow
from the sigma reading, a library softmax for the fixed-sigma mode, a direct numpy
restatement, and the invariants the paper states."""
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import ref
from paper_2407_08454_amd import synth


def _one_set(K, V, pivot, **kw):
    """Merge all n rows as a single set with the given pivot."""
    n = K.shape[0]
    st = np.array([[[0, n]]], np.int32)
    pv = np.array([[[pivot]]], np.int32)
    ko, vo, w = ref.merge(K[None, None], V[None, None], "f32", st, pv, np.array([[1]], np.int32), **kw)
    return ko[0, 0, 0], vo[0, 0, 0], w[0, 0]


def test_pair_closed_form():
    # one neighbour at any distance D: sigma = D/(2 sqrt 2), so g = exp(-4)
    for scale in (1e-3, 1.0, 37.0):
        K = (np.array([[1, 2, 3, 4], [2, 0, 3, 5]], np.float32) * scale).astype(np.float32)
        V = np.array([[1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
        ko, vo, w = _one_set(K, V, 0)
        wp = 1.0 / (1.0 + math.exp(-4.0))
        assert w[0] == pytest.approx(wp, rel=1e-14) and w[1] == pytest.approx(1 - wp, rel=1e-12)
        assert wp == pytest.approx(0.982014, abs=1e-6)
        np.testing.assert_allclose(ko, wp * K[0].astype(float) + (1 - wp) * K[1].astype(float), rtol=1e-14)
        np.testing.assert_allclose(vo[:2], [2 * wp, 2 * (1 - wp)], rtol=1e-12)   # value weights times |S| = 2


@pytest.mark.parametrize("m", [3, 5, 9])
def test_equidistant_closed_form(m):
    # pivot at the origin, the m-1 others on axes at distance r: g = exp(-m^2/(m-1)^2)
    K = np.zeros((m, m), np.float32)
    for i in range(1, m):
        K[i, i] = 3.0
    V = np.eye(m, dtype=np.float32)
    ko, vo, w = _one_set(K, V, 0)
    g = math.exp(-(m * m) / float((m - 1) ** 2))
    assert w[0] == pytest.approx(1 / (1 + (m - 1) * g), rel=1e-13)
    np.testing.assert_allclose(w[1:], g / (1 + (m - 1) * g), rtol=1e-13)
    np.testing.assert_allclose(vo, m * w, rtol=1e-13)


def test_fixed_sigma_is_a_softmax_of_squared_distances():
    rng = np.random.default_rng(0)
    K = rng.standard_normal((7, 16)).astype(np.float32)
    V = rng.standard_normal((7, 16)).astype(np.float32)
    p = 4
    for sigma in (0.5, 5.0):
        ko, vo, w = _one_set(K, V, p, sigma_mode=ref.SIGMA_FIXED, sigma=sigma, value_scale_by_set_size=False)
        D2 = ((K.astype(float) - K[p].astype(float)) ** 2).sum(1)
        want = softmax(-D2 / (2 * sigma * sigma))
        np.testing.assert_allclose(w, want, rtol=1e-12)
        np.testing.assert_allclose(ko, want @ K.astype(float), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(vo, want @ V.astype(float), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_matches_direct_numpy_restatement_and_invariants(dtype):
    n, d = 300, 128
    q, k, v, _ = synth.gen_slice(7, 0, n, d, 1, 0.93, dtype)
    rng = np.random.default_rng(1)
    mass = rng.random(n)
    o = ref.identify_sets(k[None, None], mass[None, None], dtype, 0.5, 0.17, 0.12, 0.75, True, n)
    M = int(o["n_sets"][0, 0])
    st, pv = o["set_start"][0, 0], o["pivot"][0, 0]
    ko, vo, w = ref.merge(k[None, None], v[None, None], dtype, o["set_start"], o["pivot"], o["n_sets"])
    k64, v64 = synth.to_f64(k, dtype), synth.to_f64(v, dtype)
    sizes = []
    for s in range(M):
        lo, hi, p = st[s], st[s + 1], pv[s]
        m = hi - lo
        sizes.append(m)
        D = np.linalg.norm(k64[lo:hi] - k64[p], axis=1)
        ws = w[0, 0, lo:hi]
        assert ws.sum() == pytest.approx(1.0, rel=1e-13)            # Eq. (6): weights sum to 1
        assert ws[p - lo] == ws.max()                                 # the pivot has the largest weight
        if m == 1:                                                    # singleton: unchanged
            assert (ko[0, 0, s] == k64[lo]).all() and (vo[0, 0, s] == v64[lo]).all()
            continue
        sigma = D.sum() / (math.sqrt(2) * m)
        g = np.exp(-D ** 2 / (2 * sigma ** 2))
        assert ((g > 0) & (g <= 1)).all()
        order = np.argsort(D)
        assert (np.diff(ws[order]) <= 1e-18).all()                   # weights fall with distance
        np.testing.assert_allclose(ws, g / g.sum(), rtol=1e-12)
        np.testing.assert_allclose(ko[0, 0, s], (g / g.sum()) @ k64[lo:hi], rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(vo[0, 0, s], m * (g / g.sum()) @ v64[lo:hi], rtol=1e-11, atol=1e-13)
    assert max(sizes) > 4 and min(sizes) == 1
    assert (ko[0, 0, M:] == 0).all()


def test_identical_keys_give_uniform_weights():
    m, d = 6, 8
    K = np.tile(np.arange(1, d + 1, dtype=np.float32), (m, 1))
    V = np.arange(m * d, dtype=np.float32).reshape(m, d)
    ko, vo, w = _one_set(K, V, 2)
    np.testing.assert_allclose(w, 1.0 / m, rtol=1e-15)
    np.testing.assert_allclose(ko, K[0], rtol=1e-15)
    np.testing.assert_allclose(vo, V.astype(float).sum(0), rtol=1e-14)        # |S| * mean(v)
    ko, vo, w = _one_set(K, V, 2, value_scale_by_set_size=False)
    np.testing.assert_allclose(vo, V.astype(float).mean(0), rtol=1e-14)


def test_weights_are_scale_invariant_and_pivot_dependent():
    rng = np.random.default_rng(5)
    K = rng.standard_normal((9, 12)).astype(np.float32)
    V = rng.standard_normal((9, 12)).astype(np.float32)
    _, _, w1 = _one_set(K, V, 3)
    _, _, w2 = _one_set((K * 4).astype(np.float32), V, 3)          # times 4 is exact in fp32
    np.testing.assert_allclose(w1, w2, rtol=1e-13)
    _, _, w3 = _one_set(K, V, 5)
    assert int(np.argmax(w3)) == 5 and int(np.argmax(w1)) == 3


def test_threshold_one_makes_the_pass_an_identity():
    n, d = 64, 16
    q, k, v, _ = synth.gen_slice(9, 0, n, d, 1, 0.95, "f16")
    mass = ref.attn_mass(q[None], k[None, None], "f16")
    o = ref.identify_sets(k[None, None], mass, "f16", 1.0, 0.1, 0.1, 1.0, True, n)
    assert o["n_sets"][0, 0] == n
    ko, vo, w = ref.merge(k[None, None], v[None, None], "f16", o["set_start"], o["pivot"], o["n_sets"])
    assert (ko[0, 0] == k.astype(np.float64)).all() and (vo[0, 0] == v.astype(np.float64)).all()
    assert (w == 1).all()


def test_whole_pass_on_the_small_workload_meets_the_budget():
    cfg = synth.CONFIGS[1]
    Q, K, V, _ = synth.gen_config(cfg)
    mass = ref.attn_mass(Q, K, "f32")
    o = ref.identify_sets(K, mass, "f32", 0.5, 0.17, 0.12, 0.75, True, 256)
    assert o["status"][0, 0] == ref.SLICE_OK and 148 < o["n_sets"][0, 0] <= 256
    ko, vo, w = ref.merge(K, V, "f32", o["set_start"], o["pivot"], o["n_sets"])
    assert np.isfinite(ko).all() and np.isfinite(vo).all()
    assert w[0, 0].sum() == pytest.approx(float(o["n_sets"][0, 0]), rel=1e-12)
