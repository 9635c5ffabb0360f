"""ctypes wrapper around the fp64 CPU oracle (oracle/kvm_ref.c).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: imported only by tests/, the smoke check and
the benchmark's cpu_baseline leg.  It knows nothing of the GPU library.

Arrays are numpy: storage dtypes "f32" (float32), "f16" (float16), "bf16" (uint16 bit
patterns).  All outputs are fp64 / int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvm_ref.c")
_LIB = os.path.join(_HERE, "libkvm_ref.so")
_DTYPE = {"f32": 0, "f16": 1, "bf16": 2}
SLICE_OK, SLICE_FALLBACK, SLICE_INFEASIBLE, SLICE_TRUNCATED = 0, 1, 2, 4
SIGMA_MEAN_DIST, SIGMA_FIXED = 0, 1
WEIGHTS_GAUSSIAN, WEIGHTS_AVERAGE = 0, 1
PIVOT_MAX_SCORE, PIVOT_LAST, PIVOT_RANDOM = 0, 1, 2
SETS_ADJACENT, SETS_ANCHOR = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP across slices)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.kvm_ref_half_to_double.restype = ctypes.c_double
        _lib.kvm_ref_half_to_double.argtypes = [ctypes.c_uint16]
        _lib.kvm_ref_bf16_to_double.restype = ctypes.c_double
        _lib.kvm_ref_bf16_to_double.argtypes = [ctypes.c_uint16]
        _lib.kvm_ref_splitmix64_at.restype = ctypes.c_uint64
        _lib.kvm_ref_splitmix64_at.argtypes = [ctypes.c_uint64]
        _lib.kvm_ref_random_offset.restype = ctypes.c_int
        _lib.kvm_ref_random_offset.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_storage(x, dtype):
    want = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]
    if x.dtype != want or not x.flags.c_contiguous:
        raise ValueError(f"expected contiguous {want} array for dtype {dtype}")


def _lens(seq_lens, B):
    if seq_lens is None:
        return None
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    assert sl.shape == (B,)
    return sl


def half_to_double(bits: int) -> float:
    return _load().kvm_ref_half_to_double(bits)


def bf16_to_double(bits: int) -> float:
    return _load().kvm_ref_bf16_to_double(bits)


def splitmix64_at(z: int) -> int:
    return int(_load().kvm_ref_splitmix64_at(z & 0xFFFFFFFFFFFFFFFF))


def random_offset(seed: int, slice_index: int, first_token: int, m: int) -> int:
    return int(_load().kvm_ref_random_offset(seed & 0xFFFFFFFFFFFFFFFF, slice_index, first_token, m))


def num_threads() -> int:
    return int(_load().kvm_ref_num_threads())


def set_num_threads(k: int) -> None:
    """Threads the oracle's loops over slices use from now on (the OpenMP runtime's own switch)."""
    _load().kvm_ref_set_num_threads(int(k))


def attn_mass(Q, K, dtype: str, G: int = 1, seq_lens=None):
    """Q (B, H*G, N, d), K (B, H, N, d) -> mass (B, H, N) fp64."""
    lib = _load()
    _check_storage(Q, dtype)
    _check_storage(K, dtype)
    B, H, N, d = K.shape
    assert Q.shape == (B, H * G, N, d)
    sl = _lens(seq_lens, B)
    mass = np.empty((B, H, N), dtype=np.float64)
    lib.kvm_ref_attn_mass.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 4
    rc = lib.kvm_ref_attn_mass(B, H, G, N, d, _DTYPE[dtype], _ptr(sl), _ptr(Q), _ptr(K), _ptr(mass))
    if rc:
        raise RuntimeError(f"kvm_ref_attn_mass failed: {rc}")
    return mass


def row_lse(Q, K, dtype: str, G: int = 1, seq_lens=None):
    """Q (B, H*G, N, d), K (B, H, N, d) -> natural-log softmax denominators (B, H*G, N) fp64."""
    lib = _load()
    _check_storage(Q, dtype)
    _check_storage(K, dtype)
    B, H, N, d = K.shape
    assert Q.shape == (B, H * G, N, d)
    sl = _lens(seq_lens, B)
    lse = np.empty((B, H * G, N), dtype=np.float64)
    lib.kvm_ref_row_lse.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 4
    rc = lib.kvm_ref_row_lse(B, H, G, N, d, _DTYPE[dtype], _ptr(sl), _ptr(Q), _ptr(K), _ptr(lse))
    if rc:
        raise RuntimeError(f"kvm_ref_row_lse failed: {rc}")
    return lse


def attn_mass_append(q_new, K, mass, dtype: str, G: int = 1, seq_lens=None):
    """q_new (B, H*G, d), K (B, H, N, d), mass (B, H, N) -> mass with the newest token's attention row added (fp64 copy)."""
    lib = _load()
    _check_storage(q_new, dtype)
    _check_storage(K, dtype)
    B, H, N, d = K.shape
    assert q_new.shape == (B, H * G, d)
    sl = _lens(seq_lens, B)
    out = np.array(mass, dtype=np.float64, order="C", copy=True)
    assert out.shape == (B, H, N)
    lib.kvm_ref_attn_mass_append.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 4
    rc = lib.kvm_ref_attn_mass_append(B, H, G, N, d, _DTYPE[dtype], _ptr(sl), _ptr(q_new), _ptr(K), _ptr(out))
    if rc:
        raise RuntimeError(f"kvm_ref_attn_mass_append failed: {rc}")
    return out


def identify_sets(K, mass, dtype: str, budget: float, recent_ratio: float, heavy_ratio: float,
                  threshold: float, enforce_budget: bool = True, cap_rows: int | None = None,
                  seq_lens=None, pivot_rule: int = PIVOT_MAX_SCORE, pivot_seed: int = 0,
                  set_rule: int = SETS_ADJACENT):
    """K (B, H, N, d), mass (B, H, N) -> dict of index maps (see kvm_ref.c)."""
    lib = _load()
    _check_storage(K, dtype)
    B, H, N, d = K.shape
    mass = np.ascontiguousarray(mass, dtype=np.float64)
    assert mass.shape == (B, H, N)
    if cap_rows is None:
        cap_rows = N
    sl = _lens(seq_lens, B)
    out = dict(
        set_id=np.empty((B, H, N), np.int32),
        set_start=np.empty((B, H, cap_rows + 1), np.int32),
        pivot=np.empty((B, H, cap_rows), np.int32),
        n_sets=np.empty((B, H), np.int32),
        status=np.empty((B, H), np.int32),
        sim=np.empty((B, H, N), np.float64),
        protected=np.empty((B, H, N), np.uint8),
        min_removed_sim=np.empty((B, H), np.float64),
        anchor_margin=np.full((B, H), np.inf, np.float64),
        cap_rows=cap_rows,
    )
    lib.kvm_ref_identify_sets.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] + [ctypes.c_double] * 4 + \
        [ctypes.c_int] * 3 + [ctypes.c_uint64, ctypes.c_int] + [ctypes.c_void_p] * 11
    rc = lib.kvm_ref_identify_sets(B, H, N, d, _DTYPE[dtype], _ptr(sl), float(budget), float(recent_ratio),
                                   float(heavy_ratio), float(threshold), int(bool(enforce_budget)), int(set_rule),
                                   int(pivot_rule), int(pivot_seed), cap_rows,
                                   _ptr(K), _ptr(mass), _ptr(out["set_id"]), _ptr(out["set_start"]),
                                   _ptr(out["pivot"]), _ptr(out["n_sets"]), _ptr(out["status"]),
                                   _ptr(out["sim"]), _ptr(out["protected"]), _ptr(out["min_removed_sim"]),
                                   _ptr(out["anchor_margin"]))
    if rc:
        raise RuntimeError(f"kvm_ref_identify_sets failed: {rc}")
    return out


def merge(K, V, dtype: str, set_start, pivot, n_sets, sigma_mode: int = SIGMA_MEAN_DIST,
          sigma: float = 0.0, value_scale_by_set_size: bool = True, seq_lens=None,
          weights: int = WEIGHTS_GAUSSIAN):
    """-> (K_out, V_out (B, H, cap_rows, d) fp64 with rows >= n_sets zero, w (B, H, N))."""
    lib = _load()
    _check_storage(K, dtype)
    _check_storage(V, dtype)
    B, H, N, d = K.shape
    set_start = np.ascontiguousarray(set_start, dtype=np.int32)
    pivot = np.ascontiguousarray(pivot, dtype=np.int32)
    n_sets = np.ascontiguousarray(n_sets, dtype=np.int32)
    cap_rows = pivot.shape[-1]
    assert set_start.shape == (B, H, cap_rows + 1) and n_sets.shape == (B, H)
    sl = _lens(seq_lens, B)
    K_out = np.zeros((B, H, cap_rows, d), np.float64)
    V_out = np.zeros((B, H, cap_rows, d), np.float64)
    w = np.empty((B, H, N), np.float64)
    lib.kvm_ref_merge.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                       ctypes.c_double, ctypes.c_int] + [ctypes.c_void_p] * 8
    rc = lib.kvm_ref_merge(B, H, N, d, _DTYPE[dtype], _ptr(sl), cap_rows, int(weights), int(sigma_mode), float(sigma),
                           int(bool(value_scale_by_set_size)), _ptr(K), _ptr(V), _ptr(set_start), _ptr(pivot),
                           _ptr(n_sets), _ptr(K_out), _ptr(V_out), _ptr(w))
    if rc:
        raise RuntimeError(f"kvm_ref_merge failed: {rc}")
    return K_out, V_out, w


def evict(K, V, mass, dtype: str, budget: float, recent_ratio: float, cap_rows: int, seq_lens=None):
    """Comparison workload (eviction by score) -> (kept (B, H, cap_rows), n_kept (B, H), K_out, V_out fp64)."""
    lib = _load()
    _check_storage(K, dtype)
    _check_storage(V, dtype)
    B, H, N, d = K.shape
    mass = np.ascontiguousarray(mass, dtype=np.float64)
    sl = _lens(seq_lens, B)
    kept = np.empty((B, H, cap_rows), np.int32)
    n_kept = np.empty((B, H), np.int32)
    K_out = np.zeros((B, H, cap_rows, d), np.float64)
    V_out = np.zeros((B, H, cap_rows, d), np.float64)
    lib.kvm_ref_evict.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p, ctypes.c_double, ctypes.c_double, ctypes.c_int] + \
        [ctypes.c_void_p] * 7
    rc = lib.kvm_ref_evict(B, H, N, d, _DTYPE[dtype], _ptr(sl), float(budget), float(recent_ratio), int(cap_rows),
                           _ptr(K), _ptr(V), _ptr(mass), _ptr(kept), _ptr(n_kept), _ptr(K_out), _ptr(V_out))
    if rc:
        raise RuntimeError(f"kvm_ref_evict failed: {rc}")
    return kept, n_kept, K_out, V_out


def evict_merge_values(K, V, mass, dtype: str, budget: float, recent_ratio: float, cap_rows: int, seq_lens=None):
    """Comparison workload (value-only merging into the nearest kept token)
    -> (kept, n_kept, K_out, V_out fp64, count (B, H, cap_rows))."""
    lib = _load()
    _check_storage(K, dtype)
    _check_storage(V, dtype)
    B, H, N, d = K.shape
    mass = np.ascontiguousarray(mass, dtype=np.float64)
    sl = _lens(seq_lens, B)
    kept = np.empty((B, H, cap_rows), np.int32)
    n_kept = np.empty((B, H), np.int32)
    count = np.empty((B, H, cap_rows), np.int32)
    K_out = np.zeros((B, H, cap_rows, d), np.float64)
    V_out = np.zeros((B, H, cap_rows, d), np.float64)
    lib.kvm_ref_evict_merge_values.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p, ctypes.c_double, ctypes.c_double,
                                                                     ctypes.c_int] + [ctypes.c_void_p] * 8
    rc = lib.kvm_ref_evict_merge_values(B, H, N, d, _DTYPE[dtype], _ptr(sl), float(budget), float(recent_ratio),
                                        int(cap_rows), _ptr(K), _ptr(V), _ptr(mass), _ptr(kept), _ptr(n_kept),
                                        _ptr(K_out), _ptr(V_out), _ptr(count))
    if rc:
        raise RuntimeError(f"kvm_ref_evict_merge_values failed: {rc}")
    return kept, n_kept, K_out, V_out, count
