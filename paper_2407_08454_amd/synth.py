"""Seeded synthetic Q/K/V generators for the KV-merging compression pass.

This module holds input recipes only: random draws, the AR(1) key recurrence that
imitates the high adjacent-token key similarity the paper observes (Section 3.1),
rounding to the storage dtype, and padding.  It contains none of the method's
arithmetic (no attention, no cosine similarity, no merging) and is shared by the CPU
oracle's tests and the GPU path's tests / benchmark so that both read identical bits.

Every slice (one (batch, layer, KV-head) triple) owns a random stream derived from
(seed, slice index), so a single slice can be regenerated without the others.

Storage dtypes: "f32" -> numpy float32, "f16" -> numpy float16, "bf16" -> numpy uint16
holding bfloat16 bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

import math
import os

import numpy as np
from scipy.signal import lfilter

RESET_RATE = 1.0 / 32.0          # Poisson rate of fresh key draws, per token
PAD_VALUE = 1.0e4                # finite garbage written into padded positions

# The five workloads: shapes of the models the paper evaluates (Section 5.1), with the
# two KV budgets it reports.  "layers" x "batch" is folded into the leading B axis.
CONFIGS = {
    1: dict(name="single-head-512", layers=1, batch=1, H_kv=1, G=1, N=512, d=128,
            dtype="f32", rho=0.95, budgets=(0.5,), seed=0, seq_lens=None),
    2: dict(name="llama2-7b-4096", layers=32, batch=1, H_kv=32, G=1, N=4096, d=128,
            dtype="f16", rho=None, budgets=(0.5, 0.35), seed=1, seq_lens=None),
    3: dict(name="llama2-13b-4096", layers=40, batch=1, H_kv=40, G=1, N=4096, d=128,
            dtype="bf16", rho=None, budgets=(0.35,), seed=2, seq_lens=None),
    4: dict(name="mistral-7b-gqa-16384", layers=32, batch=1, H_kv=8, G=4, N=16384, d=128,
            dtype="bf16", rho=None, budgets=(0.5,), seed=3, seq_lens=None),
    5: dict(name="llama2-7b-ragged-b4", layers=32, batch=4, H_kv=32, G=1, N=16384, d=128,
            dtype="f16", rho=None, budgets=(0.35,), seed=4,
            seq_lens=(4096, 8192, 12288, 16384)),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array once to the storage dtype."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def storage_numpy_dtype(dtype: str):
    return {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]


def _slice_rng(seed: int, slice_index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed, spawn_key=(slice_index,))))


def ar1_keys(rng: np.random.Generator, n: int, d: int, rho: float) -> np.ndarray:
    """k_0 ~ N(0,I); k_t = rho k_{t-1} + sqrt(1-rho^2) eps_t; at every t >= 1 a fresh
    N(0,I) draw replaces k_t with probability 1 - exp(-RESET_RATE)."""
    eps = rng.standard_normal((n, d), dtype=np.float32)
    u = rng.random(n)
    reset = u < -math.expm1(-RESET_RATE)
    if n:
        reset[0] = True
    x = eps.astype(np.float64) * math.sqrt(1.0 - rho * rho)
    x[reset] = eps[reset]
    out = np.empty((n, d), dtype=np.float64)
    starts = np.flatnonzero(reset)
    ends = np.append(starts[1:], n)
    a = np.array([1.0, -rho])
    b = np.array([1.0])
    for s, e in zip(starts, ends):
        out[s:e] = lfilter(b, a, x[s:e], axis=0)
    return out.astype(np.float32)


def gen_slice(seed: int, slice_index: int, n: int, d: int, G: int = 1, rho: float | None = None,
              dtype: str = "f32", N: int | None = None):
    """One slice: Q (G, N, d), K (N, d), V (N, d) in storage dtype, and the rho used.

    Positions >= n (padding up to N) hold PAD_VALUE.  If rho is None it is drawn from
    U(0.85, 0.99) as the first draw of the slice's stream.
    """
    N = n if N is None else N
    rng = _slice_rng(seed, slice_index)
    r = float(rng.uniform(0.85, 0.99))
    if rho is None:
        rho = r
    k = ar1_keys(rng, n, d, rho)
    q = rng.standard_normal((G, n, d), dtype=np.float32)
    v = rng.standard_normal((n, d), dtype=np.float32)
    if N > n:
        pad = lambda a, shape: np.concatenate(
            [a, np.full(shape, PAD_VALUE, dtype=np.float32)], axis=-2)
        k = pad(k, (N - n, d))
        v = pad(v, (N - n, d))
        q = pad(q, (G, N - n, d))
    return to_storage(q, dtype), to_storage(k, dtype), to_storage(v, dtype), rho


def config_dims(cfg: dict, layers: int | None = None):
    """(B, H_kv, G, N, d, seq_lens[B] or None) with layers folded into B.

    B index = layer * batch + b, so seq_lens repeats the batch's lengths per layer.
    """
    L = cfg["layers"] if layers is None else layers
    B = L * cfg["batch"]
    sl = None
    if cfg["seq_lens"] is not None:
        sl = np.tile(np.asarray(cfg["seq_lens"], dtype=np.int32), L)
    return B, cfg["H_kv"], cfg["G"], cfg["N"], cfg["d"], sl


def _gen_chunk(args):
    """Worker: generate a run of slices (module-level so a spawned process can import it)."""
    seed, first, count, lens, d, G, rho, dtype, N = args
    return [gen_slice(seed, first + i, lens[i], d, G, rho, dtype, N)[:3] for i in range(count)]


def gen_config(cfg: dict, layers: int | None = None, layer_offset: int = 0, workers: int | None = None):
    """Full tensors of a workload: Q (B, H_kv*G, N, d), K, V (B, H_kv, N, d), seq_lens.

    Slice index = ((layer_offset*batch + B index) * H_kv + h): generating a subset of
    the layers yields the same bits those layers have in the full workload.  Large
    workloads are generated by a pool of spawned worker processes (no fork: the caller
    may already hold a GPU context).
    """
    B, H, G, N, d, sl = config_dims(cfg, layers)
    npdt = storage_numpy_dtype(cfg["dtype"])
    Q = np.empty((B, H * G, N, d), dtype=npdt)
    K = np.empty((B, H, N, d), dtype=npdt)
    V = np.empty((B, H, N, d), dtype=npdt)
    base = layer_offset * cfg["batch"] * H
    total = B * H
    lens_all = [N if sl is None else int(sl[bh // H]) for bh in range(total)]

    def place(first, triples):
        for i, (q, k, v) in enumerate(triples):
            b, h = divmod(first + i, H)
            Q[b, h * G:(h + 1) * G] = q
            K[b, h] = k
            V[b, h] = v

    if workers is None:
        workers = min(16, os.cpu_count() or 1)
    chunk = max(1, min(8, (64 * 4096) // max(N, 1)))
    jobs = [(cfg["seed"], base + f, min(chunk, total - f), lens_all[f:f + chunk], d, G, cfg["rho"],
             cfg["dtype"], N) for f in range(0, total, chunk)]
    if workers <= 1 or total * N <= 64 * 4096:
        for j in jobs:
            place(j[1] - base, _gen_chunk(j))
    else:
        import multiprocessing as mp
        from concurrent.futures import ProcessPoolExecutor
        with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
            for j, res in zip(jobs, ex.map(_gen_chunk, jobs)):
                place(j[1] - base, res)
    return Q, K, V, sl


def gen_config_layers(cfg: dict, workers: int | None = None):
    """The same tensors one layer at a time (for workloads too large to hold on the host at once):
    yields (Q, K, V, seq_lens) of layer 0, 1, ..., each with the bits gen_config gives that layer.
    One pool of spawned worker processes serves all layers."""
    B, H, G, N, d, sl = config_dims(cfg, 1)
    npdt = storage_numpy_dtype(cfg["dtype"])
    total = B * H
    lens_all = [N if sl is None else int(sl[bh // H]) for bh in range(total)]
    if workers is None:
        workers = min(16, os.cpu_count() or 1)
    chunk = max(1, min(8, (64 * 4096) // max(N, 1)))
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    with ProcessPoolExecutor(max_workers=max(workers, 1), mp_context=mp.get_context("spawn")) as ex:
        for layer in range(cfg["layers"]):
            base = layer * total
            jobs = [(cfg["seed"], base + f, min(chunk, total - f), lens_all[f:f + chunk], d, G, cfg["rho"],
                     cfg["dtype"], N) for f in range(0, total, chunk)]
            Q = np.empty((B, H * G, N, d), dtype=npdt)
            K = np.empty((B, H, N, d), dtype=npdt)
            V = np.empty((B, H, N, d), dtype=npdt)
            for j, res in zip(jobs, ex.map(_gen_chunk, jobs)):
                for i, (q, k, v) in enumerate(res):
                    b, h = divmod(j[1] - base + i, H)
                    Q[b, h * G:(h + 1) * G] = q
                    K[b, h] = k
                    V[b, h] = v
            yield Q, K, V, sl


def slice_of(Q, K, V, b: int, h: int, G: int):
    """Views of one slice out of full tensors: Q (G, N, d), K (N, d), V (N, d)."""
    return Q[b, h * G:(h + 1) * G], K[b, h], V[b, h]
