"""Thin Python binding of libkvm.so (the C ABI of include/kvm.h).

Argument marshalling only: every step of the pass runs in the library's HIP kernels.
torch supplies device memory and the stream.  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvm.so")

KVM_F32, KVM_F16, KVM_BF16 = 0, 1, 2
KVM_OK = 0
KVM_ERR_INVALID_ARG, KVM_ERR_UNSUPPORTED, KVM_ERR_WORKSPACE, KVM_ERR_LAUNCH = 1, 2, 3, 4
KVM_SLICE_FALLBACK, KVM_SLICE_INFEASIBLE, KVM_SLICE_TRUNCATED = 1, 2, 4
KVM_SIGMA_MEAN_DIST, KVM_SIGMA_FIXED = 0, 1
KVM_WEIGHTS_GAUSSIAN, KVM_WEIGHTS_AVERAGE = 0, 1
KVM_PIVOT_MAX_SCORE, KVM_PIVOT_LAST, KVM_PIVOT_RANDOM = 0, 1, 2
KVM_SETS_ADJACENT, KVM_SETS_ANCHOR = 0, 1

EXPORTS = ("kvm_params_for_budget", "kvm_out_capacity", "kvm_workspace_bytes", "kvm_attn_mass",
           "kvm_attn_mass_from_lse", "kvm_attn_mass_append", "kvm_sim_append",
           "kvm_attn_mass_sim", "kvm_identify_sets", "kvm_merge", "kvm_merge_refresh", "kvm_merge_static", "kvm_evict", "kvm_evict_merge_values", "kvm_profile_enable", "kvm_profile_collect", "kvm_profile_disable",
           "kvm_last_error", "kvm_version")

_TORCH_DTYPE = {torch.float32: KVM_F32, torch.float16: KVM_F16, torch.bfloat16: KVM_BF16}


class KvmShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("G", ctypes.c_int32), ("N", ctypes.c_int32),
                ("d", ctypes.c_int32), ("dtype", ctypes.c_int32), ("seq_lens", ctypes.c_void_p)]


class KvmParams(ctypes.Structure):
    _fields_ = [("budget", ctypes.c_double), ("recent_ratio", ctypes.c_double), ("heavy_ratio", ctypes.c_double),
                ("threshold", ctypes.c_float), ("sigma_mode", ctypes.c_int32), ("sigma", ctypes.c_float),
                ("value_scale_by_set_size", ctypes.c_int32), ("enforce_budget", ctypes.c_int32),
                ("weights", ctypes.c_int32), ("pivot_rule", ctypes.c_int32), ("pivot_seed", ctypes.c_uint64),
                ("set_rule", ctypes.c_int32), ("sim_given", ctypes.c_int32)]


class KvmKernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int32), ("total_ms", ctypes.c_float)]


class KvmError(RuntimeError):
    def __init__(self, fn, code, msg):
        super().__init__(f"{fn} failed with status {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libkvm.so; raises if it has not been built (python -m paper_2407_08454_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2407_08454_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    P, S = ctypes.c_void_p, ctypes.c_size_t
    lib.kvm_params_for_budget.argtypes = [ctypes.c_double, ctypes.POINTER(KvmParams)]
    lib.kvm_params_for_budget.restype = ctypes.c_int
    lib.kvm_out_capacity.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)]
    lib.kvm_out_capacity.restype = ctypes.c_int32
    lib.kvm_workspace_bytes.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)]
    lib.kvm_workspace_bytes.restype = S
    lib.kvm_attn_mass.argtypes = [ctypes.POINTER(KvmShape), P, P, P, P, S, P]
    lib.kvm_attn_mass.restype = ctypes.c_int
    lib.kvm_attn_mass_sim.argtypes = [ctypes.POINTER(KvmShape), P, P, P, P, P, S, P]
    lib.kvm_attn_mass_sim.restype = ctypes.c_int
    lib.kvm_attn_mass_from_lse.argtypes = [ctypes.POINTER(KvmShape), P, P, P, P, P, S, P]
    lib.kvm_attn_mass_from_lse.restype = ctypes.c_int
    lib.kvm_attn_mass_append.argtypes = [ctypes.POINTER(KvmShape), P, P, P, P, S, P]
    lib.kvm_attn_mass_append.restype = ctypes.c_int
    lib.kvm_sim_append.argtypes = [ctypes.POINTER(KvmShape), P, P, P]
    lib.kvm_sim_append.restype = ctypes.c_int
    lib.kvm_identify_sets.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)] + [P] * 9 + [S, P]
    lib.kvm_identify_sets.restype = ctypes.c_int
    lib.kvm_merge.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)] + [P] * 9 + [S, P]
    lib.kvm_merge.restype = ctypes.c_int
    lib.kvm_merge_refresh.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)] + [P] * 13 + [S, P]
    lib.kvm_merge_refresh.restype = ctypes.c_int
    lib.kvm_merge_static.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)] + [P] * 9
    lib.kvm_merge_static.restype = ctypes.c_int
    lib.kvm_evict.argtypes = [ctypes.POINTER(KvmShape), ctypes.POINTER(KvmParams)] + [P] * 8 + [S, P]
    lib.kvm_evict.restype = ctypes.c_int
    lib.kvm_evict_merge_values.argtypes = lib.kvm_evict.argtypes
    lib.kvm_evict_merge_values.restype = ctypes.c_int
    lib.kvm_profile_enable.argtypes = [ctypes.c_int32]
    lib.kvm_profile_enable.restype = ctypes.c_int
    lib.kvm_profile_collect.argtypes = [ctypes.POINTER(KvmKernelTime), ctypes.c_int32]
    lib.kvm_profile_collect.restype = ctypes.c_int32
    lib.kvm_profile_disable.argtypes = []
    lib.kvm_profile_disable.restype = ctypes.c_int
    lib.kvm_last_error.restype = ctypes.c_char_p
    lib.kvm_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(fn, rc):
    if rc != KVM_OK:
        raise KvmError(fn, rc, load_library().kvm_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def kvm_params_for_budget(budget: float) -> KvmParams:
    p = KvmParams()
    _check("kvm_params_for_budget", load_library().kvm_params_for_budget(float(budget), ctypes.byref(p)))
    return p


def make_params(budget, recent_ratio, heavy_ratio, threshold=0.75, sigma_mode=KVM_SIGMA_MEAN_DIST, sigma=0.0,
                value_scale_by_set_size=True, enforce_budget=True, weights=KVM_WEIGHTS_GAUSSIAN,
                pivot_rule=KVM_PIVOT_MAX_SCORE, pivot_seed=0, set_rule=KVM_SETS_ADJACENT, sim_given=False) -> KvmParams:
    return KvmParams(float(budget), float(recent_ratio), float(heavy_ratio), float(threshold), int(sigma_mode),
                     float(sigma), int(bool(value_scale_by_set_size)), int(bool(enforce_budget)), int(weights),
                     int(pivot_rule), int(pivot_seed), int(set_rule), int(bool(sim_given)))


def make_shape(K: torch.Tensor, G: int = 1, seq_lens: torch.Tensor | None = None) -> KvmShape:
    """Shape descriptor of a contiguous (B, H_kv, N, d) cache tensor."""
    if K.dim() != 4 or not K.is_contiguous():
        raise ValueError("K must be a contiguous (B, H_kv, N, d) tensor")
    if K.dtype not in _TORCH_DTYPE:
        raise ValueError(f"unsupported dtype {K.dtype}")
    B, H, N, d = K.shape
    if seq_lens is not None:
        if seq_lens.dtype != torch.int32 or seq_lens.shape != (B,) or seq_lens.device != K.device:
            raise ValueError("seq_lens must be an int32 tensor of shape (B,) on K's device")
    shape = KvmShape(B, H, int(G), N, d, _TORCH_DTYPE[K.dtype], None if seq_lens is None else seq_lens.data_ptr())
    shape._seq_lens_ref = seq_lens          # the descriptor holds a raw pointer: keep the tensor alive
    return shape


def kvm_out_capacity(shape: KvmShape, params: KvmParams) -> int:
    cap = load_library().kvm_out_capacity(ctypes.byref(shape), ctypes.byref(params))
    if cap < 0:
        raise KvmError("kvm_out_capacity", KVM_ERR_INVALID_ARG, load_library().kvm_last_error().decode())
    return cap


def kvm_workspace_bytes(shape: KvmShape, params: KvmParams | None = None) -> int:
    return load_library().kvm_workspace_bytes(ctypes.byref(shape), None if params is None else ctypes.byref(params))


def _same_device(*ts):
    dev = None
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous and on the GPU")
        dev = dev or t.device
        if t.device != dev:
            raise ValueError("tensors must share one device")


def _check_attn_operands(shape: KvmShape, Q, K, mass):
    B, H, G, N, d = shape.B, shape.H_kv, shape.G, shape.N, shape.d
    if tuple(Q.shape) != (B, H * G, N, d) or tuple(K.shape) != (B, H, N, d) or tuple(mass.shape) != (B, H, N):
        raise ValueError("operand shapes do not match the shape descriptor")
    if mass.dtype != torch.float32 or Q.dtype != K.dtype or _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")


def kvm_attn_mass(shape: KvmShape, Q, K, mass, ws):
    """mass (B, H_kv, N) float32 <- aggregated attention score of every key."""
    _same_device(Q, K, mass, ws)
    _check_attn_operands(shape, Q, K, mass)
    _check("kvm_attn_mass", load_library().kvm_attn_mass(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(mass), _ptr(ws),
                                                         ws.numel() * ws.element_size(), _stream()))


def kvm_attn_mass_sim(shape: KvmShape, Q, K, mass, sim, ws):
    """kvm_attn_mass, and sim (B, H_kv, N) float32 <- cosine similarity of every key to the one before it."""
    _same_device(Q, K, mass, sim, ws)
    _check_attn_operands(shape, Q, K, mass)
    if sim.dtype != torch.float32 or tuple(sim.shape) != (shape.B, shape.H_kv, shape.N):
        raise ValueError("sim must be float32 of shape (B, H_kv, N)")
    _check("kvm_attn_mass_sim", load_library().kvm_attn_mass_sim(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(mass), _ptr(sim),
                                                                 _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def kvm_attn_mass_from_lse(shape: KvmShape, Q, K, row_lse, mass, ws):
    """The same map from the caller's row statistics: row_lse (B, H_kv*G, N) float32, natural logarithms."""
    _same_device(Q, K, row_lse, mass, ws)
    _check_attn_operands(shape, Q, K, mass)
    if row_lse.dtype != torch.float32 or tuple(row_lse.shape) != (shape.B, shape.H_kv * shape.G, shape.N):
        raise ValueError("row_lse must be float32 of shape (B, H_kv*G, N)")
    _check("kvm_attn_mass_from_lse",
           load_library().kvm_attn_mass_from_lse(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(row_lse), _ptr(mass), _ptr(ws),
                                                 ws.numel() * ws.element_size(), _stream()))


def kvm_attn_mass_append(shape: KvmShape, q_new, K, mass, ws):
    """mass (B, H_kv, N) float32 += the attention row of the newest token (its key already stored at n_b - 1)."""
    _same_device(q_new, K, mass, ws)
    B, H, G, N, d = shape.B, shape.H_kv, shape.G, shape.N, shape.d
    if tuple(q_new.shape) != (B, H * G, d) or tuple(K.shape) != (B, H, N, d) or tuple(mass.shape) != (B, H, N):
        raise ValueError("operand shapes do not match the shape descriptor")
    if mass.dtype != torch.float32 or q_new.dtype != K.dtype or _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")
    _check("kvm_attn_mass_append",
           load_library().kvm_attn_mass_append(ctypes.byref(shape), _ptr(q_new), _ptr(K), _ptr(mass), _ptr(ws),
                                               ws.numel() * ws.element_size(), _stream()))


def kvm_sim_append(shape: KvmShape, K, sim):
    """sim[b, h, n_b - 1] <- cosine similarity of the newest key and its predecessor; nothing else is written."""
    _same_device(K, sim)
    B, H, N, d = shape.B, shape.H_kv, shape.N, shape.d
    if tuple(K.shape) != (B, H, N, d) or tuple(sim.shape) != (B, H, N):
        raise ValueError("operand shapes do not match the shape descriptor")
    if sim.dtype != torch.float32 or _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")
    _check("kvm_sim_append", load_library().kvm_sim_append(ctypes.byref(shape), _ptr(K), _ptr(sim), _stream()))


def kvm_identify_sets(shape: KvmShape, params: KvmParams, K, mass, set_id, set_start, pivot, n_sets, sim_opt,
                      slice_status, ws):
    _same_device(K, mass, set_id, set_start, pivot, n_sets, sim_opt, slice_status, ws)
    B, H, N, d = shape.B, shape.H_kv, shape.N, shape.d
    cap = kvm_out_capacity(shape, params)
    want = {"K": (K, (B, H, N, d)), "mass": (mass, (B, H, N)), "set_id": (set_id, (B, H, N)),
            "set_start": (set_start, (B, H, cap + 1)), "pivot": (pivot, (B, H, cap)), "n_sets": (n_sets, (B, H)),
            "slice_status": (slice_status, (B, H))}
    if sim_opt is not None:
        want["sim_opt"] = (sim_opt, (B, H, N))
    for name, (t, shp) in want.items():
        if tuple(t.shape) != shp:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {shp}")
    for t in (set_id, set_start, pivot, n_sets, slice_status):
        if t.dtype != torch.int32:
            raise ValueError("index maps must be int32")
    if mass.dtype != torch.float32 or (sim_opt is not None and sim_opt.dtype != torch.float32):
        raise ValueError("mass and sim must be float32")
    if _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")
    _check("kvm_identify_sets", load_library().kvm_identify_sets(
        ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(mass), _ptr(set_id), _ptr(set_start), _ptr(pivot),
        _ptr(n_sets), _ptr(sim_opt), _ptr(slice_status), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def _check_merge_operands(shape, params, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, ws=None):
    _same_device(K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, ws)
    B, H, N, d = shape.B, shape.H_kv, shape.N, shape.d
    cap = kvm_out_capacity(shape, params)
    want = {"K": (K, (B, H, N, d)), "V": (V, (B, H, N, d)), "set_start": (set_start, (B, H, cap + 1)),
            "pivot": (pivot, (B, H, cap)), "n_sets": (n_sets, (B, H)), "K_out": (K_out, (B, H, cap, d)),
            "V_out": (V_out, (B, H, cap, d))}
    if w_opt is not None:
        want["w_opt"] = (w_opt, (B, H, N))
    for name, (t, shp) in want.items():
        if tuple(t.shape) != shp:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {shp}")
    for t in (set_start, pivot, n_sets):
        if t.dtype != torch.int32:
            raise ValueError("index maps must be int32")
    if not (K.dtype == V.dtype == K_out.dtype == V_out.dtype) or _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")
    if w_opt is not None and w_opt.dtype != torch.float32:
        raise ValueError("w_opt must be float32")


def kvm_merge(shape: KvmShape, params: KvmParams, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, ws):
    _check_merge_operands(shape, params, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, ws)
    _check("kvm_merge", load_library().kvm_merge(
        ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(V), _ptr(set_start), _ptr(pivot), _ptr(n_sets),
        _ptr(K_out), _ptr(V_out), _ptr(w_opt), None if ws is None else _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def kvm_merge_refresh(shape: KvmShape, params: KvmParams, K, V, prev_set_id, prev_set_start, prev_pivot, prev_n_sets,
                      set_start, pivot, n_sets, K_out, V_out, n_changed, ws):
    """K_out / V_out, merged with the previous maps, become the compacted cache of the new maps: rows of sets
    that did not change move to their new index, the others are merged again."""
    _check_merge_operands(shape, params, K, V, set_start, pivot, n_sets, K_out, V_out, None, ws)
    _same_device(prev_set_id, prev_set_start, prev_pivot, prev_n_sets, n_changed)
    B, H, N = shape.B, shape.H_kv, shape.N
    for t, other, shp in ((prev_set_id, None, (B, H, N)), (prev_set_start, set_start, None), (prev_pivot, pivot, None),
                          (prev_n_sets, n_sets, None)) + (((n_changed, None, (B, H)),) if n_changed is not None else ()):
        if t.dtype != torch.int32 or tuple(t.shape) != (shp if shp is not None else tuple(other.shape)):
            raise ValueError("previous maps must be int32 tensors shaped like the new ones")
    _check("kvm_merge_refresh", load_library().kvm_merge_refresh(
        ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(V), _ptr(prev_set_id), _ptr(prev_set_start),
        _ptr(prev_pivot), _ptr(prev_n_sets), _ptr(set_start), _ptr(pivot), _ptr(n_sets), _ptr(K_out), _ptr(V_out),
        _ptr(n_changed), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def kvm_merge_static(shape: KvmShape, params: KvmParams, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt):
    """kvm_merge without a workspace: the work plan lives in a buffer built into the library."""
    _check_merge_operands(shape, params, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt)
    _check("kvm_merge_static", load_library().kvm_merge_static(
        ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(V), _ptr(set_start), _ptr(pivot), _ptr(n_sets),
        _ptr(K_out), _ptr(V_out), _ptr(w_opt), _stream()))


def _evict(fn: str, shape: KvmShape, params: KvmParams, K, V, mass, kept, n_kept, K_out, V_out, ws):
    _same_device(K, V, mass, kept, n_kept, K_out, V_out, ws)
    B, H, N, d = shape.B, shape.H_kv, shape.N, shape.d
    cap = kvm_out_capacity(shape, params)
    want = {"K": (K, (B, H, N, d)), "V": (V, (B, H, N, d)), "mass": (mass, (B, H, N)), "kept": (kept, (B, H, cap)),
            "n_kept": (n_kept, (B, H)), "K_out": (K_out, (B, H, cap, d)), "V_out": (V_out, (B, H, cap, d))}
    for name, (t, shp) in want.items():
        if tuple(t.shape) != shp:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {shp}")
    if kept.dtype != torch.int32 or n_kept.dtype != torch.int32 or mass.dtype != torch.float32:
        raise ValueError("kept and n_kept must be int32, mass float32")
    if not (K.dtype == V.dtype == K_out.dtype == V_out.dtype) or _TORCH_DTYPE[K.dtype] != shape.dtype:
        raise ValueError("dtype mismatch")
    _check(fn, getattr(load_library(), fn)(
        ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(V), _ptr(mass), _ptr(kept), _ptr(n_kept), _ptr(K_out),
        _ptr(V_out), None if ws is None else _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def kvm_evict(shape: KvmShape, params: KvmParams, K, V, mass, kept, n_kept, K_out, V_out, ws):
    """Comparison workload: keep the recent window and the largest scores, gather their rows."""
    _evict("kvm_evict", shape, params, K, V, mass, kept, n_kept, K_out, V_out, ws)


def kvm_evict_merge_values(shape: KvmShape, params: KvmParams, K, V, mass, kept, n_kept, K_out, V_out, ws):
    """Comparison workload: as kvm_evict, the evicted values averaged into the nearest kept token's value."""
    _evict("kvm_evict_merge_values", shape, params, K, V, mass, kept, n_kept, K_out, V_out, ws)


def kvm_profile_enable(max_launches: int):
    _check("kvm_profile_enable", load_library().kvm_profile_enable(int(max_launches)))


def kvm_profile_collect() -> dict:
    """{kernel name: (launches, total milliseconds)} since the last collect."""
    recs = (KvmKernelTime * 16)()
    n = load_library().kvm_profile_collect(recs, 16)
    return {recs[i].name.decode(): (recs[i].launches, recs[i].total_ms) for i in range(n)}


def kvm_profile_disable():
    _check("kvm_profile_disable", load_library().kvm_profile_disable())


class Buffers:
    """Caller-owned device buffers for one shape/params pair (allocated once with torch)."""

    def __init__(self, shape: KvmShape, params: KvmParams, device, dtype, with_debug: bool = False, with_sim: bool = False):
        B, H, N, d = shape.B, shape.H_kv, shape.N, shape.d
        cap = kvm_out_capacity(shape, params)
        i32 = dict(dtype=torch.int32, device=device)
        self.cap = cap
        self.mass = torch.empty((B, H, N), dtype=torch.float32, device=device)
        self.set_id = torch.empty((B, H, N), **i32)
        self.set_start = torch.empty((B, H, cap + 1), **i32)
        self.pivot = torch.empty((B, H, cap), **i32)
        self.n_sets = torch.empty((B, H), **i32)
        self.status = torch.empty((B, H), **i32)
        self.K_out = torch.empty((B, H, cap, d), dtype=dtype, device=device)
        self.V_out = torch.empty((B, H, cap, d), dtype=dtype, device=device)
        self.sim = torch.empty((B, H, N), dtype=torch.float32, device=device) if with_debug or with_sim else None
        self.w = torch.empty((B, H, N), dtype=torch.float32, device=device) if with_debug else None
        self.ws = torch.empty(max(kvm_workspace_bytes(shape, params), 256), dtype=torch.uint8, device=device)


def compress(shape: KvmShape, params: KvmParams, Q, K, V, buf: Buffers, sim_from_score_pass: bool = False):
    """One pass of the whole hot path: three library calls on the current stream.
    sim_from_score_pass (adjacent rule only): the similarities come out of the score pass
    (kvm_attn_mass_sim) and kvm_identify_sets skips its scan of K."""
    if sim_from_score_pass and params.set_rule == KVM_SETS_ADJACENT and not params.sim_given:
        if buf.sim is None:
            raise ValueError("sim_from_score_pass needs Buffers(..., with_sim=True)")
        kvm_attn_mass_sim(shape, Q, K, buf.mass, buf.sim, buf.ws)
        given = KvmParams.from_buffer_copy(params)
        given.sim_given = 1
        kvm_identify_sets(shape, given, K, buf.mass, buf.set_id, buf.set_start, buf.pivot, buf.n_sets, buf.sim,
                          buf.status, buf.ws)
    else:
        kvm_attn_mass(shape, Q, K, buf.mass, buf.ws)
        kvm_identify_sets(shape, params, K, buf.mass, buf.set_id, buf.set_start, buf.pivot, buf.n_sets, buf.sim,
                          buf.status, buf.ws)
    kvm_merge(shape, params, K, V, buf.set_start, buf.pivot, buf.n_sets, buf.K_out, buf.V_out, buf.w, buf.ws)
