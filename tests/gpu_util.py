"""Helpers for the GPU parity tests: numpy <-> device tensors, calls through the C ABI
binding, and the comparison metrics.  Nothing here computes any part of the method."""
from __future__ import annotations

import numpy as np
import torch

from paper_2407_08454_amd import binding as kb

TOL = 2e-3                      # max relative error for mass and merged K/V (fp32 accumulation)
# Merged rows are stored in the cache dtype: one round-to-nearest adds up to one unit
# roundoff (2^-24, 2^-11, 2^-8) on top of the arithmetic tolerance.
UNIT_ROUNDOFF = {"f32": 2.0 ** -24, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}
MANT_BITS = {"f32": 23, "f16": 10, "bf16": 7}
MIN_EXP = {"f32": -126, "f16": -14, "bf16": -126}
NEAR = 1e-6                     # similarities this close to the threshold may decide either way

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def lens_dev(seq_lens):
    return None if seq_lens is None else torch.as_tensor(np.asarray(seq_lens, dtype=np.int32)).cuda()


def gpu_mass(Q, K, dtype, G=1, seq_lens=None):
    Qd, Kd = to_dev(Q, dtype), to_dev(K, dtype)
    sl = lens_dev(seq_lens)
    sh = kb.make_shape(Kd, G, sl)
    B, H, N, _ = K.shape
    mass = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(kb.kvm_workspace_bytes(sh), 256), dtype=torch.uint8, device="cuda")
    kb.kvm_attn_mass(sh, Qd, Kd, mass, ws)
    torch.cuda.synchronize()
    return mass.cpu().numpy()


def gpu_mass_from_lse(Q, K, row_lse32, dtype, G=1, seq_lens=None):
    Qd, Kd = to_dev(Q, dtype), to_dev(K, dtype)
    sl = lens_dev(seq_lens)
    sh = kb.make_shape(Kd, G, sl)
    B, H, N, _ = K.shape
    mass = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(kb.kvm_workspace_bytes(sh), 256), dtype=torch.uint8, device="cuda")
    ld = torch.from_numpy(np.ascontiguousarray(row_lse32, dtype=np.float32)).cuda()
    kb.kvm_attn_mass_from_lse(sh, Qd, Kd, ld, mass, ws)
    torch.cuda.synchronize()
    return mass.cpu().numpy()


def gpu_mass_append(q_new, K, mass32, dtype, G=1, seq_lens=None):
    qd, Kd = to_dev(q_new, dtype), to_dev(K, dtype)
    sl = lens_dev(seq_lens)
    sh = kb.make_shape(Kd, G, sl)
    mass = torch.from_numpy(np.ascontiguousarray(mass32, dtype=np.float32)).cuda()
    ws = torch.empty(max(kb.kvm_workspace_bytes(sh), 256), dtype=torch.uint8, device="cuda")
    kb.kvm_attn_mass_append(sh, qd, Kd, mass, ws)
    torch.cuda.synchronize()
    return mass.cpu().numpy()


def gpu_identify(K, mass32, dtype, params, seq_lens=None, want_sim=True):
    Kd = to_dev(K, dtype)
    sl = lens_dev(seq_lens)
    sh = kb.make_shape(Kd, 1, sl)
    B, H, N, _ = K.shape
    cap = kb.kvm_out_capacity(sh, params)
    i32 = dict(dtype=torch.int32, device="cuda")
    o = dict(set_id=torch.full((B, H, N), -7, **i32), set_start=torch.full((B, H, cap + 1), -7, **i32),
             pivot=torch.full((B, H, cap), -7, **i32), n_sets=torch.full((B, H), -7, **i32),
             status=torch.full((B, H), -7, **i32),
             sim=torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda") if want_sim else None)
    ws = torch.empty(max(kb.kvm_workspace_bytes(sh, params), 256), dtype=torch.uint8, device="cuda")
    md = torch.from_numpy(np.ascontiguousarray(mass32, dtype=np.float32)).cuda()
    kb.kvm_identify_sets(sh, params, Kd, md, o["set_id"], o["set_start"], o["pivot"], o["n_sets"], o["sim"],
                         o["status"], ws)
    torch.cuda.synchronize()
    out = {k: (None if v is None else v.cpu().numpy()) for k, v in o.items()}
    out["cap_rows"] = cap
    return out


def gpu_merge(K, V, dtype, params, set_start, pivot, n_sets, seq_lens=None, want_w=True):
    Kd, Vd = to_dev(K, dtype), to_dev(V, dtype)
    sl = lens_dev(seq_lens)
    sh = kb.make_shape(Kd, 1, sl)
    B, H, N, d = K.shape
    cap = kb.kvm_out_capacity(sh, params)
    assert pivot.shape[-1] == cap
    Ko = torch.zeros((B, H, cap, d), dtype=TORCH_DT[dtype], device="cuda")
    Vo = torch.zeros((B, H, cap, d), dtype=TORCH_DT[dtype], device="cuda")
    w = torch.zeros((B, H, N), dtype=torch.float32, device="cuda") if want_w else None
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    ws = torch.empty(max(kb.kvm_workspace_bytes(sh, params), 256), dtype=torch.uint8, device="cuda")
    kb.kvm_merge(sh, params, Kd, Vd, i32(set_start), i32(pivot), i32(n_sets), Ko, Vo, w, ws)
    torch.cuda.synchronize()
    return to_host_f64(Ko), to_host_f64(Vo), (None if w is None else w.cpu().numpy()), Ko, Vo


def assert_mass_close(got32, want64, lens, N, what=""):
    """Elementwise relative error on valid positions; exact zero on padding."""
    B, H, _ = want64.shape
    worst = 0.0
    for b in range(B):
        n = N if lens is None else int(lens[b])
        g, w = got32[b, :, :n].astype(np.float64), want64[b, :, :n]
        assert (got32[b, :, n:] == 0).all(), f"{what}: padding of batch {b} is not zero"
        if n:
            assert np.isfinite(g).all(), f"{what}: non-finite mass"
            err = np.abs(g - w) / w
            worst = max(worst, float(err.max()))
    assert worst <= TOL, f"{what}: mass relative error {worst:.3e} > {TOL}"
    return worst


def row_rel_err(got64, want64):
    """Per row: max |x - ref| / max |ref| (the row-normalised error)."""
    num = np.abs(got64 - want64).max(axis=-1)
    den = np.abs(want64).max(axis=-1)
    den = np.where(den == 0, 1.0, den)
    return num / den


def kv_tol(dtype):
    return TOL + UNIT_ROUNDOFF[dtype]


def storage_ulp(x64, dtype):
    """Spacing of the storage format at |x| (elementwise)."""
    e = np.floor(np.log2(np.maximum(np.abs(x64), 2.0 ** MIN_EXP[dtype])))
    return 2.0 ** (e - MANT_BITS[dtype])


def ulp_excess(got64, want64, dtype):
    """Per row: max over elements of (|got - want| - 1 ulp(want)) / max|want|.  A correctly
    rounded fp32-accumulated result stays within one ulp of the exact value; what is left is
    arithmetic error, which must be tiny."""
    den = np.abs(want64).max(axis=-1, keepdims=True)
    den = np.where(den == 0, 1.0, den)
    return (np.maximum(np.abs(got64 - want64) - storage_ulp(want64, dtype), 0.0) / den).max(axis=-1)


def compare_maps(g, o, lens, N, eps, what=""):
    """Bit-exact comparison of the index maps of every slice.  A slice whose boundary flags
    differ only at positions whose oracle similarity lies within NEAR of the (effective)
    threshold is counted as excused; any other difference fails.  Returns (#excused slices,
    #near-threshold similarities seen)."""
    B, H, _ = o["set_id"].shape
    cap = o["cap_rows"]
    excused = near_total = 0
    for b in range(B):
        n = N if lens is None else int(lens[b])
        for h in range(H):
            tag = f"{what} slice ({b},{h})"
            eff = eps
            if o["status"][b, h] & kb.KVM_SLICE_FALLBACK and np.isfinite(o["min_removed_sim"][b, h]):
                eff = o["min_removed_sim"][b, h]
            near = np.abs(o["sim"][b, h, 1:n] - eps) <= NEAR
            if eff != eps:
                near |= np.abs(o["sim"][b, h, 1:n] - eff) <= NEAR
            near_total += int(near.sum())
            same = (np.array_equal(g["set_id"][b, h], o["set_id"][b, h]) and g["n_sets"][b, h] == o["n_sets"][b, h]
                    and np.array_equal(g["set_start"][b, h], o["set_start"][b, h])
                    and np.array_equal(g["pivot"][b, h], o["pivot"][b, h]) and g["status"][b, h] == o["status"][b, h])
            if same:
                continue
            gb = np.diff(g["set_id"][b, h, :n]) != 0
            ob = np.diff(o["set_id"][b, h, :n]) != 0
            diff = np.flatnonzero(gb != ob)
            assert len(diff) and near[diff].all(), \
                f"{tag}: maps differ away from the threshold (n_sets {g['n_sets'][b, h]} vs {o['n_sets'][b, h]}, " \
                f"first boundary difference at {diff[:5] + 1}, status {g['status'][b, h]} vs {o['status'][b, h]})"
            excused += 1
    return excused, near_total


def check_partition(g, lens, N, cap_rows, what=""):
    """Validity of GPU index maps on their own: contiguous, disjoint, covering; pivots inside."""
    B, H, _ = g["set_id"].shape
    for b in range(B):
        n = N if lens is None else int(lens[b])
        for h in range(H):
            sid, M = g["set_id"][b, h], int(g["n_sets"][b, h])
            assert (sid[n:] == -1).all(), what
            if n == 0:
                assert M == 0
                continue
            assert sid[0] == 0 and sid[n - 1] == M - 1, what
            d = np.diff(sid[:n])
            assert ((d == 0) | (d == 1)).all(), what
            k = min(M, cap_rows)
            st, pv = g["set_start"][b, h], g["pivot"][b, h]
            starts = np.flatnonzero(np.concatenate([[True], d == 1]))
            assert np.array_equal(st[:k], starts[:k]), what
            ends = np.append(starts[1:], n)
            assert ((pv[:k] >= starts[:k]) & (pv[:k] < ends[:k])).all(), what
