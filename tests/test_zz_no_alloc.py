"""kvm_merge_static -- the merge for callers that cannot allocate -- against kvm_merge, through
the C ABI.  Both run the same kernels, so the outputs have to be bit-identical; the call is
made twice in a row, the second time on a smaller input, because the built-in buffer keeps
the first call's plan.  This file is collected last: a failure here must not hide others."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2407_08454_amd import binding as kb
from paper_2407_08454_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _maps_from_the_oracle(K, Q, dtype, params, lens, cap):
    mass = ref.attn_mass(Q, K, dtype, seq_lens=lens)
    return ref.identify_sets(K, mass.astype(np.float32).astype(np.float64), dtype, params.budget, params.recent_ratio,
                             params.heavy_ratio, params.threshold, True, cap, lens)


def _both(B, H, N, lens, dtype, seed):
    Q = np.empty((B, H, N, 128), synth.storage_numpy_dtype(dtype))
    K, V = np.empty_like(Q), np.empty_like(Q)
    for b in range(B):
        for h in range(H):
            q, k, v, _ = synth.gen_slice(seed, b * H + h, lens[b], 128, 1, None, dtype, N)
            Q[b, h], K[b, h], V[b, h] = q[0], k, v
    params = kb.kvm_params_for_budget(0.5)
    Kd, Vd = gu.to_dev(K, dtype), gu.to_dev(V, dtype)
    sl = gu.lens_dev(lens)
    sh = kb.make_shape(Kd, 1, sl)
    cap = kb.kvm_out_capacity(sh, params)
    o = _maps_from_the_oracle(K, Q, dtype, params, lens, cap)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    st, pv, ns = i32(o["set_start"]), i32(o["pivot"]), i32(o["n_sets"])
    tdt = gu.TORCH_DT[dtype]
    out = []
    for static in (False, True):
        Ko = torch.full((B, H, cap, 128), 7.0, dtype=tdt, device="cuda")
        Vo = torch.full((B, H, cap, 128), 7.0, dtype=tdt, device="cuda")
        w = torch.full((B, H, N), -1.0, dtype=torch.float32, device="cuda")
        if static:
            kb.kvm_merge_static(sh, params, Kd, Vd, st, pv, ns, Ko, Vo, w)
        else:
            ws = torch.empty(max(kb.kvm_workspace_bytes(sh, params), 256), dtype=torch.uint8, device="cuda")
            kb.kvm_merge(sh, params, Kd, Vd, st, pv, ns, Ko, Vo, w, ws)
        torch.cuda.synchronize()
        out.append((Ko, Vo, w))
    (k0, v0, w0), (k1, v1, w1) = out
    assert torch.equal(k0.view(torch.int16 if dtype != "f32" else torch.int32), k1.view(torch.int16 if dtype != "f32" else torch.int32))
    assert torch.equal(v0.view(torch.int16 if dtype != "f32" else torch.int32), v1.view(torch.int16 if dtype != "f32" else torch.int32))
    assert torch.equal(w0.view(torch.int32), w1.view(torch.int32))
    # and against the oracle, to the bar of the merge tests
    rk, rv, _ = ref.merge(K, V, dtype, o["set_start"], o["pivot"], o["n_sets"], seq_lens=lens)
    for b in range(B):
        for h in range(H):
            M = min(int(o["n_sets"][b, h]), cap)
            if M == 0:
                continue
            assert gu.row_rel_err(gu.to_host_f64(k1[b, h, :M]), rk[b, h, :M]).max() <= gu.kv_tol(dtype)
            assert gu.row_rel_err(gu.to_host_f64(v1[b, h, :M]), rv[b, h, :M]).max() <= gu.kv_tol(dtype)
            assert gu.ulp_excess(gu.to_host_f64(k1[b, h, :M]), rk[b, h, :M], dtype).max() <= 2e-5
            assert gu.ulp_excess(gu.to_host_f64(v1[b, h, :M]), rv[b, h, :M], dtype).max() <= 2e-5


def test_merge_static_twice_in_a_row_the_second_call_smaller():
    print("kvm_merge_static: 3 x 2 slices, N=1500 ragged, f16", flush=True)
    _both(3, 2, 1500, [1500, 777, 0], "f16", 71)
    print("kvm_merge_static: 1 x 2 slices, N=300, bf16", flush=True)
    _both(1, 2, 300, [300], "bf16", 72)
