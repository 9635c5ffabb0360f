"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before any launch (no GPU needed: these calls return
before touching the device)."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from paper_2407_08454_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kvm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(kvm_[a-z_]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = kb.load_library()
    names = _declared()
    assert names == set(kb.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert re.fullmatch(r"\d+\.\d+\.\d+", lib.kvm_version().decode())


def test_header_is_plain_c_and_matches_the_binding_structs(tmp_path):
    """The header has to compile as C99 and as C++ on its own, and the ctypes mirror of its two
    structs has to have the sizes and field offsets the C compiler gives them."""
    import subprocess
    fields = {"kvm_shape": [f[0] for f in kb.KvmShape._fields_], "kvm_params": [f[0] for f in kb.KvmParams._fields_]}
    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "kvm.h"', 'int main(void) {']
    for st, names in fields.items():
        lines.append(f'  printf("{st} %zu\\n", sizeof({st}));')
        for n in names:
            lines.append(f'  printf("{st}.{n} %zu\\n", offsetof({st}, {n}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st, cls in (("kvm_shape", kb.KvmShape), ("kvm_params", kb.KvmParams)):
        assert int(got[st]) == ctypes.sizeof(cls)
        for n in fields[st]:
            assert int(got[f"{st}.{n}"]) == getattr(cls, n).offset, f"{st}.{n}"


def test_presets_follow_the_printed_hyperparameters():
    p = kb.kvm_params_for_budget(0.5)
    assert (p.budget, p.recent_ratio, p.heavy_ratio, p.threshold) == (0.5, 0.17, 0.12, 0.75)
    p = kb.kvm_params_for_budget(0.35)
    assert (p.budget, p.recent_ratio, p.heavy_ratio, p.threshold) == (0.35, 0.08, 0.02, 0.75)
    assert p.enforce_budget == 1 and p.value_scale_by_set_size == 1 and p.sigma_mode == kb.KVM_SIGMA_MEAN_DIST
    assert (p.weights, p.pivot_rule, p.pivot_seed, p.set_rule) == (kb.KVM_WEIGHTS_GAUSSIAN, kb.KVM_PIVOT_MAX_SCORE, 0,
                                                                   kb.KVM_SETS_ADJACENT)
    p = kb.kvm_params_for_budget(0.25)
    assert p.recent_ratio + p.heavy_ratio < 0.25
    with pytest.raises(kb.KvmError):
        kb.kvm_params_for_budget(0.0)
    with pytest.raises(kb.KvmError):
        kb.kvm_params_for_budget(1.5)


def _shape(**kw):
    d = dict(B=2, H_kv=3, G=1, N=100, d=128, dtype=kb.KVM_F16, seq_lens=None)
    d.update(kw)
    return kb.KvmShape(**d)


def test_capacity_and_workspace():
    p = kb.kvm_params_for_budget(0.35)
    assert kb.kvm_out_capacity(_shape(N=4096), p) == 1433 == math.floor(0.35 * 4096)
    p.enforce_budget = 0
    assert kb.kvm_out_capacity(_shape(N=4096), p) == 4096
    sh = _shape(B=4, H_kv=8, G=4, N=1000)
    need = kb.kvm_workspace_bytes(sh, p)
    assert need >= 4 * 8 * 4 * 1000 * 4 and need >= 4 * 8 * 1000 * 13
    assert kb.kvm_workspace_bytes(_shape(d=64), p) == 0


def test_host_detectable_errors_return_before_any_launch():
    lib = kb.load_library()
    p = kb.kvm_params_for_budget(0.5)
    one = ctypes.c_void_p(256)            # never dereferenced: the calls fail before any launch

    def attn(sh, Q=one, K=one, mass=one, ws=one, nbytes=1 << 30):
        return lib.kvm_attn_mass(ctypes.byref(sh), Q, K, mass, ws, nbytes, None)

    assert attn(_shape(d=64)) == kb.KVM_ERR_UNSUPPORTED and b"head dimension" in lib.kvm_last_error()
    assert attn(_shape(dtype=7)) == kb.KVM_ERR_UNSUPPORTED
    assert attn(_shape(G=0)) == kb.KVM_ERR_INVALID_ARG
    assert attn(_shape(N=-1)) == kb.KVM_ERR_INVALID_ARG
    assert attn(_shape(), Q=None) == kb.KVM_ERR_INVALID_ARG
    assert attn(_shape(), ws=None) == kb.KVM_ERR_WORKSPACE
    assert attn(_shape(), nbytes=16) == kb.KVM_ERR_WORKSPACE and b"workspace" in lib.kvm_last_error()
    assert lib.kvm_attn_mass(None, one, one, one, one, 0, None) == kb.KVM_ERR_INVALID_ARG

    def attn_lse(sh, row_lse=one, ws=one, nbytes=1 << 30):
        return lib.kvm_attn_mass_from_lse(ctypes.byref(sh), one, one, row_lse, one, ws, nbytes, None)

    assert attn_lse(_shape(d=64)) == kb.KVM_ERR_UNSUPPORTED
    assert attn_lse(_shape(), row_lse=None) == kb.KVM_ERR_INVALID_ARG and b"row_lse" in lib.kvm_last_error()
    assert attn_lse(_shape(), nbytes=16) == kb.KVM_ERR_WORKSPACE and b"kvm_attn_mass_from_lse" in lib.kvm_last_error()
    assert attn_lse(_shape(N=0), row_lse=None, ws=None) == kb.KVM_OK          # nothing to do

    def attn_sim(sh, sim=one, ws=one, nbytes=1 << 30):
        return lib.kvm_attn_mass_sim(ctypes.byref(sh), one, one, one, sim, ws, nbytes, None)

    assert attn_sim(_shape(d=64)) == kb.KVM_ERR_UNSUPPORTED
    assert attn_sim(_shape(), sim=None) == kb.KVM_ERR_INVALID_ARG and b"sim" in lib.kvm_last_error()
    assert attn_sim(_shape(), nbytes=16) == kb.KVM_ERR_WORKSPACE and b"kvm_attn_mass_sim" in lib.kvm_last_error()
    assert attn_sim(_shape(N=0), sim=None, ws=None) == kb.KVM_OK              # nothing to do

    def append(sh, q=one, ws=one, nbytes=1 << 30):
        return lib.kvm_attn_mass_append(ctypes.byref(sh), q, one, one, ws, nbytes, None)

    assert append(_shape(d=64)) == kb.KVM_ERR_UNSUPPORTED
    assert append(_shape(), q=None) == kb.KVM_ERR_INVALID_ARG and b"q_new" in lib.kvm_last_error()
    assert append(_shape(), nbytes=16) == kb.KVM_ERR_WORKSPACE and b"kvm_attn_mass_append" in lib.kvm_last_error()
    assert append(_shape(N=0), q=None, ws=None) == kb.KVM_OK                     # nothing to do

    def ident(sh, pr, ws=one, nbytes=1 << 30, K=one):
        return lib.kvm_identify_sets(ctypes.byref(sh), ctypes.byref(pr), K, one, one, one, one, one, None, one, ws,
                                     nbytes, None)

    bad = kb.make_params(0.5, 0.4, 0.3)                  # conserved fraction above the budget
    assert ident(_shape(), bad) == kb.KVM_ERR_INVALID_ARG and b"exceeds the budget" in lib.kvm_last_error()
    assert ident(_shape(), kb.make_params(1.5, 0.1, 0.1)) == kb.KVM_ERR_INVALID_ARG
    assert ident(_shape(), kb.make_params(0.5, 0.1, 0.1, threshold=float("nan"))) == kb.KVM_ERR_INVALID_ARG
    assert ident(_shape(), kb.make_params(0.5, 0.1, 0.1, sigma_mode=5)) == kb.KVM_ERR_UNSUPPORTED
    assert ident(_shape(), kb.make_params(0.5, 0.1, 0.1, weights=2)) == kb.KVM_ERR_UNSUPPORTED
    assert ident(_shape(), kb.make_params(0.5, 0.1, 0.1, pivot_rule=3)) == kb.KVM_ERR_UNSUPPORTED
    assert ident(_shape(), kb.make_params(0.5, 0.1, 0.1, set_rule=2)) == kb.KVM_ERR_UNSUPPORTED and \
        b"set_rule" in lib.kvm_last_error()
    given = kb.make_params(0.5, 0.1, 0.1, sim_given=True)
    assert ident(_shape(), given) == kb.KVM_ERR_INVALID_ARG and b"sim_given" in lib.kvm_last_error()   # no sim_opt passed
    assert lib.kvm_sim_append(ctypes.byref(_shape()), None, one, None) == kb.KVM_ERR_INVALID_ARG
    assert lib.kvm_sim_append(ctypes.byref(_shape(d=64)), one, one, None) == kb.KVM_ERR_UNSUPPORTED
    assert lib.kvm_sim_append(ctypes.byref(_shape(N=0)), None, None, None) == kb.KVM_OK
    assert ident(_shape(), p, K=None) == kb.KVM_ERR_INVALID_ARG
    assert ident(_shape(), p, nbytes=8) == kb.KVM_ERR_WORKSPACE

    def merge(sh, pr, K=one, ws=one, nbytes=1 << 30):
        return lib.kvm_merge(ctypes.byref(sh), ctypes.byref(pr), K, one, one, one, one, one, one, None, ws, nbytes, None)

    assert merge(_shape(), kb.make_params(0.5, 0.1, 0.1, sigma_mode=kb.KVM_SIGMA_FIXED, sigma=0.0)) == kb.KVM_ERR_INVALID_ARG
    assert merge(_shape(), p, K=None) == kb.KVM_ERR_INVALID_ARG
    assert merge(_shape(d=256), p) == kb.KVM_ERR_UNSUPPORTED
    assert merge(_shape(), p, ws=None) == kb.KVM_ERR_WORKSPACE
    assert merge(_shape(), p, nbytes=4) == kb.KVM_ERR_WORKSPACE

    def merge_static(sh, pr, K=one):
        return lib.kvm_merge_static(ctypes.byref(sh), ctypes.byref(pr), K, one, one, one, one, one, one, None, None)

    assert merge_static(_shape(), p, K=None) == kb.KVM_ERR_INVALID_ARG
    assert merge_static(_shape(d=256), p) == kb.KVM_ERR_UNSUPPORTED
    assert merge_static(_shape(N=0), p, K=None) == kb.KVM_OK                      # nothing to do
    # 2^16 slices of 2049 plan entries each do not fit the built-in buffer of 2^21: refused, nothing launched
    assert merge_static(_shape(B=2 ** 10, H_kv=2 ** 6, N=2 ** 17), p) == kb.KVM_ERR_WORKSPACE
    assert b"built-in buffer" in lib.kvm_last_error()

    two = ctypes.c_void_p(32)

    def refresh(sh, pr, K=one, new=two, ws=one, nbytes=1 << 30):
        return lib.kvm_merge_refresh(ctypes.byref(sh), ctypes.byref(pr), K, one, one, one, one, one, new, new, new, one, one, None,
                                     ws, nbytes, None)

    assert refresh(_shape(), p, K=None) == kb.KVM_ERR_INVALID_ARG
    assert refresh(_shape(), p, new=one) == kb.KVM_ERR_INVALID_ARG and b"different buffers" in lib.kvm_last_error()
    assert refresh(_shape(d=256), p) == kb.KVM_ERR_UNSUPPORTED
    assert refresh(_shape(), p, ws=None) == kb.KVM_ERR_WORKSPACE
    assert refresh(_shape(), p, nbytes=4) == kb.KVM_ERR_WORKSPACE
    assert refresh(_shape(N=0), p, K=None) == kb.KVM_OK                           # nothing to do

    for fn in (lib.kvm_evict, lib.kvm_evict_merge_values):                        # the two comparison workloads
        def evict(sh, pr, K=one, ws=one, nbytes=1 << 30):
            return fn(ctypes.byref(sh), ctypes.byref(pr), K, one, one, one, one, one, one, ws, nbytes, None)
        assert evict(_shape(), p, K=None) == kb.KVM_ERR_INVALID_ARG
        assert evict(_shape(d=256), p) == kb.KVM_ERR_UNSUPPORTED
        assert evict(_shape(), p, ws=None) == kb.KVM_ERR_WORKSPACE
        assert evict(_shape(), p, nbytes=8) == kb.KVM_ERR_WORKSPACE
        assert evict(_shape(B=0), p, K=None) == kb.KVM_OK


def test_binding_refuses_mismatched_tensors_on_the_host():
    import torch
    K = torch.zeros((1, 2, 8, 128), dtype=torch.float16)
    sh = kb.make_shape(K)
    assert (sh.B, sh.H_kv, sh.N, sh.d, sh.dtype) == (1, 2, 8, 128, kb.KVM_F16)
    with pytest.raises(ValueError):
        kb.make_shape(K[:, :, ::2])                       # not contiguous
    with pytest.raises(ValueError):
        kb.make_shape(K.to(torch.float64))
    with pytest.raises(ValueError):                       # CPU tensors never reach the library
        kb.kvm_attn_mass(sh, K, K, torch.zeros((1, 2, 8)), torch.zeros(1024, dtype=torch.uint8))


def test_layer_by_layer_generation_gives_the_bits_of_the_whole_workload():
    """Large workloads are generated one layer at a time on the host; the layers must be the ones
    the whole-workload generator gives (same seeds per slice)."""
    from paper_2407_08454_amd import synth
    cfg = dict(name="tiny", layers=3, batch=2, H_kv=2, G=2, N=64, d=128, dtype="bf16", rho=None, budgets=(0.5,), seed=7,
               seq_lens=(40, 64))
    Q, K, V, sl = synth.gen_config(cfg, workers=1)
    layers = list(synth.gen_config_layers(cfg, workers=1))
    assert len(layers) == 3
    for layer, (q, k, v, s) in enumerate(layers):
        rows = slice(layer * 2, layer * 2 + 2)                   # layers are folded into the batch axis
        assert np.array_equal(q, Q[rows]) and np.array_equal(k, K[rows]) and np.array_equal(v, V[rows])
        assert np.array_equal(s, sl[rows])
