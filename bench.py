#!/usr/bin/env python3
"""Benchmark of the whole KV-merging compression pass on one MI355X.

A step = one pass of the hot path (kvm_attn_mass, kvm_identify_sets, kvm_merge) over every
(layer, KV-head) slice of the workload, inputs resident in HBM.  The default workload is the
Llama2-7B shape (32 layers x 32 KV heads, N = 4096, d = 128, fp16, budget 0.5) on seeded
synthetic Q/K/V.  Prints one JSON line; `roofline` describes the dominant kernel from HIP
events recorded by the library on its launch stream inside the timed region, `cpu_baseline`
is the fp64 oracle timed on the host cores on a sample of the same slices.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA = {"f16": 2.5e15, "bf16": 2.5e15, "f32": 157.3e12}   # dense matrix peaks, FLOP/s
PEAK_HBM = 8.0e12                                               # B/s
METRIC = "KV tokens compressed/sec (all layers x heads) at Llama2-7B N=4096"

def kernel_sources_sha256() -> str:
    """Hash of the HIP sources the library is built from: the stamp of the counter measurements under profiles/."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2407_08454_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload: str) -> dict:
    """{kernel: (bytes fetched, bytes written) per launch} from profiles/hbm_traffic_<workload>.md (FETCH_SIZE /
    WRITE_SIZE counter runs; hardware counters cannot be read from inside this process).  Empty when the file is
    missing or was measured on other kernel sources than the ones in the tree: the figures would be stale."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.md")
    if not os.path.exists(path):
        return {}
    out, stamp = {}, None
    for line in open(path):
        if line.startswith("sources_sha256:"):
            stamp = line.split(":", 1)[1].strip()
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 3 and cells[0].endswith("_kernel") and cells[1].isdigit() and cells[2].isdigit():
            out[cells[0]] = (int(cells[1]), int(cells[2]))
    return out if stamp == kernel_sources_sha256() else {}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload id (2 = the headline Llama2-7B shape)")
    ap.add_argument("--layers", type=int, default=None, help="generate only this many layers (not the headline run)")
    ap.add_argument("--budget", type=float, default=0.5)
    ap.add_argument("--threshold", type=float, default=None, help="similarity threshold (default: the preset's 0.75)")
    ap.add_argument("--cpu-slices", type=int, default=512, help="slices the oracle is timed on (0 = skip)")
    ap.add_argument("--sim-from-score-pass", action="store_true",
                    help="similarities written by the score pass (kvm_attn_mass_sim) instead of kvm_identify_sets' own scan of K")
    ap.add_argument("--no-profile", action="store_true", help="no per-kernel events inside the timed region")
    ap.add_argument("--weights", choices=["gaussian", "average"], default="gaussian",
                    help="merge weights (average = the average weighted merging of Section 4.2)")
    ap.add_argument("--pivot", choices=["max-score", "last", "random"], default="max-score",
                    help="pivot rule (last = largest index, Section 4.2; random = Section 5.4)")
    ap.add_argument("--method", choices=["merge", "evict", "evict-merge-values", "append"], default="merge",
                    help="evict = the comparison workload: attention mass, then plain eviction by score (kvm_evict); "
                         "evict-merge-values = the same with the evicted values averaged into the nearest kept token "
                         "(kvm_evict_merge_values); "
                         "append = decode-time refresh: one more query row added to the scores (kvm_attn_mass_append), "
                         "then sets and merge again")
    ap.add_argument("--sets", choices=["adjacent", "anchor"], default="adjacent",
                    help="reading of Algorithm 1 (anchor = similarity to the set's top token; no budget fallback)")
    ap.add_argument("--row-stats", choices=["computed", "given"], default="computed",
                    help="given = the softmax row statistics are an input, as left behind by a prefill attention kernel "
                         "(kvm_attn_mass_from_lse: only the column-sum pass runs)")
    ap.add_argument("--sigma", type=float, default=None, help="fixed sigma (Section 5.4) instead of the per-set one")
    ap.add_argument("--keys", choices=["ar1", "identical"], default="ar1",
                    help="identical = every key of a slice equals its first key: the degenerate case in which all free "
                         "tokens of a slice form one merging set (worst case of the merge kernel, not the headline)")
    ap.add_argument("--gen-workers", type=int, default=None,
                    help="processes that generate the inputs (1 = in this process, e.g. under a profiler)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of K before the timed region (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every (layer, head) slice is independent, so more GPUs "
              "would each take a share of the slices with no exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2407_08454_amd import binding as kb
    from paper_2407_08454_amd import synth

    cfg = synth.CONFIGS[args.config]
    dtype = cfg["dtype"]
    t0 = time.time()
    Q, K, V, lens = synth.gen_config(cfg, layers=args.layers, workers=args.gen_workers)
    gen_s = time.time() - t0
    B, H, G, N, d = K.shape[0], cfg["H_kv"], cfg["G"], cfg["N"], cfg["d"]
    n_per_b = np.full(B, N, np.int64) if lens is None else lens.astype(np.int64)
    token_slices = int(n_per_b.sum()) * H

    torch.cuda.set_device(0)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]

    def dev(x):
        if dtype == "bf16":
            return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(x).cuda()

    if args.keys == "identical":
        K[:] = K[:, :, :1]
    Qd, Kd, Vd = dev(Q), dev(K), dev(V)
    sl = None if lens is None else torch.from_numpy(lens).cuda()
    params = kb.kvm_params_for_budget(args.budget)
    if args.threshold is not None:
        params.threshold = args.threshold
    params.weights = {"gaussian": kb.KVM_WEIGHTS_GAUSSIAN, "average": kb.KVM_WEIGHTS_AVERAGE}[args.weights]
    params.pivot_rule = {"max-score": kb.KVM_PIVOT_MAX_SCORE, "last": kb.KVM_PIVOT_LAST,
                         "random": kb.KVM_PIVOT_RANDOM}[args.pivot]
    if args.sigma is not None:
        params.sigma_mode, params.sigma = kb.KVM_SIGMA_FIXED, args.sigma
    if args.sets == "anchor":
        params.set_rule = kb.KVM_SETS_ANCHOR
    variant = (f"sets {args.sets}, weights {args.weights}, pivot {args.pivot}, "
               f"sigma {'per set' if args.sigma is None else args.sigma}"
               + ("" if args.threshold is None else f", threshold {args.threshold}"))
    shape = kb.make_shape(Kd, G, sl)
    buf = kb.Buffers(shape, params, "cuda", tdt, with_sim=args.sim_from_score_pass)

    row_lse = sim_carried = None
    if args.row_stats == "given":
        # stand-in for what a prefill attention kernel leaves behind: natural-log softmax denominators,
        # made here with library calls before anything is timed
        variant += "; row statistics given by the caller"
        row_lse = torch.empty((B, H * G, N), dtype=torch.float32, device="cuda")
        upper = torch.triu(torch.ones((N, N), dtype=torch.bool, device="cuda"), 1)
        for b in range(B):
            for hq in range(H * G):
                s_ = (Qd[b, hq].float() @ Kd[b, hq // G].float().T) * (1.0 / d ** 0.5)
                row_lse[b, hq] = torch.logsumexp(s_.masked_fill_(upper, float("-inf")), dim=1)
        del upper, s_

    append = args.method == "append"
    if append:
        # Decode-time loop on a growing sequence: the prompt is the workload minus the tokens that the
        # warm-up and timed steps append; its whole pass runs once, untimed.  Every step then appends one
        # token: one query row added to the scores, one new similarity, sets identified again (similarities
        # carried), and the compacted cache brought up to date (kvm_merge_refresh).
        variant += "; decode-time refresh (per token: one query row, one similarity, sets, cache refresh)"
        grow = args.warmup + args.steps
        if lens is not None or grow >= N:
            print("bench.py: --method append needs a workload of equal lengths longer than warmup + steps", file=sys.stderr)
            return 2
        sl = torch.full((B,), N - grow, dtype=torch.int32, device="cuda")
        shape = kb.make_shape(Kd, G, sl)
        kb.kvm_attn_mass(shape, Qd, Kd, buf.mass, buf.ws)
        sim_carried = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        maps = [(buf.set_id, buf.set_start, buf.pivot, buf.n_sets),
                tuple(torch.empty_like(t) for t in (buf.set_id, buf.set_start, buf.pivot, buf.n_sets))]
        cur = [0]
        kb.kvm_identify_sets(shape, params, Kd, buf.mass, *maps[0], sim_carried, buf.status, buf.ws)
        kb.kvm_merge(shape, params, Kd, Vd, maps[0][1], maps[0][2], maps[0][3], buf.K_out, buf.V_out, None, buf.ws)
        params.sim_given = 0 if args.sets == "anchor" else 1       # the anchor rule needs the key norms of a scan
        n_now = [N - grow]
        # the appended tokens' query rows, one contiguous (B, H G, d) block per step
        q_steps = Qd[:, :, N - grow:N].permute(2, 0, 1, 3).contiguous()

    # on request the similarities come out of the score pass (kvm_attn_mass_sim) and the sets' own scan of K is skipped
    fused = (args.sim_from_score_pass and args.sets == "adjacent" and row_lse is None and not append
             and args.method == "merge")
    params_sets = params
    if fused:
        variant += "; adjacent similarities written by the score pass"
        sim_carried = buf.sim
        params_sets = kb.KvmParams.from_buffer_copy(params)
        params_sets.sim_given = 1

    def attn_mass():
        if append:
            sl.add_(1)                                          # the token's key and value are already in K, V
            n_now[0] += 1
            q_new = q_steps[n_now[0] - 1 - (N - grow)]
            kb.kvm_attn_mass_append(shape, q_new, Kd, buf.mass, buf.ws)
            kb.kvm_sim_append(shape, Kd, sim_carried)
        elif fused:
            kb.kvm_attn_mass_sim(shape, Qd, Kd, buf.mass, sim_carried, buf.ws)
        elif row_lse is None:
            kb.kvm_attn_mass(shape, Qd, Kd, buf.mass, buf.ws)
        else:
            kb.kvm_attn_mass_from_lse(shape, Qd, Kd, row_lse, buf.mass, buf.ws)

    evict = args.method in ("evict", "evict-merge-values")
    if evict:
        evict_call = kb.kvm_evict if args.method == "evict" else kb.kvm_evict_merge_values
        variant = ("comparison workload: eviction by score" if args.method == "evict" else
                   "comparison workload: eviction by score, evicted values averaged into the nearest kept token") + \
            ("; row statistics given by the caller" if row_lse is not None else "")
        # kept positions go where the pivots would, their count where the set count would
        def rest():
            evict_call(shape, params, Kd, Vd, buf.mass, buf.pivot, buf.n_sets, buf.K_out, buf.V_out, buf.ws)
        buf.status.zero_()
    def identify():
        if append:
            new = maps[1 - cur[0]]
            kb.kvm_identify_sets(shape, params, Kd, buf.mass, *new, sim_carried, buf.status, buf.ws)
        else:
            kb.kvm_identify_sets(shape, params_sets, Kd, buf.mass, buf.set_id, buf.set_start, buf.pivot, buf.n_sets,
                                 sim_carried, buf.status, buf.ws)

    def merge():
        if append:
            old, new = maps[cur[0]], maps[1 - cur[0]]
            kb.kvm_merge_refresh(shape, params, Kd, Vd, *old, new[1], new[2], new[3], buf.K_out, buf.V_out, None, buf.ws)
            cur[0] = 1 - cur[0]
        else:
            kb.kvm_merge(shape, params, Kd, Vd, buf.set_start, buf.pivot, buf.n_sets, buf.K_out, buf.V_out, None, buf.ws)

    for _ in range(args.warmup):
        attn_mass()
        if evict:
            rest()
        else:
            identify()
            merge()
    torch.cuda.synchronize()
    if args.calibration_copy:          # reads and writes K.numel() * element_size bytes exactly once
        copy = torch.empty_like(Kd)
        copy.copy_(Kd)
        torch.cuda.synchronize()
        del copy

    if not args.no_profile:
        kb.kvm_profile_enable(12 * args.steps)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in ev:
        e[0].record()
        attn_mass()
        e[1].record()
        if evict:
            e[2].record()
            rest()
        else:
            identify()
            e[2].record()
            merge()
        e[3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = [sum(e[i].elapsed_time(e[i + 1]) for e in ev) for i in range(3)]
    kernels = {}
    if not args.no_profile:
        kernels = {k: v[1] / max(v[0], 1) for k, v in kb.kvm_profile_collect().items()}
        kb.kvm_profile_disable()

    n_sets = (maps[cur[0]][3] if append else buf.n_sets).cpu().numpy().astype(np.int64)
    status = buf.status.cpu().numpy()
    M_total = int(n_sets.sum())

    # ---- roofline of the dominant kernel -----------------------------------------------------
    esz = 4 if dtype == "f32" else 2
    # algorithmic work per launch: one causal QK^T for each attention kernel; bytes streamed once
    flops_attn = float(sum(G * n * (n + 1) * d for n in n_per_b) * H)
    bytes_cos = float(token_slices * d * esz + token_slices * 4)
    bytes_merge = float(2 * token_slices * d * esz + 2 * M_total * d * esz + 8 * M_total)
    roofline = None
    hbm = {}
    if args.keys == "identical":
        variant += "; identical keys (one merging set per slice)"
    headline = (args.keys == "ar1" and args.config == 2 and args.layers is None and args.budget == 0.5 and args.weights == "gaussian"
                and args.pivot == "max-score" and args.sigma is None and args.threshold is None and args.sets == "adjacent" and args.method == "merge" and row_lse is None and not fused)

    counters = measured_traffic("llama2-7b_n4096_f16") if headline else {}

    def traffic(name):
        return float(sum(counters[name])) if name in counters else None

    if kernels:
        dom = max(kernels, key=kernels.get)
        if dom.startswith("attn"):
            ach = flops_attn / (kernels[dom] * 1e-3)
            roofline = {"kernel": dom, "bound": "mfma", "achieved": ach / 1e12, "peak": PEAK_MFMA[dtype] / 1e12,
                        "unit": "TFLOP/s", "frac": ach / PEAK_MFMA[dtype], "traffic": traffic(dom),
                        "algorithmic_flops": flops_attn, "ms_per_launch": kernels[dom]}
        else:
            byts = bytes_merge if dom == "merge_kernel" else bytes_cos
            ach = byts / (kernels[dom] * 1e-3)
            roofline = {"kernel": dom, "bound": "hbm", "achieved": ach / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                        "frac": ach / PEAK_HBM, "traffic": traffic(dom), "algorithmic_bytes": byts,
                        "ms_per_launch": kernels[dom]}
        bytes_app = float(token_slices * d * esz + G * token_slices * 4)     # K once, the scores written
        for name, byts in (("cosine_scan_kernel", bytes_cos), ("merge_kernel", bytes_merge),
                           ("append_scores_kernel", bytes_app)):
            if name in kernels:
                hbm[name] = {"algorithmic_GB": byts / 1e9, "traffic": traffic(name), "ms": kernels[name],
                             "GB/s": byts / (kernels[name] * 1e-3) / 1e9,
                             "frac_of_hbm_peak": byts / (kernels[name] * 1e-3) / PEAK_HBM}

    # the stages as wholes: stage (a) counted once (one causal QK^T is the method's work, both score passes are
    # charged to it), stages (b)+(c) together against the bytes they have to move
    # (K twice, V once, merged rows, scores, similarities and maps: 3 n d s + 2 M d s + 20 n per slice)
    stage_fractions = None
    if not append and not evict and stage_ms[0] > 0:
        # (with the similarities written by the score pass, stage (b) no longer reads K: 2 n d s instead of 3)
        bytes_bc = float((2 if fused else 3) * token_slices * d * esz + 2 * M_total * d * esz + 20 * token_slices)
        stage_fractions = {
            "attn_mass_of_mfma_peak": flops_attn / (stage_ms[0] / args.steps * 1e-3) / PEAK_MFMA[dtype],
            "identify_plus_merge_of_hbm_peak": bytes_bc / ((stage_ms[1] + stage_ms[2]) / args.steps * 1e-3) / PEAK_HBM,
            "identify_plus_merge_algorithmic_GB": bytes_bc / 1e9,
        }

    # ---- the oracle on the host cores, on a sample of the same slices --------------------------
    cpu = None
    if args.cpu_slices > 0 and evict:
        print("bench.py: no CPU baseline leg for the comparison workloads (use --cpu-slices 0)", file=sys.stderr)
    if args.cpu_slices > 0 and not evict:
        from oracle import ref

        def oracle_pass(S):
            """The oracle's whole pass (or one decode-time refresh) on S slices spread over layers and heads."""
            idx = np.linspace(0, B * H - 1, S).astype(int)
            Ks = np.ascontiguousarray(K.reshape(B * H, N, d)[idx])[:, None]
            Vs = np.ascontiguousarray(V.reshape(B * H, N, d)[idx])[:, None]
            Qs = np.ascontiguousarray(Q.reshape(B * H, G, N, d)[idx])
            ls = None if lens is None else lens[idx // H]
            t0 = time.perf_counter()
            if append:
                # scores before the step: seeded positive numbers (the oracle's time does not depend on them)
                m0 = np.random.default_rng(0).random((S, 1, N)) + 0.01
                qn = np.ascontiguousarray(Qs[:, :, N - 1] if ls is None else
                                          np.stack([Qs[i, :, max(int(n) - 1, 0)] for i, n in enumerate(ls)]))
                m = ref.attn_mass_append(qn, Ks, m0, dtype, G=G, seq_lens=ls)
            else:
                m = ref.attn_mass(Qs, Ks, dtype, G=G, seq_lens=ls)
            o = ref.identify_sets(Ks, m.astype(np.float32).astype(np.float64), dtype, params.budget, params.recent_ratio,
                                  params.heavy_ratio, params.threshold, True, buf.cap, ls, pivot_rule=params.pivot_rule,
                                  pivot_seed=params.pivot_seed, set_rule=params.set_rule)
            ref.merge(Ks, Vs, dtype, o["set_start"], o["pivot"], o["n_sets"], params.sigma_mode, params.sigma,
                      bool(params.value_scale_by_set_size), seq_lens=ls, weights=params.weights)
            secs = time.perf_counter() - t0
            toks = S if append else int(N * S if ls is None else ls.sum())
            return toks / secs, secs

        what = "one decode-time refresh" if append else "whole pass"
        S = min(args.cpu_slices, B * H)
        cores = ref.num_threads()
        rate, secs = oracle_pass(S)
        cpu = {"value": rate, "unit": "token-slices/s", "cores": cores, "kind": "oracle", "cpu_model": cpu_model(),
               "sample": f"{S} of {B * H} slices (evenly spaced over layers and heads), {what} in fp64, "
                         f"{secs:.1f} s wall on {cores} OpenMP threads"}
        # the same on one core, on a sample cut down by the core count so that it takes about as long
        S1 = max(1, min(S, S // max(cores, 1)))
        ref.set_num_threads(1)
        rate1, secs1 = oracle_pass(S1)
        ref.set_num_threads(cores)
        cpu["single_core"] = {"value": rate1, "unit": "token-slices/s", "cores": 1,
                              "sample": f"{S1} of {B * H} slices, {what} in fp64, {secs1:.1f} s wall on one thread"}

    metric, work = (METRIC if args.config == 2 else METRIC.split(" at ")[0]), token_slices
    refresh = None
    if append:                                              # one token per slice and step
        metric, work = "decode-time refresh: appended tokens/sec (all layers x heads) at Llama2-7B N=4096", B * H
        # what the last step's refresh had to do: sets merged again, kept rows whose index changed
        o_sid, o_st, o_pv, o_ns = (t.cpu().numpy().reshape(B * H, -1) for t in maps[1 - cur[0]])
        _, n_st, n_pv, n_ns = (t.cpu().numpy().reshape(B * H, -1) for t in maps[cur[0]])
        again = moved = 0
        for i in range(B * H):
            M, Mo = int(n_ns[i, 0]), int(o_ns[i, 0])
            lo, hi, pv = n_st[i, :M], n_st[i, 1:M + 1], n_pv[i, :M]
            so = np.clip(o_sid[i, lo], 0, max(Mo - 1, 0))
            same = (o_st[i, so] == lo) & (o_st[i, so + 1] == hi) & (o_pv[i, so] == pv)
            again += int((~same).sum())
            moved += int((same & (so != np.arange(M))).sum())
        refresh = {"sets_merged_again_per_slice": again / (B * H), "rows_moved_per_slice": moved / (B * H),
                   "rows_per_slice": M_total / (B * H), "moved_GB": 4.0 * moved * d * esz / 1e9}
    out = {
        "metric": metric, "value": work / (ms_per_step * 1e-3), "unit": "token-slices/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {cfg['name']}: {B // cfg['batch']} layers x {H} KV heads, "
                               f"G={G}, N={N}, d={d}, {dtype}, budget {args.budget}, AR(1) keys seed {cfg['seed']}; {variant}",
                   "slices": B * H, "token_slices_per_step": token_slices, "merged_rows_per_step": M_total,
                   "mean_M_over_n": M_total / token_slices, "slices_with_fallback": int((status != 0).sum()),
                   # merged length over original length per layer (the layer-wise compression ratio of Section 3.2)
                   "M_over_n_per_layer": [round(float(x), 4) for x in
                                          (n_sets.reshape(-1, cfg["batch"], H).sum((1, 2)) /
                                           (n_per_b.reshape(-1, cfg["batch"]).sum(1) * H))]},
        "roofline": roofline, "cpu_baseline": cpu, "stage_fractions": stage_fractions,
        "stage_ms": {"attn_mass": stage_ms[0] / args.steps, "identify_sets": stage_ms[1] / args.steps,
                     "merge": stage_ms[2] / args.steps},
        "kernel_ms": kernels, "hbm_kernels": hbm, "input_generation_s": gen_s,
    }
    if refresh is not None:
        out["last_refresh"] = refresh
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
