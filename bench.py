#!/usr/bin/env python3
"""Benchmark of the FastGen hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input: attention
profiling + policy choice + compaction of the prompt (stage 1), then S decode steps over the
compressed caches (stage 2). Inputs are resident in HBM before the timed region starts.
Prints ONE JSON line: the headline metric is profiled prompt tokens/s (stage 1); decode
attention steps/s, the roofline objects and the CPU oracle baseline ride along. The workload
is the largest configuration that fits one GPU (llama65b_b2); short side runs of the other
bf16 configurations are reported under "other_configs".
"""
from __future__ import annotations

import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15   # flop/s, dense, MI355X
PEAK_HBM = 8.0e12         # B/s
TIMING_SAMPLE = 8         # decode steps between two timed ones (an event record costs microseconds)

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy of
# known size (factors 2.00 / 1.00); the commands and raw counter values are in
# profiles/hbm_traffic_<workload>_pmc.md. Offline numbers: the counters cannot be read inside
# a timed run. "sweeps" = both sweeps together, "decode_attn" = per launch over the first 16
# decode steps.
MEASURED_TRAFFIC = {
    # (FETCH_SIZE KiB x 2 + WRITE_SIZE KiB) x 1024 of sweep 1 + sweep 2; of fg_decode_partial_kernel
    "llama65b_b2": {"sweeps": (26371393 * 2 + 655360 + 32501777 * 2 + 2129920) * 1024.0,
                    "decode_attn": (9837948 * 2 + 274801) * 1024.0},
    "llama7b_b1": {"sweeps": (717242 * 2 + 16384 + 736650 * 2 + 53248) * 1024.0,
                   "decode_attn": (263969 * 2 + 10228) * 1024.0},
    "llama7b_b16": {"sweeps": (6642435 * 2 + 131072 + 5898438 * 2 + 425984) * 1024.0,
                    "decode_attn": (2102048 * 2 + 87862) * 1024.0},
    "llama13b_b4": {"sweeps": (8408802 * 2 + 204800 + 9147482 * 2 + 665600) * 1024.0,
                    "decode_attn": (4289956 * 2 + 96794) * 1024.0},
}

BASELINE_INDEX = {"tiny": 0, "llama7b_b1": 1, "llama7b_b16": 2, "llama13b_b4": 3, "llama65b_b2": 4}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama65b_b2",
                    help="default: the largest single-GPU configuration (BASELINE configs[4])")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short side runs of the other bf16 configurations (extra keys of the line)")
    ap.add_argument("--decode-steps", type=int, default=-1, help="override S (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--cache-tokens", type=int, default=0, help="cache pool capacity in tokens (0 = worst case)")
    ap.add_argument("--group-size", type=int, default=1,
                    help="query heads per K/V head (grouped-query variant of the workload; not a BASELINE config)")
    ap.add_argument("--forced-policy", type=int, default=-1, help="every unit uses this policy (non-adaptive baselines)")
    ap.add_argument("--cpu-sample-units", type=int, default=0, help="0 = sized for ~20 s")
    ap.add_argument("--probe-every", type=int, default=0,
                    help="N > 0: every N-th decode step runs with the stability probe (fastgen_decode_step_probe)")
    return ap.parse_args()


def decode_bytes(lens_before, policy, d, e):
    """Algorithmic HBM bytes of one decode step: (attention kernel, whole step).
    Per unit with L = held tokens including the new one: K^ and V^ rows 2*L*d*e; q, k_new,
    v_new read and o written 4*d*e; the appended row 2*d*e; for the policies that keep
    cumulative scores (those with `frequent`) the float64 logit of every held token written
    once (8*L). The update adds: positions and classes (5*L) for the policies that evict, logits
    read (8*L) and cumulative scores read+written (16*L) for those with `frequent`."""
    import numpy as np
    L = lens_before.astype(np.int64) + 1
    scored = (policy == 2) | (policy == 3)
    attn = 2 * L * d * e + 5 * d * e + np.where(scored, 8 * L, 0)
    upd = d * e + np.where(policy < 4, 5 * L, 0) + np.where(scored, 24 * L, 0)
    return int(attn.sum()), int(attn.sum() + upd.sum())


def run_workload(w, args, steps, warmup, dev="cuda:0"):
    """Generates the workload's inputs on the device, runs `warmup` untimed and `steps` timed
    passes of the whole path, and returns the measurements (plus what the CPU leg needs)."""
    import numpy as np
    import torch
    from paper_2310_01801_amd import binding, synth

    U, n, d, S, B = w.num_units, w.prompt_len, w.head_dim, w.steps, w.batch
    e = 2 if w.dtype == "bf16" else 4
    G = max(1, args.group_size)

    t0 = time.time()
    plan = synth.unit_plan(w)
    cls_p, cls_d = synth.token_classes(w)
    units = list(range(U))
    Q, K, V = synth.prompt_batch(w, plan, cls_p, units, dev)
    q, k, v = synth.decode_batch(w, plan, cls_d, units, dev) if S > 0 else (None, None, None)
    if G > 1:
        Q = torch.cat([synth.prompt_group_queries(w, plan, cls_p, u, G, dev) for u in units])
        if S > 0:
            q = torch.cat([synth.decode_group_queries(w, plan, cls_d, u, G, dev) for u in units], dim=1).contiguous()
    cls_p_d = torch.from_numpy(cls_p).to(dev)
    cls_d_d = torch.from_numpy(cls_d).to(dev)
    out = torch.empty((U * G, d), dtype=w.torch_dtype, device=dev)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    cfg = binding.make_config(U, B, d, w.torch_dtype, n, S, w.T, w.r_l, w.r_f, 0.0, args.forced_policy,
                              args.cache_tokens, None, G)
    workspace = torch.empty(binding.fastgen_workspace_bytes(cfg), dtype=torch.uint8, device=dev)

    def one_pass(timing=False):
        fg = binding.FastGen(cfg, dev, workspace=workspace)
        if timing:
            fg.fastgen_enable_timing(TIMING_SAMPLE)   # every phase of stage 1, every 8th decode step
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        pol, rec, cnt = fg.fastgen_profile(Q, K, cls_p_d)
        fg.fastgen_compact(K, V)
        ev[1].record()
        for t in range(S):
            if args.probe_every > 0 and t % args.probe_every == 0:
                fg.fastgen_decode_step_probe(q[t], k[t], v[t], cls_d_d[t], out)
            else:
                fg.fastgen_decode_step(q[t], k[t], v[t], cls_d_d[t], out)
        ev[2].record()
        torch.cuda.synchronize()
        res = dict(stage1_ms=ev[0].elapsed_time(ev[1]), stage2_ms=ev[1].elapsed_time(ev[2]),
                   policy=pol, timing=fg.fastgen_read_timing() if timing else None)
        fg.close()
        return res

    for _ in range(warmup):
        one_pass()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    runs = [one_pass(timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start

    s1 = float(np.median([r["stage1_ms"] for r in runs]))
    s2 = float(np.median([r["stage2_ms"] for r in runs]))
    # per-phase device time (HIP events recorded by the library on the launch stream)
    phase = {name: float(np.median([r["timing"][name][0] for r in runs])) for name in binding.PHASES}
    launches = {name: runs[0]["timing"][name][1] for name in binding.PHASES}
    traffic = MEASURED_TRAFFIC.get(w.name, {}) if (args.forced_policy < 0 and G == 1) else {}

    # ---- roofline of the profiling sweeps (matrix-core bound)
    flop_sweep = float(d) * n * (n + 1) * U * G   # causal QK^T, one sweep
    sweeps_ms = phase["sweep1"] + phase["sweep2"]
    mfma_achieved = 2 * flop_sweep / (sweeps_ms * 1e-3)
    roof_profile = dict(kernel="fg_profile_mfma_kernel (both sweeps)", bound="mfma",
                        achieved=mfma_achieved / 1e12, peak=PEAK_BF16_MFMA / 1e12, unit="TFLOP/s",
                        frac=mfma_achieved / PEAK_BF16_MFMA, traffic=traffic.get("sweeps"),
                        avg_launch_ms=sweeps_ms / 2, flop_per_launch=flop_sweep)

    # ---- roofline of the decode attention kernel (HBM bound): one untimed replay logs lengths
    roof_decode = None
    if S > 0:
        fg = binding.FastGen(cfg, dev, workspace=workspace)
        pol, _, _ = fg.fastgen_profile(Q, K, cls_p_d)
        fg.fastgen_compact(K, V)
        pol_np = pol.cpu().numpy()
        attn_b = step_b = 0
        held = []
        n_timed = 0
        for t in range(S):
            if t % TIMING_SAMPLE == 0:   # the steps whose kernels the timed passes measure
                lens = fg.fastgen_export_state(lengths_only=True)["lengths"].cpu().numpy()
                a_b, s_b = decode_bytes(lens, pol_np, d, e)
                attn_b += a_b
                step_b += s_b
                n_timed += 1
                held.append(int(lens.sum()))
            fg.fastgen_decode_step(q[t], k[t], v[t], cls_d_d[t], out)
        torch.cuda.synchronize()
        fg.close()
        attn_ms = phase["decode_attn"] / max(1, launches["decode_attn"])
        upd_ms = phase["decode_update"] / max(1, launches["decode_update"])
        bw = (attn_b / n_timed) / (attn_ms * 1e-3)
        roof_decode = dict(kernel="fg_decode_partial_kernel", bound="hbm", achieved=bw / 1e9,
                           peak=PEAK_HBM / 1e9, unit="GB/s", frac=bw / PEAK_HBM,
                           traffic=traffic.get("decode_attn"),
                           avg_launch_ms=attn_ms, bytes_per_launch=attn_b / n_timed,
                           timed_launches=launches["decode_attn"], update_kernel_avg_ms=upd_ms,
                           whole_step_GBps=(step_b / n_timed) / ((attn_ms + upd_ms) * 1e-3) / 1e9,
                           mean_held_tokens_per_unit=float(np.mean(held)) / U,
                           full_cache_tokens_per_unit=n + (S + 1) / 2)
    pol_hist = np.bincount(runs[0]["policy"].cpu().numpy(), minlength=5).tolist()
    res = dict(w=w, wall=wall, ms_per_step=wall * 1e3 / steps, stage1_ms=s1, stage2_ms=s2,
               tokens_per_s=B * n / (s1 * 1e-3), decode_steps_per_s=(S / (s2 * 1e-3)) if S > 0 else None,
               phase=phase, launches=launches, roof_profile=roof_profile, roof_decode=roof_decode,
               pol_hist=pol_hist, gen_s=gen_s, sweeps_ms=sweeps_ms, plan=plan, cls_p=cls_p, cls_d=cls_d)
    del Q, K, V, q, k, v, workspace, out, runs
    gc.collect()
    torch.cuda.empty_cache()
    return res


def describe(w, S):
    idx = BASELINE_INDEX.get(w.name)
    tag = f"BASELINE configs[{idx}]" if idx is not None else "not a BASELINE config"
    if w.name == "llama65b_b2":
        tag += ", the largest single-GPU configuration"
    return (f"{w.name}: {w.layers} layers x {w.heads} heads, batch {w.batch}, head_dim {w.head_dim}, {w.dtype}, "
            f"prompt {w.prompt_len}, {S} decode steps, T={w.T}, r_l={w.r_l}, r_f={w.r_f} ({tag})")


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for --gpus {args.gpus}); "
              "the path shards by head/sequence with no exchange step, see DESIGN.md", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2310_01801_amd import binding, synth

    binding.load_library()  # no fallback: fails if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    if args.decode_steps >= 0:
        w = w.scaled(steps=args.decode_steps)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    m = run_workload(w, args, args.steps, args.warmup, dev)
    roof_profile, roof_decode = m["roof_profile"], m["roof_decode"]

    # ---- what library kernels reach on this machine, next to the published peaks (context only)
    ref = reference_rates(dev)
    roof_profile["box_reference"] = {"bf16_gemm_8192_TFLOPs": ref["gemm_tflops"], **pipe_microbenchmarks(dev)}
    if roof_decode:
        roof_decode["box_reference"] = {"device_copy_1GiB_GBps_read_plus_write": ref["copy_gbps"]}
    # the dominant kernel: the one the device spends most of a pass in
    decode_total_ms = (roof_decode["avg_launch_ms"] * w.steps) if roof_decode else 0.0
    dominant = roof_decode if (roof_decode and decode_total_ms > m["sweeps_ms"]) else roof_profile

    # ---- the other bf16 configurations, short side runs (1 warm-up + 3 timed passes each)
    others = None
    if (not args.no_other_configs and args.forced_policy < 0 and args.group_size <= 1 and args.decode_steps < 0
            and args.probe_every == 0):
        others = {}
        for name in ("llama7b_b1", "llama7b_b16", "llama13b_b4", "llama65b_b2"):
            if name == w.name:
                continue
            o = run_workload(synth.WORKLOADS[name], args, 3, 1, dev)
            rd = o["roof_decode"]
            others[name] = {
                "workload": describe(o["w"], o["w"].steps), "prompt_tokens_per_s": o["tokens_per_s"],
                "decode_attn_steps_per_s": o["decode_steps_per_s"], "stage1_ms": o["stage1_ms"],
                "stage2_ms": o["stage2_ms"], "pct_mfma": 100 * o["roof_profile"]["frac"],
                "pct_hbm": 100 * rd["frac"], "sweeps_ms": o["sweeps_ms"],
                "decode_attn_avg_launch_ms": rd["avg_launch_ms"], "decode_update_avg_launch_ms": rd["update_kernel_avg_ms"],
                "whole_step_GBps": rd["whole_step_GBps"], "policy_histogram": o["pol_hist"],
                "traffic": {"sweeps": o["roof_profile"]["traffic"], "decode_attn": rd["traffic"]}}

    # ---- CPU oracle on a bounded sample (never tuned; reported, not a target)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, m["plan"], m["cls_p"], m["cls_d"], args.cpu_sample_units)

    line = {
        "metric": "profiled prompt tokens/s; decode attn steps/s; % MFMA and % HBM roofline",
        "value": m["tokens_per_s"], "unit": "prompt tokens/s (stage 1: profile + select + compact, all heads)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": describe(w, w.steps), "units": w.num_units,
                   "query_heads_per_unit": max(1, args.group_size),
                   "policy_histogram": m["pol_hist"], "input_generation_s": m["gen_s"]},
        "decode_attn_steps_per_s": m["decode_steps_per_s"],
        "stage1_ms": m["stage1_ms"], "stage2_ms": m["stage2_ms"],
        "phase_ms": m["phase"], "phase_launches": m["launches"],
        "pct_mfma": 100 * roof_profile["frac"],
        "pct_hbm": 100 * roof_decode["frac"] if roof_decode else None,
        "roofline": dominant, "roofline_profile": roof_profile, "roofline_decode": roof_decode,
        "cpu_baseline": cpu, "other_configs": others,
    }
    print(json.dumps(line))


def reference_rates(dev):
    """A large bf16 GEMM (hipBLASLt through torch) and a 1 GiB device copy, timed with events:
    the practical ceilings of this machine for matrix-core and HBM bound work."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    a = torch.randn((8192, 8192), device=dev, dtype=torch.bfloat16)
    b = torch.randn((8192, 8192), device=dev, dtype=torch.bfloat16)
    for _ in range(3):
        torch.matmul(a, b)
    ev[0].record()
    for _ in range(10):
        torch.matmul(a, b)
    ev[1].record()
    torch.cuda.synchronize()
    gemm = 10 * 2 * 8192.0 ** 3 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12
    del a, b
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev[0].record()
    for _ in range(5):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    copy = 5 * 2 * float(1 << 30) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    del src, dst
    return dict(gemm_tflops=gemm, copy_gbps=copy)


def pipe_microbenchmarks(dev):
    """Register-only micro-benchmarks of one wave-step of the sweeps (16 MFMAs of 32x32x16 bf16
    and the softmax arithmetic of their 32 results per lane), three waves per SIMD: the matrix
    pipe alone, the vector ALU alone, and both as the sweeps issue them. They give the rate the
    matrix pipe sustains on this machine and show how far its work overlaps with the vector ALU's."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "paper_2310_01801_amd", "libfgubench.so")
    if not os.path.exists(path):
        return {"pipe_microbenchmarks": None}
    lib = ctypes.CDLL(path)
    lib.fg_ubench_run.restype = ctypes.c_int
    lib.fg_ubench_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    blocks, iters = 768 * 4, 2000
    out = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
    clk = torch.zeros(2 * blocks, dtype=torch.int64, device=dev)
    res = {}
    for mode, name in ((1, "mfma_only"), (2, "softmax_valu_only_sweep1"), (3, "mfma_then_softmax_sweep1"),
                       (4, "mfma_then_softmax_sweep2")):
        ns, mhz = ctypes.c_double(), ctypes.c_double()
        rc = lib.fg_ubench_run(mode, blocks, iters, out.data_ptr(), clk.data_ptr(),
                               torch.cuda.current_stream().cuda_stream, ctypes.byref(ns), ctypes.byref(mhz))
        if rc != 0:
            return {"pipe_microbenchmarks": f"failed with HIP error {rc}"}
        res[name + "_ns_per_wave_step"] = ns.value
        # the shader clock the chip held meanwhile (cycle counter / 100 MHz counter)
        res[name + "_shader_MHz"] = mhz.value
    flop = 16 * 2 * 32 * 32 * 16   # one wave-step of MFMAs
    simds = 1024
    res["mfma_only_TFLOPs"] = flop * simds / res["mfma_only_ns_per_wave_step"] / 1e3
    res["sweep1_ceiling_frac_of_2.5PF"] = flop * simds / res["mfma_then_softmax_sweep1_ns_per_wave_step"] / 1e3 / 2500.0
    res["sweep2_ceiling_frac_of_2.5PF"] = flop * simds / res["mfma_then_softmax_sweep2_ns_per_wave_step"] / 1e3 / 2500.0
    return {"pipe_microbenchmarks": res}


def cpu_baseline(w, plan, cls_p, cls_d, sample_units):
    """Times the float64 oracle (profile + compact + all decode steps) on a seeded sample of
    units on the host, and extrapolates to the whole workload. The oracle is one numpy process:
    its matrix products run on the BLAS thread pool, everything else on one core; `cores` is
    the average number of busy cores measured over the sample (process CPU time / wall time)."""
    import numpy as np
    from oracle import fastgen_oracle as fo
    from paper_2310_01801_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = 1
    rng = np.random.default_rng(1234)
    scale = float(np.float32(1.0 / math.sqrt(w.head_dim)))
    budget_s, used, done = 20.0, 0.0, 0
    t_prof = t_dec = 0.0
    order = rng.permutation(w.num_units)
    limit = sample_units if sample_units > 0 else w.num_units
    cpu_busy = 0.0
    for u in order[:limit]:
        u = int(u)
        b = u // w.units_per_seq
        Qu, Ku, Vu = (synth.to_f64(x) for x in synth.prompt_unit(w, plan, cls_p, u))
        if w.steps > 0:
            qu, ku, vu = (synth.to_f64(x) for x in synth.decode_unit(w, plan, cls_d, u))
        c0 = time.process_time()
        t0 = time.perf_counter()
        prof = fo.profile_unit(Qu, Ku, cls_p[b], w.T, w.r_l, w.r_f, scale)
        cache = fo.compact_unit(Ku, Vu, cls_p[b], prof)
        t1 = time.perf_counter()
        for t in range(w.steps):
            fo.decode_step(cache, qu[t], ku[t], vu[t], int(cls_d[t, b]), t, w.r_l, w.r_f, scale)
        t2 = time.perf_counter()
        t_prof += t1 - t0
        t_dec += t2 - t1
        used += t2 - t0
        done += 1
        cpu_busy += time.process_time() - c0
        if sample_units <= 0 and used > budget_s:
            break
    full_prof = t_prof * w.num_units / done
    full_dec = t_dec * w.num_units / done
    return {"value": w.batch * w.prompt_len / full_prof, "unit": "prompt tokens/s (stage 1), extrapolated",
            "cores": round(cpu_busy / max(used, 1e-9), 2), "kind": "oracle",
            "sample": f"{done} of {w.num_units} units (seeded), every decode step; "
                      f"{t_prof:.2f} s stage 1 + {t_dec:.2f} s stage 2 measured, scaled by {w.num_units}/{done}; "
                      f"single-process numpy, BLAS thread pool of {threads}, `cores` = process CPU time / wall time",
            "decode_attn_steps_per_s": (w.steps / full_dec) if w.steps > 0 and full_dec > 0 else None,
            "blas_threads": threads, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
