#!/usr/bin/env python3
"""Benchmark of the HBP SpMV hot path on one MI355X.

A step is one hbp_spmv call: the SpMV-part kernel plus the combine kernel over one resident
matrix.  Prints ONE JSON line.  GFLOP/s follows the paper's convention 2 nnz / t with t
including the combine step (Section 4.3).
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size), or None."""
    import glob
    import re
    for path in glob.glob(os.path.join(ROOT, "profiles", "*_pmc.md")):
        for line in open(path):
            m = re.match(r"TRAFFIC_BYTES_PER_LAUNCH kernel=(\S+) workload=(\S+) bytes=(\d+)", line)
            if m and m.group(1) == kernel and m.group(2) == workload:
                return int(m.group(3))
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (default: the 27-point stencil)")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--rows-per-block", type=int, default=0)
    ap.add_argument("--cols-per-block", type=int, default=0)
    ap.add_argument("--num-workers", type=int, default=-1)
    ap.add_argument("--fixed-q8", type=int, default=-2)
    ap.add_argument("--claim-chunk", type=int, default=0)
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--rounds", type=int, default=0)
    ap.add_argument("--slot-weight", type=int, default=-1)
    ap.add_argument("--group-weight", type=int, default=-1)
    ap.add_argument("--combine-unit-slots", type=int, default=0)
    ap.add_argument("--hash-shift", type=int, default=-1)
    ap.add_argument("--round-weight", type=int, default=-1)
    ap.add_argument("--column-weight", type=int, default=-1)
    ap.add_argument("--heavy-group-rounds", type=int, default=0)
    ap.add_argument("--dtype", choices=("f32", "f64"), default="f32",
                    help="value type: f32 is the headline metric; f64 runs the fp64 variant on the same pattern")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-csr", action="store_true", help="skip the CSR baselines and the study legs")
    ap.add_argument("--no-study", action="store_true",
                    help="skip the plain 2D-partition and length-key legs (keeps a kernel trace to the HBP layout alone)")
    ap.add_argument("--builds", type=int, default=3, help="timed hbp_build repetitions")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference dispatch for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2504_08860_amd as H
    from paper_2504_08860_amd.presets import preset
    from workloads import make_config, widen_to_f64

    torch.cuda.set_device(0)
    t0 = time.time()
    m = make_config(args.config, args.scale)
    log(f"[bench] generated {m.name}: {m.n_rows} x {m.n_cols}, nnz {m.nnz} in {time.time() - t0:.1f}s")
    f64 = args.dtype == "f64"
    vb = 8 if f64 else 4
    if f64:
        m = widen_to_f64(m)
    hbp_build, hbp_spmv, hbp_spmv_timed, hbp_csr_spmv = (
        (H.hbp_build_f64, H.hbp_spmv_f64, H.hbp_spmv_timed_f64, H.hbp_csr_spmv_f64) if f64
        else (H.hbp_build, H.hbp_spmv, H.hbp_spmv_timed, H.hbp_csr_spmv))
    params = preset(args.config, args.dtype)
    if args.rows_per_block: params["rows_per_block"] = args.rows_per_block
    if args.cols_per_block: params["cols_per_block"] = args.cols_per_block
    if args.num_workers >= 0: params["num_workers"] = args.num_workers
    if args.fixed_q8 >= -1: params["fixed_fraction_q8"] = args.fixed_q8
    if args.claim_chunk: params["claim_chunk"] = args.claim_chunk
    if args.threads: params["threads_per_worker"] = args.threads
    if args.rounds: params["rounds_per_batch"] = args.rounds
    if args.slot_weight >= 0: params["slot_weight"] = args.slot_weight
    if args.group_weight >= 0: params["group_weight"] = args.group_weight
    if args.combine_unit_slots: params["combine_unit_slots"] = args.combine_unit_slots
    if args.hash_shift >= 0: params["hash_shift"] = args.hash_shift
    if args.round_weight >= 0: params["round_weight"] = args.round_weight
    if args.column_weight >= 0: params["column_weight"] = args.column_weight
    if args.heavy_group_rounds: params["heavy_group_rounds"] = args.heavy_group_rounds
    overridden = params != preset(args.config, args.dtype) or f64

    dev = lambda a: torch.from_numpy(a).cuda()
    ptr, col, val, x = dev(m.ptr), dev(m.col), dev(m.val), dev(m.x)
    y = torch.empty(m.n_rows, device="cuda", dtype=x.dtype)
    torch.cuda.synchronize()

    # preprocessing time (validation off, allocation and synchronisation included)
    build_ms = []
    h = None
    for _ in range(max(1, args.builds)):
        if h is not None:
            H.hbp_free(h)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h = hbp_build(ptr, col, val, m.n_rows, m.n_cols, validate=False, **params)
        torch.cuda.synchronize()
        build_ms.append((time.perf_counter() - t0) * 1e3)
    info = H.hbp_get_info(h)
    log(f"[bench] R={info.rows_per_block} C={info.cols_per_block} W={info.group_width} a={info.hash_shift} "
        f"blocks={info.blocks} slots={info.slots} groups={info.groups} P={info.num_workers} "
        f"fixed_q8={info.fixed_fraction_q8} threads={info.threads_per_worker} build_ms={[round(b, 2) for b in build_ms]}")

    if args.calibrate_copy:  # a copy kernel of known size: 2^28 bytes read, 2^28 bytes written
        src = torch.empty(1 << 26, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # the timed region: exactly K steps between synchronisations
    for _ in range(args.warmup):
        hbp_spmv(h, x, y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        hbp_spmv(h, x, y)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations from HIP events recorded on the launch stream
    ms_part, ms_comb, ms_call = hbp_spmv_timed(h, x, y, max(20, min(args.steps, 200)))
    gflops = 2.0 * m.nnz / (ms_per_step * 1e-3) / 1e9
    # algorithmic bytes of the whole call, as stored: col+data per nonzero, slot/group/block
    # metadata, x once, y once (the partial sums written and re-read are extra traffic, not counted)
    alg_call = info.bytes_layout + vb * m.n_cols + vb * m.n_rows
    csr_equiv = (4 + vb) * m.nnz + 4 * (m.n_rows + 1) + vb * m.n_cols + vb * m.n_rows
    eff_gbs = alg_call / (ms_per_step * 1e-3) / 1e9
    part_gbs = info.bytes_spmv_part / (ms_part * 1e-3) / 1e9

    out = {
        "metric": f"HBP SpMV GFLOP/s ({'fp64' if f64 else 'fp32'}, 2*nnz/t, t = SpMV part + combine)",
        "value": round(gflops, 2), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"config {args.config}: {m.name}, {m.n_rows}x{m.n_cols}, nnz {m.nnz}"
                               + ("" if args.scale == 1.0 else f" (scale {args.scale})"),
                   "rows_per_block": info.rows_per_block, "cols_per_block": info.cols_per_block,
                   "group_width": info.group_width, "hash_shift": info.hash_shift, "blocks": info.blocks,
                   "slots": info.slots, "groups": info.groups, "workers": info.num_workers,
                   "fixed_fraction_q8": info.fixed_fraction_q8, "claim_chunk": info.claim_chunk,
                   "threads_per_worker": info.threads_per_worker, "rounds_per_batch": info.rounds_per_batch, "slot_weight": info.slot_weight, "group_weight": info.group_weight,
                   "combine_unit_slots": info.combine_unit_slots, "combine_units": info.combine_units,
                   "round_weight": info.round_weight, "column_weight": info.column_weight, "heavy_group_rounds": info.heavy_group_rounds},
        "roofline": {"bound": "hbm", "kernel": "k_spmv_part", "achieved": round(part_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(part_gbs / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic("k_spmv_part", m.name) if args.scale == 1.0 and not overridden else None,
                     "bytes_per_launch": info.bytes_spmv_part, "ms_per_launch": round(ms_part, 5)},
        "whole_call": {"effective_GBps": round(eff_gbs, 1), "frac_of_hbm_peak": round(eff_gbs / HBM_PEAK_GBS, 4),
                       "algorithmic_bytes": alg_call, "csr_equivalent_bytes": csr_equiv,
                       "ms_spmv_part": round(ms_part, 5), "ms_combine": round(ms_comb, 5),
                       "ms_call_events": round(ms_call, 5),
                       "note": "back-to-back calls; x, y and the partial sums stay in the 256 MB last-level cache"},
        "hbp_build_ms": round(min(build_ms), 3),
    }

    if not args.no_csr:
        for kind, name in ((0, "csr_scalar"), (1, "csr_vector")):
            for _ in range(5):
                hbp_csr_spmv(kind, ptr, col, val, x, y)
            torch.cuda.synchronize()
            reps = max(5, min(50, args.steps))
            t0 = time.perf_counter()
            for _ in range(reps):
                hbp_csr_spmv(kind, ptr, col, val, x, y)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / reps
            out[name] = {"ms": round(ms, 5), "GFLOPs": round(2.0 * m.nnz / (ms * 1e-3) / 1e9, 2),
                         "hbp_speedup": round(ms / ms_per_step, 3)}

    if not args.no_csr and not args.no_study:
        # Section 4's second baseline: the same 2D partition without the hash reorder and with an
        # all-fixed schedule, and the diagnostic of Section 4.1 for both layouts (mean over the
        # groups of the standard deviation of their rows' lengths)
        def group_len_std(handle):
            seg_len = H.hbp_export(handle, "seg_len").astype(np.float64)
            gs = H.hbp_export(handle, "group_slot").astype(np.int64)
            cnt = np.diff(gs).astype(np.float64)
            s1 = np.add.reduceat(seg_len, gs[:-1])
            s2 = np.add.reduceat(seg_len * seg_len, gs[:-1])
            var = np.maximum(s2 / cnt - (s1 / cnt) ** 2, 0.0)
            return float(np.sqrt(var).mean())
        plain_params = dict(params, fixed_fraction_q8=256)
        hp = hbp_build(ptr, col, val, m.n_rows, m.n_cols, validate=False, no_reorder=True, **plain_params)
        for _ in range(5):
            hbp_spmv(hp, x, y)
        torch.cuda.synchronize()
        p_part, p_comb, p_call = hbp_spmv_timed(hp, x, y, max(5, min(50, args.steps)))
        ms = p_part + p_comb
        out["plain_2d"] = {"ms": round(ms, 5), "ms_spmv_part": round(p_part, 5), "ms_combine": round(p_comb, 5),
                           "GFLOPs": round(2.0 * m.nnz / (ms * 1e-3) / 1e9, 2),
                           "hbp_speedup": round(ms / (ms_part + ms_comb), 3),
                           "group_len_std": {"hbp": round(group_len_std(h), 4), "plain_2d": round(group_len_std(hp), 4)}}
        H.hbp_free(hp)
        # hash study (Section 5's outlook): the same schedule and kernels with the rows of a block
        # ordered by their length itself, which no hash of the length can improve on
        hl = hbp_build(ptr, col, val, m.n_rows, m.n_cols, validate=False, key_length=True, **params)
        for _ in range(5):
            hbp_spmv(hl, x, y)
        torch.cuda.synchronize()
        l_part, l_comb, l_call = hbp_spmv_timed(hl, x, y, max(5, min(50, args.steps)))
        out["length_key"] = {"ms": round(l_part + l_comb, 5), "ms_spmv_part": round(l_part, 5), "ms_combine": round(l_comb, 5),
                             "speedup_over_hbp": round((ms_part + ms_comb) / (l_part + l_comb), 3),
                             "group_len_std": round(group_len_std(hl), 4),
                             "groups": H.hbp_get_info(hl).groups}
        H.hbp_free(hl)

    if not args.no_cpu_baseline:
        import oracle
        reps, times = 5, []
        for _ in range(reps):
            t0 = time.perf_counter()
            oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
            times.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        o = oracle.OracleHbp(m.ptr, m.col, m.val, m.n_rows, m.n_cols, R=info.rows_per_block, C=info.cols_per_block,
                             W=info.group_width, num_workers=info.num_workers)
        o_build = time.perf_counter() - t0
        o.close()
        med = sorted(times)[len(times) // 2]
        out["cpu_baseline"] = {"value": round(2.0 * m.nnz / med / 1e9, 3), "unit": "GFLOP/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"whole workload, oracle CSR SpMV ({'extended-precision' if f64 else 'fp64'} accumulate) median of {reps} runs; "
                                         f"oracle HBP build once: {o_build * 1e3:.0f} ms",
                               "host_cpus": os.cpu_count()}
    H.hbp_free(h)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
