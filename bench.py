#!/usr/bin/env python3
"""Benchmark of the HBP SpMV hot path on one MI355X.

A step is one hbp_spmv call: the SpMV-part kernel plus the combine kernel over one resident
matrix.  Prints ONE JSON line.  GFLOP/s follows the paper's convention 2 nnz / t with t
including the combine step (Section 4.3).

The headline workload is the largest of the five (configuration 5, the irregular 4M x 1M matrix),
built with the library's own choice of block parameters (nothing passed to hbp_build); the other
large workloads are measured the same way and reported under "per_config".
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
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc summaries
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size), or None."""
    import glob
    import re
    for path in glob.glob(os.path.join(ROOT, "profiles", "*_pmc.md")):
        for line in open(path):
            m = re.match(r"TRAFFIC_BYTES_PER_LAUNCH kernel=(\S+) workload=(\S+) bytes=(\d+)", line)
            if m and m.group(1) == kernel and m.group(2) == workload:
                return int(m.group(3))
    return None


class Bench:
    """One workload resident on the GPU, and the measurements taken on it."""

    def __init__(self, number, scale, dtype, steps, warmup):
        import torch
        from workloads import make_config, widen_to_f64
        import paper_2504_08860_amd as H
        self.H, self.torch = H, torch
        self.number, self.steps, self.warmup = number, steps, warmup
        t0 = time.time()
        m = make_config(number, scale)
        self.f64 = dtype == "f64"
        if self.f64:
            m = widen_to_f64(m)
        self.m = m
        log(f"[bench] generated {m.name}: {m.n_rows} x {m.n_cols}, nnz {m.nnz} in {time.time() - t0:.1f}s")
        self.vb = 8 if self.f64 else 4
        self.build_fn, self.spmv_fn, self.timed_fn, self.csr_fn = (
            (H.hbp_build_f64, H.hbp_spmv_f64, H.hbp_spmv_timed_f64, H.hbp_csr_spmv_f64) if self.f64
            else (H.hbp_build, H.hbp_spmv, H.hbp_spmv_timed, H.hbp_csr_spmv))
        dev = lambda a: torch.from_numpy(a).cuda()
        self.ptr, self.col, self.val, self.x = dev(m.ptr), dev(m.col), dev(m.val), dev(m.x)
        self.y = torch.empty(m.n_rows, device="cuda", dtype=self.x.dtype)
        torch.cuda.synchronize()

    def build(self, **params):
        return self.build_fn(self.ptr, self.col, self.val, self.m.n_rows, self.m.n_cols, validate=False, **params)

    def timed_builds(self, reps, **params):
        """(handle, [ms per build]): validation off, allocation and synchronisation included."""
        ms, h = [], None
        for _ in range(max(1, reps)):
            if h is not None:
                self.H.hbp_free(h)
            self.torch.cuda.synchronize()
            t0 = time.perf_counter()
            h = self.build(**params)
            self.torch.cuda.synchronize()
            ms.append((time.perf_counter() - t0) * 1e3)
        return h, ms

    def wall_ms_per_step(self, h, steps, warmup):
        for _ in range(warmup):
            self.spmv_fn(h, self.x, self.y)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.spmv_fn(h, self.x, self.y)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def kernel_ms(self, h, iters):
        """(SpMV part, combine, whole call) by HIP events on the launch stream."""
        return self.timed_fn(h, self.x, self.y, iters)

    def leg(self, iters=30, **params):
        """Build with `params`, time the two kernels, free: a comparison leg."""
        h = self.build(**params)
        for _ in range(5):
            self.spmv_fn(h, self.x, self.y)
        self.torch.cuda.synchronize()
        part, comb, _ = self.kernel_ms(h, iters)
        info = self.H.hbp_get_info(h)
        out = {"ms": round(part + comb, 5), "ms_spmv_part": round(part, 5), "ms_combine": round(comb, 5),
               "GFLOPs": round(2.0 * self.m.nnz / ((part + comb) * 1e-3) / 1e9, 2)}
        return h, info, out

    def algorithmic_bytes(self, info):
        """(whole call, SpMV part alone, CSR equivalent): bytes the method has to move, as stored: column +
        value per nonzero, slot/group/block metadata, x once, y once.  The partial sums, written by the
        SpMV part and read back by the combine part, are traffic the method adds and are not counted."""
        m, vb = self.m, self.vb
        call = info.bytes_layout + vb * m.n_cols + vb * m.n_rows
        part = info.bytes_spmv_part - vb * info.slots
        csr = (4 + vb) * m.nnz + 4 * (m.n_rows + 1) + vb * m.n_cols + vb * m.n_rows
        return call, part, csr

    def csr_baselines(self, reps):
        """Thread per row, wavefront per row, and the power-of-two lanes per row nearest the mean row length."""
        m = self.m
        mean = m.nnz / max(1, m.n_rows)
        near = min((2, 4, 8, 16, 32), key=lambda k: abs(k - mean))
        out = {}
        for kind, name in ((0, "csr_scalar"), (1, "csr_vector"), (near, f"csr_{near}_lanes_per_row")):
            for _ in range(3):
                self.csr_fn(kind, self.ptr, self.col, self.val, self.x, self.y)
            self.torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                self.csr_fn(kind, self.ptr, self.col, self.val, self.x, self.y)
            self.torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / reps
            out[name] = {"ms": round(ms, 5), "GFLOPs": round(2.0 * m.nnz / (ms * 1e-3) / 1e9, 2)}
        best = min(out, key=lambda k: out[k]["ms"])
        return out, best

    def group_len_std(self, h):
        """Section 4.1's diagnostic: mean over the groups of the standard deviation of their rows' lengths."""
        import numpy as np
        H = self.H
        seg_len = H.hbp_export(h, "seg_len").astype(np.float64)
        gs = H.hbp_export(h, "group_slot").astype(np.int64)
        cnt = np.diff(gs).astype(np.float64)
        s1 = np.add.reduceat(seg_len, gs[:-1])
        s2 = np.add.reduceat(seg_len * seg_len, gs[:-1])
        var = np.maximum(s2 / cnt - (s1 / cnt) ** 2, 0.0)
        return float(np.sqrt(var).mean())

    def summary(self, h, info, ms_per_step, ms_part, ms_comb):
        m = self.m
        call_b, part_b, csr_b = self.algorithmic_bytes(info)
        t_kernels = (ms_part + ms_comb) * 1e-3
        return {"workload": f"config {self.number}: {m.name}, {m.n_rows}x{m.n_cols}, nnz {m.nnz}",
                "GFLOPs": round(2.0 * m.nnz / (ms_per_step * 1e-3) / 1e9, 2), "ms_per_step": round(ms_per_step, 5),
                "ms_spmv_part": round(ms_part, 5), "ms_combine": round(ms_comb, 5),
                "whole_call_frac_of_hbm_peak": round(call_b / t_kernels / 1e9 / HBM_PEAK_GBS, 4),
                "spmv_part_frac_of_hbm_peak": round(part_b / (ms_part * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "algorithmic_bytes": call_b, "csr_equivalent_bytes": csr_b,
                "rows_per_block": info.rows_per_block, "cols_per_block": info.cols_per_block,
                "rounds_per_batch": info.rounds_per_batch, "hash_shift": info.hash_shift,
                "slots": info.slots, "groups": info.groups, "blocks": info.blocks}

    def close(self):
        del self.ptr, self.col, self.val, self.x, self.y
        self.torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, help="headline workload 1..5 (default: the largest, the irregular 4M x 1M matrix)")
    ap.add_argument("--others", type=str, default="2,3,4", help="workloads also measured and reported under per_config ('' = none)")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--tuned", action="store_true", help="headline with the hand-picked block sizes of presets.py instead of the library's choice")
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
    ap.add_argument("--no-csr", action="store_true", help="skip the CSR baselines and the comparison legs")
    ap.add_argument("--no-study", action="store_true", help="skip the comparison legs (keeps a kernel trace to the headline layout alone)")
    ap.add_argument("--builds", type=int, default=3, help="timed hbp_build repetitions")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference dispatch for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    import paper_2504_08860_amd as H
    from paper_2504_08860_amd.presets import tuned_block_sizes

    torch.cuda.set_device(0)
    params = {}
    if args.tuned: params.update(tuned_block_sizes(args.config, args.dtype))
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
    library_choice = not params and not args.tuned

    B = Bench(args.config, args.scale, args.dtype, args.steps, args.warmup)
    m = B.m
    h, build_ms = B.timed_builds(args.builds, **params)
    info = H.hbp_get_info(h)
    log(f"[bench] R={info.rows_per_block} C={info.cols_per_block} W={info.group_width} a={info.hash_shift} rounds={info.rounds_per_batch} "
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
    ms_per_step = B.wall_ms_per_step(h, args.steps, args.warmup)
    # per-kernel durations from HIP events recorded on the launch stream
    ms_part, ms_comb, ms_call = B.kernel_ms(h, max(20, min(args.steps, 200)))
    head = B.summary(h, info, ms_per_step, ms_part, ms_comb)
    call_b, part_b, csr_b = B.algorithmic_bytes(info)
    part_gbs = part_b / (ms_part * 1e-3) / 1e9
    call_gbs = call_b / ((ms_part + ms_comb) * 1e-3) / 1e9
    traffic = {k: measured_traffic(k, m.name) for k in ("k_spmv_part", "k_combine")} if args.scale == 1.0 and library_choice and not B.f64 else {}

    out = {
        "metric": f"HBP SpMV GFLOP/s ({'fp64' if B.f64 else 'fp32'}, 2*nnz/t, t = SpMV part + combine)",
        "value": head["GFLOPs"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": head["workload"] + ("" if args.scale == 1.0 else f" (scale {args.scale})"),
                   "parameters": "chosen by the library from the matrix" if library_choice else "given on the command line / presets.py",
                   "rows_per_block": info.rows_per_block, "cols_per_block": info.cols_per_block,
                   "group_width": info.group_width, "hash_shift": info.hash_shift, "blocks": info.blocks,
                   "slots": info.slots, "groups": info.groups, "workers": info.num_workers,
                   "fixed_fraction_q8": info.fixed_fraction_q8, "claim_chunk": info.claim_chunk,
                   "threads_per_worker": info.threads_per_worker, "rounds_per_batch": info.rounds_per_batch,
                   "slot_weight": info.slot_weight, "group_weight": info.group_weight,
                   "combine_unit_slots": info.combine_unit_slots, "combine_units": info.combine_units,
                   "round_weight": info.round_weight, "column_weight": info.column_weight, "heavy_group_rounds": info.heavy_group_rounds},
        # the dominant kernel; its algorithmic bytes leave out the partial sums it writes (extra traffic of the method)
        "roofline": {"bound": "hbm", "kernel": "k_spmv_part", "achieved": round(part_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(part_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic.get("k_spmv_part"),
                     "bytes_per_launch": part_b, "ms_per_launch": round(ms_part, 5)},
        # the whole call, t = SpMV part + combine (Section 4.3): the number to judge the path by
        "whole_call": {"effective_GBps": round(call_gbs, 1), "frac_of_hbm_peak": round(call_gbs / HBM_PEAK_GBS, 4),
                       "algorithmic_bytes": call_b, "csr_equivalent_bytes": csr_b,
                       "ms_spmv_part": round(ms_part, 5), "ms_combine": round(ms_comb, 5), "ms_call_events": round(ms_call, 5),
                       "traffic_spmv_part_plus_combine": (traffic.get("k_spmv_part") + traffic.get("k_combine"))
                       if traffic.get("k_spmv_part") and traffic.get("k_combine") else None,
                       "note": "back-to-back calls: x and y (and, on the smaller workloads, part of the partial sums) stay in "
                               "the 256 MB last-level cache; the matrix stream does not fit and comes from HBM every step"},
        "hbp_build_ms": round(min(build_ms), 3),
    }

    if not args.no_csr:
        csr, best = B.csr_baselines(max(5, min(30, args.steps)))
        out["csr"] = csr
        out["csr_best"] = {"kernel": best, "ms": csr[best]["ms"], "hbp_speedup": round(csr[best]["ms"] / ms_per_step, 3)}

    if not args.no_csr and not args.no_study:
        base = ms_part + ms_comb
        legs = {}
        # the hand-picked block sizes (rows, columns, rounds per batch) against the library's choice
        hx, ix, o = B.leg(**tuned_block_sizes(args.config, args.dtype))
        o.update(rows_per_block=ix.rows_per_block, cols_per_block=ix.cols_per_block, rounds_per_batch=ix.rounds_per_batch,
                 headline_over_this=round(o["ms"] / base, 3))
        legs["tuned_block_sizes"] = o
        H.hbp_free(hx)
        # Section 3.1's block of 512 rows x 4096 columns
        hx, ix, o = B.leg(rows_per_block=512, cols_per_block=4096, **{k: v for k, v in params.items() if k not in ("rows_per_block", "cols_per_block")})
        o.update(slots=ix.slots, headline_speedup=round(o["ms"] / base, 3))
        legs["paper_block_size_512x4096"] = o
        H.hbp_free(hx)
        # Section 3.3 read literally: equal block counts per worker, one ticket counter over the rest
        hx, ix, o = B.leg(paper_schedule=True, **params)
        o.update(first_ticket_block=ix.first_ticket_block, blocks=ix.blocks, headline_speedup=round(o["ms"] / base, 3))
        legs["paper_schedule"] = o
        H.hbp_free(hx)
        # this library's schedule without / with a larger competitive share
        for name, q8 in (("all_fixed", 256), ("competitive_quarter", 192)):
            hx, ix, o = B.leg(**dict(params, fixed_fraction_q8=q8))
            o.update(headline_speedup=round(o["ms"] / base, 3))
            legs[name] = o
            H.hbp_free(hx)
        # Section 4's second baseline: the same 2D partition without the hash reorder, all fixed
        hx, ix, o = B.leg(no_reorder=True, **dict(params, fixed_fraction_q8=256))
        o.update(headline_speedup=round(o["ms"] / base, 3), group_len_std=round(B.group_len_std(hx), 4))
        legs["plain_2d"] = o
        H.hbp_free(hx)
        # hash study (Section 5's outlook): rows ordered by their length itself; one shift per block
        for name, kw in (("length_key", dict(key_length=True)), ("block_shift", dict(block_shift=True))):
            hx, ix, o = B.leg(**dict(params, **kw))
            o.update(headline_speedup=round(o["ms"] / base, 3), group_len_std=round(B.group_len_std(hx), 4))
            legs[name] = o
            H.hbp_free(hx)
        legs["headline_group_len_std"] = round(B.group_len_std(h), 4)
        out["legs"] = legs

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
                               "sample": f"whole workload, oracle CSR SpMV ({'extended-precision' if B.f64 else 'fp64'} accumulate) median of {reps} runs; "
                                         f"oracle HBP build once: {o_build * 1e3:.0f} ms",
                               "host_cpus": os.cpu_count()}
    H.hbp_free(h)
    B.close()

    # the other large workloads, measured the same way (library's choice of parameters)
    per_config = [dict(head, hbp_build_ms=round(min(build_ms), 3),
                       csr_best_ms=out.get("csr_best", {}).get("ms"), csr_speedup=out.get("csr_best", {}).get("hbp_speedup"))]
    others = [int(c) for c in args.others.split(",") if c.strip()] if args.scale == 1.0 and library_choice else []
    for number in others:
        if number == args.config:
            continue
        Bo = Bench(number, 1.0, args.dtype, args.steps, args.warmup)
        ho, bms = Bo.timed_builds(2)
        io = H.hbp_get_info(ho)
        step = Bo.wall_ms_per_step(ho, max(20, min(args.steps, 100)), min(args.warmup, 10))
        p_ms, c_ms, _ = Bo.kernel_ms(ho, 30)
        entry = Bo.summary(ho, io, step, p_ms, c_ms)
        entry["hbp_build_ms"] = round(min(bms), 3)
        if not args.no_csr:
            csr, best = Bo.csr_baselines(5)
            entry["csr_best_ms"], entry["csr_best_kernel"], entry["csr_speedup"] = csr[best]["ms"], best, round(csr[best]["ms"] / step, 3)
            if not args.no_study:
                hx, ix, o = Bo.leg(paper_schedule=True)
                entry["paper_schedule_ms"] = o["ms"]
                H.hbp_free(hx)
                hx, ix, o = Bo.leg(**tuned_block_sizes(number, args.dtype))
                entry["tuned_block_sizes_ms"] = o["ms"]
                H.hbp_free(hx)
                hx, ix, o = Bo.leg(no_reorder=True, fixed_fraction_q8=256)
                entry["plain_2d_ms"] = o["ms"]
                H.hbp_free(hx)
        H.hbp_free(ho)
        Bo.close()
        per_config.append(entry)
    per_config.sort(key=lambda e: e["workload"])
    out["per_config"] = per_config
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
