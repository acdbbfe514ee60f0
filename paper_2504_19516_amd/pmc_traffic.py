"""HBM traffic of the prefill gate/up GEMM and of the decode layer-step from rocprofv3 byte counters.

Takes the counter CSVs of two runs of the benchmark with the copy-kernel reference switched on,

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir1> -o out -- python3 bench.py --split 224 --steps 5 --warmup 1 --no-cpu-baseline --no-serving --pmc-probe
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir2> -o out -- python3 bench.py --split 224 --steps 5 --warmup 1 --no-cpu-baseline --no-serving --pmc-probe

scales each counter by what it reads for the copy kernel (which moves a known number of bytes
each way) and prints the per-launch figures of the gate/up GEMM and the per-step sum over the
decode phase's kernels. With --json it also writes the record bench.py reports as
roofline.traffic and roofline_decode.traffic.

    python -m paper_2504_19516_amd.pmc_traffic <fetch.csv> <write.csv> --prefill-cus 224 [--json] [--l2 <l2.csv>]

--l2 takes the CSV of a third pass with the L2 request counters (--pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum, same command) and
prints requests, hits and misses per launch of every kernel.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re
import subprocess

COPY_BYTES = 512 << 20                     # bench.py --pmc-probe: bytes read (and bytes written) per copy launch
GATEUP_KERNEL = "gemm_wreg_kernel"         # the 256 x 256 prefill tile; its SwiGLU instantiation is the gate/up GEMM
# SwiGLU epilogue = first template argument 3 (the second is the tile's wave rows: 2 = 256 x 256), demangled or mangled name
GATEUP_PATTERN = r"gemm_wreg_kernel<3, 2>|gemm_wreg_kernelILi3ELi2E"
COPY_KERNEL = "copy_kernel"
# kernels that only the decode phase launches; one attn_decode_mfma launch = one decode layer-step.
# (Its embedding and first RMSNorm launches share kernels with the prefill phase and are left out:
# 64 rows, under 2 MB per step.)
DECODE_STEP_KERNEL = "attn_decode_mfma_kernel"
DECODE_KERNELS = (r"attn_decode_mfma_kernel", r"attn_decode_merge_kernel", r"decode_qkv_finish_kernel", r"reduce_resid_norm_kernel",
                  r"reduce_swiglu_kernel", r"gemm_dl_kernel<64, |gemm_dl_kernelILi64E", r"gemm_skinny_kernel")


def per_kernel(path, counter, queue_of=None):
    """kernel name -> counter values, one per launch. With queue_of (a kernel-name pattern), only the launches on the
    hardware queue that carries most launches of that kernel are kept: the benchmark also runs its time-multiplexed
    reference (other streams, other launch shapes), which is not what the stored figures describe."""
    recs = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                recs.append((r["Kernel_Name"], float(r["Counter_Value"]), r.get("Queue_Id", "")))
    keep = None
    if queue_of is not None:
        queues = collections.Counter(q for name, _, q in recs if re.search(queue_of, name))
        if queues:
            keep = queues.most_common(1)[0][0]
    rows = collections.defaultdict(list)
    for name, v, q in recs:
        if keep is None or q == keep:
            rows[name].append(v)
    return rows


def pick(rows, needle, pattern=None):
    vals = []
    for name, v in rows.items():
        if needle in name and (pattern is None or re.search(pattern, name)):
            vals += v
    return vals


def git_head():
    try:
        return subprocess.run(["git", "rev-parse", "--short", "HEAD"], cwd=os.path.dirname(os.path.abspath(__file__)), capture_output=True,
                              text=True, check=True).stdout.strip()
    except Exception:
        return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_csv")
    ap.add_argument("write_csv")
    ap.add_argument("--prefill-cus", type=int, required=True)
    ap.add_argument("--json", action="store_true")
    ap.add_argument("--list", action="store_true", help="also print every kernel's mean bytes per launch")
    ap.add_argument("--l2", default=None, help="counter CSV of a TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum pass")
    ap.add_argument("--commit", default=None, help="commit of the kernels that were measured (default: this checkout's HEAD)")
    args = ap.parse_args()
    out = {}
    lines = []
    for counter, path in (("FETCH_SIZE", args.fetch_csv), ("WRITE_SIZE", args.write_csv)):
        rows = per_kernel(path, counter)
        prefill_rows = per_kernel(path, counter, GATEUP_PATTERN)              # the prefill partition's queue
        decode_rows = per_kernel(path, counter, DECODE_STEP_KERNEL)           # the decode partition's queue
        copy = pick(rows, COPY_KERNEL)
        # the benchmark also runs the copy kernel on smaller buffers (its bandwidth probes of the decode
        # partition); the reference launches are the largest ones
        copy = [v for v in copy if v >= 0.75 * max(copy)] if copy else copy
        gate = pick(prefill_rows, GATEUP_KERNEL, GATEUP_PATTERN)
        if not copy or not gate:
            raise SystemExit(f"{counter}: kernels not found in {path} (copy launches {len(copy)}, gate/up launches {len(gate)})")
        copy_mean, gate_mean = sum(copy) / len(copy), sum(gate) / len(gate)
        factor = COPY_BYTES / copy_mean                     # bytes per counter unit
        steps = len(pick(decode_rows, DECODE_STEP_KERNEL))
        dec_units = sum(sum(v) for name, v in decode_rows.items() if any(re.search(pat, name) for pat in DECODE_KERNELS))
        if not steps:
            raise SystemExit(f"{counter}: no decode step found in {path}")
        out[counter] = dict(copy_counter=copy_mean, factor_bytes_per_unit=factor, gateup_counter=gate_mean,
                            gateup_bytes=gate_mean * factor, launches=len(gate), decode_bytes=dec_units / steps * factor, decode_steps=steps)
        lines.append(f"{counter}: copy kernel reads {copy_mean:.1f} per launch for {COPY_BYTES} bytes -> {factor:.2f} bytes per unit; "
                     f"gate/up GEMM {gate_mean:.1f} per launch over {len(gate)} launches -> {gate_mean * factor / 1e6:.1f} MB")
    total = out["FETCH_SIZE"]["gateup_bytes"] + out["WRITE_SIZE"]["gateup_bytes"]
    lines.append(f"gate/up GEMM HBM traffic per launch: {total / 1e6:.1f} MB "
                 f"(read {out['FETCH_SIZE']['gateup_bytes'] / 1e6:.1f}, written {out['WRITE_SIZE']['gateup_bytes'] / 1e6:.1f})")
    if args.list:
        for counter, path in (("FETCH_SIZE", args.fetch_csv), ("WRITE_SIZE", args.write_csv)):
            rows = per_kernel(path, counter)
            f = out[counter]["factor_bytes_per_unit"]
            lines.append(f"{counter}, mean per launch:")
            for name, v in sorted(rows.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
                if sum(v) / len(v) * f >= 1e5:
                    lines.append(f"  {sum(v) / len(v) * f / 1e6:10.1f} MB  x {len(v):4d}  {name[:90]}")
    dec_total = out["FETCH_SIZE"]["decode_bytes"] + out["WRITE_SIZE"]["decode_bytes"]
    lines.append(f"decode layer-step HBM traffic (its own kernels, mean of {out['FETCH_SIZE']['decode_steps']} steps): {dec_total / 1e6:.1f} MB "
                 f"(read {out['FETCH_SIZE']['decode_bytes'] / 1e6:.1f}, written {out['WRITE_SIZE']['decode_bytes'] / 1e6:.1f})")
    if args.l2:
        req, hit, miss = (per_kernel(args.l2, n) for n in ("TCC_REQ_sum", "TCC_HIT_sum", "TCC_MISS_sum"))
        lines.append("L2 (all 8 XCDs summed), mean per launch: requests, hits, misses (millions), hit rate")
        for name, v in sorted(req.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
            r, h, m = (sum(x[name]) / len(x[name]) / 1e6 for x in (req, hit, miss))
            if r >= 0.05:
                lines.append(f"  {r:9.2f} {h:9.2f} {m:9.2f}  {100 * h / r:5.1f} %  x {len(v):4d}  {name[:80]}")
    print("\n".join(lines))
    if args.json:
        rec = dict(workload="config2", prefill_cus=args.prefill_cus, gateup_hbm_bytes_per_launch=total,
                   read_bytes=out["FETCH_SIZE"]["gateup_bytes"], written_bytes=out["WRITE_SIZE"]["gateup_bytes"],
                   decode_hbm_bytes_per_step=dec_total, decode_read_bytes=out["FETCH_SIZE"]["decode_bytes"],
                   decode_written_bytes=out["WRITE_SIZE"]["decode_bytes"],
                   fetch_factor=out["FETCH_SIZE"]["factor_bytes_per_unit"], write_factor=out["WRITE_SIZE"]["factor_bytes_per_unit"],
                   measured_at_commit=args.commit or git_head())
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data", "pmc_traffic.json")
        with open(path, "w") as f:
            json.dump(rec, f, indent=1)
        print("wrote", path)


if __name__ == "__main__":
    main()
