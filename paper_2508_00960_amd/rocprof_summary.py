"""Turns rocprofv3 output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2508_00960_amd.rocprof_summary trace   --workload c4 --dir out/prof_c4 --bench out/prof_c4.json
    python -m paper_2508_00960_amd.rocprof_summary traffic --workload c4 --fetch out/pmc_fetch_c4 --write out/pmc_write_c4 \
                                                           --bench out/pmc_fetch_c4.json
    python -m paper_2508_00960_amd.rocprof_summary mfma    --workload c4 --dir out/pmc_mfma_c4 --bench out/pmc_mfma_c4.json

Each mode prints the summary (redirect it into profiles/ffn_step_<workload>_<kind>.txt).  The directories are what
`rocprofv3 --output-format csv -d <dir> -o <workload>` wrote; --bench is the JSON line bench.py printed in the same
run.  Kernel dispatches are matched to the names bench.py gives its launches by kernel family (which template of
the library), launches per step, and number of workgroups; nothing here knows a workload's shapes.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

FAMILIES = [
    # (substrings of the kernel's name, demangled or not, family, prefixes of the bench names it can carry)
    (("gemm_mfma_fwd_kernel",), "fwd", ("layer update + thin compression",)),
    (("gemm_mfma_tail_kernel",), "tail", ("weight + compressor gradients |",)),
    (("gemm_mfma_table_kernel",), "table", ("weight + compressor gradients of all layers",)),
    (("table_upload_kernel",), "upload", ("parameter table",)),
    (("gemm_mfma_kernel<0, 0", "gemm_mfma_kernelILi0ELi0E"), "kc_kc", ("layer update", "compression")),
    (("gemm_mfma_kernel<0, 1", "gemm_mfma_kernelILi0ELi1E"), "kc_km", ("input gradient", "error compression")),
    (("gemm_mfma_kernel<1, 1", "gemm_mfma_kernelILi1ELi1E"), "km_km", ("weight + compressor gradients", "weight gradients", "compressor gradient")),
    (("thin_product_kernel",), "thin", ("compression",)),
    (("reduce_scatter_kernel",), "rs", ("reduce-scatter",)),
    (("sgd_kernel",), "sgd", ("SGD update",)),
    (("mse_delta_kernel",), "mse", ("output error",)),
    (("colsum_kernel",), "colsum", ("bias gradient",)),
    (("loss_kernel",), "loss", ("loss",)),
    (("gemm_generic_kernel",), "generic", ()),
    (("fill_zero_kernel",), "fill", ("clear",)),
    (("copy_kernel",), "copy", ()),
]


def family_of(kernel_name):
    if "phantom" not in kernel_name:        # the library's kernels live in namespace phantom
        return None, ()
    for needles, fam, prefixes in FAMILIES:
        if any(n in kernel_name for n in needles):
            return fam, prefixes
    return None, ()


def short(kernel_name):
    fam, _ = family_of(kernel_name)
    if fam is None:
        return kernel_name.split("(")[0][-60:]
    name = kernel_name.split("(")[0]
    name = name.replace("void phantom::", "").replace("phantom::", "")
    if name.startswith("_ZN7phantom"):      # a name the profiler's demangler gave up on (the bfloat16 type): make it readable
        import re
        m = re.match(r"_ZN7phantom\d+([a-z_]+)I(.*?)EEv", name)
        if m:
            args = m.group(2).replace("DF16b", "@,").replace("Lb0E", "0,").replace("Lb1E", "1,")
            args = re.sub(r"Li(\d+)E", r"\1,", args).replace("f", "float,").replace("@", "bf16").rstrip(",")
            name = f"{m.group(1)}<{args}>"
    return name[:70]


def one_file(directory, suffix):
    hits = glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True)
    if not hits:
        raise SystemExit(f"no *{suffix} under {directory}")
    return hits[0]


def expected_workgroups(row):
    """Workgroup counts a launch of this bench row may have: one per 128 x 128 tile, or one per pair of tiles."""
    single = dual = 0
    for m, n in (("M", "N"), ("M2", "N2"), ("M3", "N3")):
        tm, tn = -(-row.get(m, 0) // 128), -(-row.get(n, 0) // 128)
        single += tm * tn * row["groups"]
        dual += -(-tm // 2) * tn * row["groups"]
    thin = -(-row.get("M", 0) // 32) * row["groups"]
    first_dual = -(--(-row.get("M", 0) // 128) // 2) * -(-row.get("N", 0) // 128) * row["groups"]
    return single, {single, dual, thin, first_dual, -(-row.get("M", 0) // 128) * -(-row.get("N", 0) // 128) * row["groups"]}


def carries_pair(kernel_name):
    """Is this an instance of gemm_mfma_kernel built for two products in one launch (template argument PAIR)?"""
    import re
    m = re.search(r"gemm_mfma_kernel<([^>]*)>", short(kernel_name))
    if not m:
        return None
    args = [a.strip() for a in m.group(1).split(",")]
    return len(args) >= 7 and args[6] in ("1", "true")


def match_rows(groups, rows):
    """groups: {(kernel name, workgroups): calls}; rows: bench.py's kernel table.  Returns {(kernel, wgs): row}."""
    out = {}
    used = set()
    order = {fam: i for i, (_, fam, _) in enumerate(FAMILIES)}
    fam_groups = collections.defaultdict(list)
    for key, calls in groups.items():
        fam, prefixes = family_of(key[0])
        if fam and prefixes:
            fam_groups[(fam, prefixes)].append((key, calls))
    # families whose kernel can carry one kind of launch only come first (the thin kernel before the general product)
    for (fam, prefixes), items in sorted(fam_groups.items(), key=lambda kv: (len(kv[0][1]), order[kv[0][0]])):
        cand = [r for r in rows if id(r) not in used and any(r["name"].startswith(p) for p in prefixes)
                and not (fam in ("kc_kc", "km_km", "kc_km") and "|" in r["name"]) and not (fam == "kc_kc" and "thin" in r["name"])]
        items.sort(key=lambda kv: (-kv[1], kv[0][1]))
        left = []
        for key, calls in items:            # first the launches whose workgroup count is exactly what a row's shapes give
            hit = [r for r in cand if id(r) not in used and key[1] in expected_workgroups(r)[1]]
            pair = carries_pair(key[0])
            if pair is not None and any(("M2" in r) == pair for r in hit):     # a launch of two products has a second shape
                hit = [r for r in hit if ("M2" in r) == pair]
            if len(hit) >= 1:
                hit.sort(key=lambda r: abs(expected_workgroups(r)[0] - key[1]))
                out[key] = hit[0]
                used.add(id(hit[0]))
            else:
                left.append((key, calls))
        rest = sorted((r for r in cand if id(r) not in used), key=lambda r: (-r["launches_per_step"], expected_workgroups(r)[0]))
        for (key, _), row in zip(left, rest):
            out[key] = row
            used.add(id(row))
        for key, _ in left[len(rest):]:     # more kinds of dispatch than names (a rider adds a workgroup): the nearest name
            if cand:
                out[key] = min(cand, key=lambda r: abs(expected_workgroups(r)[0] - key[1]))
    return out


def load_bench(path):
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line.startswith("{"):
                return json.loads(line)
    raise SystemExit(f"no JSON line in {path}")


def trace(args):
    rows = list(csv.DictReader(open(one_file(args.dir, "kernel_trace.csv"))))
    bench = load_bench(args.bench)
    agg = collections.defaultdict(list)
    for r in rows:
        wgs = (int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])) // \
              (int(r["Workgroup_Size_X"]) * int(r["Workgroup_Size_Y"]) * int(r["Workgroup_Size_Z"]))
        agg[(r["Kernel_Name"], wgs)].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    named = match_rows({k: len(v) for k, v in agg.items()}, bench["kernels"])
    own = {k: v for k, v in agg.items() if family_of(k[0])[0] is not None}
    total = sum(sum(v) for v in own.values())
    print(f"# rocprofv3 kernel-trace summary: phantom_ffn_step, workload {bench['config']['workload']}")
    print("# command (from the repository root on the GPU box, after cd /tmp; export TMPDIR=/tmp):")
    print(f"#   {args.command}")
    print(f"#   python -m paper_2508_00960_amd.rocprof_summary trace --workload {args.workload} --dir {args.dir} --bench {args.bench}")
    print("# (bench.py runs warm-up, a graph capture, the timed graph replays, eager timing and an event-bracketed pass; every dispatch of")
    print("#  the library's kernels in the process is counted; the dense comparison, the other workloads and the oracle are switched off)")
    print("# per (kernel, workgroups per launch): kernel | bench.py's name of the launch | workgroups | calls | total ms | average us | % of the library's kernel time | min us | max us")
    print()
    for k, v in sorted(own.items(), key=lambda kv: -sum(kv[1])):
        row = named.get(k)
        label = "-" if row is None else f"{row['name']} M={row['M']} N={row['N']} K={row['K']} x{row['groups']}"
        print(f"{short(k[0]):<72} | {label:<92} | {k[1]:>6} | {len(v):>5} | {sum(v) / 1e6:>8.3f} | {sum(v) / len(v) / 1e3:>8.2f} | "
              f"{100 * sum(v) / total:>5.2f} | {min(v) / 1e3:>7.2f} | {max(v) / 1e3:>7.2f}")
    print()
    print("# the same launches timed live by bench.py in this run with HIP events around each (under the profiler, which adds to the event latency): average us per launch")
    for r in bench["kernels"]:
        extra = f"  ({r['tflops']} TFLOP/s)" if "tflops" in r else ""
        print(f"#   {r['name']:<64} M={r['M']} N={r['N']} K={r['K']} x{r['groups']}: {r['avg_us']:.2f}{extra}")
    print(f"# whole step under the profiler (HIP graph replay): {bench['ms_per_step'] * 1e3:.1f} us = {bench['value']:.1f} TFLOP/s")
    dom = bench["roofline"]
    print(f"# dominant launch (bench.py's roofline object): {dom['kernel']}: {dom['avg_us']} us between its events, "
          f"{dom['achieved']} {dom['unit']} = {dom['frac']:.3f} of the {dom['bound']} peak")


def counters(directory):
    rows = list(csv.DictReader(open(one_file(directory, "counter_collection.csv"))))
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in rows:
        wgs = int(r["Grid_Size"]) // int(r["Workgroup_Size"])
        agg[(r["Kernel_Name"], wgs)][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def traffic(args):
    import bench as bench_py
    bench = load_bench(args.bench)
    F, W = counters(args.fetch), counters(args.write)
    # calibration: the one 256 MiB device copy of bench.py --calibrate-copy (262144 KiB read, 262144 KiB written); bench.py's
    # other large copies (measured_copy_gbs) move 1 GiB each, so the calibration copy is the smallest of the large ones
    known = 256 * 1024
    big_f = [min(v["FETCH_SIZE"]) for k, v in F.items() if family_of(k[0])[0] is None and max(v["FETCH_SIZE"]) > 50000]
    big_w = [min(v["WRITE_SIZE"]) for k, v in W.items() if family_of(k[0])[0] is None and max(v["WRITE_SIZE"]) > 50000]
    if not big_f or not big_w:
        raise SystemExit("calibration copy not found (run bench.py with --calibrate-copy)")
    cal_f, cal_w = min(big_f), min(big_w)
    sf, sw = known / cal_f, known / cal_w
    named = match_rows({k: len(v["FETCH_SIZE"]) for k, v in F.items()}, bench["kernels"])
    print(f"# HBM traffic per launch, workload {bench['config']['workload']}, from two rocprofv3 counter passes:")
    print(f"#   {args.command.replace('COUNTER', 'FETCH_SIZE').replace('OUTDIR', args.fetch)}")
    print(f"#   {args.command.replace('COUNTER', 'WRITE_SIZE').replace('OUTDIR', args.write)}")
    print(f"#   python -m paper_2508_00960_amd.rocprof_summary traffic --workload {args.workload} --fetch {args.fetch} --write {args.write} --bench {args.bench}")
    print("# (after cd /tmp; export TMPDIR=/tmp; each pass under timeout -s KILL 180)")
    print(f"# kernel sources: {bench_py.kernel_sources_hash()}")
    print(f"# calibration: the 256 MiB device-to-device copy of --calibrate-copy (262144 KiB read, 262144 KiB written) reads FETCH_SIZE = {cal_f:.1f} and WRITE_SIZE = {cal_w:.1f}")
    print(f"#   -> bytes = FETCH_SIZE x 1024 x {sf:.4f}, bytes = WRITE_SIZE x 1024 x {sw:.4f}")
    print("# columns: workload kernel M N K groups fetch_bytes write_bytes   | raw FETCH_SIZE, WRITE_SIZE (KiB per dispatch, average), algorithmic bytes, traffic / algorithmic")
    for k, row in sorted(named.items(), key=lambda kv: kv[1]["name"]):
        if k not in W or "algorithmic_bytes" not in row:
            continue
        f_raw = sum(F[k]["FETCH_SIZE"]) / len(F[k]["FETCH_SIZE"])
        w_raw = sum(W[k]["WRITE_SIZE"]) / len(W[k]["WRITE_SIZE"])
        fb, wb = f_raw * 1024 * sf, w_raw * 1024 * sw
        alg = row["algorithmic_bytes"]
        print(f"{args.workload} {row['name'].replace(' ', '_')} {row['M']} {row['N']} {row['K']} {row['groups']} {fb:.0f} {wb:.0f}   | "
              f"{f_raw:.1f} {w_raw:.1f} {alg:.0f} {(fb + wb) / alg:.3f}")
    print("# (algorithmic bytes: each operand of each product of the launch read once, its output written once; what an epilogue reads or writes besides,")
    print("#  the saved sigma' or ReLU bits, the target, the output error, and a rider's tensors are not in that figure)")
    for k, v in F.items():
        fam = family_of(k[0])[0]
        if fam in ("rs", "sgd", "fill", "thin") and k in W:
            f_raw = sum(v["FETCH_SIZE"]) / len(v["FETCH_SIZE"])
            w_raw = sum(W[k]["WRITE_SIZE"]) / len(W[k]["WRITE_SIZE"])
            print(f"# {short(k[0])} ({k[1]} workgroups): fetch {f_raw * 1024 * sf:.0f} B, write {w_raw * 1024 * sw:.0f} B per launch")


def mfma(args):
    bench = load_bench(args.bench)
    C = counters(args.dir)
    named = match_rows({k: len(next(iter(v.values()))) for k, v in C.items()}, bench["kernels"])
    print(f"# rocprofv3 counter pass: matrix-core utilisation and LDS activity per kernel of phantom_ffn_step, workload {bench['config']['workload']}")
    print(f"#   {args.command}")
    print(f"#   python -m paper_2508_00960_amd.rocprof_summary mfma --workload {args.workload} --dir {args.dir} --bench {args.bench}")
    print("# MfmaUtil: share of the whole dispatch (launch, first tile and epilogue included) during which the matrix cores are busy.")
    print("# SQ_INSTS_VALU_MFMA_MOPS_BF16 counts 512 FLOP each: \"MFMA GFLOP\" is what the matrix cores executed, padding of ragged tiles included.")
    print("# columns: kernel | bench.py's name | workgroups | dispatches | MfmaUtil % | MFMA GFLOP per dispatch | SQ_ACTIVE_INST_LDS | SQ_LDS_BANK_CONFLICT (cycles per dispatch) | conflicts / LDS-active")
    for k, v in sorted(C.items(), key=lambda kv: kv[0][0]):
        if family_of(k[0])[0] is None:
            continue
        avg = lambda name: (sum(v[name]) / len(v[name])) if name in v else float("nan")
        row = named.get(k)
        label = "-" if row is None else row["name"]
        lds, conf = avg("SQ_ACTIVE_INST_LDS"), avg("SQ_LDS_BANK_CONFLICT")
        print(f"{short(k[0]):<72} | {label:<64} | {k[1]:>6} | {len(next(iter(v.values()))):>4} | {avg('MfmaUtil'):>5.1f} | "
              f"{avg('SQ_INSTS_VALU_MFMA_MOPS_BF16') * 512e-9:>8.2f} | {lds:>10.0f} | {conf:>8.0f} | {conf / lds if lds else 0:.3f}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["trace", "traffic", "mfma"])
    ap.add_argument("--workload", required=True)
    ap.add_argument("--dir")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--bench", required=True)
    ap.add_argument("--command", default="", help="the rocprofv3 command line that produced the input, to be quoted in the summary")
    args = ap.parse_args()
    {"trace": trace, "traffic": traffic, "mfma": mfma}[args.mode](args)


if __name__ == "__main__":
    main()
