#!/usr/bin/env python3
"""Benchmark of the phantom-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]

A "step" is one pass of the whole hot path over one batch of synthetic input that already sits in
HBM.  The default workload is benchmark configuration 4, the largest single-GPU one: n=16384, p=16
(shard 1024), k=64, batch 4096, 8 layers, GELU, MSE, bf16 storage / fp32 accumulate, rank 0 with the 15
peers' phantom buffers seeded; its step is a training step through phantom_ffn_step (forward through
every layer, loss, backward through every layer, SGD).
Prints ONE JSON line: whole-step throughput (TFLOP/s from the algorithmic FLOP count
6*B*s*(s+p*k) per layer and rank, and samples/s), the roofline of the dominant kernel measured
with HIP events around each of its launches, the CPU oracle timed on a bounded sample, the
dense network of equal width (and one rank's tensor-parallel share of it) through the same kernels, and
the other benchmark configurations (2, 3 and the forward sweep 5) as extra keys.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0         # MI355X HBM3E, published
SETTLE_S = 0.3                # untimed load before every timed region, beyond the --warmup steps (see time_steps)

WORKLOADS = {
    # name: (n, p, k, batch, layers, act, dtype, rank, mode, lr)
    "c1": (256, 4, 8, 32, 2, "relu", "f32", -1, "train", 1e-2),
    "c2": (4096, 8, 32, 1024, 4, "relu", "bf16", -1, "no_update", 0.0),
    "c3": (32768, 64, 16, 2048, 1, "relu", "bf16", 0, "no_update", 0.0),
    "c4": (16384, 16, 64, 4096, 8, "gelu", "bf16", 0, "train", 1e-3),
    "c5k4": (8192, 8, 4, 8192, 6, "relu", "bf16", 0, "forward", 0.0),
    "c5k16": (8192, 8, 16, 8192, 6, "relu", "bf16", 0, "forward", 0.0),
    "c5k64": (8192, 8, 64, 8192, 6, "relu", "bf16", 0, "forward", 0.0),
    "c5k256": (8192, 8, 256, 8192, 6, "relu", "bf16", 0, "forward", 0.0),
    # configuration 2 generalised to more ranks on the one device (grouped products, in-memory gather / reduce)
    "a16": (8192, 16, 32, 1024, 4, "relu", "bf16", -1, "no_update", 0.0),
    "a32": (8192, 32, 16, 1024, 4, "relu", "bf16", -1, "no_update", 0.0),
    "a64": (16384, 64, 8, 512, 4, "relu", "bf16", -1, "no_update", 0.0),
    # layers of different widths and phantom widths (Section IV, first paragraph): two more entries, the widths
    # n_0 .. n_L and k_1 .. k_L; here configuration 2 with every other layer twice as wide
    "w4": (4096, 8, 32, 1024, 4, "relu", "bf16", -1, "no_update", 0.0, (4096, 8192, 4096, 8192, 4096), (32, 64, 32, 64)),
}


def layer_shapes(n, p, k, L, widths=(), ks=()):
    """(si, so, k) of every layer: inputs and outputs held by one rank, phantom width."""
    widths = widths or (n,) * (L + 1)
    ks = ks or (k,) * L
    return [(widths[l] // p, widths[l + 1] // p, ks[l]) for l in range(L)]


def flops_per_step(shapes, p, B, mode, groups):
    q = p - 1
    # multiply-adds of one forward on one rank (Section IV-A): local update, decompression, compression
    per = sum(B * (so * si + q * so * k + (k * si if q else 0)) for si, so, k in shapes)
    passes = 1 if mode == "forward" else 3           # backward costs twice the forward (Section IV-B)
    return 2.0 * per * passes * groups


def bytes_per_step(shapes, p, B, mode, groups, e):
    """Algorithmic bytes: every input and weight read once, every output written once, storage type."""
    q = p - 1
    total = 0
    for si, so, k in shapes:
        W = so * si + q * so * k + (k * si if q else 0) + so
        fwd = e * (B * si + B * so + q * k * B + (B * k if q else 0) + W)
        bwd = e * (2 * B * si + 2 * B * so + 2 * q * k * B + (B * k if q else 0) + 2 * W)
        total += fwd if mode == "forward" else fwd + bwd
    return float(total * groups)


class Bench:
    """Device-resident tensors of one workload and a closure that runs one step through the C ABI."""

    def __init__(self, name, seeded=True, seed=0):
        import numpy as np
        import torch
        import paper_2508_00960_amd as ph
        import phantom_inputs as pin
        from helpers import empty, empty_f32, to_gpu, to_gpu_f32, workspace

        spec = WORKLOADS[name] if isinstance(name, str) else name
        n, p, k, B, L, act, dt, rank, mode, lr = spec[:10]
        widths, ks = (spec[10], spec[11]) if len(spec) > 10 else ((), ())
        self.cfg = dict(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dt, rank=rank, mode=mode, lr=lr,
                        widths=tuple(widths), ks=tuple(ks))
        self.shapes = layer_shapes(n, p, k, L, widths, ks)
        self.ph, self.torch = ph, torch
        self.prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dt, rank=rank, widths=tuple(widths), ks=tuple(ks))
        self.pc = ph.make_problem(n, p, k, B, L, act, dt, rank, widths=tuple(widths), ks=tuple(ks))
        self.groups = p if rank < 0 else 1
        self.mode, self.lr = mode, lr
        self.ws = workspace(ph.workspace_bytes(self.pc))
        q = p - 1
        has = q > 0
        tdt = torch.float32 if dt == "f32" else torch.bfloat16
        lead = (p,) if rank < 0 else ()
        names = ["Lw", "bias"] + (["Cw", "Dw"] if has else [])
        if seeded:
            data = pin.all_rank_step_inputs(self.prob, seed) if rank < 0 else pin.one_rank_step_inputs(self.prob, seed)
            self.host = data
            self.W = {nm: [to_gpu(P[nm], dt) for P in data["layers"]] for nm in names}
            self.G = [to_gpu(P["G"], dt) for P in data["layers"]] if (has and rank >= 0) else None
            self.dg = [to_gpu(P["dg_own"], dt) for P in data["layers"]] if (has and rank >= 0) else None
            self.X0, self.T = to_gpu(data["X0"], dt), to_gpu(data["T"], dt)
        else:
            # same shapes and distributions, drawn on the GPU (used for the side measurements only)
            gen = torch.Generator(device="cuda").manual_seed(seed)
            def uni(shape, bound):
                return ((torch.rand(shape, device="cuda", generator=gen) * 2 - 1) * bound).to(tdt)
            def nrm(shape, scale=1.0):
                return (torch.randn(shape, device="cuda", generator=gen) * scale).to(tdt)
            def layer_weights(si, so, kl):
                shapes = {"Lw": (lead + (so, si), si ** -0.5), "bias": (lead + (so,), si ** -0.5)}
                if has:
                    shapes["Cw"] = (lead + (kl, si), si ** -0.5)
                    shapes["Dw"] = (lead + (q, so, kl), kl ** -0.5)
                return {nm: uni(*shapes[nm]) for nm in names}
            per_layer = [layer_weights(*sh) for sh in self.shapes]
            self.W = {nm: [d[nm] for d in per_layer] for nm in names}
            self.G = [nrm((q, B, kl)) for _, _, kl in self.shapes] if (has and rank >= 0) else None
            self.dg = [nrm((B, kl), 1.0 / B) for _, _, kl in self.shapes] if (has and rank >= 0) else None
            self.X0, self.T = nrm(lead + (B, self.shapes[0][0])), nrm(lead + (B, self.shapes[-1][1]))
        self.M = None
        if dt == "bf16" and mode == "train":
            self.M = {nm: [w.float() for w in self.W[nm]] for nm in names}
        self.loss = empty_f32((4,))
        self.flops = flops_per_step(self.shapes, p, B, mode, self.groups)
        self.bytes = bytes_per_step(self.shapes, p, B, mode, self.groups, 4 if dt == "f32" else 2)

    def step(self):
        W, M = self.W, self.M or {}
        self.ph.ffn_step(self.pc, self.X0, self.T, W["Lw"], W.get("Cw"), W.get("Dw"), W["bias"],
                         Lw_master=M.get("Lw"), Cw_master=M.get("Cw"), Dw_master=M.get("Dw"),
                         bias_master=M.get("bias"), G=self.G, dg_own=self.dg, loss=self.loss, lr=self.lr,
                         mode=self.mode, workspace=self.ws)

    def time_steps(self, steps, warmup, graph=True):
        """(ms per step, launch mode).  Warm-up untimed, then exactly `steps` steps between device syncs."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        # The device's clocks take a few hundred milliseconds of load to settle (the first 20 steps after an idle
        # period run about 8 % slower than the same steps later): more untimed steps until SETTLE_S have passed.
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < SETTLE_S:
            for _ in range(10):
                self.step()
            torch.cuda.synchronize()
        run, how = self.step, "eager"
        if graph:
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    self.step()
                torch.cuda.current_stream().wait_stream(side)
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    self.step()
                g.replay()
                torch.cuda.synchronize()
                run, how = g.replay, "hip_graph"
            except Exception as exc:   # capture is an optimisation of the launch path, not of the kernels
                print(f"[bench] graph capture failed, timing eager launches: {exc}", file=sys.stderr)
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, how

    def profile(self, steps):
        """Per-kernel times from HIP events around every launch (eager launches)."""
        self.torch.cuda.synchronize()
        self.ph.profile_begin(steps * 64 * self.prob.layers + 64)
        for _ in range(steps):
            self.step()
        return self.ph.profile_end()


EMPTY_LAUNCH = "(empty launch)"


def kernel_table(entries, steps, esize):
    """Adds per-launch averages, FLOP and algorithmic bytes to the raw profile entries.

    avg_us is the time between the HIP events around a launch, as measured: it includes about 2 us of
    launch latency that rocprofv3's kernel duration does not, so every rate derived from it is on the
    low side.  What the same pair of events reads around a kernel that does nothing is reported
    beside it (`empty_launch_us`), not subtracted.
    """
    out = []
    empty = [e for e in entries if e["name"] == EMPTY_LAUNCH]
    overhead = empty[0]["total_ms"] * 1e3 / empty[0]["calls"] if empty else 0.0
    for e in entries:
        if e["name"] == EMPTY_LAUNCH:
            continue
        avg_us = e["total_ms"] * 1e3 / e["calls"]
        row = dict(name=e["name"], M=e["M"], N=e["N"], K=e["K"], groups=e["groups"],
                   launches_per_step=e["calls"] / steps, avg_us=round(avg_us, 3))
        if e["K"] > 0:
            out_e = 4 if "gradients" in e["name"] or e["name"] == "compressor gradient" else esize
            flops, byts = 0.0, 0.0
            # the third and fourth product of a launch are the input gradient and / or the error compression riding with
            # the weight gradients: storage type out
            for M, N, K, oe in ((e["M"], e["N"], e["K"], out_e), (e.get("M2", 0), e.get("N2", 0), e.get("K2", 0), out_e),
                                (e.get("M3", 0), e.get("N3", 0), e.get("K3", 0), esize),
                                (e.get("M4", 0), e.get("N4", 0), e.get("K4", 0), esize)):
                flops += 2.0 * M * N * K * e["groups"]
                byts += (esize * (M + N) * K + oe * M * N) * e["groups"]
            if e.get("K2", 0):
                row.update(M2=e["M2"], N2=e["N2"], K2=e["K2"])
            if e.get("K3", 0):
                row.update(M3=e["M3"], N3=e["N3"], K3=e["K3"])
            if e.get("K4", 0):
                row.update(M4=e["M4"], N4=e["N4"], K4=e["K4"])
            row.update(tflops=round(flops / avg_us * 1e-6, 2), gbs=round(byts / avg_us * 1e-3, 1),
                       flops=flops, bytes=byts)
        out.append(row)
    return out, overhead


def kernel_sources_hash():
    """sha256 (first 16 hex digits) over the HIP sources the library is built from, in name order."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2508_00960_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, row):
    """HBM bytes per launch of one kernel, from the committed rocprofv3 counter summary of this workload
    (profiles/ffn_step_<workload>_hbm_traffic.txt); None if there is none, if it has no line for this kernel,
    or if it was taken from other kernel sources than the ones in the tree (its "# kernel sources:" line).

    The summary holds one line per (workload, kernel, shape): FETCH_SIZE and WRITE_SIZE per dispatch,
    already scaled by what the same counters read for a copy of known size in the same run.
    """
    path = os.path.join(ROOT, "profiles", f"ffn_step_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    key = [workload, row["name"].replace(" ", "_"), str(row["M"]), str(row["N"]), str(row["K"]), str(row["groups"])]
    found, fresh = None, False
    with open(path) as f:
        for line in f:
            w = line.split()
            if line.startswith("# kernel sources:"):
                fresh = w[-1] == kernel_sources_hash()
            if len(w) >= 8 and not line.startswith("#") and w[:6] == key:
                found = float(w[6]) + float(w[7])
    return found if fresh else None


def vendor_gemm_reference(c, shapes, groups):
    """Context only, never part of `value`: what the vendor GEMM library (hipBLASLt / rocBLAS through torch.matmul)
    takes for the bare matrix products of ONE layer of this workload at the same shapes and operand layouts,
    without bias, activation, sigma' or any fusion, one product per call (torch.bmm over the ranks held).
    Shows what a product of this shape costs on this chip apart from this library's kernels."""
    import torch
    si, so, k = shapes[-1]
    B, q = c["batch"], c["p"] - 1
    Kc = si + q * k

    def r(*shape):
        return torch.randn(*((groups,) + shape), device="cuda", dtype=torch.bfloat16)

    def time_us(fn, iters=30):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    xcat, wcat, delta = r(B, Kc), r(so, Kc), r(B, so)
    out = {"layer update [B,Kc]x[so,Kc]^T": time_us(lambda: torch.bmm(xcat, wcat.transpose(1, 2)))}
    if q:
        x, cw = r(B, si), r(k, si)
        out["compression [B,si]x[k,si]^T"] = time_us(lambda: torch.bmm(x, cw.transpose(1, 2)))
    if c["mode"] != "forward":
        lc, dcat = r(so + (k if q else 0), si), r(B, so + (k if q else 0))
        out["input gradient [B,so+k]x[so+k,si]"] = time_us(lambda: torch.bmm(dcat, lc))
        out["weight gradients [B,so]^Tx[B,Kc]"] = time_us(lambda: torch.bmm(delta.transpose(1, 2), xcat))
        if q:
            dw, dg, x = r(so, q * k), r(B, k), r(B, si)
            out["error compression [B,so]x[so,(p-1)k]"] = time_us(lambda: torch.bmm(delta, dw))
            out["compressor gradient [B,k]^Tx[B,si]"] = time_us(lambda: torch.bmm(dg.transpose(1, 2), x))
    total = sum(out.values())
    return {"per_layer_us": {name: round(us, 2) for name, us in out.items()}, "layer_us": round(total, 2),
            "step_ms_products_only": total * c["layers"] * 1e-3,
            "what": "torch.bmm (vendor GEMM library) on the bare products of the last layer's shapes, one call each, "
                    "no epilogues; context, not a target and not this library's path"}


def cpu_baseline(bench, sample_batch):
    """The fp64 oracle as it stands on the host cores, on a batch subset of the same workload."""
    import phantom_inputs as pin
    from oracle import oracle
    c = bench.cfg
    prob = pin.Problem(n=c["n"], p=c["p"], k=c["k"], batch=sample_batch, layers=c["layers"], act=c["act"],
                       dtype=c["dtype"], rank=c["rank"], widths=c["widths"], ks=c["ks"])
    all_ranks = c["rank"] < 0
    data = pin.all_rank_step_inputs(prob, 0) if all_ranks else pin.one_rank_step_inputs(prob, 0)
    def once():
        if c["mode"] == "forward":
            oracle.ffn_forward(c["act"], data["X0"], data["layers"], c["dtype"], all_ranks)
        else:
            oracle.ffn_step(c["act"], data["X0"], data["T"], data["layers"], c["lr"], c["dtype"], all_ranks)

    # at least 10 s of oracle work (or 20 passes), so that the figure is not a start-up artefact
    t0 = time.perf_counter()
    reps = 0
    while reps < 20 and (reps == 0 or time.perf_counter() - t0 < 10.0):
        once()
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    fl = flops_per_step(bench.shapes, c["p"], sample_batch, c["mode"], bench.groups)
    return {"value": fl / dt * 1e-12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": round(dt, 2), "passes": reps, "samples_per_s": sample_batch / dt,
            "sample": f"same workload with batch {sample_batch} of {c['batch']} (all layers, fp64), "
                      f"mean of {reps} passes ({dt * reps:.0f} s of host time)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4", choices=sorted(WORKLOADS))
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-vendor-reference", action="store_true", help="skip the torch.bmm timings of the bare products")
    ap.add_argument("--no-others", action="store_true", help="skip the other benchmark configurations (extra keys)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy: the dispatch of known size that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the other ranks of phantom parallelism are emulated "
              "as buffers on it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # what a plain device-to-device copy reaches on this machine (1 GiB read + 1 GiB written per pass): the measured
    # companion of the published HBM peak that the roofline below is priced against
    src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) * 1e-9
    del src, dst

    b = Bench(args.workload)
    c = b.cfg
    # exactly `steps` steps between device synchronisations, twice: as replays of one captured HIP graph and as eager
    # launches on the stream.  The same kernels run either way; the headline is the faster way of launching them
    # (dependent kernels of a graph replay start later after each other than the same kernels on a stream do here
    # when each runs for tens of microseconds; launch-bound workloads gain from the graph instead).
    ms_graph, how = b.time_steps(args.steps, args.warmup, graph=not args.no_graph)
    ms_eager, _ = b.time_steps(args.steps, 2, graph=False) if how == "hip_graph" else (ms_graph, how)
    ms = min(ms_graph, ms_eager)
    if ms_eager < ms_graph:
        how = "eager"
    tflops = b.flops / ms * 1e-9
    esize = 4 if c["dtype"] == "f32" else 2

    prof_steps = max(5, min(args.steps, 50))
    table, event_overhead_us = kernel_table(b.profile(prof_steps), prof_steps, esize)
    products = [r for r in table if "flops" in r]
    dom = max(products, key=lambda r: r["avg_us"] * r["launches_per_step"])
    ridge = MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if dom["flops"] / dom["bytes"] >= ridge or c["dtype"] == "f32":
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": dom["tflops"] / MFMA_PEAK_TFLOPS}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["gbs"] / HBM_PEAK_GBS}
    roof.update(traffic=measured_traffic(args.workload, dom), kernel=f"{dom['name']} M={dom['M']} N={dom['N']} K={dom['K']} x{dom['groups']}",
                avg_us=dom["avg_us"], launches_per_step=dom["launches_per_step"],
                flop_per_launch=dom["flops"], algorithmic_bytes_per_launch=dom["bytes"])

    out = {
        "metric": "phantom-layer fwd+bwd TFLOP/s and samples/s per GPU; % of bf16 MFMA peak",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_s": SETTLE_S,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if c["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: phantom FFN n={c['n']} p={c['p']} (shard {c['n'] // c['p']}) "
                               f"k={c['k']} batch={c['batch']} layers={c['layers']} {c['act']} "
                               f"{'all ranks emulated on the GPU' if c['rank'] < 0 else 'rank %d with seeded peer buffers' % c['rank']}, "
                               f"step = {c['mode']}",
                   "launch": how, "n": c["n"], "p": c["p"], "k": c["k"], "global_batch": c["batch"],
                   "layers": c["layers"], "activation": c["act"],
                   **({"widths": list(c["widths"]), "ks": list(c["ks"])} if c["widths"] else {})},
        "samples_per_s": c["batch"] / ms * 1e3,
        "ms_per_step_eager": ms_eager, "ms_per_step_hip_graph": ms_graph,
        "pct_mfma_peak": 100.0 * tflops / MFMA_PEAK_TFLOPS,
        "pct_hbm_peak": 100.0 * (b.bytes / ms * 1e-6) / HBM_PEAK_GBS,
        "algorithmic_flop_per_step": b.flops, "algorithmic_bytes_per_step": b.bytes,
        "roofline": roof,
        "empty_launch_us": round(event_overhead_us, 3),
        "measured_copy_gbs": round(copy_gbs, 1),
        "kernels": [{{"flops": "flop", "bytes": "algorithmic_bytes"}.get(k_, k_): v for k_, v in r.items()} for r in table],
    }

    if not args.no_dense:
        # the dense network of equal width and depth (p = 1: n x n weight blocks) through the same kernels ...
        d = Bench((c["n"], 1, 0, c["batch"], c["layers"], c["act"], c["dtype"], 0, c["mode"], c["lr"],
                   c["widths"], ()), seeded=False)
        dms, dhow = d.time_steps(max(5, args.steps // 4), 2, graph=not args.no_graph)
        out["dense_equal_width"] = {"ms_per_step": dms, "tflops": d.flops / dms * 1e-9, "launch": dhow,
                                    "flop_per_step": d.flops, "phantom_speedup": dms / ms,
                                    "what": f"{c['layers']} dense layers {c['n']} x {c['n']}, batch {c['batch']}, step = {c['mode']}"}
        del d
        torch.cuda.empty_cache()
        # ... and one rank's share of that network under tensor parallelism: an [n/p, n] block of every layer
        # applied to the full-width activation (one layer timed, times the depth)
        if c["p"] > 1 and not c["widths"]:
            t = Bench((c["n"], 1, 0, c["batch"], 1, c["act"], c["dtype"], 0, c["mode"], c["lr"],
                       (c["n"], c["n"] // c["p"]), ()), seeded=False)
            tms, thow = t.time_steps(max(10, args.steps // 2), 3, graph=not args.no_graph)
            out["dense_tensor_parallel_share"] = {
                "ms_per_layer": tms, "ms_per_step": tms * c["layers"], "tflops": t.flops / tms * 1e-9, "launch": thow,
                "flop_per_layer": t.flops, "phantom_speedup": tms * c["layers"] / ms,
                "what": f"one layer [{c['n'] // c['p']} x {c['n']}] on batch {c['batch']}, step = {c['mode']}, x {c['layers']} layers"}
            del t
            torch.cuda.empty_cache()
    if not args.no_vendor_reference:
        out["vendor_gemm_reference"] = vendor_gemm_reference(c, b.shapes, b.groups)
    if not args.no_others:
        # the other benchmark configurations, same measurement (HIP graph replays between device syncs), inputs of
        # the same shapes and distributions drawn on the GPU
        others = {}
        for name in ("c2", "c3", "c5k4", "c5k16", "c5k64", "c5k256"):
            if name == args.workload:
                continue
            o = Bench(name, seeded=False)
            oms, ohow = o.time_steps(max(20, args.steps), 5, graph=not args.no_graph)
            if ohow == "hip_graph":
                oeager, _ = o.time_steps(max(20, args.steps), 2, graph=False)
                if oeager < oms:
                    oms, ohow = oeager, "eager"
            oc = o.cfg
            others[name] = {"ms_per_step": oms, "tflops": o.flops / oms * 1e-9, "pct_mfma_peak": 100.0 * o.flops / oms * 1e-9 / MFMA_PEAK_TFLOPS,
                            "pct_hbm_peak": 100.0 * (o.bytes / oms * 1e-6) / HBM_PEAK_GBS,
                            "samples_per_s": oc["batch"] / oms * 1e3, "launch": ohow,
                            "what": f"n={oc['n']} p={oc['p']} k={oc['k']} batch={oc['batch']} layers={oc['layers']} {oc['act']} "
                                    f"{'all ranks' if oc['rank'] < 0 else 'rank 0'} step={oc['mode']}"}
            del o
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    if not args.no_cpu_baseline:
        sample = args.cpu_sample_batch or max(1, min(c["batch"], int(1.0e11 / (b.flops / c["batch"]))))
        out["cpu_baseline"] = cpu_baseline(b, sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
