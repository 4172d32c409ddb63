#!/usr/bin/env python3
"""Decode-step benchmark of the fused dictionary-decode + dequantize + GEMV path on one MI355X.

A step = every matrix-vector product of one LLaMA-3.2-3B token step (28 layers x q,k,v,o,gate,up,down + lm_head,
197 matrices, each with its own seeded activation), weights resident in HBM in compressed form.
Prints one JSON line: compressed-weight HBM GB/s (value), tokens/s, roofline of the matvec kernel (batch 1), of the
batched kernel (batch 8), the stress configuration (Student-t weights, batch 16, whole-model expansion), the same sweep
with one dictionary per matrix, and the CPU oracle timed on a sample of the same workload, against which the timed
outputs are then checked.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM traffic of the default workload's launches measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain
# 1 GiB copy in the same run; profiles/k_matvec_config4_batch1_hbm_traffic.txt): bytes read per stored byte of the
# launch, bytes written per step.  The figures belong to the kernel sources whose digest is given; with other sources
# `traffic` is reported as null rather than as a stale number.
PROFILED_TRAFFIC = {
    "csrc_sha16": "cd3cf3bfc8810c9d",
    # kernel: (bytes read per stored byte of the launch, bytes written per step: a number, or "weights" = one per weight)
    "tq::k_matvec": (1.0030, 3_620_000),                 # batch 1
    "tq::k_matvec_ring": (1.0115, 316_580_000),          # batch 8: y is 28.9 MB; partial sums go out once per quad
    "tq::k_decompress": (1.0000, "weights"),
}


def csrc_digest() -> str:
    d = os.path.join(ROOT, "paper_2509_22951_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(os.listdir(d)):
        if f.endswith((".h", ".hip", ".cpp")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100, help="untimed steps right before the timed ones")
    ap.add_argument("--prewarm-ms", type=float, default=150.0,
                    help="before the counted warm-up: the same launches repeated, uncounted, for at least this long, so that the "
                         "GPU has reached its sustained clocks whatever --warmup is (a step takes under a millisecond; the "
                         "clocks need tens of milliseconds of load)")
    ap.add_argument("--config", type=int, default=4, help="workload: config 4 = LLaMA-3.2-3B decode-step sweep")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--also-batch", type=int, default=8, help="second batch size reported under 'other_batches' (0 = none)")
    ap.add_argument("--threads", type=int, default=min(16, os.cpu_count() or 1), help="host threads for setup")
    ap.add_argument("--max-entries", type=int, default=0)
    ap.add_argument("--lmax", type=int, default=0)
    ap.add_argument("--seg-cols", type=int, default=0, help="columns per segment (0 = library default)")
    ap.add_argument("--dictionary", choices=["sequence", "matrix"], default="sequence",
                    help="sequence: one LZW dictionary runs over the matrices in sweep order and freezes when full "
                         "(the table of paper section 4 is built over all parameters); matrix: every matrix starts from the 256 singles")
    ap.add_argument("--dictionary-kind", choices=["lzw", "frequency"], default="lzw",
                    help="lzw: LZW growth with freeze (the paper's Background, the headline configuration); frequency: the "
                         "first matrix of a sequence (every matrix with --dictionary matrix) fixes the dictionary as its "
                         "most frequent byte pairs, the way the paper's section 4 picks table entries")
    ap.add_argument("--bits", type=int, default=8, choices=range(2, 9),
                    help="quantization width (paper section 3 tried 8, 6, 4, 2 and ternary); the headline is 8")
    ap.add_argument("--pack", action="store_true",
                    help="with --bits 2..4: two values per stored byte (a code then stands for up to four weights)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle (then nothing is verified either)")
    ap.add_argument("--cpu-sample-layers", type=int, default=8,
                    help="layers of the sweep the CPU oracle is timed on (8 layers = 56 matrices take about 10 s on one core)")
    ap.add_argument("--no-decompress", action="store_true", help="skip the tq_decompress pass over all matrices")
    ap.add_argument("--no-gate-up", action="store_true",
                    help="skip the leg that runs the gate/up pairs of the workload as fused silu(gate) * up products")
    ap.add_argument("--no-listing", action="store_true",
                    help="skip the leg that expands one matrix stored in the paper's own section 4 stream format")
    ap.add_argument("--no-config5", action="store_true",
                    help="skip the stress configuration (config 5: Student-t weights, batch 16, whole-model expansion)")
    ap.add_argument("--no-dependent-stages", action="store_true",
                    help="skip the side leg that runs the default sweep in dependent stages (one persistent launch, and one launch per stage)")
    ap.add_argument("--no-matrix-dictionary", action="store_true",
                    help="skip the leg that repeats the sweep with one dictionary per matrix")
    ap.add_argument("--layers", type=int, default=0, help="debug: keep only the first N layers (+ lm_head)")
    ap.add_argument("--fuse", choices=["none", "independent", "staged", "layer", "sweep"], default="sweep",
                    help="how the products of a step are grouped into launches.  sweep: the step is a list of independent "
                         "products (each has its own activation vector), so all of them go to tq_matvec_multi at once; "
                         "layer: one tq_matvec_multi per transformer layer; independent: only products that a real layer "
                         "computes from the same input (q,k,v and gate,up) share a launch; staged: the same grouping as one "
                         "staged step (tq_step_create_staged: one kernel launch, device-side hand-over between the groups); "
                         "none: one tq_matvec per matrix")
    ap.add_argument("--no-prepared-step", action="store_true",
                    help="launch through tq_matvec_multi (at most 128 matrices per kernel launch) instead of a prepared tq_step")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and replay it (takes the host's launch cost out of plans with many launches)")
    ap.add_argument("--copies", type=int, default=0,
                    help="copies of the compressed matrices in device memory that the steps rotate over, so that a workload "
                         "smaller than the caches is still read from HBM (0 = as many as make 512 MB; 1 = none, cache-resident)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, so a counter profile of this command holds a kernel of "
                         "known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


class Workload:
    """The matrices of one configuration, encoded and resident in device memory, with the byte counts of their containers."""

    def __init__(self, tq, specs, args, dictionary, opts, keep_names=(), keep_all=False):
        from inputs import make_weights
        self.specs = specs
        self.kept = {}          # index -> container bytes, for the matrices the CPU oracle will decode
        self.blobs = {}         # every container (small workloads only: further copies are made from them)
        mats = [None] * len(specs)
        workers = max(1, min(args.threads, 8))
        inner = max(1, args.threads // workers)
        opts = dict(opts)
        # One LZW dictionary over the sequence: the matrices are encoded one after the other, each starting from the
        # dictionary the previous one ended with, until the dictionary is full (Gaussian weights fill it inside the first
        # matrix) or the first layer is through; from then on it is frozen at the size it has reached, so the remaining
        # matrices no longer depend on each other and are encoded in parallel.
        cap = args.max_entries or tq.TQ_MAX_ENTRIES_DEVICE
        prev, n_chain = None, 0

        def keep(i, blob):
            if specs[i].name in keep_names:
                self.kept[i] = blob
            if keep_all:
                self.blobs[i] = blob

        while n_chain < min(7, len(specs)):
            i = n_chain
            blob = tq.tq_encode(make_weights(specs[i]), n_threads=args.threads,
                                dict_from=prev if dictionary == "sequence" else None, **opts)
            mats[i] = tq.Matrix(blob)
            keep(i, blob)
            prev = blob
            n_chain += 1
            if dictionary != "sequence" or mats[i].info["n_entries"] == cap:
                break
        if dictionary == "sequence":
            opts["max_entries"] = mats[n_chain - 1].info["n_entries"]
        rest = sorted(range(n_chain, len(specs)), key=lambda i: -specs[i].rows * specs[i].cols)

        def encode(i):
            return i, tq.tq_encode(make_weights(specs[i]), n_threads=inner,
                                   dict_from=prev if dictionary == "sequence" else None, **opts)

        with ThreadPoolExecutor(workers) as ex:
            for i, blob in ex.map(encode, rest):
                mats[i] = tq.Matrix(blob)                   # validates, uploads, frees nothing on the hot path later
                keep(i, blob)
        self.mats, self.opts, self.prev, self.dictionary = mats, opts, prev, dictionary
        self.infos = infos = [m.info for m in mats]
        # Bytes the kernels must read from HBM: code stream, unit offsets and scales of every matrix, and every distinct
        # dictionary once (matrices encoded as one sequence hold the same dictionary; the library stores one copy).
        # The matrices of a chain hold growing dictionaries, all later ones the last of them.
        dict_bytes = sum(i["dict_bytes"] for i in (infos[:n_chain] if dictionary == "sequence" else infos))
        self.stored_bytes = sum(i["compressed_bytes"] - i["dict_bytes"] for i in infos) + dict_bytes
        self.n_codes = sum(i["n_codes"] for i in infos)
        self.n_real_codes = sum(i["n_real_codes"] for i in infos)
        # The method's own bytes: the codes of the parse (the padding codes that even out the 64 lane streams of a unit
        # are this layout's overhead, not the method's), unit offsets, scales, dictionaries.
        self.algorithmic_bytes = self.stored_bytes - 2 * (self.n_codes - self.n_real_codes)
        self.n_weights = sum(s.rows * s.cols for s in specs)

    def close(self):
        for m in self.mats:
            m.close()
        self.mats = []


def launch_groups(specs, fuse):
    """Launch plan: consecutive matrices that a transformer layer computes from the same input are independent."""
    groups, cur = [], []
    for i, s in enumerate(specs):
        kind = s.name.split(".")[-1]
        joins = bool(cur) and (
            fuse == "sweep" or
            (fuse == "layer" and s.name.split(".")[0] == specs[cur[-1]].name.split(".")[0]) or
            (fuse == "independent" and (
                (kind in ("k_proj", "v_proj") and specs[cur[-1]].name.split(".")[-1] in ("q_proj", "k_proj")) or
                (kind == "up_proj" and specs[cur[-1]].name.split(".")[-1] == "gate_proj"))))
        if joins:
            cur.append(i)
        else:
            if cur:
                groups.append(cur)
            cur = [i]
    groups.append(cur)
    return groups


def timed_block(step, steps, warmup, prewarm_ms, torch, spread_steps=100):
    """prewarm (uncounted, by wall time) -> warmup steps -> `steps` steps timed as one block, by wall clock and by HIP events
    on the launch stream -> the same steps once more with an event between every two (median / min / max)."""
    t0 = time.perf_counter()
    n_pre = 0
    while (time.perf_counter() - t0) * 1e3 < prewarm_ms:
        for _ in range(10):
            step()
        n_pre += 10
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = e0.elapsed_time(e1) / steps
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(min(steps, spread_steps) + 1)]
    marks[0].record()
    for e in marks[1:]:
        step()
        e.record()
    torch.cuda.synchronize()
    each = sorted(a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:]))
    spread = {"median": round(each[len(each) // 2], 4), "min": round(each[0], 4), "max": round(each[-1], 4), "n": len(each)}
    return wall_ms, ev_ms, spread, n_pre


def roofline_block(kernel, wl, ev_ms, n_launches, traffic=None, extra_bytes=0, note=None):
    """achieved = algorithmic bytes per launch / mean launch duration (HIP events on the launch stream around the timed
    steps, launches back to back).  extra_bytes: algorithmic bytes written (the expansion writes the matrix)."""
    alg = wl.algorithmic_bytes + extra_bytes
    ach = alg / ev_ms / 1e6
    return {
        "bound": "hbm", "kernel": kernel,
        "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
        "traffic": traffic,
        "algorithmic_bytes_per_launch": round(alg / n_launches),
        "stored_bytes_per_launch": round((wl.stored_bytes + extra_bytes) / n_launches),
        "padding_frac": round(1 - wl.n_real_codes / wl.n_codes, 4),
        "frac_on_stored_bytes": round((wl.stored_bytes + extra_bytes) / ev_ms / 1e6 / HBM_PEAK_GBS, 4),
        "launch_us": round(ev_ms * 1e3 / n_launches, 1),
        "note": note or "achieved = algorithmic bytes per launch (codes of the parse without the layout's padding codes, unit "
                        "offsets, scales, each distinct dictionary once) / mean launch duration from HIP events on the launch "
                        "stream; traffic = HBM bytes per launch from the FETCH_SIZE/WRITE_SIZE counter runs under profiles/ "
                        "(null off the profiled workload or when the kernel sources have changed since)",
    }


class Runner:
    """Times the products of a workload at one batch size in the launch plan the arguments ask for."""

    def __init__(self, tq, torch, wl, mat_sets, args, dev, stream):
        self.tq, self.torch, self.wl, self.mat_sets, self.args, self.dev, self.stream = tq, torch, wl, mat_sets, args, dev, stream
        self.groups = launch_groups(wl.specs, "independent" if args.fuse == "staged" else args.fuse)

    def make_io(self, batch):
        from inputs import make_activations
        xs, ys = [], []
        for s in self.wl.specs:
            bits, _ = make_activations(s, batch)
            xs.append(self.torch.from_numpy(bits.view(np.int16).copy()).to(self.dev))
            ys.append(self.torch.empty((batch, s.rows), dtype=self.torch.float32, device=self.dev))
        return xs, ys

    def run(self, batch, steps, warmup, prewarm_ms):
        tq, torch, args, stream = self.tq, self.torch, self.args, self.stream
        xs, ys = self.make_io(batch)
        extra = [0]   # kernel launches per step relative to tq_matvec_multi's

        def calls_for(ms, count):
            calls = []            # one per group; each takes the stream to launch on
            if args.fuse == "staged":   # every group a stage of one staged step
                order = [i for g in self.groups for i in g]
                st = tq.Step([ms[i].handle for i in order], [xs[i].data_ptr() for i in order], [ys[i].data_ptr() for i in order], batch,
                             stages=[k for k, g in enumerate(self.groups) for _ in g])
                if count:
                    extra[0] += st.info["n_launches"] - len(self.groups)
                return [lambda s, st=st: st.launch(s)]
            for g in self.groups:
                if len(g) == 1:   # one matrix: its description travels in the kernel arguments
                    m, xp, yp = ms[g[0]], xs[g[0]].data_ptr(), ys[g[0]].data_ptr()
                    calls.append(lambda s, m=m, xp=xp, yp=yp: m.matvec(xp, yp, batch, s))
                elif args.no_prepared_step:
                    mc = tq.MultiCall([ms[i].handle for i in g], [xs[i].data_ptr() for i in g],
                                      [ys[i].data_ptr() for i in g], batch)
                    calls.append(lambda s, mc=mc: mc.launch(s))
                else:   # the same products as a prepared step: buffers fixed, jobs in device memory, up to 896 matrices per launch
                    st = tq.Step([ms[i].handle for i in g], [xs[i].data_ptr() for i in g], [ys[i].data_ptr() for i in g], batch)
                    if count:
                        extra[0] += st.info["n_launches"] - (-(-len(g) // 128))
                    calls.append(lambda s, st=st: st.launch(s))
            return calls

        def stepper(calls):
            def eager_step():
                for c in calls:
                    c(stream)
            if not args.graph:
                return eager_step
            eager_step()
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                cap = torch.cuda.current_stream().cuda_stream
                for c in calls:      # the same calls, issued on the capturing stream
                    c(cap)
            return graph.replay

        steppers = [stepper(calls_for(ms, k == 0)) for k, ms in enumerate(self.mat_sets)]
        turn = [0]

        def step():   # copy after copy
            steppers[turn[0] % len(steppers)]()
            turn[0] += 1

        wall_ms, ev_ms, spread, n_pre = timed_block(step, steps, warmup, prewarm_ms, torch)
        # tq_matvec_multi serves up to 128 matrices per kernel launch; a prepared step may need fewer launches (or more,
        # where the matrices of a group go to different kernels)
        n_launches = sum(-(-len(g) // 128) for g in self.groups) + extra[0]
        return dict(wall_ms=wall_ms, ev_ms=ev_ms, spread=spread, prewarm_steps=n_pre, n_launches=n_launches, xs=xs, ys=ys)


def expansion_leg(tq, torch, wl, args, dev, stream, keep_output=False):
    """tq_decompress of every matrix of the workload into one device buffer, matrix after matrix."""
    out = torch.empty(wl.n_weights, dtype=torch.int8, device=dev)
    offs = np.cumsum([0] + [s.rows * s.cols for s in wl.specs])
    handles, ptrs = [m.handle for m in wl.mats], [out.data_ptr() + int(o) for o in offs[:-1]]
    dstep = None if args.no_prepared_step else tq.Step(handles, None, ptrs, decompress=True)

    def expand():
        if dstep is None:
            tq.tq_decompress_multi(handles, ptrs, stream)
        else:
            dstep.launch(stream)
    for _ in range(5):
        expand()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        expand()
    e1.record()
    torch.cuda.synchronize()
    d_ms = e0.elapsed_time(e1) / reps
    n_launches = -(-len(wl.mats) // 128) if dstep is None else dstep.info["n_launches"]
    res = {"ms_per_model": round(d_ms, 3), "kernel_launches": n_launches,
           "GBps_read_plus_write": round((wl.algorithmic_bytes + wl.n_weights) / d_ms / 1e6, 1),
           "GBps_written": round(wl.n_weights / d_ms / 1e6, 1),
           "roofline": roofline_block("tq::k_decompress", wl, d_ms, n_launches, extra_bytes=wl.n_weights,
                                      note="read + write: algorithmic bytes read (as for the product) plus one byte written per "
                                           "weight, per launch / mean launch duration from HIP events on the launch stream")}
    return res, (out, offs) if keep_output else None


def gate_up_leg(wl, args, dev, stream):
    """The gate/up pairs of the workload (up to 8 layers of them) as fused products: one container of interleaved rows
    per pair, silu(gate) * up in the kernel's epilogue, against the same pairs as two separate products each."""
    import torch

    import paper_2509_22951_amd as tq
    from inputs import make_activations, make_weights
    specs, mats = wl.specs, wl.mats
    pairs = [(i, i + 1) for i in range(len(specs) - 1)
             if specs[i].name.endswith("gate_proj") and specs[i + 1].name.endswith("up_proj")][:8]
    if not pairs:
        return None
    batch = args.batch
    prev = wl.prev if wl.dictionary == "sequence" else None
    fused = [tq.Matrix(tq.tq_encode_gate_up(make_weights(specs[g]), make_weights(specs[u]), n_threads=args.threads,
                                            dict_from=prev, **wl.opts)) for g, u in pairs]
    xs = [torch.from_numpy(make_activations(specs[g], batch)[0].view(np.int16).copy()).to(dev) for g, _ in pairs]
    ys = [torch.empty((batch, specs[g].rows), dtype=torch.float32, device=dev) for g, _ in pairs]
    y2 = [torch.empty((batch, specs[g].rows), dtype=torch.float32, device=dev) for g, _ in pairs]
    hs, xp, yp = [m.handle for m in fused], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
    sep = tq.MultiCall([mats[i].handle for p in pairs for i in p], [x.data_ptr() for x in xs for _ in (0, 1)],
                       [y.data_ptr() for pair in zip(ys, y2) for y in pair], batch)

    def timed(f, reps=100):
        for _ in range(100):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # the encoding above left the GPU idle: both forms are timed twice, alternating, and the better time counts
    t_fused = t_sep = float("inf")
    for _ in range(2):
        t_sep = min(t_sep, timed(lambda: sep.launch(stream)))
        t_fused = min(t_fused, timed(lambda: tq.tq_matvec_gate_up_multi(hs, xp, yp, batch, stream)))
    nbytes = sum(m.info["compressed_bytes"] - m.info["dict_bytes"] for m in fused)
    for m in fused:
        m.close()
    return {"pairs": len(pairs), "batch": batch, "weights": sum(2 * specs[g].rows * specs[g].cols for g, _ in pairs),
            "fused_ms": round(t_fused, 4), "two_products_ms": round(t_sep, 4),
            "fused_GBps": round(nbytes / t_fused / 1e6, 1)}


def listing_leg(specs, mats, dev, stream):
    """The paper's section 4 stream format, literally: table of the most frequent windows of 4 values over the first
    matrix of the workload, the largest of its first matrices compressed with it, expanded on the device.
    The quantized values come from the containers of the workload (tq_decompress); nothing of that is timed."""
    import torch

    import paper_2509_22951_amd as tq

    def quantized_bytes(i):
        out = torch.empty((specs[i].rows, specs[i].cols), dtype=torch.int8, device=dev)
        mats[i].decompress(out.data_ptr(), stream)
        torch.cuda.synchronize()
        return out.cpu().numpy().view(np.uint8).reshape(-1)

    first = specs[0]
    i_big = max(range(min(8, len(specs))), key=lambda i: specs[i].rows * specs[i].cols)
    big = specs[i_big]
    q_first = quantized_bytes(0)
    table = tq.tq_listing_build_table([q_first])
    values = quantized_bytes(i_big)
    words = tq.tq_listing_compress(values, table)
    h = tq.Listing(words, table)
    out = torch.empty(values.size, dtype=torch.uint8, device=dev)
    for _ in range(20):
        h.decompress(out.data_ptr(), stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 100
    e0.record()
    for _ in range(reps):
        h.decompress(out.data_ptr(), stream)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    ok = bool(torch.equal(out.cpu(), torch.from_numpy(values)))
    info = h.info
    h.close()
    moved = 2 * info["n_words"] + info["n_values"]
    return {"workload": f"{big.name} ({big.rows}x{big.cols}) in the paper's section 4 format, table from {first.name}",
            "values": info["n_values"], "words": info["n_words"], "table_entries": info["n_table"],
            "groups_in_table": round(1 - info["n_escapes"] / max(info["n_tokens"], 1), 4),
            "bytes_per_value": round(2 * info["n_words"] / max(info["n_values"], 1), 3),
            "us": round(us, 1), "GBps_read_plus_write": round(moved / us / 1e3, 1), "exact": ok}


def cpu_baseline_and_verification(wl, args, infos, timed_ys, expanded, torch):
    """The CPU oracle on a bounded sample of the workload (timed: sequential decode + float64 product, one thread, then
    the same sample over the host's threads), and, with the oracle's results in hand, the check of what the GPU was
    timed on: every row of the timed outputs of the sample matrices and of the other matrices kept for it (last layer,
    lm_head) against the oracle's float64 products, and the same matrices of the timed expansion against the oracle's
    decoded bytes, bit for bit.  For the first layer the oracle also quantizes the generated weights itself, so the
    whole chain weights -> container -> output is covered there."""
    from inputs import make_activations, make_weights
    from oracle import oracle as O
    specs = wl.specs
    sample = sorted(i for i in wl.kept if specs[i].name in {s.name for s in specs[:7 * args.cpu_sample_layers]})
    others = sorted(i for i in wl.kept if i not in sample)
    t0 = time.perf_counter()
    sb, refs = 0, {}
    for i in sample:
        _, x = make_activations(specs[i], args.batch)
        refs[i] = O.matvec_from_blob(wl.kept[i], x)                 # oracle: sequential decode, then float64 GEMV
        sb += infos[i]["compressed_bytes"]
    dt = time.perf_counter() - t0
    sw = sum(specs[i].rows * specs[i].cols for i in sample)
    out = {
        "value": round(sb / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {args.cpu_sample_layers} layers of the sweep ({len(sample)} matrices, {sw} weights, {dt:.2f} s): decode + "
                  f"float64 GEMV, batch {args.batch}; whole sweep extrapolates to {dt * wl.n_weights / sw:.1f} s/token",
        "tokens_per_s_extrapolated": round(args.batch / (dt * wl.n_weights / sw), 4),
    }
    # the same sample once more, the matrices (independent of each other) spread over the host's threads
    n_thr = max(1, min(args.threads, len(sample)))
    work = [(wl.kept[i], make_activations(specs[i], args.batch)[1]) for i in sample]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=n_thr) as pool:
        list(pool.map(lambda bx: O.matvec_from_blob(*bx), work))
    dt_all = time.perf_counter() - t0
    model = next((l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name")), "unknown")
    out["all_threads"] = {"value": round(sb / dt_all / 1e9, 3), "unit": "GB/s", "threads": n_thr,
                          "seconds": round(dt_all, 2), "os_cpu_count": os.cpu_count(), "cpu": model}

    # ---- verification of the timed buffers (not timed itself)
    decoded = {}

    def product_of(i):
        Q, s = O.decode_blob(wl.kept[i])
        decoded[i] = Q
        _, x = make_activations(specs[i], args.batch)
        rows = specs[i].rows
        cuts = [(a, min(rows, a + 8192)) for a in range(0, rows, 8192)]
        with ThreadPoolExecutor(max_workers=max(1, args.threads)) as pool:
            return np.concatenate(list(pool.map(lambda ab: O.gemv_f64(Q[ab[0]:ab[1]], s[ab[0]:ab[1]], x), cuts)), axis=1)

    for i in others:
        refs[i] = product_of(i)
    worst, rows_checked, ok = 0.0, 0, True
    for i, ref in refs.items():
        got = timed_ys[i].cpu().numpy().astype(np.float64)
        scale = np.abs(ref).max(axis=1, keepdims=True)
        err = float((np.abs(got - ref) / np.maximum(scale, 1e-300)).max()) if np.isfinite(got).all() else float("inf")
        worst = max(worst, err)
        ok = ok and err <= 1e-3
        rows_checked += ref.shape[1]
    verified = {"outputs": ok, "matrices": len(refs), "rows": rows_checked, "worst_rel_err": float(f"{worst:.3e}"),
                "tolerance": 1e-3, "against": "oracle decode of the container + float64 product, every row of the timed y buffers of "
                                              "the sample layers, the last layer and lm_head"}
    quant_ok = True
    for i in sorted(refs)[:7]:      # first layer: the oracle quantizes the generated weights itself
        if i not in decoded:
            decoded[i] = O.decode_blob(wl.kept[i])[0]
        Qo, _ = O.quantize_rows(make_weights(specs[i]), args.bits)
        quant_ok = quant_ok and np.array_equal(Qo, decoded[i])
    verified["first_layer_containers_hold_the_oracles_quantized_weights"] = bool(quant_ok)
    if expanded is not None:
        buf, offs = expanded
        exact = True
        for i in sorted(refs):
            if i not in decoded:
                decoded[i] = O.decode_blob(wl.kept[i])[0]
            dev_q = buf[int(offs[i]):int(offs[i + 1])].view(specs[i].rows, specs[i].cols)
            exact = exact and bool(torch.equal(dev_q, torch.from_numpy(decoded[i]).to(dev_q.device)))
        verified["expansion_bit_exact"] = exact
        ok = ok and exact
    verified["ok"] = bool(ok and quant_ok)
    return out, verified


def main():
    args = parse_args()
    if args.pack and args.bits > 4:
        sys.exit("--pack takes --bits 2..4")
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path is a single-GPU kernel; row- or column-parallel "
              "sharding over several GPUs is a design note, not built). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2509_22951_amd as tq
    from inputs import CONFIGS, config_matrices

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    tq.load()
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream

    def specs_of(config):
        specs = config_matrices(config)
        if args.layers:
            specs = [s for s in specs if s.name == "lm_head" or int(s.name[1:3]) < args.layers]
        return specs

    specs = specs_of(args.config)
    t_setup = time.time()
    # ---- encode (host, off the hot path): generate -> quantize -> dictionary-code, a few matrices at a time.
    # Kept for the CPU oracle: the first layers (its timed sample), the last layer and lm_head (verification only).
    keep_names = set() if args.no_cpu_baseline else ({s.name for s in specs[:7 * args.cpu_sample_layers]} | {s.name for s in specs[-8:]})
    opts = dict(max_entries=args.max_entries, lmax=args.lmax, seg_cols=args.seg_cols, dictionary=args.dictionary_kind,
                bits=0 if args.bits == 8 else args.bits, pack=args.pack)
    small = sum(s.rows * s.cols for s in specs) < 400_000_000 and args.copies != 1   # small workload: further copies are made below
    wl = Workload(tq, specs, args, args.dictionary, opts, keep_names, keep_all=small)
    infos = wl.infos

    # Cold-cache protocol: a workload that fits the caches is held in several copies and step k reads copy k mod N.
    n_copies = args.copies if args.copies > 0 else (-(-512_000_000 // wl.stored_bytes) if small else 1)
    if not small:
        n_copies = 1
    mat_sets = [wl.mats] + [[tq.Matrix(wl.blobs[i]) for i in range(len(specs))] for _ in range(n_copies - 1)]
    wl.blobs.clear()
    setup_s = time.time() - t_setup

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    runner = Runner(tq, torch, wl, mat_sets, args, dev, stream)
    main_run = runner.run(args.batch, args.steps, args.warmup, args.prewarm_ms)
    wall_ms, ev_ms, n_launches = main_run["wall_ms"], main_run["ev_ms"], main_run["n_launches"]

    def kernel_name(batch, packed=False):
        return "tq::k_matvec" if batch <= 2 else "tq::k_matvec_ring"

    default_workload = (args.config == 4 and args.batch == 1 and args.fuse == "sweep" and args.dictionary == "sequence"
                        and args.dictionary_kind == "lzw" and args.bits == 8 and not args.pack and not args.no_prepared_step
                        and not (args.max_entries or args.lmax or args.seg_cols or args.layers or args.copies))
    digest_matches = PROFILED_TRAFFIC["csrc_sha16"] == csrc_digest()

    def profiled_traffic(kernel, n_launches, batch=1):
        """HBM bytes per launch as the counter runs under profiles/ measured them, for the workload they were taken on."""
        if not (default_workload and digest_matches) or (kernel == "tq::k_matvec_ring" and batch != 8):
            return None
        per_stored, written = PROFILED_TRAFFIC[kernel]
        return round((per_stored * wl.stored_bytes + (wl.n_weights if written == "weights" else written)) / n_launches)

    others = {}
    if args.also_batch and args.also_batch != args.batch:
        r2 = runner.run(args.also_batch, max(3, args.steps // 2), args.warmup, args.prewarm_ms)
        others[str(args.also_batch)] = {
            "ms_per_step": round(r2["wall_ms"], 4), "GBps": round(wl.algorithmic_bytes / r2["wall_ms"] / 1e6, 1),
            "tokens_per_s": round(args.also_batch / (r2["wall_ms"] * 1e-3), 1), "step_ms": r2["spread"],
            "roofline": roofline_block(kernel_name(args.also_batch), wl, r2["ev_ms"], r2["n_launches"],
                                       profiled_traffic(kernel_name(args.also_batch), r2["n_launches"], args.also_batch))}
        del r2

    decompress, expanded = None, None
    if not args.no_decompress:
        decompress, expanded = expansion_leg(tq, torch, wl, args, dev, stream, keep_output=not args.no_cpu_baseline)
        decompress["roofline"]["traffic"] = profiled_traffic("tq::k_decompress", decompress["kernel_launches"])

    listing = None
    if not args.no_listing:
        listing = listing_leg(specs, wl.mats, dev, stream)
    gate_up = None
    if not args.no_gate_up:
        gate_up = gate_up_leg(wl, args, dev, stream)

    traffic = profiled_traffic("tq::k_matvec", n_launches)
    gbps = wl.algorithmic_bytes / wall_ms / 1e6
    result = {
        "metric": "compressed-weight HBM GB/s of the fused decode+dequant+GEMV decode-step sweep (% of 8 TB/s peak in "
                  "roofline.frac; tokens/s alongside)",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": f"bf16 activations x {'int8' if args.bits == 8 else str(args.bits) + '-bit'} weights, fp32 accumulate",
        "data": "synthetic",
        "tokens_per_s": round(args.batch / (wall_ms * 1e-3), 1),
        "step_ms": main_run["spread"],   # one event pair per step, in a pass of its own after the timed region
        "config": {
            "workload": f"config {args.config}: {CONFIGS[args.config]['desc']}, batch {args.batch}",
            "matrices": len(specs), "weights": wl.n_weights,
            "value_counts": "algorithmic bytes: the codes of the parse, unit offsets, scales, each distinct dictionary once "
                            "(the padding codes of the layout are left out; stored_bytes includes them)",
            "algorithmic_bytes": wl.algorithmic_bytes, "stored_bytes": wl.stored_bytes,
            "raw_int8_bytes": wl.n_weights, "stored_over_raw_int8": round(wl.stored_bytes / wl.n_weights, 4),
            "bytes_per_weight": round(wl.algorithmic_bytes / wl.n_weights, 4),
            "stored_bytes_per_weight": round(wl.stored_bytes / wl.n_weights, 4),
            "weights_per_code": round(wl.n_weights / wl.n_codes, 4),
            "weights_per_real_code": round(wl.n_weights / wl.n_real_codes, 4),
            "padding_frac": round(1 - wl.n_real_codes / wl.n_codes, 4),
            "GBps_on_stored_bytes": round(wl.stored_bytes / wall_ms / 1e6, 1),
            "dictionary_entries": infos[-1]["n_entries"], "lmax": infos[0]["lmax"], "seg_cols": infos[0]["seg_cols"],
            "dictionary": args.dictionary, "dictionary_kind": args.dictionary_kind, "bits": args.bits,
            "packing": "nibbles" if args.pack else "none", "fuse": args.fuse, "prepared_step": not args.no_prepared_step,
            "kernel_launches_per_step": n_launches,
            "hip_graph": bool(args.graph),
            "prewarm_ms": args.prewarm_ms, "prewarm_steps": main_run["prewarm_steps"],
            "cache": (f"cold: the steps rotate over {n_copies} copies of the compressed matrices ({n_copies * wl.stored_bytes / 1e6:.0f} MB)" if n_copies > 1
                      else "cold: one step streams more than the caches hold" if wl.stored_bytes >= 512_000_000
                      else "cache-resident: the same compressed bytes are read again every step"),
            # activations read and outputs written per step: beside the compressed bytes, not part of `value`
            "x_bytes_per_step": sum(2 * args.batch * s.cols for s in specs),
            "y_bytes_per_step": sum(4 * args.batch * s.rows for s in specs),
        },
        "roofline": roofline_block(kernel_name(args.batch), wl, ev_ms, n_launches, traffic),
        "other_batches": others,
        "decompress": decompress,
        "gate_up_fused": gate_up,
        "listing_format": listing,
        "setup_s": round(setup_s, 1),
        "paper_context": "context only, no target: the paper times whole evaluation questions end to end (section 5, Tables 2-4; "
                         "Xeon Gold 6130 + Tesla V100-SXM2 32 GB, compressed path on the CPU): LLaMA-3.2-3B at 8 bits 0.56-1.29 s per "
                         "question compressed against 0.20-0.33 s uncompressed; it reports no throughput of this path",
    }

    # ---- the same sweep with a real layer's dependencies respected: q,k,v | o | gate,up | down per layer, then lm_head
    def dependent_stages_leg():
        import copy
        out = {"plan": "the products that a layer can run side by side form a stage; a stage starts when the one before it has "
                       "stored its outputs"}
        for fuse, key in (("staged", "one_persistent_launch"), ("independent", "one_launch_per_stage")):
            a2 = copy.copy(args)
            a2.fuse, a2.graph = fuse, False
            r = Runner(tq, torch, wl, mat_sets[:1], a2, dev, stream)
            rr = r.run(args.batch, max(3, args.steps // 2), max(2, args.warmup // 2), min(args.prewarm_ms, 50.0))
            out["stages"] = len(r.groups)
            out[key] = {"ms_per_step": round(rr["wall_ms"], 4), "tokens_per_s": round(args.batch / (rr["wall_ms"] * 1e-3), 1),
                        "GBps": round(wl.algorithmic_bytes / rr["wall_ms"] / 1e6, 1),
                        "frac": round(wl.algorithmic_bytes / rr["wall_ms"] / 1e6 / HBM_PEAK_GBS, 4),
                        "kernel_launches_per_step": rr["n_launches"], "step_ms": rr["spread"]}
            del rr, r
        return out

    def optional_leg(name, fn):   # a failure in a side leg is reported in the line instead of losing the line
        try:
            result[name] = fn()
        except Exception as e:   # noqa: BLE001
            result[name] = {"error": f"{type(e).__name__}: {e}"}

    if default_workload and not args.no_dependent_stages:
        optional_leg("dependent_stages", dependent_stages_leg)

    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["verified"] = cpu_baseline_and_verification(wl, args, infos, main_run["ys"], expanded, torch)
    else:
        result["verified"] = None
    del expanded, main_run
    for ms in mat_sets:
        for m in ms:
            m.close()
    wl.mats = []
    torch.cuda.empty_cache()

    # ---- the same sweep with one dictionary per matrix (what "built greedily from the matrix" says literally)
    def matrix_dictionary_leg():
        wm = Workload(tq, specs, args, "matrix", opts)
        rm = Runner(tq, torch, wm, [wm.mats], args, dev, stream).run(args.batch, args.steps, args.warmup, args.prewarm_ms)
        out = {
            "dictionary": "matrix", "ms_per_step": round(rm["wall_ms"], 4), "tokens_per_s": round(args.batch / (rm["wall_ms"] * 1e-3), 1),
            "GBps": round(wm.algorithmic_bytes / rm["wall_ms"] / 1e6, 1), "bytes_per_weight": round(wm.algorithmic_bytes / wm.n_weights, 4),
            "step_ms": rm["spread"], "roofline": roofline_block(kernel_name(args.batch), wm, rm["ev_ms"], rm["n_launches"])}
        del rm
        wm.close()
        torch.cuda.empty_cache()
        return out

    if default_workload and not args.no_matrix_dictionary:
        optional_leg("dictionary_per_matrix", matrix_dictionary_leg)

    # ---- the stress configuration: config 5 (Student-t weights), batch 16, and the expansion of the whole model
    def config5_leg():
        s5 = specs_of(5)
        w5 = Workload(tq, s5, args, "sequence", opts)
        r5 = Runner(tq, torch, w5, [w5.mats], args, dev, stream).run(16, max(3, args.steps // 2), args.warmup, args.prewarm_ms)
        d5, _ = expansion_leg(tq, torch, w5, args, dev, stream)
        out = {
            "workload": f"config 5: {CONFIGS[5]['desc']}, batch 16", "ms_per_step": round(r5["wall_ms"], 4),
            "tokens_per_s": round(16 / (r5["wall_ms"] * 1e-3), 1), "GBps": round(w5.algorithmic_bytes / r5["wall_ms"] / 1e6, 1),
            "bytes_per_weight": round(w5.algorithmic_bytes / w5.n_weights, 4), "stored_bytes_per_weight": round(w5.stored_bytes / w5.n_weights, 4),
            "weights_per_real_code": round(w5.n_weights / w5.n_real_codes, 4), "dictionary_entries": w5.infos[-1]["n_entries"],
            "lmax": w5.infos[0]["lmax"], "step_ms": r5["spread"],
            "roofline": roofline_block(kernel_name(16), w5, r5["ev_ms"], r5["n_launches"]), "decompress": d5}
        del r5
        w5.close()
        return out

    if default_workload and not args.no_config5:
        optional_leg("config5", config5_leg)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
