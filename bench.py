#!/usr/bin/env python3
"""Benchmark of the paged decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3] [--kernel auto]

A step is one decode iteration of the attention executor over every resident
layer: per layer adr_decode_step = the append of the new token, the partition
pass and the log-sum-exp merge (--separate-append: adr_kv_append, then
adr_decode_attention).  Sequences grow by one token per step.
Prints ONE JSON line: whole-job attended-KV bandwidth (algorithmic bytes of K
and V attended per second, inputs resident in HBM), the roofline of the
dominant kernel from HIP events on the launch stream, the fp64 oracle timed
on the host cores as a baseline, and (object "corun") the same attention steps
next to a compute-bound neighbour: a bf16 8192^3 matrix product on a second
stream, with the compute units shared freely and split by queue masks, for the
matrix-core kernel and for the vector-ALU kernel.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import tempfile
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2503_20552_amd as adr  # noqa: E402
import workloads as W  # noqa: E402

HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernel per launch, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this command (see profiles/), scaled by the same counters'
# reading on adr_probe_copy.  A profiler run cannot happen inside this script, so the
# figure is carried here together with the hash of the kernel sources it was taken
# with (`python bench.py --csrc-hash` prints the current one): with other sources the
# line reports traffic null rather than a stale number.
MEASURED_TRAFFIC_BYTES = {
    # (workload, kernel[, "fp8"]): (bytes per launch, hash of csrc/ at the time, summary under profiles/)
    (3, 'decode_stream_kernel'): (2344273634, '6766cd555ffaca53', 'profiles/decode_stream_kernel_workload3.md'),
    (5, 'decode_stream_kernel'): (10533352777, '6766cd555ffaca53', 'profiles/decode_stream_kernel_workloads2_5_bf16.md'),
    (2, 'decode_stream_kernel'): (1447104494, '6766cd555ffaca53', 'profiles/decode_stream_kernel_workloads2_5_bf16.md'),
    (5, 'decode_stream_kernel', 'fp8'): (5456117949, '6766cd555ffaca53', 'profiles/decode_stream_kernel_workload5_fp8.md'),
    (3, 'decode_stream_kernel', 'fp8'): (1214961475, '6766cd555ffaca53', 'profiles/decode_stream_kernel_workload5_fp8.md'),
    (4, 'decode_mfma_kernel'): (347841203, '6766cd555ffaca53', 'profiles/decode_mfma_kernel_workload4.md'),
}


def csrc_hash() -> str:
    """Hash of the library's kernel sources (what a traffic figure was measured with)."""
    d = os.path.join(ROOT, "paper_2503_20552_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def build_state(wl: W.Workload, layers: int, total_steps: int, fp8: bool = False, length_bound: int = 0):
    dev = "cuda:0"
    b = W.make_batch(wl, device=dev, headroom_tokens=total_steps + 1)

    def as_cache(k, v):
        if not fp8:
            return adr.KVCache(k, v)
        k8, ks = W.quantize_pool_fp8(k, b.used)      # host-style quantiser (library casts), on the device
        v8, vs = W.quantize_pool_fp8(v, b.used)
        return adr.KVCache(k8, v8, ks, vs)

    caches = [as_cache(b.k_cache, b.v_cache)]
    for i in range(1, layers):
        caches.append(as_cache(*W.layer_pools(wl, b, i, dev)))
    if fp8:
        b.k_cache = b.v_cache = None                 # the bf16 originals are not needed any more
        torch.cuda.empty_cache()
    # one grouped q|k|v buffer per step, as the executor receives it
    width = (wl.Hq + 2 * wl.Hkv) * wl.d
    qkv = W.randn_bf16((wl.B, width), wl.seed + 7, dev)
    q = qkv[:, :wl.Hq * wl.d].view(wl.B, wl.Hq, wl.d)
    k_new = qkv[:, wl.Hq * wl.d:(wl.Hq + wl.Hkv) * wl.d].view(wl.B, wl.Hkv, wl.d)
    v_new = qkv[:, (wl.Hq + wl.Hkv) * wl.d:].view(wl.B, wl.Hkv, wl.d)
    steps = np.arange(total_steps, dtype=np.int32)[:, None]
    positions = torch.as_tensor(b.lens_before[None, :] + steps).to(torch.int32).to(dev).contiguous()
    seq_lens = (positions + 1).contiguous()
    table = torch.as_tensor(b.block_table).to(dev)
    max_len = int(b.lens_before.max()) + total_steps
    if length_bound > max_len:
        # the bound a serving system knows (its context limit), not the batch's own maximum: the table is
        # padded to it, nothing else changes
        pages = -(-length_bound // wl.page_size)
        wide = torch.zeros((wl.B, pages), dtype=table.dtype, device=dev)
        wide[:, :table.shape[1]] = table
        table, max_len = wide, length_bound
    return dict(batch=b, caches=caches, q=q, k_new=k_new, v_new=v_new, positions=positions,
                seq_lens=seq_lens, table=table, max_len=max_len)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="resident layer caches (0 = the workload's)")
    ap.add_argument("--kernel", default="auto", choices=["auto", "valu", "mfma"])
    ap.add_argument("--partition", type=int, default=-1, help="partition tokens (-1 = the workload's)")
    ap.add_argument("--cache-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: caches quantised to e4m3 bytes with one fp32 scale per (page, kv-head)")
    ap.add_argument("--separate-append", action="store_true",
                    help="adr_kv_append then adr_decode_attention per layer instead of one adr_decode_step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-corun", action="store_true", help="leave the colocation object out of the line")
    ap.add_argument("--corun-steps", type=int, default=3, help="attention steps per colocation measurement")
    ap.add_argument("--csrc-hash", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--corun-gemm", action="store_true",
                    help="colocation measurement: the attention steps on one stream while bf16 8192^3 matrix "
                         "products run on another; prints its own JSON line (alone and contended rates)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (all layers: append, attention, merge) into a HIP graph and replay "
                         "it; prints its own JSON line with eager and replayed times and the CPU time spent "
                         "enqueueing a step either way")
    ap.add_argument("--graph-table", action="store_true",
                    help="record the step for batch capacities on an interval grid (adr_graph_table_*) and replay "
                         "the smallest fit for several batch sizes; prints its own JSON line: per capacity the GPU "
                         "time of a step and the CPU time to enqueue it, eager and replayed, and what a table "
                         "recorded for a masked stream costs with and without ADR_GRID_CUS")
    ap.add_argument("--attention-cus", type=int, default=0,
                    help="with --corun-gemm: the attention on a stream masked to the first N compute units, the "
                         "matrix products on the others (0 = two plain streams)")
    ap.add_argument("--cu-sweep", action="store_true",
                    help="with --corun-gemm: repeat the measurement with the attention confined to 32, 64, ... "
                         "compute units and the matrix products to the others")
    ap.add_argument("--length-bound", type=int, default=0,
                    help="pass this bound on the lengths (max_seq_len) instead of the batch's own maximum, when it "
                         "is larger: what a serving system with a fixed context limit would pass")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also launch adr_probe_copy once on 1 GiB (calibrates profiler byte counters)")
    args = ap.parse_args()
    if args.csrc_hash:
        print(csrc_hash())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    adr.load_library()  # fails loudly when the HIP library is missing

    wl = W.WORKLOADS[args.workload]
    layers = args.layers or wl.layers
    part = wl.partition_tokens if args.partition < 0 else args.partition
    flags = {"auto": adr.KERNEL_AUTO, "valu": adr.KERNEL_VALU, "mfma": adr.KERNEL_MFMA}[args.kernel]
    K, Wm = args.steps, args.warmup
    total_steps = K + Wm

    t0 = time.time()
    fp8 = args.cache_dtype == "fp8"
    st = build_state(wl, layers, total_steps, fp8, args.length_bound)
    b = st["batch"]
    elem = 1 if fp8 else 2
    torch.cuda.synchronize()
    log("workload %d %s: B=%d Hq=%d Hkv=%d d=%d layers=%d partition=%d pool=%d pages (%.1f GB K+V resident) "
        "lengths %s; set-up %.1f s" % (wl.ident, wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, layers, part, b.num_pages,
                                      layers * 2 * st["caches"][0].k.numel() * elem / 1e9, W.describe_lengths(b.seq_lens),
                                      time.time() - t0))
    out = torch.empty((wl.B, wl.Hq, wl.d), dtype=torch.bfloat16, device="cuda:0")
    ws_bytes = adr.adr_decode_workspace_bytes(wl.B, wl.Hq, wl.d, st["max_len"], part)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda:0")
    # K and V of one token in one layer (+ an fp8 page's two scales per kv-head, shared by its 16 tokens)
    bytes_per_token = 2 * wl.Hkv * wl.d * elem + (2 * wl.Hkv * 4 / wl.page_size if fp8 else 0)

    def one_step(s, events=None, pos=None, seq=None, kernel_flags=None):
        if pos is None:
            pos, seq = st["positions"][s], st["seq_lens"][s]
        kf = flags if kernel_flags is None else kernel_flags
        for li, cache in enumerate(st["caches"]):
            if events is None and not args.separate_append:
                # append and attention in one call (the token index is seq - 1 = pos)
                adr.adr_decode_step(out, st["q"], st["k_new"], st["v_new"], cache, st["table"], seq, wl.scale,
                                    st["max_len"], part, ws, None, kf)
                continue
            adr.adr_kv_append(cache, st["k_new"], st["v_new"], st["table"], pos)
            if events is None:
                adr.adr_decode_attention(out, st["q"], cache, st["table"], seq, wl.scale, st["max_len"],
                                         part, ws, None, kf)
            else:   # the same three kernels in the same order, with events around the partition pass and the merge
                # (the workspace's control area is clear: every earlier call left it so, which saves the
                # attention call its clearing kernel, as the append does inside adr_decode_step)
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record()
                adr.adr_decode_attention(out, st["q"], cache, st["table"], seq, wl.scale, st["max_len"],
                                         part, ws, None, kf | adr.PARTIALS_ONLY | adr.WORKSPACE_READY)
                e1.record()
                adr.adr_decode_merge(out, seq, st["max_len"], part, ws)
                e2.record()
                events.append((e0, e1, e2))

    if args.probe_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        adr.adr_probe_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    if args.corun_gemm:
        return corun_gemm(args, wl, st, one_step, bytes_per_token, layers, part)
    if args.graph:
        return graph_replay(args, wl, st, one_step, out, bytes_per_token, layers, part)
    if args.graph_table:
        return graph_table(args, wl, st, out, ws, bytes_per_token, layers, part, flags)

    for s in range(Wm):
        one_step(s)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(Wm, Wm + K):
        one_step(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    tokens_per_step = [int(b.lens_before.sum()) + wl.B * (s + 1) for s in range(Wm, Wm + K)]
    attended_tokens = layers * sum(tokens_per_step)          # (token, layer) pairs attended
    kv_bytes = attended_tokens * bytes_per_token
    value = kv_bytes / elapsed / 1e9

    # the same K steps again, instrumented: HIP events on the launch stream around each pass
    events = []
    for s in range(Wm, Wm + K):
        one_step(s, events)
    torch.cuda.synchronize()
    attn_ms = np.array([e0.elapsed_time(e1) for e0, e1, _ in events])
    merge_ms = np.array([e1.elapsed_time(e2) for _, e1, e2 in events])
    bytes_per_launch = kv_bytes / (layers * K)
    achieved = bytes_per_launch / (attn_ms.mean() * 1e-3) / 1e9
    # the library says which kernel it runs for this shape
    kernel_name = adr.adr_kernel_name(adr.adr_decode_kernel_choice(st["caches"][0], wl.B, wl.Hq, st["max_len"],
                                                                   part, flags))
    traffic, traffic_source = None, None
    default_shape = layers == wl.layers and part == wl.partition_tokens and not args.length_bound
    entry = MEASURED_TRAFFIC_BYTES.get((wl.ident, kernel_name, "fp8") if fp8 else (wl.ident, kernel_name))
    if entry and default_shape and entry[1] == csrc_hash():
        traffic, traffic_source = entry[0], entry[2]
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": traffic_source,
                "avg_kernel_ms": round(float(attn_ms.mean()), 5),
                "median_kernel_ms": round(float(np.median(attn_ms)), 5), "launches": int(len(attn_ms)),
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "merge_avg_ms": round(float(merge_ms.mean()), 5)}
    log("partition pass %.4f ms avg (min %.4f, max %.4f), merge %.4f ms avg" % (
        attn_ms.mean(), attn_ms.min(), attn_ms.max(), merge_ms.mean()))

    corun = None
    if not args.no_corun and not fp8 and wl.d == 128:
        corun = corun_summary(args, wl, st, one_step, bytes_per_token, layers)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, st, Wm, bytes_per_token)

    line = {
        "metric": "decode_attention_attended_kv_bandwidth",
        "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.cache_dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d Hq=%d Hkv=%d d=%d page=%d %s cache, %d resident layers, partition %d + LSE "
                               "merge, lengths %s" % (wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, wl.page_size,
                                                      "fp8-e4m3" if fp8 else "bf16", layers, part, wl.lengths),
                   "kernel": args.kernel, "layers": layers, "partition_tokens": part,
                   "cache_dtype": args.cache_dtype, "max_seq_len": st["max_len"]},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "attended_tokens_per_s": round(attended_tokens / elapsed, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "corun": corun,
    }
    print(json.dumps(line), flush=True)
    return 0


class Neighbour:
    """The compute-bound neighbour of Sec. 3.3's colocation: bf16 n x n x n products, back to back."""

    def __init__(self, wl, n=8192, dev="cuda:0"):
        self.n = n
        self.a = W.randn_bf16((n, n), wl.seed + 50, dev)
        self.b = W.randn_bf16((n, n), wl.seed + 51, dev)
        self.c = torch.empty((n, n), dtype=torch.bfloat16, device=dev)
        self.flop = 2.0 * n ** 3

    def product(self):
        torch.matmul(self.a, self.b, out=self.c)

    def alone_ms(self, stream, reps=8):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            self.product()
            e0.record()
            for _ in range(reps):
                self.product()
            e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def tflops(self, ms):
        return round(self.flop / ms / 1e9, 1)


def side_by_side(attention_pass, attn_stream, nb, nb_stream, attn_alone_ms, gemm_alone_ms):
    """The attention pass on one stream while products run on the other from before its start to after
    its end.  Returns (attention ms, mean ms of the products that ran wholly inside the attention's
    window, how many those were)."""
    def ev():
        return torch.cuda.Event(enable_timing=True)
    # enough products to cover the attention pass even if it slows down fourfold
    n_gemm = max(4, int(math.ceil(4.0 * attn_alone_ms / gemm_alone_ms)) + 2)
    marks = [ev() for _ in range(n_gemm + 1)]
    c0, c1 = ev(), ev()
    with torch.cuda.stream(nb_stream):
        marks[0].record()
        for i in range(n_gemm):
            nb.product()
            marks[i + 1].record()
    with torch.cuda.stream(attn_stream):
        c0.record(); attention_pass(); c1.record()
    torch.cuda.synchronize()
    inside = [marks[i].elapsed_time(marks[i + 1]) for i in range(n_gemm)
              if c0.elapsed_time(marks[i]) >= 0 and marks[i + 1].elapsed_time(c1) >= 0]
    return c0.elapsed_time(c1), (float(np.mean(inside)) if inside else None), len(inside)


def corun_summary(args, wl, st, one_step, bytes_per_token, layers):
    """The colocation half of the target (Sec. 3.3), short enough for the default run: the attention
    steps alone and next to the neighbour, (i) on two plain streams and (ii) with the compute units
    split by queue masks, each for the matrix-core kernel the library picks and for the vector-ALU
    kernel (whose arithmetic does not compete for the matrix pipe the neighbour is using)."""
    b = st["batch"]
    Wm, K = args.warmup, args.corun_steps
    steps = list(range(Wm, Wm + min(K, args.steps)))
    tokens = [int(b.lens_before.sum()) + wl.B * (s + 1) for s in steps]
    kv_bytes = layers * sum(tokens) * bytes_per_token
    total_cus = torch.cuda.get_device_properties(0).multi_processor_count
    nb = Neighbour(wl)
    kernels = {"matrix_core": None}
    G = wl.Hq // wl.Hkv
    if G in (1, 2, 4, 8):
        kernels["vector_alu"] = adr.KERNEL_VALU

    def gbps(ms):
        return round(kv_bytes / ms / 1e6, 1)

    def measure(attn_stream, nb_stream):
        row = {}
        gemm_ms = nb.alone_ms(nb_stream)
        row["gemm_alone_TFLOPs"] = nb.tflops(gemm_ms)
        for name, kf in kernels.items():
            def attention_pass():
                for s in steps:
                    one_step(s, kernel_flags=kf)
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(attn_stream):
                attention_pass()                                     # warm-up on this stream
                a0.record(); attention_pass(); a1.record()
            torch.cuda.synchronize()
            alone_ms = a0.elapsed_time(a1)
            co_ms, gemm_co_ms, n_inside = side_by_side(attention_pass, attn_stream, nb, nb_stream, alone_ms, gemm_ms)
            row[name] = {"attention_alone_GBps": gbps(alone_ms), "attention_contended_GBps": gbps(co_ms),
                         "contended_pct_of_hbm_peak": round(100 * kv_bytes / co_ms / 1e6 / HBM_PEAK_GBS, 1),
                         "gemm_contended_TFLOPs": nb.tflops(gemm_co_ms) if gemm_co_ms else None,
                         "gemms_inside_attention_window": n_inside}
        return row

    for _ in range(3):
        nb.product()
    torch.cuda.synchronize()
    res = {"neighbour": "bf16 %d^3 torch.matmul on a second stream, back to back" % nb.n,
           "attention_steps_per_measurement": len(steps), "total_cus": total_cus}
    res["plain_streams"] = measure(torch.cuda.Stream(), torch.cuda.Stream())        # default priority, both
    res["cu_split"] = []
    for n_attn in (192, 224):
        if n_attn >= total_cus:
            continue
        ha = adr.adr_stream_create_cu_mask([i < n_attn for i in range(total_cus)])
        hb = adr.adr_stream_create_cu_mask([i >= n_attn for i in range(total_cus)])
        try:
            row = {"attention_cus": n_attn, "gemm_cus": total_cus - n_attn}
            row.update(measure(torch.cuda.ExternalStream(ha), torch.cuda.ExternalStream(hb)))
            res["cu_split"].append(row)
        finally:
            torch.cuda.synchronize()
            adr.adr_stream_destroy(ha)
            adr.adr_stream_destroy(hb)
        log("corun split %s" % json.dumps(row))
    log("corun plain streams %s" % json.dumps(res["plain_streams"]))
    return res


def corun_gemm(args, wl, st, one_step, bytes_per_token, layers, part):
    """Attention and a compute-bound neighbour sharing the GPU (the paper's colocation of the
    attention executor with prefill, Sec. 3.3): stream A runs the K timed steps, stream B runs
    bf16 8192 x 8192 x 8192 products back to back.  Each is timed alone and then together; the
    contended figures count only work that overlapped the other stream's activity.
    --attention-cus N confines the attention to N compute units and the products to the rest."""
    K, Wm = args.steps, args.warmup
    b = st["batch"]
    if args.cu_sweep:
        return cu_sweep(args, wl, st, one_step, bytes_per_token, layers, part)
    total_cus = torch.cuda.get_device_properties(0).multi_processor_count
    nb = Neighbour(wl)
    tokens = [int(b.lens_before.sum()) + wl.B * (s + 1) for s in range(Wm, Wm + K)]
    kv_bytes = layers * sum(tokens) * bytes_per_token
    handles = []
    if args.attention_cus:
        n_attn = args.attention_cus
        handles = [adr.adr_stream_create_cu_mask([i < n_attn for i in range(total_cus)]),
                   adr.adr_stream_create_cu_mask([i >= n_attn for i in range(total_cus)])]
        sa, sb = (torch.cuda.ExternalStream(h) for h in handles)
    else:
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()      # default priority, both

    def attention_pass():
        for s in range(Wm, Wm + K):
            one_step(s)

    for _ in range(3):
        nb.product()
    with torch.cuda.stream(sa):
        for s in range(Wm):
            one_step(s)
    torch.cuda.synchronize()
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(sa):
        a0.record(); attention_pass(); a1.record()
    torch.cuda.synchronize()
    attn_alone_ms = a0.elapsed_time(a1)
    gemm_alone_ms = nb.alone_ms(sb, reps=20 if not handles else 6)
    attn_co_ms, gemm_co_ms, n_inside = side_by_side(attention_pass, sa, nb, sb, attn_alone_ms, gemm_alone_ms)
    torch.cuda.synchronize()
    for h in handles:
        adr.adr_stream_destroy(h)
    line = {
        "metric": "decode_attention_attended_kv_bandwidth_colocated", "unit": "GB/s",
        "value": round(kv_bytes / attn_co_ms / 1e6, 1), "n_gpus": 1, "steps": K, "warmup": Wm,
        "higher_is_better": True, "dtype": args.cache_dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d Hq=%d Hkv=%d d=%d, %d layers, partition %d, kernel %s; neighbour: bf16 %d^3 "
                               "torch.matmul on a second stream" % (wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, layers,
                                                                   part, args.kernel, nb.n),
                   "attention_cus": args.attention_cus or total_cus,
                   "gemm_cus": total_cus - args.attention_cus if args.attention_cus else total_cus},
        "attention_alone_GBps": round(kv_bytes / attn_alone_ms / 1e6, 1),
        "attention_contended_GBps": round(kv_bytes / attn_co_ms / 1e6, 1),
        "attention_ms_alone": round(attn_alone_ms, 4), "attention_ms_contended": round(attn_co_ms, 4),
        "gemm_alone_TFLOPs": nb.tflops(gemm_alone_ms),
        "gemm_contended_TFLOPs": nb.tflops(gemm_co_ms) if gemm_co_ms else None,
        "gemm_ms_alone": round(gemm_alone_ms, 4), "gemm_ms_contended": round(gemm_co_ms, 4) if gemm_co_ms else None,
        "gemms_inside_attention_window": n_inside,
    }
    print(json.dumps(line), flush=True)
    return 0


def graph_replay(args, wl, st, one_step, out, bytes_per_token, layers, part):
    """Sec. 3.2.2: the executor's per-layer kernels are launched from a pre-recorded graph, because
    launching them one by one costs more CPU time than the kernels take on the GPU.  One step (every
    layer's append, attention and merge) is recorded once, with the per-step inputs (positions,
    lengths) in fixed device buffers that are overwritten before each replay."""
    K, Wm = args.steps, args.warmup
    b = st["batch"]
    pos_buf = st["positions"][0].clone()
    seq_buf = st["seq_lens"][0].clone()
    tokens = [int(b.lens_before.sum()) + wl.B * (s + 1) for s in range(Wm, Wm + K)]
    kv_bytes = layers * sum(tokens) * bytes_per_token

    def timed(run_step):
        torch.cuda.synchronize()
        cpu = 0.0
        t0 = time.perf_counter()
        for s in range(Wm, Wm + K):
            c0 = time.perf_counter()
            run_step(s)
            cpu += time.perf_counter() - c0
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / K * 1e3, cpu / K * 1e3

    for s in range(Wm):
        one_step(s)
    eager_ms, eager_cpu_ms = timed(lambda s: one_step(s))
    eager_out = out.clone()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        one_step(0, pos=pos_buf, seq=seq_buf)             # warm the stream before recording
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        one_step(0, pos=pos_buf, seq=seq_buf)

    def replay(s):
        pos_buf.copy_(st["positions"][s])
        seq_buf.copy_(st["seq_lens"][s])
        graph.replay()

    # the caches now hold the tokens of the eager pass at these positions already: the replays
    # rewrite the same bytes, so the last step's output must equal the eager one bit for bit
    graph_ms, graph_cpu_ms = timed(replay)
    same = bool(torch.equal(out, eager_out))
    n_launch = layers * 3
    line = {
        "metric": "decode_attention_attended_kv_bandwidth_graph_replay", "unit": "GB/s",
        "value": round(kv_bytes / (graph_ms * K) / 1e6, 1), "n_gpus": 1, "steps": K, "warmup": Wm,
        "higher_is_better": True, "dtype": args.cache_dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d Hq=%d Hkv=%d d=%d, %d layers, partition %d; one HIP graph of %d kernel "
                               "launches per step" % (wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, layers, part, n_launch)},
        "eager_GBps": round(kv_bytes / (eager_ms * K) / 1e6, 1),
        "eager_ms_per_step": round(eager_ms, 4), "graph_ms_per_step": round(graph_ms, 4),
        "cpu_enqueue_ms_per_step_eager": round(eager_cpu_ms, 4),
        "cpu_enqueue_ms_per_step_graph": round(graph_cpu_ms, 4),
        "cpu_enqueue_us_per_layer_eager": round(eager_cpu_ms / layers * 1e3, 2),
        "cpu_enqueue_us_per_layer_graph": round(graph_cpu_ms / layers * 1e3, 2),
        "gpu_us_per_layer_graph": round(graph_ms / layers * 1e3, 2),
        "replayed_output_equals_eager": same,
    }
    print(json.dumps(line), flush=True)
    return 0 if same else 1


def graph_table(args, wl, st, out, ws, bytes_per_token, layers, part, flags):
    """Sec. 3.2.2 to its sketch: steps recorded for capacities on an interval grid, the smallest fit
    replayed for a batch of n rows (surplus rows padded).  For each capacity: GPU time per step and CPU
    time to enqueue one, eager (one adr_decode_step per layer) against one graph launch."""
    K, Wm = args.steps, args.warmup
    b = st["batch"]
    interval = max(wl.B // 4, 1)
    seq_buf = st["seq_lens"][0].clone()
    side = torch.cuda.Stream()

    def make_table(stream, table_flags):
        return adr.GraphTable(out, st["q"], st["k_new"], st["v_new"], st["caches"], st["table"], seq_buf, wl.scale,
                              st["max_len"], part, ws, interval, wl.B, stream, flags=table_flags)

    def set_rows(step, n):
        seq = st["seq_lens"][step].clone()
        seq[n:] = 0
        seq_buf.copy_(seq)
        return int(st["seq_lens"][step][:n].sum().item())

    def timed(fn, stream):
        torch.cuda.synchronize()
        cpu = 0.0
        t0 = time.perf_counter()
        with torch.cuda.stream(stream):
            for _ in range(K):
                c0 = time.perf_counter()
                fn()
                cpu += time.perf_counter() - c0
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / K * 1e3, cpu / K * 1e3

    def eager(n):
        for cache in st["caches"]:
            adr.adr_decode_step(out[:n], st["q"][:n], st["k_new"][:n], st["v_new"][:n], cache, st["table"][:n],
                                seq_buf[:n], wl.scale, st["max_len"], part, ws, None, flags)

    table = make_table(side, flags)
    rows = []
    # every timed step rewrites the same token slots, so the caches stay as they are
    for n in sorted({wl.B, wl.B - 1, 3 * wl.B // 4, wl.B // 2 + 1, wl.B // 4, 1}):
        cap = table.capacity(n)
        tokens = set_rows(Wm, n)
        for _ in range(Wm):
            eager(n)
            table.launch(n, side)
        eager_ms, eager_cpu = timed(lambda: eager(n), side)
        want = out[:n].clone()
        graph_ms, graph_cpu = timed(lambda: table.launch(n, side), side)
        same = bool(torch.equal(out[:n], want)) and bool(torch.all(out[n:cap] == 0))
        rows.append({"rows": n, "capacity": cap, "attended_tokens_per_layer": tokens,
                     "eager_ms_per_step": round(eager_ms, 4), "graph_ms_per_step": round(graph_ms, 4),
                     "cpu_enqueue_us_per_layer_eager": round(eager_cpu / layers * 1e3, 2),
                     "cpu_enqueue_us_per_step_graph": round(graph_cpu * 1e3, 2),
                     "gpu_us_per_layer_graph": round(graph_ms / layers * 1e3, 2),
                     "graph_GBps": round(layers * tokens * bytes_per_token / graph_ms / 1e6, 1),
                     "replayed_output_equals_eager": same})
        log("graph table: %s" % json.dumps(rows[-1]))
    table.destroy()

    # a table for a stream confined to three quarters of the compute units: the recording cannot ask the
    # stream for its mask, so without ADR_GRID_CUS the grid is sized for the whole chip
    total_cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_masked = 3 * total_cus // 4
    handle = adr.adr_stream_create_cu_mask([i < n_masked for i in range(total_cus)])
    masked = torch.cuda.ExternalStream(handle)
    set_rows(Wm, wl.B)
    masked_rows = {}
    try:
        eager_ms, _ = timed(lambda: eager(wl.B), masked)        # asks the stream: grid of n_masked workgroups
        masked_rows["eager_ms_per_step"] = round(eager_ms, 4)
        for name, f in (("graph_grid_for_whole_chip", flags), ("graph_with_ADR_GRID_CUS", flags | adr.GRID_CUS(n_masked))):
            t = make_table(masked, f)
            for _ in range(Wm):
                t.launch(wl.B, masked)
            ms, _ = timed(lambda: t.launch(wl.B, masked), masked)
            masked_rows[name + "_ms_per_step"] = round(ms, 4)
            torch.cuda.synchronize()
            t.destroy()
    finally:
        torch.cuda.synchronize()
        adr.adr_stream_destroy(handle)
    line = {"metric": "decode_step_graph_table", "unit": "ms", "n_gpus": 1, "steps": K, "warmup": Wm,
            "dtype": args.cache_dtype, "data": "synthetic",
            "config": {"workload": "%s: B=%d Hq=%d Hkv=%d d=%d, %d layers, partition %d; capacities %s" % (
                wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, layers, part, list(range(interval, wl.B + 1, interval)))},
            "rows": rows, "masked_stream": dict(masked_rows, attention_cus=n_masked)}
    print(json.dumps(line), flush=True)
    return 0 if all(r["replayed_output_equals_eager"] for r in rows) else 1


def cu_sweep(args, wl, st, one_step, bytes_per_token, layers, part):
    """Sec. 3.3's question on this chip: how much attention bandwidth does a fraction of the compute
    units obtain, and what does the neighbour lose?  The attention runs on a stream whose queue is
    masked to the first n compute-unit bits, the matrix products on a stream masked to the rest."""
    K, Wm = args.steps, args.warmup
    b = st["batch"]
    total_cus = torch.cuda.get_device_properties(0).multi_processor_count
    nb = Neighbour(wl)
    tokens = [int(b.lens_before.sum()) + wl.B * (s + 1) for s in range(Wm, Wm + K)]
    kv_bytes = layers * sum(tokens) * bytes_per_token

    def attention_pass():
        for s in range(Wm, Wm + K):
            one_step(s)

    for s in range(Wm):
        one_step(s)
    for _ in range(3):
        nb.product()
    torch.cuda.synchronize()
    rows = []
    for n_attn in range(32, total_cus + 1, 32):
        ha = adr.adr_stream_create_cu_mask([i < n_attn for i in range(total_cus)])
        sa = torch.cuda.ExternalStream(ha)
        row = {"attention_cus": n_attn, "gemm_cus": total_cus - n_attn}
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(sa):
            attention_pass()                      # warm-up on this stream
            a0.record(); attention_pass(); a1.record()
        torch.cuda.synchronize()
        alone_ms = a0.elapsed_time(a1)
        row["attention_alone_GBps"] = round(kv_bytes / alone_ms / 1e6, 1)
        if n_attn < total_cus:
            hb = adr.adr_stream_create_cu_mask([i >= n_attn for i in range(total_cus)])
            sb = torch.cuda.ExternalStream(hb)
            gemm_ms = nb.alone_ms(sb)
            row["gemm_alone_TFLOPs"] = nb.tflops(gemm_ms)
            co_ms, gemm_co_ms, n_inside = side_by_side(attention_pass, sa, nb, sb, alone_ms, gemm_ms)
            row["attention_contended_GBps"] = round(kv_bytes / co_ms / 1e6, 1)
            row["gemm_contended_TFLOPs"] = nb.tflops(gemm_co_ms) if gemm_co_ms else None
            row["gemms_inside_attention_window"] = n_inside
            del sb
            adr.adr_stream_destroy(hb)
        del sa
        adr.adr_stream_destroy(ha)
        log("cu sweep: %s" % json.dumps(row))
        rows.append(row)
    line = {"metric": "decode_attention_bandwidth_vs_compute_units", "unit": "GB/s", "n_gpus": 1, "steps": K,
            "warmup": Wm, "dtype": args.cache_dtype, "data": "synthetic",
            "config": {"workload": "%s: B=%d Hq=%d Hkv=%d d=%d, %d layers, partition %d, kernel %s; neighbour: bf16 "
                                   "%d^3 torch.matmul on the complementary compute units" % (
                                       wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, layers, part, args.kernel, nb.n)},
            "total_cus": total_cus, "rows": rows}
    print(json.dumps(line), flush=True)
    return 0


def cpu_baseline(wl, st, step, bytes_per_token):
    """The fp64 oracle, untuned, on this machine's host cores over a bounded sample:
    whole layers of the same workload at the first timed step's lengths, as many
    as give roughly 10-30 s of CPU work."""
    import oracle
    try:    # the same source built for this machine's CPU (same bits; the flags the baseline is quoted with)
        build = oracle.use_native_build(tempfile.mkdtemp(prefix="adr_oracle_"))
    except Exception as e:  # no compiler on this machine: the portable build that travelled with the tree
        log("native oracle build failed (%s); timing the portable build" % e)
        build = "gcc -O2 -fopenmp (portable build)"
    b = st["batch"]
    seq = st["seq_lens"][step].cpu().numpy()
    pairs_per_layer = int(seq.sum()) * wl.Hq                 # (token, q-head) dot products and V sums
    n_layers = int(min(len(st["caches"]), max(1, round(4e8 / max(pairs_per_layer, 1)))))
    qh = W.bits(st["q"].contiguous())
    dt, threads = 0.0, 1
    for li in range(n_layers):
        cache = st["caches"][li]
        kh, vh = W.bits(cache.k), W.bits(cache.v)           # device -> host copy, not timed
        scales = {}
        if cache.k_scale is not None:
            scales = dict(k_scale=W.bits(cache.k_scale), v_scale=W.bits(cache.v_scale))
        t0 = time.perf_counter()
        _, _, threads = oracle.decode_attention(qh, kh, vh, b.block_table, seq, wl.scale, **scales)
        dt += time.perf_counter() - t0
        del kh, vh
    tokens = int(seq.sum()) * n_layers
    gbs = tokens * bytes_per_token / dt / 1e9
    log("cpu oracle: %d layer(s), %d attended tokens, %.2f s on %d threads -> %.3f GB/s" % (
        n_layers, tokens, dt, threads, gbs))
    return {"value": round(gbs, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": "fp64 oracle over %d of %d layers, all %d requests (%d attended token-layers), %.2f s wall"
                      % (n_layers, len(st["caches"]), wl.B, tokens, dt),
            "build": build,
            "attended_tokens_per_s": round(tokens / dt, 1)}


if __name__ == "__main__":
    sys.exit(main())
