#!/usr/bin/env python3
"""Benchmark of the int4 compressed-domain decode-attention hot path on one MI355X.

A step = one pass of the whole hot path for one layer of the workload:
  quantise-append of one new token per sequence (Sec. 2.1)  ->  fused int4 SDPA over seq_len tokens
  (Alg. 1, Eq. 6), through the one-call entry point tq_sdpa_int4_append_decode (the decode kernel takes
  the new token in itself; --two-calls times tq_quantize_kv + tq_sdpa_int4_decode instead).
Inputs are resident in HBM before the timed region.  Steps rotate over several distinct KV
caches so that the 256 MB Infinity Cache cannot serve the stream (one 128K layer is 168 MB).

Prints ONE JSON line.  `value` is microseconds per decode step (lower is better); the same line
carries effective GB/s (packed int4 + scales + zero-points actually needed, divided by time),
the roofline block for the dominant kernel (timed with stream events), the
unfused GPU comparator and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published
PROBE_SRC = ROOT / "bench_probe.hip"
PROBE_LIB = ROOT / "libbench_probe.so"


def build_probe():
    """Compiles the benchmark's read-bandwidth probe (bench_probe.hip) for gfx950; returns the library's path."""
    import subprocess
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           str(PROBE_SRC), "-o", str(PROBE_LIB) + f".tmp{os.getpid()}"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on bench_probe.hip:\n" + res.stderr)
    os.replace(cmd[-1], PROBE_LIB)
    return PROBE_LIB


def load_probe():
    """bench_probe_read_stream(src, bytes, sink, stream) of the built probe library (built here if it is missing)."""
    import ctypes
    if not PROBE_LIB.exists():
        build_probe()
    f = ctypes.CDLL(str(PROBE_LIB)).bench_probe_read_stream
    f.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    f.restype = ctypes.c_int
    return f


def dist(xs):
    """median / p10 / p90 of a list of batch means (microseconds)."""
    xs = sorted(xs)
    pick = lambda f: xs[min(len(xs) - 1, max(0, round(f * (len(xs) - 1))))]
    return {"median": round(statistics.median(xs), 3), "p10": round(pick(0.1), 3), "p90": round(pick(0.9), 3),
            "batches": len(xs)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="llama128k",
                    help="tiny | llama8k | llama128k (default, the headline shape) | gqa16_128k (the same with 128 query heads: "
                         "the 16-row tile) | gemma32k | global512_32k (d=512, GQA 32: "
                         "the head_dim 512 matrix-core kernel) | varlen8 (8 sequences of "
                         "the llama shape with their own lengths in [4096, 32768], per-sequence append + decode) | paged8 (the same "
                         "over a pool of 256-token pages in random order) | varlen256 (256 sequences of 64 ... 1024 tokens of the llama "
                         "shape: every (sequence, KV head) row is one chunk, no merge kernel) | varlen256_2k (the same with 64 ... 2048 tokens: "
                         "chunks planned on the device, merge kernel of one block per sequence and four query heads) | sweep80 "
                         "(80 layers x batch 4 of the llama128k shape, append + attend per layer) | prefill128k (the prefill arm: "
                         "one bulk tq_quantize_kv of a 128K layer)")
    ap.add_argument("--layers", type=int, default=80, help="sweep80 only: number of layers")
    ap.add_argument("--buffers", type=int, default=8, help="distinct KV caches the steps rotate over")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--group-size", type=int, default=32,
                    help="quantisation group: 32 (the paper's), 64 or 128 (fixed-length workloads in a contiguous cache)")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--window", type=int, default=0, help="sliding window: attend only the last N tokens (0 = all)")
    ap.add_argument("--n-queries", type=int, default=1,
                    help="query tokens per sequence and step (2..8: the step appends that many tokens and attends "
                         "them causally, as in speculative verification; fixed-length workloads)")
    ap.add_argument("--two-calls", action="store_true",
                    help="time the step as tq_quantize_kv + tq_sdpa_int4_decode instead of tq_sdpa_int4_append_decode")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-baseline", action="store_true", help="skip the unfused GPU comparator")
    ap.add_argument("--no-check", action="store_true", help="skip the sampled oracle check")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the read-stream probe")
    ap.add_argument("--batches", type=int, default=7,
                    help="further batches of --steps steps (and of --steps kernel launches) timed after the first, for the "
                         "median / p10 / p90 the line reports next to `value`")
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed run of the step loop before the warm-up steps: the GPU's clocks take some tens of "
                         "milliseconds of sustained load to settle (a cold start reads 36 us per launch, falling to "
                         "29.5 us within about 40 ms)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain device copy of packed_bytes (reference point for HBM byte counters)")
    return ap.parse_args()


def sweep(args):
    """Full decode-step attention sweep: the Llama-70B shape x `layers` layers x batch 4 at 128K, every
    (layer, batch element) with its own seed; a step appends one token per sequence per layer
    (tq_quantize_kv) and attends (tq_sdpa_int4_decode), layer after layer on one stream."""
    import numpy as np
    import torch

    import paper_2604_16957_amd as tq
    import tq_workloads as wl

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    L, B = args.layers, 4
    base = wl.WORKLOADS["llama128k"]
    S, Hq, Hkv, d = base.seq_len, base.n_q_heads, base.n_kv_heads, base.head_dim
    steps = args.steps if args.steps != 400 else 5
    warmup = args.warmup if args.warmup != 40 else 6      # (about 60 ms: the clocks settle)
    samples = {(0, 0), (L - 1, B - 1)}           # (layer, batch element) pairs checked against the oracle
    kept = {}
    caches, qs, news = [], [], []
    kb = torch.empty((B, Hkv, S, d), dtype=torch.float16, device=dev)
    vb = torch.empty_like(kb)
    for l in range(L):
        q4 = torch.empty((B, Hq, d), dtype=torch.float16, device=dev)
        for b in range(B):
            q, k, v = wl.make_inputs(wl.layer_workload(l, b), device=dev)
            q4[b], kb[b], vb[b] = q[0], k[0], v[0]
            if (l, b) in samples:
                kept[(l, b)] = (q.cpu(), k.cpu(), v.cpu())
            del q, k, v
        c = tq.KVCache(B, Hkv, d, S)
        tq.tq_quantize_kv(c, kb[:, :, :S - 1].contiguous(), vb[:, :, :S - 1].contiguous(), 0)
        news.append((kb[:, :, S - 1:].contiguous(), vb[:, :, S - 1:].contiguous()))
        caches.append(c)
        qs.append(q4)
        if l % 10 == 9:
            torch.cuda.synchronize()
            print(f"# sweep: {l + 1}/{L} layers resident", file=sys.stderr, flush=True)
    del kb, vb
    torch.cuda.synchronize()
    ws = torch.empty(tq.tq_workspace_bytes(B, Hq, d), dtype=torch.uint8, device=dev)
    outs = torch.empty((L, B, Hq, d), dtype=torch.float16, device=dev)
    alpha = base.attn_scale
    packed = L * B * base.packed_bytes

    def step():
        for l in range(L):
            if args.two_calls:
                tq.tq_quantize_kv(caches[l], news[l][0], news[l][1], S - 1)
                tq.tq_sdpa_int4_decode(caches[l], qs[l], S, alpha, out=outs[l], workspace=ws)
            else:
                tq.tq_sdpa_int4_append_decode(caches[l], news[l][0], news[l][1], qs[l], S, alpha, out=outs[l], workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / steps
    # the dominant kernel: events around the first launch of each layer's decode, one more step
    fused = tq.tq_decode_launches(caches[0], Hq, S, alpha) == 1
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
    n_splits = 0
    for l in range(L):
        tq.tq_quantize_kv(caches[l], news[l][0], news[l][1], S - 1)
        evs[l][0].record()
        if fused:
            tq.tq_sdpa_int4_decode(caches[l], qs[l], S, alpha, out=outs[l], workspace=ws)
        else:
            n_splits = tq.tq_sdpa_int4_partial(caches[l], qs[l], S, alpha, ws)
        evs[l][1].record()
        if not fused:
            tq.tq_sdpa_int4_reduce(B, Hq, d, n_splits, ws, outs[l])
    torch.cuda.synchronize()
    k_us = [a.elapsed_time(b) * 1e3 for a, b in evs]
    kernel_us = statistics.fmean(k_us)
    per_launch = B * base.packed_bytes
    achieved = per_launch / (kernel_us * 1e-6) / 1e9

    cpu = check = None
    if not args.no_cpu or not args.no_check:
        import oracle
        worst_abs = worst_rel = 0.0
        exact = True
        t_cpu = []
        for (l, b), (q0, k0, v0) in sorted(kept.items()):
            kc, ks, kz = oracle.quantize(k0.numpy())
            vc, vs, vz = oracle.quantize(v0.numpy())
            t = time.perf_counter()
            ref = oracle.attend_packed(q0.numpy(), kc, ks, kz, vc, vs, vz, seq_len=S, alpha=alpha,
                                       nthreads=oracle.default_threads())
            t_cpu.append(time.perf_counter() - t)
            got = outs[l, b].cpu().numpy().astype(np.float64)
            diff = got - ref[0]
            worst_abs = max(worst_abs, float(np.abs(diff).max()))
            worst_rel = max(worst_rel, float(np.linalg.norm(diff) / np.linalg.norm(ref)))
            exact = exact and bool(np.array_equal(caches[l].k_codes[b].cpu().numpy(), kc[0])
                                   and np.array_equal(caches[l].v_codes[b].cpu().numpy(), vc[0]))
        check = {"sampled_layer_batch": sorted(kept), "max_abs": worst_abs, "rel_l2": worst_rel,
                 "codes_bit_exact": exact, "ok": worst_abs <= 2e-3 and worst_rel <= 1e-3 and exact}
        if not args.no_cpu:
            cpu = {"value": round(statistics.fmean(t_cpu) * 1e6 * L * B, 1), "unit": "us/decode-step",
                   "cores": oracle.default_threads(), "kind": "oracle",
                   "sample": f"{len(t_cpu)} of the {L * B} (layer, batch element) attention calls timed whole "
                             f"(fp64 naive softmax over the packed cache), mean x {L * B}; appends not included"}
    line = {
        "metric": "us_per_decode_step (int4 SDPA, all layers, append + fused attention)",
        "value": round(ms_per_step * 1e3, 1), "unit": "us/decode-step", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 codes + fp16 scale/zero in HBM; fp16 MFMA/VALU inputs, fp32 accumulate, fp16 out",
        "data": "synthetic",
        "config": {"workload": f"sweep{L}: llama128k shape x {L} layers x batch {B}, one token appended per sequence per layer",
                   "batch": B, "layers": L, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d, "seq_len": S,
                   "attn_scale": alpha, "group_size": 32, "n_splits": n_splits, "decode_launches": 1 if fused else 2,
                   "step_calls": "tq_quantize_kv + tq_sdpa_int4_decode" if args.two_calls else "tq_sdpa_int4_append_decode"},
        "effective_GBps": round(packed / (ms_per_step * 1e-3) / 1e9, 1),
        "pct_of_hbm_peak": round(100 * packed / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "packed_bytes_per_step": packed,
        "roofline": {"bound": "hbm", "kernel": "decode_partial_mfma_kernel, one launch per layer (batch 4)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "kernel_us_mean": round(kernel_us, 2), "kernel_us_median": round(statistics.median(k_us), 2),
                     "algorithmic_bytes_per_launch": per_launch},
        "cpu_baseline": cpu, "oracle_check": check,
    }
    print(json.dumps(line), flush=True)


def prefill(args):
    """The prefill arm of Sec. 3.3 (quantize -> store): one bulk tq_quantize_kv of a whole 128K layer of the
    llama128k shape (537 MB of fp16 K and V in, 168 MB of codes, scales and zero-points out), over rotating
    destination caches; codes checked bit for bit against the oracle on a slice."""
    import numpy as np
    import torch

    import paper_2604_16957_amd as tq
    import tq_workloads as wl

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS["llama128k"]
    S, B, Hkv, d = w.seq_len, w.batch, w.n_kv_heads, w.head_dim
    GS = args.group_size
    _, k, v = wl.make_inputs(w, device=dev)
    caches = [tq.KVCache(B, Hkv, d, S, group_size=GS) for _ in range(4)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(n):
        e0.record()
        for i in range(n):
            tq.tq_quantize_kv(caches[i % 4], k, v, 0)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    steps = args.steps if args.steps != 400 else 100
    spent = 0.0
    while spent < args.settle_ms * 1e3:
        spent += timed(50) * 50
    for _ in range(args.warmup):
        tq.tq_quantize_kv(caches[0], k, v, 0)
    us = timed(steps)
    batches = [us] + [timed(steps) for _ in range(args.batches)]
    moved = 2 * B * Hkv * S * d * 2 + tq.tq_kv_bytes_grouped(B, Hkv, S, d, GS)
    check = None
    if not args.no_check:
        import oracle
        n = 4096                                   # the first tokens of every KV head
        kc, ks, kz = oracle.quantize(k[:, :, :n].cpu().numpy(), group=GS)
        c = caches[(steps - 1) % 4]
        check = {"tokens": n, "codes_bit_exact": bool(np.array_equal(c.k_codes[:, :, :n].cpu().numpy(), kc) and
                                                       np.array_equal(c.k_scale[:, :, :n].cpu().numpy().view(np.uint16), ks.view(np.uint16)) and
                                                       np.array_equal(c.k_zero[:, :, :n].cpu().numpy().view(np.uint16), kz.view(np.uint16)))}
        check["ok"] = check["codes_bit_exact"]
    achieved = moved / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "us_per_bulk_quantise (one 128K layer, K and V)", "value": round(us, 2), "unit": "us/fill",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 6), "step_us": dist(batches),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp16 in; fp32 arithmetic of Eq. 2-3; int4 codes + fp16 scale/zero out", "data": "synthetic",
        "config": {"workload": "prefill128k", "batch": B, "n_kv_heads": Hkv, "head_dim": d, "seq_len": S, "group_size": GS},
        "roofline": {"bound": "hbm", "kernel": "quantize_append_kernel (the whole tq_quantize_kv call)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": moved},
        "cpu_baseline": None, "oracle_check": check}))


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build targets one GPU; run with --gpus 1 (no multi-GPU path exists).")
    if args.workload == "prefill128k":
        import torch
        if not torch.cuda.is_available():
            sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback.")
        return prefill(args)
    if args.workload == "sweep80":
        import torch
        if not torch.cuda.is_available():
            sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback.")
        return sweep(args)
    import numpy as np
    import torch

    import paper_2604_16957_amd as tq
    import tq_workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback.")
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    paged = args.workload == "paged8"             # varlen8 with the sequences scattered over a pool of 256-token pages
    many = args.workload in ("varlen256", "varlen256_2k")   # many short sequences: 256 of 64 ... 1024 (2048) tokens
    varlen = args.workload == "varlen8" or paged or many
    PT = 256
    if many:
        w = wl.custom(args.workload, batch=256, n_q_heads=64, n_kv_heads=8, head_dim=128,
                      seq_len=2048 if args.workload == "varlen256_2k" else 1024, seed=1200, outlier_channels=4)
    elif varlen:   # continuous batching: 8 sequences of the llama shape, lengths drawn in [4096, 32768]
        w = wl.custom("paged8" if paged else "varlen8", batch=8, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=32768, seed=1100,
                      outlier_channels=4)
    else:
        w = wl.WORKLOADS[args.workload]
    S, B, Hq, Hkv, d = w.seq_len, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    lens = None
    if varlen:
        g = torch.Generator().manual_seed(w.seed + 5)
        lens = torch.randint(64 if many else 4096, S + 1, (B,), generator=g, dtype=torch.int32)
        lens[0] = S                               # the bound is attained
        lens_dev, pos_dev = lens.to(dev), (lens - 1).to(dev)

    GS = args.group_size
    if GS != 32 and lens is not None:
        sys.exit("bench.py: --group-size is offered for the fixed-length workloads")
    NQ = args.n_queries
    if NQ > 1 and (lens is not None or args.window > 0):
        sys.exit("bench.py: --n-queries is offered for the fixed-length workloads without a window")

    # ---- resident inputs: `buffers` caches, each pre-filled with S-NQ tokens; the step appends the last NQ
    caches, qs, news = [], [], []
    for i in range(args.buffers):
        wi = wl.Workload(**{**w.__dict__, "seed": w.seed + 7777 * i})
        q, k, v = wl.make_inputs(wi, device=dev)
        if paged:                                 # a pool with exactly the pages the sequences need, in random order
            gp = torch.Generator().manual_seed(w.seed + 99 + i)
            table = torch.randperm(B * (S // PT), generator=gp).to(torch.int32).reshape(B, S // PT).to(dev)
            c = tq.KVCache(B * (S // PT), Hkv, d, PT)
            c.table = table
            tq.tq_quantize_kv_paged(c, table, k[:, :, :S - 1].contiguous(), v[:, :, :S - 1].contiguous(),
                                    torch.zeros(B, dtype=torch.int32, device=dev))
        else:
            c = tq.KVCache(B, Hkv, d, S, group_size=GS)
            tq.tq_quantize_kv(c, k[:, :, :S - NQ].contiguous(), v[:, :, :S - NQ].contiguous(), 0)
        news.append((k[:, :, S - NQ:].contiguous(), v[:, :, S - NQ:].contiguous()))
        caches.append(c)
        qs.append(q if NQ == 1 else wl.make_queries(wi, NQ, device=dev))
        del k, v
    torch.cuda.synchronize()
    ws = torch.empty(tq.tq_workspace_bytes(B * NQ, Hq, d), dtype=torch.uint8, device=dev)
    out = torch.empty_like(qs[0])
    packed_bytes = tq.tq_kv_bytes_grouped(B, Hkv, S, d, GS) if lens is None else \
        int(lens.sum()) * Hkv * (w.packed_bytes // (B * Hkv * S))
    kw = dict(n_splits=args.n_splits, variant=args.variant)
    if args.window > 0:                           # sliding window: only the attended tokens are streamed
        if lens is not None:
            sys.exit("bench.py: --window is offered for the fixed-length workloads")
        kw["window"] = args.window
        packed_bytes = packed_bytes // S * min(S, args.window)

    def append(j):                                # the step's new token goes to the end of every sequence
        if lens is None:
            tq.tq_quantize_kv(caches[j], news[j][0], news[j][1], S - NQ)
        elif paged:
            tq.tq_quantize_kv_paged(caches[j], caches[j].table, news[j][0], news[j][1], pos_dev)
        else:
            tq.tq_quantize_kv_varlen(caches[j], news[j][0], news[j][1], pos_dev)

    def decode(j):
        if lens is None:
            tq.tq_sdpa_int4_decode(caches[j], qs[j], S, w.attn_scale, out=out, workspace=ws, **kw)
        elif paged:
            tq.tq_sdpa_int4_decode_paged(caches[j], caches[j].table, qs[j], lens_dev, S, w.attn_scale, out=out,
                                         workspace=ws, **kw)
        else:
            tq.tq_sdpa_int4_decode_varlen(caches[j], qs[j], lens_dev, S, w.attn_scale, out=out, workspace=ws, **kw)

    one_call = lens is None and not args.two_calls

    def step(i):
        j = i % args.buffers
        if one_call:                              # the step's token is quantised, stored and attended by one call
            tq.tq_sdpa_int4_append_decode(caches[j], news[j][0], news[j][1], qs[j], S, w.attn_scale, out=out,
                                          workspace=ws, **kw)
        elif lens is not None and not args.two_calls:
            if paged:
                tq.tq_sdpa_int4_append_decode_paged(caches[j], caches[j].table, news[j][0], news[j][1], qs[j], lens_dev, S,
                                                    w.attn_scale, out=out, workspace=ws, **kw)
            else:
                tq.tq_sdpa_int4_append_decode_varlen(caches[j], news[j][0], news[j][1], qs[j], lens_dev, S, w.attn_scale,
                                                     out=out, workspace=ws, **kw)
        else:
            append(j)
            decode(j)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def settle(fn):
        """Runs fn(i) untimed for --settle-ms of GPU time: measurements start from settled clocks."""
        i, spent = 0, 0.0
        while spent < args.settle_ms:
            e0.record()
            for _ in range(200):
                fn(i)
                i += 1
            e1.record()
            torch.cuda.synchronize()
            spent += e0.elapsed_time(e1)

    def timed(fn, n):
        """microseconds per call of n consecutive fn(i) between two events on the launch stream"""
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    # ---- timed region: (settling run,) W warm-up steps, then exactly K steps between synchronisations: `value`.
    #      Further batches of K steps follow for the spread.
    settle(step)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    us_per_step = timed(step, args.steps)
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = us_per_step * 1e-3
    step_batches = [us_per_step] + [timed(step, args.steps) for _ in range(args.batches)]

    # ---- dominant kernel: stream events around each of its launches.  Where the decode call is ONE
    #      launch (partials and chunk merge in the same kernel) that launch is timed; otherwise phase 1,
    #      the partial kernel, which tq_sdpa_int4_partial launches on its own.
    fused = (not paged) and tq.tq_decode_launches(caches[0], Hq, S, w.attn_scale, n_queries=NQ, **kw) == 1
    if args.workload == "varlen256_2k":           # (the launch count above is that of a common length; these lengths
        fused = False                             # take chunks planned on the device and the merge kernel)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    n_splits = 0 if paged else tq.tq_sdpa_int4_partial(caches[0], qs[0], S, w.attn_scale, ws, **kw)
    lo = max(0, S - args.window) if args.window > 0 else 0     # first attended token

    def dominant(j):
        if fused or lens is not None:             # (no separate phase-1 entry point takes per-sequence lengths)
            decode(j)
        else:
            tq.tq_sdpa_int4_partial(caches[j], qs[j], S, w.attn_scale, ws, **kw)

    for i in range(args.steps):
        j = i % args.buffers
        append(j)
        evs[i][0].record()
        dominant(j)
        evs[i][1].record()
        if not fused and lens is None:
            tq.tq_sdpa_int4_reduce(B * NQ, Hq, d, n_splits, ws, out)
    torch.cuda.synchronize()
    k_us = [a.elapsed_time(b) * 1e3 for a, b in evs]
    kernel_us_bracketed = statistics.fmean(k_us)
    # Average launch duration: `steps` launches of that kernel in a row between two events.  This is the
    # figure the roofline uses; it agrees with rocprofv3's kernel trace of the step loop, whereas an
    # event pair around every single launch (kept as `kernel_us_bracketed_*`) adds the latency of the
    # two event packets, about 2 us, to each measurement.
    settle(lambda i: dominant(i % args.buffers))
    # (Batches of at least 200 launches, whatever K is: the kernel's average duration does not depend on K, and in a
    #  batch of 20 the two event records and the first launch's start-up weigh 0.3 - 1 us per launch on it.)
    kernel_launches = max(args.steps, 200)
    kernel_batches = [timed(lambda i: dominant(i % args.buffers), kernel_launches) for _ in range(1 + args.batches)]
    kernel_us = statistics.fmean(kernel_batches)     # average launch duration over all timed launches
    achieved = packed_bytes / (kernel_us * 1e-6) / 1e9

    # ---- what the machine delivers for a read-once stream of this size: the library's read probe (non-temporal
    #      loads, nothing else) over rotating buffers of the same number of bytes, timed like the kernel
    ceiling = None
    unit16 = 16 << 20
    probe_bytes = packed_bytes // unit16 * unit16
    if probe_bytes > 0 and not args.no_ceiling:
        bufs = [torch.empty(probe_bytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(args.buffers)]
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        probe = load_probe()
        stream = torch.cuda.current_stream().cuda_stream

        def read(i):
            if probe(bufs[i % args.buffers].data_ptr(), probe_bytes, sink.data_ptr(), stream) != 0:
                sys.exit("bench.py: the read probe rejected its arguments or failed to launch")

        settle(read)
        probe_us = statistics.fmean(timed(read, args.steps) for _ in range(1 + args.batches))
        probe_gbps = probe_bytes / (probe_us * 1e-6) / 1e9
        ceiling = {"kernel": "bench_probe.hip: read-only stream, non-temporal loads, 256 blocks", "bytes_per_launch": probe_bytes,
                   "us_per_launch": round(probe_us, 3), "GBps": round(probe_gbps, 1),
                   "frac_of_peak": round(probe_gbps / HBM_PEAK_GBPS, 4),
                   "decode_kernel_vs_this": round(achieved / probe_gbps, 4)}
        del bufs

    if args.calibrate_copy:      # known traffic: reads packed_bytes, writes packed_bytes
        src = torch.empty(packed_bytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(6):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- unfused comparator on the same inputs
    baseline = None
    if not args.no_baseline and lens is None and NQ == 1:
        dense = torch.empty(tq.tq_dense_scratch_bytes(B, Hkv, S, d), dtype=torch.uint8, device=dev)
        nb = max(5, min(40, args.steps // 5))

        def unfused(i):
            j = i % args.buffers
            tq.tq_dequant_then_attend(caches[j], qs[j], S, w.attn_scale, out=out, workspace=ws, dense_scratch=dense)

        def fused_call(i):                        # the fused call, timed the same way on the same inputs
            j = i % args.buffers
            tq.tq_sdpa_int4_decode(caches[j], qs[j], S, w.attn_scale, out=out, workspace=ws, **kw)

        for i in range(3):
            unfused(i)
        torch.cuda.synchronize()
        base_us = statistics.median(timed(unfused, nb) for _ in range(3))
        settle(fused_call)
        fused_us = statistics.median(timed(fused_call, args.steps) for _ in range(3))
        # what the unfused path moves: phase 1 reads the packed cache and writes dense fp16 K^ and V^, phase 2 reads them
        dense_bytes = tq.tq_dense_scratch_bytes(B, Hkv, S, d)
        moved = packed_bytes + 2 * dense_bytes
        baseline = {"name": "tq_dequant_then_attend (dense fp16)", "us_per_call": round(base_us, 2),
                    "fused_decode_us_per_call": round(fused_us, 2), "fused_speedup": round(base_us / fused_us, 2),
                    "calls": nb, "bytes_moved_per_call": moved,
                    "GBps_on_bytes_moved": round(moved / (base_us * 1e-6) / 1e9, 1),
                    "frac_of_hbm_peak_on_bytes_moved": round(moved / (base_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                    "byte_ratio_unfused_over_fused": round(moved / packed_bytes, 2)}
        del dense

    # ---- CPU oracle on the host cores (reported baseline, never the target) + sampled parity check
    cpu = None
    check = None
    if not args.no_cpu or not args.no_check:
        import oracle
        q0, k0, v0 = wl.make_inputs(w, device="cpu")           # the named workload's own bits
        if NQ > 1:
            q0 = wl.make_queries(w, NQ, device="cpu")
        kc, ks, kz = oracle.quantize(k0.numpy(), group=GS)
        vc, vs, vz = oracle.quantize(v0.numpy(), group=GS)
        threads = oracle.default_threads()
        reps, times = 3, []
        ref = None
        def oracle_attend():
            if NQ > 1:                            # query token t attends the first S - (NQ - 1 - t) tokens
                rows = [oracle.attend_packed(q0.numpy()[:, t], kc, ks, kz, vc, vs, vz, seq_len=S - (NQ - 1 - t),
                                             alpha=w.attn_scale, nthreads=threads) for t in range(NQ)]
                return np.stack(rows, axis=1)
            if lens is None:
                return oracle.attend_packed(q0.numpy(), *[a[:, :, lo:] for a in (kc, ks, kz, vc, vs, vz)], seq_len=S - lo,
                                            alpha=w.attn_scale, nthreads=threads)
            return np.concatenate([oracle.attend_packed(q0.numpy()[b:b + 1], *[a[b:b + 1] for a in (kc, ks, kz, vc, vs, vz)],
                                                        seq_len=int(lens[b]), alpha=w.attn_scale, nthreads=threads)
                                   for b in range(B)], axis=0)

        for _ in range(reps if not args.no_cpu else 1):
            t = time.perf_counter()
            ref = oracle_attend()
            times.append(time.perf_counter() - t)
        if not args.no_cpu:
            cpu = {"value": round(statistics.median(times) * 1e6, 1), "unit": "us/decode-step", "cores": threads,
                   "kind": "oracle",
                   "sample": f"whole {w.name} layer (attention over the packed cache, fp64 naive softmax), "
                             f"median of {reps} runs; quantise-append not included"}
        if not args.no_check:
            if paged:
                table = caches[0].table
                c = tq.KVCache(B * (S // PT), Hkv, d, PT)
                tq.tq_quantize_kv_paged(c, table, k0.to(dev), v0.to(dev), torch.zeros(B, dtype=torch.int32, device=dev))
                o = tq.tq_sdpa_int4_decode_paged(c, table, q0.to(dev), lens_dev, S, w.attn_scale, workspace=ws, **kw)
                # read the pool back through the table: [B][pages][H_kv][PT][..] -> [B][H_kv][S][..]
                back = lambda t: t[table.long()].permute(0, 2, 1, 3, 4).reshape(B, Hkv, S, -1).cpu().numpy()
                got_k, got_v = back(c.k_codes), back(c.v_codes)
            else:
                c = tq.KVCache(B, Hkv, d, S, group_size=GS)
                tq.tq_quantize_kv(c, k0.to(dev), v0.to(dev), 0)
                if lens is None:
                    o = tq.tq_sdpa_int4_decode(c, q0.to(dev), S, w.attn_scale, workspace=ws, **kw)
                else:
                    o = tq.tq_sdpa_int4_decode_varlen(c, q0.to(dev), lens_dev, S, w.attn_scale, workspace=ws, **kw)
                got_k, got_v = c.k_codes.cpu().numpy(), c.v_codes.cpu().numpy()
            torch.cuda.synchronize()
            diff = o.cpu().numpy().astype(np.float64) - ref
            check = {"max_abs": float(np.abs(diff).max()), "rel_l2": float(np.linalg.norm(diff) / np.linalg.norm(ref)),
                     "codes_bit_exact": bool(np.array_equal(got_k, kc) and np.array_equal(got_v, vc))}
            check["ok"] = check["max_abs"] <= 2e-3 and check["rel_l2"] <= 1e-3 and check["codes_bit_exact"]

    line = {
        "metric": "us_per_decode_step (int4 SDPA, one layer, append + fused attention)",
        "value": round(us_per_step, 3), "unit": "us/decode-step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "step_us": dist(step_batches), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 codes + fp16 scale/zero in HBM; fp16 MFMA/VALU inputs, fp32 accumulate, fp16 out",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d,
                   "seq_len": S, "seq_lens": None if lens is None else lens.tolist() if B <= 16 else
                   {"count": B, "min": int(lens.min()), "max": int(lens.max()), "sum": int(lens.sum()), "seed": w.seed + 5}, "attn_scale": w.attn_scale, "group_size": GS, "kv_buffers_rotated": args.buffers,
                   "n_splits": n_splits, "variant": args.variant, "window": args.window, "n_queries": NQ,
                   "step_calls": ("tq_sdpa_int4_append_decode" if one_call else
                                  "tq_sdpa_int4_append_decode_paged" if paged and not args.two_calls else
                                  "tq_sdpa_int4_append_decode_varlen" if lens is not None and not args.two_calls else
                                  "tq_quantize_kv_paged + tq_sdpa_int4_decode_paged" if paged else
                                  "tq_quantize_kv_varlen + tq_sdpa_int4_decode_varlen" if lens is not None else
                                  "tq_quantize_kv + tq_sdpa_int4_decode"),
                   "decode_launches": 1 if fused else 2},
        "effective_GBps": round(packed_bytes / (us_per_step * 1e-6) / 1e9, 1),
        "pct_of_hbm_peak": round(100 * packed_bytes / (us_per_step * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
        "packed_bytes_per_step": packed_bytes,
        "host_wall_ms_timed_region": round(wall_ms, 2),
        "settle_ms_before_warmup": args.settle_ms,
        "roofline": {"bound": "hbm",
                     "kernel": ("decode_partial_mfma_kernel: fused int4 attention over the chunks + in-kernel chunk merge "
                                "(the whole tq_sdpa_int4_decode call)" if fused else
                                "partial kernel (phase 1 of the decode)" if lens is None else
                                "the whole tq_sdpa_int4_decode_paged call (partial kernel + merge kernel)" if paged else
                                "the whole tq_sdpa_int4_decode_varlen call (partial kernel + merge kernel)"),
                     "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None, "traffic_source": None, "kernel_us_mean": round(kernel_us, 3),
                     "kernel_us": dist(kernel_batches), "kernel_launches_per_batch": kernel_launches,
                     "kernel_us_bracketed_mean": round(kernel_us_bracketed, 3),
                     "kernel_us_bracketed_median": round(statistics.median(k_us), 3),
                     "algorithmic_bytes_per_launch": packed_bytes,
                     "measured_read_stream": ceiling},
        "cpu_baseline": cpu,
        "unfused_gpu_baseline": baseline,
        "oracle_check": check,
    }
    if d == 512:
        # GQA 32 on one KV head: every fetched byte is used by 32 query heads (21 MB of cache for 2.1 GFLOP), so the
        # arithmetic, not the memory system, is what the shape asks for: 4 flops per (query head, token, element).
        # The head_dim 512 kernel runs both contractions on the matrix cores (fp16 operands: the dense fp16 peak);
        # the generic kernel (--variant 1) dequantises and multiplies on the vector ALU (the fp32 vector peak).
        flops = 4.0 * B * Hq * S * d
        tf = flops / (kernel_us * 1e-6) / 1e12
        bound, peak = ("alu", 157.3) if args.variant == 1 else ("mfma", 2500.0)
        line["roofline"].update({"bound": bound, "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s",
                                 "frac": round(tf / peak, 4), "algorithmic_flops_per_launch": flops})
    prof = ROOT / "profiles" / "traffic.json"
    if prof.exists():
        try:
            t = json.loads(prof.read_text()).get(w.name)
            if t:          # measured with rocprofv3 --pmc, see profiles/*_hbm_traffic.txt: NOT measured in this run
                line["roofline"]["traffic"] = t["total_bytes"]
                line["roofline"]["traffic_source"] = ("profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                                      "bench, kept with their commands in profiles/*_hbm_traffic.txt; not measured in this run")
                line["roofline"]["traffic_detail"] = t
        except Exception:
            pass
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
