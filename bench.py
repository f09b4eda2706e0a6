#!/usr/bin/env python3
"""Throughput of the mixed-tenant per-tenant-layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_ffn]

One "step" is one pass of the whole hot path (router, residency resolve, grouped GEMMs
with fused epilogues, attention, LayerNorm) over one seeded synthetic batch that is already
resident in HBM.  Prints ONE JSON line: tokens/s per layer (whole job), plus
  roofline     – the dominant kernel (grouped bf16 MFMA GEMM): algorithmic FLOP per launch
                 / its average launch duration measured with HIP events on the compute
                 stream, against the 2.5 PFLOP/s dense bf16 peak
  cpu_baseline – the fp64 oracle timed on this machine's host cores on a bounded sample.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3     # fp32 vector
PEAK_HBM_GBS = 8000.0       # HBM3E, published


def measured_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (each scaled by a copy kernel of known size in the same run, see --copy-calibration).  The figure is
    not known to this program: it is read from the committed summary of those counter runs, the line
    `traffic_bytes_per_launch[<workload>] = <bytes>` of a file under profiles/, and reported together with
    that file's name; None where no summary covers the workload."""
    import glob
    import re
    pat = re.compile(r"^\s*traffic_bytes_per_launch\[" + re.escape(workload) + r"\]\s*=\s*([0-9.eE+]+)")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(path) as fh:
            for line in fh:
                m = pat.match(line)
                if m:
                    return float(m.group(1)), os.path.relpath(path, ROOT)
    return None, None


def linear_flops_per_token(wl) -> float:
    """2 * (weight elements touched) per token and layer, matrices only."""
    import synth
    d, f = wl.d_model, wl.d_ff
    if wl.block in (synth.BLOCK_FFN, synth.BLOCK_ADAPTER):
        return 4.0 * d * f
    return 2.0 * (4 * d * d + 2 * d * f) + 4.0 * d * wl.adapter_rank


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 200 steps: the synchronisation in front of the timed region costs the first steps about a millisecond in all
    # (a 50-step run of the default workload reads 5 % slower than its own median step); 0.1 s of timed work
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bert_ffn")
    ap.add_argument("--cpu-sample", type=int, default=256, help="requests the oracle is timed on (0 = skip)")
    ap.add_argument("--tenants", type=int, default=0, help="override the workload's tenant count (host-tier runs at reduced size)")
    ap.add_argument("--slots", type=int, default=0, help="override the number of HBM slots")
    ap.add_argument("--images", type=int, default=-1,
                    help="host-tier workloads: distinct weight sets in pinned memory; tenant t owns set t mod IMAGES "
                         "(default: 500 for hbert_10k, whose 10 000 images of 14 MB exceed what can be pinned; 0 = one per tenant)")
    ap.add_argument("--decode", type=int, default=0, metavar="G",
                    help="DEC_PRELN workloads: after the timed steps also prefill the batch into a key/value cache and "
                         "time G decode steps (one new token per request and step); reported under \"decode\"")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="bert_ffn only: also time the vendor library (torch's linear = hipBLASLt) on DENSE problems of the "
                         "two launches' sizes (one weight matrix for all rows, no gather, no ragged tiles) and on 8192^3 with "
                         "random and with all-zero operands; reported under \"vendor_dense_gemm\" as context for roofline.frac")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB (a kernel of known HBM traffic that "
                         "scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the same run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; collectives and sharding are not part of it "
              "(run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth
    import paper_2504_17449_amd as hmi
    from paper_2504_17449_amd import harness

    wl = synth.WORKLOADS[args.workload]
    if args.tenants or args.slots:
        wl = wl.scaled(name=wl.name + "_scaled", n_tenants=args.tenants or wl.n_tenants,
                       hbm_slots=args.slots or wl.hbm_slots)
    images = args.images if args.images >= 0 else (500 if wl.name == "hbert_10k" else 0)
    if images:
        wl = wl.scaled(n_images=images)
    torch.cuda.set_device(0)
    t0 = time.time()
    ids, lens, x = harness.batch_to_device(wl)
    N = int(lens.sum())
    pool = harness.create_pool(wl, max_tokens=N)
    harness.load_tenants(pool, wl, workers=16)
    y = torch.empty_like(x)
    print(f"[bench] {wl.name}: R={len(ids)} N={N} tenants={wl.n_tenants} distinct={len(set(ids.tolist()))} "
          f"image={pool.image_bytes / 1e6:.2f} MB setup={time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    # A pool with a host tier sees a different batch of tenant ids every step (same lengths and
    # hidden states, so N is fixed).  Its requests arrive one by one at the library's request queue,
    # which forms the batches, runs them in order and prefetches the next batch's tenants on the
    # copy stream while the current batch computes (the paper's dispatcher rule, Sec. 4.2, and its
    # coarse-grained pipelining, Sec. 6.2).
    n_batches = args.warmup + 3 * args.steps + 2
    batches = [ids] if not wl.host_tier else [synth.batch_ids_lens(wl, b)[0] for b in range(n_batches)]
    counter = [0]
    queue = None
    if wl.host_tier:
        queue = hmi.Queue(pool, len(ids), N, max_waiting_batches=2)
        off = np.concatenate([[0], np.cumsum(lens)])
        rows = [x[off[r]:off[r + 1]] for r in range(len(ids))]

        def push_batch(b):
            cur = batches[b % len(batches)]
            for r in range(len(cur)):
                assert queue.push(int(cur[r]), rows[r]) is not None

        push_batch(0)

    def step():
        b = counter[0]
        counter[0] += 1
        if wl.host_tier:
            push_batch(b + 1)       # its first request closes batch b, which is full
            queue.run()             # batch b; batch b + 1 is prefetched under it
        else:
            pool.stack_forward(0, wl.n_layers, x, y, ids, lens)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stats0 = pool.stats()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    stats1 = pool.stats()
    ms_per_step = elapsed * 1e3 / args.steps
    ms_per_layer = ms_per_step / wl.n_layers
    tokens_per_s = N / (ms_per_layer * 1e-3)

    # ---- spread of the step time: the same steps once more with an event after each
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    step_ev[0].record()
    for i in range(args.steps):
        step()
        step_ev[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps))
    pct = lambda q: round(per_step[min(len(per_step) - 1, int(q * len(per_step)))], 5)

    # ---- dominant kernel: same steps again with HIP events around every kernel launch
    pool.profile(True)
    for _ in range(args.steps):
        step()
    prof = pool.profile_read()
    pool.profile(False)
    gemm = prof["gemm"]
    gemm_launch_ms = gemm["ms"] / max(gemm["launches"], 1)
    launches_per_step = gemm["launches"] / args.steps
    flops_step = linear_flops_per_token(wl) * N * wl.n_layers
    flops_per_launch = flops_step / launches_per_step
    bf16 = wl.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    achieved = flops_per_launch / (gemm_launch_ms * 1e-3) / 1e12
    traffic, traffic_src = measured_traffic(wl.name)
    roofline = {"bound": "mfma" if bf16 else "alu", "kernel": "grouped_gemm", "achieved": round(achieved, 2),
                "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": traffic, "traffic_source": traffic_src,
                "avg_launch_ms": round(gemm_launch_ms, 5), "launches_per_step": launches_per_step,
                "flop_per_launch": flops_per_launch,
                "kernel_ms_per_step": {k: round(v["ms"] / args.steps, 5) for k, v in prof.items()}}
    if wl.block == synth.BLOCK_ADAPTER and bf16 and wl.n_layers == 1:
        # One fused kernel that moves 4 d bytes per token for 256 d flops per token: bound by HBM.
        # Algorithmic bytes: x in, y out, and each present tenant's image once.
        algo_bytes = 2.0 * N * wl.d_model * 2 + len(set(ids.tolist())) * pool.image_bytes
        gbs = algo_bytes / (gemm_launch_ms * 1e-3) / 1e9
        roofline.update({"bound": "hbm", "kernel": "adapter_fused", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                         "bytes_per_launch": algo_bytes})
        del roofline["flop_per_launch"]

    # ---- per-tenant output heads on the step's result (not part of the step: reported beside it)
    heads = None
    if wl.max_classes:
        scores = torch.empty((N, wl.max_classes), dtype=torch.float32, device="cuda")
        labels = torch.empty((N,), dtype=torch.int32, device="cuda")
        for _ in range(3):
            pool.head_forward(y, scores, labels)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            pool.head_forward(y, scores, labels)
        e1.record()
        torch.cuda.synchronize()
        n_pred = int((labels >= 0).sum().item())
        heads = {"ms_per_call": round(e0.elapsed_time(e1) / args.steps, 5), "predictions": n_pred,
                 "max_classes": wl.max_classes}

    # ---- the paper's whole GPU-side request path on this workload: Aggregate of looked-up tri-gram
    #      representations -> the layer stack -> the tenants' output heads (reported beside the step)
    pipeline = None
    if wl.max_classes and not wl.host_tier:
        entries = 5000
        table = harness.host_to_device(synth.plot_table(wl, entries).reshape(entries * 3, wl.d_model), wl.dtype)
        table = table.reshape(entries, 3, wl.d_model)
        frag = torch.from_numpy(synth.plot_fragment_ids(wl, entries, N)).cuda()
        xin = torch.empty_like(x)

        def request_path():
            pool.plot_aggregate(table, frag, lens, xin)
            pool.stack_forward(0, wl.n_layers, xin, y, ids, lens)
            pool.head_forward(y, None, labels)

        for _ in range(3):
            request_path()
        torch.cuda.synchronize()
        tp = time.perf_counter()
        for _ in range(args.steps):
            request_path()
        torch.cuda.synchronize()
        dtp = (time.perf_counter() - tp) / args.steps
        pipeline = {"what": "aggregate + all layers + heads", "ms_per_batch": round(dtp * 1e3, 4),
                    "requests_per_s": round(len(ids) / dtp, 1), "tokens_per_s": round(N / dtp, 1)}

    # ---- generation: prefill the same batch into a key/value cache, then G steps of one token per request
    decode = None
    if args.decode > 0 and wl.block in (synth.BLOCK_DEC_PRELN, synth.BLOCK_DEC_ADAPTER) and wl.dtype == "bf16":
        G = args.decode
        R = len(ids)
        pool.kv_create(R, int(lens.max()) + G + 3)      # the second (profiled) pass starts again from the prefill
        slots = np.arange(R, dtype=np.int32)
        pool.prefill(0, wl.n_layers, x, y, ids, lens, slots)
        xn = torch.randn((R, wl.d_model), device="cuda").to(x.dtype)
        yn = torch.empty_like(xn)
        for _ in range(3):
            pool.decode_step(0, wl.n_layers, xn, yn, ids, slots)
        torch.cuda.synchronize()
        td = time.perf_counter()
        for _ in range(G):
            pool.decode_step(0, wl.n_layers, xn, yn, ids, slots)
        torch.cuda.synchronize()
        dt = time.perf_counter() - td
        # the same steps again with the library's timing events around every launch (kernel breakdown only)
        pool.prefill(0, wl.n_layers, x, y, ids, lens, slots)
        for _ in range(3):
            pool.decode_step(0, wl.n_layers, xn, yn, ids, slots)
        pool.profile(True)
        for _ in range(G):
            pool.decode_step(0, wl.n_layers, xn, yn, ids, slots)
        torch.cuda.synchronize()
        dprof = pool.profile_read()
        pool.profile(False)
        weight_bytes = len(set(ids.tolist())) * pool.image_bytes * wl.n_layers
        if wl.block == synth.BLOCK_DEC_ADAPTER:   # plus the shared layers, read once per step
            weight_bytes += wl.n_layers * sum(int(np.prod(sh)) for _, sh, _ in synth.shared_specs(wl)) * 2
        kv_bytes = float(lens.sum() + R * (3 + G / 2)) * wl.d_model * 2 * 2 * wl.n_layers
        decode = {"steps": G, "ms_per_step": round(dt * 1e3 / G, 5), "generated_tokens_per_s": round(R * G / dt, 1),
                  "algorithmic_GB_per_step": round((weight_bytes + kv_bytes) / 1e9, 3),
                  "GB_per_s": round((weight_bytes + kv_bytes) / (dt / G) / 1e9, 1),
                  "kernel_ms_per_step": {k: round(v["ms"] / G, 5) for k, v in dprof.items()}}

    # ---- context for roofline.frac: what the vendor's dense GEMM reaches on this machine
    vendor = None
    if args.vendor_gemm and wl.block == synth.BLOCK_FFN and wl.dtype == "bf16":
        def dense_rate(M, Nn, K, zeros=False, reps=30):
            mk = (lambda *sh: torch.zeros(sh, device="cuda", dtype=torch.bfloat16)) if zeros else \
                 (lambda *sh: torch.randn(sh, device="cuda", dtype=torch.float32).mul_(0.5).to(torch.bfloat16))
            a, w, b = mk(M, K), mk(Nn, K), mk(Nn)
            for _ in range(5):
                torch.nn.functional.linear(a, w, b)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                torch.nn.functional.linear(a, w, b)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            return {"M": M, "N": Nn, "K": K, "operands": "zeros" if zeros else "random", "ms": round(ms, 5),
                    "TFLOP/s": round(2.0 * M * Nn * K / (ms * 1e-3) / 1e12, 1),
                    "frac_of_peak": round(2.0 * M * Nn * K / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        vendor = {"what": "torch.nn.functional.linear (hipBLASLt), bf16, bias, dense",
                  "ffn1_shape": dense_rate(N, wl.d_ff, wl.d_model), "ffn2_shape": dense_rate(N, wl.d_model, wl.d_ff),
                  "square_8192": dense_rate(8192, 8192, 8192), "square_8192_zero_operands": dense_rate(8192, 8192, 8192, zeros=True)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same batch
    cpu = None
    if args.cpu_sample > 0:
        from tests.oracle_side import oracle_forward
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        sample = list(range(min(args.cpu_sample, len(ids))))
        tc = time.perf_counter()
        oracle_forward(wl, ids, lens, sample)
        dt = time.perf_counter() - tc
        toks = int(lens[sample].sum()) * wl.n_layers
        cpu = {"value": round(toks / dt, 1), "unit": "tokens/s per layer", "cores": int(cores), "kind": "oracle",
               "sample": f"first {len(sample)} of {len(ids)} requests ({int(lens[sample].sum())} tokens x "
                         f"{wl.n_layers} layers), numpy fp64, {dt:.1f} s incl. regenerating their weights"}

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # one elementwise copy kernel: reads and writes copy_calibration MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- host tier: what the pipelining buys.  The same kind of steps without any prefetch (every miss is
    #      met by the forward call itself), and the prefetch traffic alone (nothing to hide it under).
    tier = None
    if wl.host_tier:
        kernels_ms = sum(v["ms"] for v in prof.values()) / args.steps
        n_probe = max(3, args.steps // 2)
        torch.cuda.synchronize()
        s0 = pool.stats()
        tn = time.perf_counter()
        for i in range(n_probe):
            pool.stack_forward(0, wl.n_layers, x, y, batches[(counter[0] + 2 + i) % len(batches)], lens)
        torch.cuda.synchronize()
        t_noprefetch = (time.perf_counter() - tn) / n_probe
        s1 = pool.stats()
        tcp = time.perf_counter()
        for i in range(n_probe):
            for layer in range(wl.n_layers):
                pool.prefetch(layer, np.unique(batches[(counter[0] + 2 + n_probe + i) % len(batches)]))
        torch.cuda.synchronize()
        t_copy = (time.perf_counter() - tcp) / n_probe
        s2 = pool.stats()
        t_step = ms_per_step * 1e-3
        hidden = max(0.0, t_copy + kernels_ms * 1e-3 - t_step)
        tier = {
            "batches": "requests pushed one by one into the library's queue; a new batch of tenant ids every step; "
                       "next batch prefetched during the current one",
            "hit_rate": round((stats1["hits"] - stats0["hits"]) /
                              max(1, stats1["hits"] - stats0["hits"] + stats1["misses"] - stats0["misses"]), 4),
            "h2d_GB_per_s": round((stats1["bytes_h2d"] - stats0["bytes_h2d"]) / elapsed / 1e9, 2),
            "h2d_MB_per_step": round((stats1["bytes_h2d"] - stats0["bytes_h2d"]) / args.steps / 1e6, 1),
            "without_prefetch": {"hit_rate": round((s1["hits"] - s0["hits"]) / max(1, s1["hits"] - s0["hits"] + s1["misses"] - s0["misses"]), 4),
                                 "ms_per_step": round(t_noprefetch * 1e3, 4),
                                 "h2d_MB_per_step": round((s1["bytes_h2d"] - s0["bytes_h2d"]) / n_probe / 1e6, 1)},
            "copy_alone_ms_per_step": round(t_copy * 1e3, 4),
            "copy_alone_GB_per_s": round((s2["bytes_h2d"] - s1["bytes_h2d"]) / n_probe / max(t_copy, 1e-9) / 1e9, 2),
            "kernels_ms_per_step": round(kernels_ms, 4),
            # share of the shorter of the two (copies, kernels) that runs hidden under the other
            "overlap_fraction": round(hidden / max(min(t_copy, kernels_ms * 1e-3), 1e-9), 3)}

    stats = pool.stats()
    if queue is not None:
        queue.close()
    pool.close()
    # what the parity tests of this workload establish (tests/test_gpu_configs.py, tests/test_gpu_parity.py)
    if wl.dtype != "bf16":
        parity_note = "fp32: every output within 1e-4 of the fp64 oracle"
    elif wl.n_layers >= 6:
        parity_note = ("bf16, six chained layers: rel-Frobenius <= 1e-2 and every |error| <= 2e-2 + half a bf16 unit of the "
                       "reference value; the flat 2e-2 max-abs bar is met by two-layer stacks of the same block and missed "
                       "by up to 3e-3 here at outputs of magnitude 4 and more, where rounding the result to bf16 alone costs 1.6e-2; "
                       "the fp32 result of the same stack (hmi_stack_forward_f32) meets both flat bars")
    else:
        parity_note = "bf16: max-abs <= 2e-2 and rel-Frobenius <= 1e-2 against the fp64 oracle"
    out = {
        "metric": "mixed-tenant tokens/sec per layer; grouped-GEMM TFLOP/s as % of bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_tenants} tenants, {len(ids)} requests, {N} tokens, "
                               f"d={wl.d_model} f={wl.d_ff} heads={wl.n_heads} layers={wl.n_layers}"
                               + (f", {wl.hbm_slots} HBM slots, tenant ids share {wl.n_images} pinned weight sets" if wl.n_images else ""),
                   "block": wl.block, "tenant_popularity": wl.popularity, "distinct_tenants": len(set(ids.tolist()))},
        "ms_per_step_p10_p50_p90": [pct(0.10), pct(0.50), pct(0.90)],
        "step_tflops": round(flops_step / (ms_per_step * 1e-3) / 1e12, 2),
        "step_frac_of_peak": round(flops_step / (ms_per_step * 1e-3) / 1e12 / peak, 4),
        "pool": stats,
        "host_tier": tier,
        "heads": heads,
        "decode": decode,
        "vendor_dense_gemm": vendor,
        "parity_note": parity_note,
        "library_override": os.environ.get("HMI_LIB_PATH") or None,   # set: another build of the library was timed (e.g. an ablation)
        "request_path": pipeline,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
