#!/usr/bin/env python3
"""Benchmark of the GQA decode-attention hot path on one MI355X.

A step is one gqa_decode_attn call (split-KV partial + combine kernels)
on the ragged long-trace batch: B=64, Hq=40, Hkv=8, D=128, KV lengths uniform
on [1024, 16384], head-major bf16 cache, inputs resident in HBM.  Calls
alternate between copies of the cache so that no call finds the previous
call's data in a cache.

Prints one JSON line: metric = KV bytes streamed per second (TB/s), with the
HBM roofline of the split-KV partial kernel (per-kernel time from HIP events
recorded inside the timed region) and the fp64 CPU oracle timed on the host
cores of the same machine.  After these headline keys (timed with exactly
--steps / --warmup) the same line carries, from the same run:
  per_config     all five named configurations (time, TB/s, kernel times, parity, oracle time)
  prefill        causal prefill at 32,768 tokens and on a ragged prompt batch
  shared_prefix  shared-prefix decode at 5 and 10 samples per prompt
--config N times one configuration only (what the rocprofv3 summaries under profiles/ use);
--no-extras prints the headline keys only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
EVENT_STRIDE = 4            # one step in four records HIP events around its kernels
HEADLINE_CONFIG = 2         # the 16K-token ragged batch the target is quoted on


PARTIAL_KERNEL_SOURCES = ("gqa_api.hip", "gqa_internal.h", "gqa_mfma_tile.h", "gqa_partial_mfma.hip")


def measured_traffic(config_index: int):
    """HBM bytes per launch of the partial kernel from the committed counter summary, or None when
    the sources the kernel is built from (its own file, the tile primitives, the shared declarations
    and the launch code) have changed since the counters were taken, when the in-tree library is
    older than those sources, or when GQA_DECODE_LIBRARY selects another build."""
    import hashlib
    if os.environ.get("GQA_DECODE_LIBRARY"):
        return None                 # another build of the library is loaded: the committed counters are not its
    path = os.path.join(ROOT, "profiles", "partial_mfma_kernel_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    h = hashlib.sha256()
    for name in PARTIAL_KERNEL_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2510_07356_amd", "csrc", name), "rb").read())
    if kv.get("source_sha256") != h.hexdigest():
        return None
    lib = os.path.join(ROOT, "paper_2510_07356_amd", "libgqa_decode.so")
    newest = max(os.path.getmtime(os.path.join(ROOT, "paper_2510_07356_amd", "csrc", n)) for n in PARTIAL_KERNEL_SOURCES)
    if not os.path.exists(lib) or os.path.getmtime(lib) < newest:
        return None
    v = kv.get(f"config{config_index}_partial_traffic_bytes")
    return int(v) if v is not None else None


def bench_shared_prefix(args) -> int:
    """Shared-prefix batch (12 prompts x 5 samples): the cascade entry point against the plain
    entry point on the same problem with every sequence holding its own copy of the prefix."""
    import torch
    from paper_2510_07356_amd import binding, workloads
    torch.cuda.set_device(0)
    sw = workloads.make_sampling_batch(tasks=args.tasks, samples=args.samples)
    w = sw.base
    devs = [binding.shared_prefix_to_device(sw) for _ in range(2)]
    d0 = devs[0]
    cp = binding.make_cascade_params(d0["q"], d0["k"], d0["v"], d0["kp"], d0["vp"], w.max_kv_len,
                                     int(sw.prefix_lens.max()), len(sw.prefix_lens), w.scale, 0, None, args.chunk)
    ws = torch.empty(binding.gqa_cascade_workspace_bytes(cp), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((w.batch, w.num_q_heads, w.head_dim), dtype=torch.float32, device="cuda:0")
    lse = torch.empty((w.batch, w.num_q_heads), dtype=torch.float32, device="cuda:0")
    calls = [binding.CascadeCall(cp, d["q"], d["kp"], d["vp"], d["prefix_lens"], d["group_start"], sw.group_start,
                                 d["k"], d["v"], d["kv_lens"], None, out, lse, ws) for d in devs]

    def timed(fns):
        for i in range(args.warmup):
            fns[i % 2]()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fns[i % 2]()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms = timed(calls)
    # the same problem without sharing
    c = sw.concatenated()
    cdevs = [binding.to_device(c) for _ in range(2)]
    pp = binding.make_params(cdevs[0]["q"], cdevs[0]["k"], cdevs[0]["v"], c.max_kv_len, c.scale, 0, None, args.chunk, 0)
    ws2 = torch.empty(binding.gqa_decode_workspace_bytes(pp), dtype=torch.uint8, device="cuda:0")
    out2 = torch.empty_like(out)
    plain = [binding.Call(pp, d["q"], d["k"], d["v"], d["kv_lens"], None, None, out2, None, ws2) for d in cdevs]
    ms_plain = timed(plain)
    calls[0](); plain[0]()
    torch.cuda.synchronize()
    result = {
        "metric": "decode_attn_kv_read_throughput", "unit": "TB/s",
        "value": round(sw.logical_kv_bytes / (ms * 1e-3) / 1e12, 4),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {args.tasks} prompts x {args.samples} samples, shared prefix stored once, "
                               f"Hq={w.num_q_heads} Hkv={w.num_kv_heads} D={w.head_dim}",
                   "logical_kv_bytes": sw.logical_kv_bytes, "physical_kv_bytes": sw.physical_kv_bytes},
        "physical_TBps": round(sw.physical_kv_bytes / (ms * 1e-3) / 1e12, 4),
        "pct_of_hbm_peak_physical": round(100 * sw.physical_kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "unshared_ms_per_step": round(ms_plain, 5),
        "speedup_vs_unshared": round(ms_plain / ms, 4),
        "max_abs_diff_vs_unshared": float((out - out2).abs().max()),
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import shared_prefix_attn
        t0 = time.perf_counter()
        ref = shared_prefix_attn(w.q, sw.kp, sw.vp, sw.prefix_lens, sw.group_start, w.k, w.v, w.kv_lens, w.scale)
        err = out.double().cpu().numpy() - ref.out
        result["parity"] = {"max_abs": float(np.abs(err).max()),
                            "rel_l2": float(np.linalg.norm(err) / np.linalg.norm(ref.out)),
                            "lse_max_abs": float(np.abs(lse.double().cpu().numpy() - ref.lse).max()),
                            "oracle_seconds": round(time.perf_counter() - t0, 3)}
    print(json.dumps(result), flush=True)
    return 0


def bench_prefill(args) -> int:
    """Causal prefill attention with the 32B head shape: one sequence of --seq-len tokens, or with
    --prompts N a padded batch of N prompts whose lengths follow the prompt recipe of the sampling
    batch (lognormal around 1,800 tokens, sigma 0.3)."""
    import numpy as np
    import torch
    from paper_2510_07356_amd import binding
    torch.cuda.set_device(0)
    Hq, Hkv, D = 40, 8, 128
    if args.prompts > 0:
        rng = np.random.default_rng([6, 0])
        lens = np.clip(np.rint(np.exp(np.log(1800.0) + 0.3 * rng.standard_normal(args.prompts))), 16, 8192).astype(np.int32)
        B, T = args.prompts, int(-(-int(lens.max()) // 256) * 256)
        seq_lens = torch.from_numpy(lens).to("cuda:0")
        what = f"causal prefill, {B} prompts of {int(lens.min())}-{int(lens.max())} tokens (sum {int(lens.sum())}) padded to {T}"
    else:
        B, T = 1, args.seq_len
        lens, seq_lens = np.array([T], dtype=np.int64), None
        what = f"causal prefill, one sequence of {T} tokens"
    g = torch.Generator(device="cuda:0").manual_seed(11)
    q = torch.randn((B, T, Hq, D), generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((B, T, Hkv, D), generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((B, T, Hkv, D), generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty((B, T, Hq, D), dtype=torch.float32, device="cuda:0")
    scale = float(np.float32(1.0 / np.sqrt(D)))
    for _ in range(args.warmup):
        binding.gqa_prefill_attn(q, k, v, scale, out, seq_lens=seq_lens)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        binding.gqa_prefill_attn(q, k, v, scale, out, seq_lens=seq_lens)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    L = lens.astype(np.float64)
    flops = float((4.0 * D * Hq * L * (L + 1) / 2.0).sum())   # two matrix products over the causal half
    tflops = flops / (ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "causal_prefill_attention_throughput", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{what}, Hq={Hq} Hkv={Hkv} D={D}", "flops": flops},
        "tokens_per_s": round(float(L.sum()) / (ms * 1e-3), 1),
        "roofline": {"kernel": "prefill_kernel", "bound": "mfma", "achieved": round(tflops, 2), "peak": 2500.0,
                     "unit": "TFLOP/s", "frac": round(tflops / 2500.0, 4), "traffic": None},
    }), flush=True)
    return 0


PROBE_MODES = {0: "non-temporal, 1 KB per load instruction (V path), 1 tile in flight",
               1: "non-temporal, operand-shaped 16 rows x 64 B (K path), 1 tile in flight",
               2: "non-temporal, 1 KB per load, then through LDS (ds_write_b128 + operand-shaped ds_read_b128)",
               3: "ordinary loads, operand-shaped, 1 tile in flight",
               4: "non-temporal, operand-shaped, 2 tiles in flight",
               5: "non-temporal, 1 KB per load, 2 tiles in flight",
               6: "non-temporal, the kernel's mix: half operand-shaped (K), half 1 KB per load (V), 1 tile in flight",
               7: "ordinary loads, the kernel's mix, 1 tile in flight",
               8: "non-temporal, the kernel's mix, the 4 wavefronts of a workgroup take the tiles of its run in turn",
               9: "non-temporal, the kernel's mix, all wavefronts take tiles in turn (chip-wide sweep)"}


def bench_probe(args) -> int:
    """Access-pattern probe (gqa_decode_stream_probe) over a buffer of the headline batch's K/V size:
    every mode at one wavefront per SIMD, then the kernel's own mix at 1 to 16 wavefronts per CU."""
    import torch
    from paper_2510_07356_amd import binding
    torch.cuda.set_device(0)
    nbytes = 2_408_591_360 // 16384 * 16384
    bufs = [torch.full((nbytes,), 1, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    sink = torch.empty(4 * 4096, dtype=torch.int32, device="cuda:0")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(workgroups, mode):
        ts = []
        for i in range(args.warmup + args.steps):
            ev0.record()
            binding.gqa_decode_stream_probe(bufs[i % 2], sink, workgroups, mode)
            ev1.record()
            ev1.synchronize()
            if i >= args.warmup:
                ts.append(ev0.elapsed_time(ev1))
        ts.sort()
        return {"best_us": round(ts[0] * 1e3, 1), "median_us": round(ts[len(ts) // 2] * 1e3, 1),
                "median_GBps": round(nbytes / ts[len(ts) // 2] / 1e6, 1)}

    rows = []
    for mode in sorted(PROBE_MODES):
        rows.append({"mode": mode, "what": PROBE_MODES[mode], "workgroups": 256, "wavefronts_per_cu": 4, **timed(256, mode)})
    for wgs in (64, 128, 512, 768, 1024):
        rows.append({"mode": 6, "what": PROBE_MODES[6], "workgroups": wgs, "wavefronts_per_cu": wgs // 64, **timed(wgs, 6)})
    print(json.dumps({"metric": "stream_probe_read_throughput", "unit": "GB/s", "bytes_per_launch": nbytes,
                      "steps": args.steps, "warmup": args.warmup, "rows": rows}), flush=True)
    return 0


def bench_decode_step(args) -> int:
    """One decode step of an L-layer model on the ragged 64-sequence batch with a paged cache: per
    layer the new token's K/V are appended (rotary included) and attention runs over that layer's
    cache.  All layers' caches stay resident (L x 2.4 GB), the step is captured once in a HIP graph
    and replayed; layer 0 is checked against the oracle."""
    import numpy as np
    import torch
    from paper_2510_07356_amd import binding, workloads
    torch.cuda.set_device(0)
    L = args.layers
    lens = workloads.ragged_lengths(2, 64, 1024, 16384)          # the lengths of the headline batch
    w = workloads.make_paged("ragged_b64_1k_16k_paged", 2, 64, 40, 8, lens, table_width=16384 // workloads.PAGE)
    base = binding.to_device(w)
    free, _ = torch.cuda.mem_get_info()
    need = (L - 1) * 2 * base["k"].numel() * 2
    if need > free - (8 << 30):
        print(f"bench.py: {L} layers need {need / 2**30:.0f} GiB of cache, {free / 2**30:.0f} GiB free", file=sys.stderr)
        return 2
    # the other layers hold the same values in memory of their own (the values do not matter for the timing)
    layers = [base] + [dict(base, k=base["k"].clone(), v=base["v"].clone()) for _ in range(L - 1)]
    positions = int(w.max_kv_len)
    d = np.arange(64, dtype=np.float64)
    ang = np.arange(positions, dtype=np.float64)[:, None] * 1.0e6 ** (-2.0 * d / 128)[None, :]
    table = np.concatenate([np.cos(ang), np.sin(ang)], axis=1).astype(np.float32)
    cs = torch.from_numpy(table).to("cuda:0")
    g = torch.Generator(device="cuda:0").manual_seed(12)
    q_in = base["q"]
    k_new = torch.randn((64, 8, 128), generator=g, device="cuda:0").to(torch.bfloat16)
    v_new = torch.randn((64, 8, 128), generator=g, device="cuda:0").to(torch.bfloat16)
    q_rot = torch.empty_like(q_in)
    params = binding.make_params(q_rot, base["k"], base["v"], positions, w.scale, w.page_size, base["block_table"], 0, 0)
    ws = torch.empty(binding.gqa_decode_workspace_bytes(params), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((64, 40, 128), dtype=torch.float32, device="cuda:0")

    def step():
        for lay in layers:
            binding.gqa_decode_kv_append(q_in, q_rot, k_new, v_new, lay["k"], lay["v"], base["kv_lens"], positions,
                                         base["block_table"], w.page_size, cs)
            binding.gqa_decode_attn(params, q_rot, lay["k"], lay["v"], base["kv_lens"], base["block_table"], None,
                                    out, None, ws)

    step()                                                        # eager once: device properties are cached
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kv_bytes = L * w.kv_bytes
    result = {
        "metric": "decode_step_kv_read_throughput", "value": round(kv_bytes / (ms * 1e-3) / 1e12, 4), "unit": "TB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{L} layers x (KV append with rotary + attention) on {w.name}: B=64 Hq=40 Hkv=8 D=128 "
                               f"kv_tokens={w.kv_tokens} per layer, paged, one HIP graph per step",
                   "layers": L, "resident_cache_bytes": L * 2 * base["k"].numel() * 2, "kv_bytes_per_step": kv_bytes},
        "pct_of_hbm_peak": round(100.0 * kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "ms_per_step_eager_launches": round(eager_ms, 4),
        "tokens_per_s_attention_only": round(64 / (ms * 1e-3), 1),
    }
    if not args.no_cpu_baseline:
        from oracle import decode_attn, kv_append
        kn = k_new.view(torch.int16).cpu().numpy().view(np.uint16)
        vn = v_new.view(torch.int16).cpu().numpy().view(np.uint16)
        q_ref = kv_append(w.q, kn, vn, w.k, w.v, w.kv_lens, cos_sin=table, block_table=w.block_table, page_size=w.page_size)
        ref = decode_attn(q_ref, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)
        binding.gqa_decode_kv_append(q_in, q_rot, k_new, v_new, base["k"], base["v"], base["kv_lens"], positions,
                                     base["block_table"], w.page_size, cs)
        binding.gqa_decode_attn(params, q_rot, base["k"], base["v"], base["kv_lens"], base["block_table"], None, out, None, ws)
        torch.cuda.synchronize()
        err = out.double().cpu().numpy() - ref.out
        result["parity"] = {"max_abs": float(np.abs(err).max()), "rel_l2": float(np.linalg.norm(err) / np.linalg.norm(ref.out))}
    print(json.dumps(result), flush=True)
    return 0


def host_cpu_description() -> str:
    """Model name of the host processor, the cores this process may run on and the cores the machine has."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    allowed = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    return f"{model}; {allowed} of {os.cpu_count()} cores available to this process"


def run_decode_config(index, steps, warmup, args, with_cpu=True, with_stream_read=False, events_every=EVENT_STRIDE):
    """Times gqa_decode_attn on one named configuration.  Returns (summary dict, details dict): the
    summary is the per-configuration entry of the JSON line, the details feed the headline keys."""
    import numpy as np
    import torch
    from paper_2510_07356_amd import binding, workloads
    w = workloads.make_config(index, layout=args.layout)
    if args.page_size > 0 and w.page_size == 0:
        # the same lengths and shape as a paged cache with a randomly permuted pool (what paging costs)
        width = -(-int(w.k.shape[2]) // args.page_size)
        w = workloads.make_paged(f"{w.name}_paged{args.page_size}", index, w.batch, w.num_q_heads, w.num_kv_heads,
                                 w.kv_lens, table_width=width, page_size=args.page_size, layout=args.layout)
    # rotate over enough copies of the cache that repeated calls cannot be served from the 256 MB
    # last-level cache or from L2: copies x K/V bytes >= 1 GiB
    copies = args.copies if args.copies > 0 else max(2, -(-(1 << 30) // max(w.kv_bytes, 1)))
    copies = min(copies, 1024)
    devs = [binding.to_device(w) for _ in range(copies)]
    params = binding.make_params(devs[0]["q"], devs[0]["k"], devs[0]["v"], w.max_kv_len, w.scale,
                                 w.page_size, devs[0]["block_table"], args.chunk, args.variant)
    host_lens = None if args.no_host_lens else w.kv_lens
    plan = binding.gqa_decode_plan_info(params, host_lens)
    ws = torch.empty(binding.gqa_decode_workspace_bytes(params), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((w.batch, w.num_q_heads, w.head_dim), dtype=torch.float32, device="cuda:0")
    lse = torch.empty((w.batch, w.num_q_heads), dtype=torch.float32, device="cuda:0")
    calls = [binding.Call(params, d["q"], d["k"], d["v"], d["kv_lens"], d["block_table"], host_lens,
                          out, lse, ws) for d in devs]
    timer = binding.Timer(steps)

    # the streaming-read ceiling over the same K buffer, measured first and for about 50 ms: the input generation
    # above ran on the host, and the chip needs some tens of milliseconds of work to reach the clocks it then
    # sustains (with 5 warm-up calls alone the first 20 calls of the headline batch read 2 % slower than later ones)
    stream_read_GBps = None
    if with_stream_read:
        kflat = devs[0]["k"].untyped_storage()
        src = torch.empty(0, dtype=torch.uint8, device="cuda:0").set_(kflat)
        sink = torch.empty(1 << 16, dtype=torch.int32, device="cuda:0")
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best, spent = float("inf"), 0.0
        while spent < 50.0:                                  # milliseconds of probe time
            ev0.record()
            binding.gqa_decode_stream_read(src, sink, 8192)
            ev1.record()
            ev1.synchronize()
            ms = ev0.elapsed_time(ev1)
            best, spent = min(best, ms), spent + max(ms, 0.01)
        stream_read_GBps = src.numel() / best / 1e6

    for i in range(warmup):
        calls[i % copies]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        # every events_every-th step carries the event records around its kernels
        calls[i % copies](timer if i % events_every == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    partial_calls, combine_calls = timer.read_calls(steps)
    timer.close()
    n_timed = len(partial_calls)
    assert n_timed == (steps + events_every - 1) // events_every
    ms_per_step = (t1 - t0) * 1e3 / steps
    partial_avg_ms, combine_avg_ms = sum(partial_calls) / n_timed, sum(combine_calls) / n_timed

    kv_bytes = w.kv_bytes
    value = kv_bytes / (ms_per_step * 1e-3) / 1e12
    achieved = kv_bytes / (partial_avg_ms * 1e-3) / 1e9
    summary = {
        "config": index, "name": w.name, "kv_bytes": kv_bytes, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "TBps": round(value, 4),
        "pct_of_hbm_peak": round(100.0 * value * 1e3 / HBM_PEAK_GBPS, 2),
        "sequences_per_s": round(w.batch / (ms_per_step * 1e-3), 1),
        "partial_kernel_us": round(partial_avg_ms * 1e3, 2), "combine_kernel_us": round(combine_avg_ms * 1e3, 2),
        "partial_kernel_frac_of_hbm_peak": round(achieved / HBM_PEAK_GBPS, 4),
        "cache_copies_rotated": copies,
    }
    if copies * kv_bytes < (1 << 30):
        summary["note"] = "copies x K/V bytes < 1 GiB: may be served from the last-level cache, not an HBM figure"
    elif kv_bytes < (64 << 20):
        summary["note"] = "launch-bound: the call is a few microseconds of traffic"
    details = {"w": w, "plan": plan, "copies": copies, "ms_per_step": ms_per_step, "value": value,
               "partial_calls": partial_calls, "partial_avg_ms": partial_avg_ms, "combine_avg_ms": combine_avg_ms,
               "n_timed": n_timed, "achieved": achieved}
    if stream_read_GBps is not None:
        details["stream_read_GBps"] = stream_read_GBps

    if with_cpu:
        from oracle import decode_attn
        reps, t_cpu_total = 0, 0.0
        while t_cpu_total < args.cpu_seconds and reps < 50:     # bounded wall time on all host cores
            t3 = time.perf_counter()
            ref = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)
            t_cpu_total += time.perf_counter() - t3
            reps += 1
        t_cpu = t_cpu_total / reps
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        calls[0]()
        torch.cuda.synchronize()
        got = out.double().cpu().numpy()
        err = got - ref.out
        live = w.kv_lens > 0
        summary["parity"] = {"max_abs": float(np.abs(err).max()),
                             "rel_l2": float(np.linalg.norm(err) / np.linalg.norm(ref.out)),
                             "lse_max_abs": float(np.abs(lse.double().cpu().numpy()[live] - ref.lse[live]).max()),
                             "finite": bool(np.isfinite(got).all())}
        summary["oracle_seconds"] = round(t_cpu, 4)
        summary["oracle_threads"] = ref.threads
        details.update(ref_threads=ref.threads, t_cpu=t_cpu, reps=reps)
    del calls, devs, ws
    torch.cuda.empty_cache()
    return summary, details


def prefill_block(args):
    """Causal prefill at 32,768 tokens and on a ragged batch of 64 prompts: TFLOP/s against the bf16 matrix peak."""
    import io
    import contextlib
    blocks = {}
    for key, extra in (("causal_32768", dict(seq_len=32768, prompts=0, steps=5, warmup=2)),
                       ("ragged_64_prompts", dict(seq_len=0, prompts=64, steps=10, warmup=2))):
        sub = argparse.Namespace(**{**vars(args), **extra})
        buf = io.StringIO()
        with contextlib.redirect_stdout(buf):
            bench_prefill(sub)
        d = json.loads(buf.getvalue().strip().splitlines()[-1])
        blocks[key] = {"workload": d["config"]["workload"], "steps": d["steps"], "ms_per_step": d["ms_per_step"],
                       "TFLOPps": d["value"], "frac_of_mfma_peak": d["roofline"]["frac"],
                       "tokens_per_s": d["tokens_per_s"]}
    return blocks


def shared_prefix_block(args):
    """Shared-prefix decode on the two sampling batches of the paper (5 and 10 samples per prompt)."""
    import io
    import contextlib
    blocks = {}
    for key, extra in (("12_prompts_x_5_samples", dict(tasks=12, samples=5, steps=100, warmup=10)),
                       ("6_prompts_x_10_samples", dict(tasks=6, samples=10, steps=100, warmup=10))):
        sub = argparse.Namespace(**{**vars(args), **extra})
        buf = io.StringIO()
        with contextlib.redirect_stdout(buf):
            bench_shared_prefix(sub)
        d = json.loads(buf.getvalue().strip().splitlines()[-1])
        blocks[key] = {"workload": d["config"]["workload"], "steps": d["steps"], "ms_per_step": d["ms_per_step"],
                       "physical_kv_bytes": d["config"]["physical_kv_bytes"],
                       "logical_kv_bytes": d["config"]["logical_kv_bytes"],
                       "physical_TBps": d["physical_TBps"], "frac_of_hbm_peak_physical": round(d["pct_of_hbm_peak_physical"] / 100, 4),
                       "unshared_ms_per_step": d["unshared_ms_per_step"], "speedup_vs_unshared": d["speedup_vs_unshared"],
                       "parity": d.get("parity")}
    return blocks


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=None,
                    help="index into the five named configurations: time only that one (default: the ragged "
                         "16K batch as the headline, then every configuration, prefill and shared prefix)")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline configuration only: no per-configuration, prefill and shared-prefix blocks")
    ap.add_argument("--chunk", type=int, default=0, help="KV tokens per share (0 = one share per workgroup)")
    ap.add_argument("--variant", type=int, default=0, help="0 = matrix-core kernel, 1 = vector-ALU kernel")
    ap.add_argument("--layout", default="head_major")
    ap.add_argument("--page-size", type=int, default=0,
                    help="run a contiguous configuration's lengths on a paged cache with this page size instead")
    ap.add_argument("--no-host-lens", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=1.5, help="wall time the oracle is repeated for, per configuration")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MIB",
                    help="also run the plain copy kernel over this many MiB, three times (counter scaling in profiles)")
    ap.add_argument("--no-stream-read", action="store_true", help="skip the streaming-read probe over one cache copy")
    ap.add_argument("--shared-prefix", action="store_true",
                    help="benchmark the shared-prefix entry point on a tasks x samples batch instead")
    ap.add_argument("--prefill", action="store_true", help="benchmark causal prefill attention instead")
    ap.add_argument("--seq-len", type=int, default=32768)
    ap.add_argument("--prompts", type=int, default=0, help="with --prefill: a ragged batch of this many prompts instead")
    ap.add_argument("--decode-step", action="store_true",
                    help="benchmark one graph-captured decode step of --layers layers (append + attention per layer)")
    ap.add_argument("--layers", type=int, default=64)
    ap.add_argument("--probe", action="store_true",
                    help="time the access-pattern probe (the evidence behind the partial kernel's load path) instead")
    ap.add_argument("--tasks", type=int, default=12)
    ap.add_argument("--samples", type=int, default=5)
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = enough for 1 GiB)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU; --gpus N with N > 1 is not supported "
              "(sequences and KV heads would shard across GPUs with no exchange)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2510_07356_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.shared_prefix:
        return bench_shared_prefix(args)
    if args.prefill:
        return bench_prefill(args)
    if args.decode_step:
        return bench_decode_step(args)
    if args.probe:
        return bench_probe(args)
    torch.cuda.set_device(0)
    binding.gqa_decode_init()
    headline = HEADLINE_CONFIG if args.config is None else args.config
    extras = args.config is None and not args.no_extras
    summary, d = run_decode_config(headline, args.steps, args.warmup, args, with_cpu=not args.no_cpu_baseline,
                                   with_stream_read=not args.no_stream_read)
    w, plan = d["w"], d["plan"]
    kv_bytes, value, ms_per_step = w.kv_bytes, d["value"], d["ms_per_step"]

    result = {
        "metric": "decode_attn_kv_read_throughput",
        "value": round(value, 4),
        "unit": "TB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name} (configs[{headline}]): B={w.batch} Hq={w.num_q_heads} Hkv={w.num_kv_heads} "
                        f"D={w.head_dim} kv_tokens={w.kv_tokens} {'paged' if w.page_size else 'contiguous'} "
                        f"{w.layout} bf16 cache",
            "kv_bytes_per_step": kv_bytes,
            "share_tokens": plan.share_tokens,
            "workgroups": plan.workgroups,
            "kernel_variant": args.variant,
            "cache_copies_rotated": d["copies"],
        },
        "pct_of_hbm_peak": round(100.0 * value * 1e3 / HBM_PEAK_GBPS, 2),
        # everything a call moves: K/V once, Q, the output, and the partial results written by the partial
        # kernel and read back by the combine kernel (at most one piece per wavefront plus one per row)
        "bytes_incl_q_out_partials": int(kv_bytes + w.batch * w.num_q_heads * w.head_dim * (2 + 4) + w.batch * w.num_q_heads * 4
                                         + 2 * (plan.workgroups * 4 + w.batch * w.num_kv_heads)
                                         * (w.num_q_heads // w.num_kv_heads) * (w.head_dim + 2) * 4),
        "sequences_per_s": round(w.batch / (ms_per_step * 1e-3), 1),
        # derived: attention-only bound on generated tokens/s if a 64-layer model made this call per layer
        "derived_tokens_per_s_64_layers": round(w.batch / (64 * ms_per_step * 1e-3), 1),
        "kernel_ms": {"partial": round(d["partial_avg_ms"], 5),
                      "partial_median": round(float(np.median(d["partial_calls"])), 5),
                      "partial_min": round(min(d["partial_calls"]), 5),
                      "combine": round(d["combine_avg_ms"], 5), "launches_timed": d["n_timed"]},
        "roofline": {
            "kernel": "partial_mfma_kernel" if args.variant == 0 else "partial_valu_kernel",
            "bound": "hbm",
            "achieved": round(d["achieved"], 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(d["achieved"] / HBM_PEAK_GBPS, 4),
            "traffic": measured_traffic(headline) if (args.variant == 0 and args.chunk == 0 and args.page_size == 0
                                                     and args.layout == "head_major") else None,
        },
    }

    if args.calibration_copy > 0:
        n = args.calibration_copy << 20
        src = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.gqa_decode_stream_copy(src, dst, 4096)
        torch.cuda.synchronize()
        result["calibration_copy_bytes"] = n
        del src, dst
    if "stream_read_GBps" in d:
        result["stream_read_probe_GBps"] = round(d["stream_read_GBps"], 1)
        result["pct_of_stream_read_probe"] = round(100.0 * value * 1e3 / d["stream_read_GBps"], 2)

    if not args.no_cpu_baseline:
        from oracle import decode_attn
        t4 = time.perf_counter()
        decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size, threads=1)
        t_one = time.perf_counter() - t4
        result["cpu_baseline"] = {
            "value": round(kv_bytes / d["t_cpu"] / 1e12, 6),
            "unit": "TB/s",
            "cores": d["ref_threads"],
            "kind": "oracle",
            "sample": f"the whole workload ({w.batch} sequences, {w.kv_tokens} KV tokens), mean of {d['reps']} runs, "
                      f"{d['t_cpu']:.3f} s wall each on {d['ref_threads']} threads; one run on a single thread: {t_one:.2f} s",
            "single_thread_value": round(kv_bytes / t_one / 1e12, 6),
            "gpu_over_cpu": round(d["t_cpu"] / (d["ms_per_step"] * 1e-3), 1),
            "host": host_cpu_description(),
        }
        result["parity"] = summary["parity"]

    if extras:
        # every named configuration with its own step count (the headline keys above keep --steps / --warmup),
        # then the two neighbouring workloads; all inside this one run so that one clock covers them
        del w, d
        per_config = []
        for i in range(5):
            inner_steps = 400 if i == 0 else 200
            s_i, _ = run_decode_config(i, inner_steps, 20, args, with_cpu=not args.no_cpu_baseline, events_every=2)
            per_config.append(s_i)
        result["per_config"] = per_config
        result["prefill"] = prefill_block(args)
        result["shared_prefix"] = shared_prefix_block(args)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
