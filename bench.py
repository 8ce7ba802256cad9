#!/usr/bin/env python3
"""Decode-step benchmark: KV append + paged GQA decode on one MI355X.

One step = one pass of the whole hot path (append, split-K plan, attention, merge) over one
batch of synthetic streams, through ``vox_decode_step``; 28 layers in sequence for the
small-backbone preset.  Prints ONE JSON line.

  value      KV-cache bytes of valid tokens read per second (GB/s), inputs resident in HBM
  roofline   the attention kernel alone: same bytes / its mean duration from HIP events
             recorded around it on the launch stream in a second timed region
  cpu_baseline  the fp64 oracle timed on the host cores over a bounded sample of the streams
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix-core rate
MULTI_WORKLOADS = ("chunk15", "chunk25", "chunk28", "prefill", "admit")
# sampling step: name -> (streams, vocabulary, settings of synth.SAMPLING_PRESETS)
SAMPLE_WORKLOADS = {"sample_small": (1024, 6564, "cosyvoice"), "sample_large": (256, 156940, "orpheus")}
METRIC = "decode-step KV GB/s & % HBM peak; stream-steps/sec at 256 streams"

def measured_traffic(workload: str):
    """HBM bytes per launch of the workload's dominant kernel, as the rocprofv3 --pmc runs
    summarised under profiles/ measured them (FETCH_SIZE, then WRITE_SIZE, each scaled by what the
    same counter reads for a plain 1 GiB device copy).  Read from the summary whose first line
    names the workload; None when there is none."""
    import glob
    import re

    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        try:
            text = open(path).read()
        except OSError:
            continue
        first = text.split("\n", 1)[0]
        if not re.search(rf"workload {re.escape(workload)}\b", first):
            continue
        m = re.search(r"traffic = (\d+) bytes per launch", text)
        if m:
            return int(m.group(1))
    return None


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def bench_multi(args, dev, emit=True):
    """Multi-token step (append of n_s new tokens per stream + causal paged attention).

    Algorithmic work per step: every context token's K and V read once per kv head
    (sum L_s * kappa bytes) and 4*Hq*D flops per (query row, visible token) pair; the roofline
    entry names whichever bound takes longer at the chip's peaks.
    """
    import copy

    import numpy as np
    import torch

    from paper_2602_00269_amd import binding, synth

    m = synth.make_multi_workload(args.workload, device=dev)
    base = m.base
    kv_bytes = base.kv_bytes_per_layer
    lens64, n64 = base.context_lens.astype(np.int64), m.new_tokens.astype(np.int64)
    pairs = int((n64 * (lens64 - n64) + n64 * (n64 + 1) // 2).sum())  # (row, visible token)
    flops = 4 * base.num_q_heads * base.head_dim * pairs
    copies = args.pool_copies
    if copies is None:
        copies = 1 if kv_bytes >= (1 << 30) else int(min(16, -(-(1 << 30) // max(1, kv_bytes))))
    pools = [(base.k_pool[0], base.v_pool[0])]
    for _ in range(1, copies):
        pools.append((base.k_pool[0].clone(), base.v_pool[0].clone()))
    sh = binding.shape_of(base, split_waves=args.split_waves)
    bt = torch.from_numpy(base.block_tables).to(dev)
    lens = torch.from_numpy(base.context_lens).to(dev)
    qo = torch.from_numpy(m.q_offsets).to(dev)
    tq = m.total_q
    ws = torch.empty(binding.paged_prefill_workspace_bytes(sh, tq), dtype=torch.uint8, device=dev)
    out = torch.zeros((tq, base.num_q_heads, base.head_dim), device=dev)

    def step(i, events=None):
        kp, vp = pools[i % copies]
        binding.kv_append_multi(sh, m.k_new, m.v_new, kp, vp, bt, lens, qo)
        binding.paged_prefill(sh, m.q, kp, vp, bt, lens, qo, base.context_lens, m.q_offsets, out,
                              ws, events=events)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9

    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    for a, b in evs:
        a.record()
        b.record()
    torch.cuda.synchronize()
    for i in range(args.steps):
        step(i, events=evs[i])
    torch.cuda.synchronize()
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    t_hbm, t_mfma = kv_bytes / (HBM_PEAK_GBPS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if t_mfma > t_hbm:
        ach = flops / (kern_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4)}
    else:
        ach = kv_bytes / (kern_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4)}
    # a batch with many single-token streams runs those through the decode kernel: the events
    # then enclose both attention kernels
    singles = int((n64 == 1).sum())
    single_steps = int(((lens64[n64 == 1] + 31) // 32).sum()) * base.num_kv_heads
    kernels = "decode_kernel<MqMath>"
    if singles >= 32 and single_steps >= 32768:  # the library's rule for splitting a batch
        kernels = "decode_kernel<MfmaMath>" + (" + decode_kernel<MqMath>" if (n64 > 1).any() else "")
    roofline.update({"kernel": kernels, "kernel_ms": round(kern_ms, 4),
                     "bytes_per_launch": kv_bytes, "flops_per_launch": flops,
                     "traffic": measured_traffic(m.name)})

    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        def bits(t):
            return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

        qb, kp, vp = bits(m.q), bits(base.k_pool[0]), bits(base.v_pool[0])

        def run(n):  # the first n streams: their tables, lengths and packed query rows
            t = time.perf_counter()
            oracle.paged_prefill(qb[: m.q_offsets[n]], kp, vp, base.block_tables[:n],
                                 base.context_lens[:n], m.q_offsets[: n + 1], base.scale,
                                 num_kv_heads=base.num_kv_heads)
            return time.perf_counter() - t

        probe_n = min(base.num_streams, 2)
        probe_t = run(probe_n)
        # the oracle's cost follows the (row, token) pairs, not the context bytes
        ppairs = (n64 * (lens64 - n64) + n64 * (n64 + 1) // 2)
        cum = np.cumsum(ppairs)
        rate = cum[probe_n - 1] / max(probe_t, 1e-6)
        n = int(np.searchsorted(cum, rate * args.cpu_seconds) + 1)
        n = max(probe_n, min(base.num_streams, n))
        secs = run(n)
        toks = int(lens64[:n].sum())
        cpu = {
            "value": round(toks * base.kv_bytes_per_token / secs / 1e9, 4),
            "unit": "GB/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"fp64 oracle multi-token attention of streams [0,{n}) of "
                      f"{base.num_streams} ({toks} context tokens, {int(m.q_offsets[n])} query "
                      f"rows), 1 pass in {secs:.2f} s",
            "cpu_model": cpu_model(),
            "host_cpus": os.cpu_count(),
        }

    line = {
        "metric": "multi-token step context KV GB/s (each context byte counted once)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": m.name,
            "streams": base.num_streams,
            "q_heads": base.num_q_heads,
            "kv_heads": base.num_kv_heads,
            "head_dim": base.head_dim,
            "layers": 1,
            "total_tokens": base.total_tokens,
            "query_rows": tq,
            "kv_bytes_per_step": kv_bytes,
            "flops_per_step": flops,
            "pool_copies": copies,
            "split_waves": args.split_waves,
        },
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if emit:
        print(json.dumps(line))
        return 0
    return line


def bench_sample(args, dev, emit=True):
    """Sampling step: one launch turns fp32 logits [S, V] into S tokens.  Algorithmic bytes: the
    logits once (S * V * 4); the kernel is one workgroup per stream."""
    import numpy as np
    import torch

    from paper_2602_00269_amd import binding, synth

    s, v, preset = SAMPLE_WORKLOADS[args.workload]
    temperature, top_p, top_k, penalty = synth.SAMPLING_PRESETS[preset]
    window = 64
    copies = 4  # distinct logits so that a small batch cannot sit in the caches
    logits = [synth.make_logits(s, v, seed=0x5EED0200 + c, device=dev) for c in range(copies)]
    hist_h = synth.make_history(s, v, window, seed=0x5EED0210)
    u_h = synth.make_uniforms(s, seed=0x5EED0211)
    hist, u = torch.from_numpy(hist_h).to(dev), torch.from_numpy(u_h).to(dev)
    prm = binding.sampling_params(temperature, top_p, penalty, top_k, s, dev)
    tokens = torch.zeros(s, dtype=torch.int32, device=dev)

    def step(i):
        binding.sample(logits[i % copies], prm, u, tokens, history=hist)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    for i, (a, b) in enumerate(evs):  # the launch goes to torch's current stream
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    nbytes = s * v * 4
    ach = nbytes / (kern_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "sample_kernel", "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                "kernel_ms": round(kern_ms, 4), "bytes_per_launch": nbytes,
                "traffic": measured_traffic(f"{args.workload}_{s}x{v}")}
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        host = logits[0].cpu().numpy()
        prm_o = oracle.sampling_params(temperature, top_p, penalty, top_k, s)
        n = min(s, 4)
        t = time.perf_counter()
        oracle.sample(host[:n], prm_o[:n], u_h[:n], history=hist_h[:n])
        rate = n / max(time.perf_counter() - t, 1e-6)
        n = int(max(n, min(s, rate * args.cpu_seconds)))
        t = time.perf_counter()
        oracle.sample(host[:n], prm_o[:n], u_h[:n], history=hist_h[:n])
        secs = time.perf_counter() - t
        cpu = {"value": round(n / secs, 1), "unit": "tokens/s", "cores": 1, "kind": "oracle",
               "sample": f"oracle sampling of streams [0,{n}) of {s} (vocabulary {v}), 1 pass in "
                         f"{secs:.2f} s", "cpu_model": cpu_model(), "host_cpus": os.cpu_count()}
    line = {
        "metric": "sampled tokens/s (one launch per batch of streams)",
        "value": round(s / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}_{s}x{v}", "streams": s, "vocab": v,
                   "settings": preset, "temperature": temperature, "top_p": top_p, "top_k": top_k,
                   "repetition_penalty": penalty, "window": window, "logit_sets": copies},
        "logits_gbps": round(nbytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if emit:
        print(json.dumps(line))
        return 0
    return line


def bench_decode(args, dev, workload, full=True, layerwise=False):
    """One decode-step workload: region A times the whole step through the production entry
    point (wall clock over all steps for the mean, HIP events between the steps for the median),
    region B the attention kernel alone between HIP events.  ``full`` adds the wave clocks, the
    read-ceiling probe and the CPU baseline and returns the whole bench line; otherwise a short
    record for the ``also`` list.  ``layerwise``: the step as a backbone would issue it, one plan
    and then one call per layer (vox_decode_plan + vox_decode_layer), instead of vox_decode_step,
    whose launches carry the neighbouring layer's append."""
    import copy

    import numpy as np
    import torch

    from paper_2602_00269_amd import binding, synth

    path = {"auto": binding.PATH_AUTO, "mfma": binding.PATH_MFMA, "valu": binding.PATH_VALU}[args.path]
    cfg = int(workload[3:])

    # ---- workload(s): distinct pool sets so small presets cannot live in the 256 MB cache
    base = synth.make_workload(cfg, device=dev, layers=args.layers)
    kv_bytes_layer = base.kv_bytes_per_layer
    copies = args.pool_copies
    if copies is None:
        copies = 1 if kv_bytes_layer * base.layers >= (1 << 30) else \
            int(min(16, -(-(1 << 30) // max(1, kv_bytes_layer * base.layers))))
    sets = [base]
    for _ in range(1, copies):  # same streams and tables, pool contents copied to fresh memory
        w = copy.copy(base)
        w.k_pool = [t.clone() for t in base.k_pool]
        w.v_pool = [t.clone() for t in base.v_pool]
        sets.append(w)
    sh = binding.shape_of(base, decode_path=path, split_waves=args.split_waves)
    bt = torch.from_numpy(base.block_tables).to(dev)
    lens = torch.from_numpy(base.context_lens).to(dev)
    host_lens = base.context_lens if args.host_lens else None
    ws = binding.alloc_workspace(sh, dev)
    outs = [[torch.zeros((base.num_streams, base.num_q_heads, base.head_dim), device=dev)
             for _ in range(base.layers)] for _ in sets]
    step_args = [binding.StepArgs(w.q, w.k_new, w.v_new, w.k_pool, w.v_pool, o)
                 for w, o in zip(sets, outs)]

    if args.rope:
        cos, sin = synth.rope_tables(base.max_blocks_per_stream * 16, base.head_dim)
        cos_d, sin_d = torch.from_numpy(cos).to(dev), torch.from_numpy(sin).to(dev)
        qkv = synth.make_qkv(base, base.seed + 7, device=dev)
        q_rot = [torch.zeros_like(t) for t in base.q]
        step_args = [binding.RopeStepArgs(qkv, q_rot, w.k_pool, w.v_pool, o, cos_d, sin_d)
                     for w, o in zip(sets, outs)]

    def eager_step(i):
        if layerwise:
            a = sets[i % copies]
            o = outs[i % copies]
            binding.decode_plan(sh, bt, lens, ws, context_lens_host=host_lens)
            for l in range(base.layers):
                binding.decode_layer(sh, l, a.q[l], a.k_new[l], a.v_new[l], a.k_pool[l],
                                     a.v_pool[l], bt, lens, o[l], ws, context_lens_host=host_lens)
        elif args.rope:
            binding.decode_step_rope(sh, step_args[i % copies], bt, lens, ws,
                                     context_lens_host=host_lens)
        else:
            binding.decode_step(sh, step_args[i % copies], bt, lens, ws,
                                context_lens_host=host_lens)

    step = eager_step
    if args.hip_graph:  # one captured step per pool set, replayed on the current stream
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graphs = []
        for c in range(copies):
            with torch.cuda.stream(side):
                eager_step(c)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                eager_step(c)
            graphs.append(g)
        torch.cuda.synchronize()

        def step(i):
            graphs[i % copies].replay()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region A: the production entry point, whole step
    for i in range(args.warmup):
        step(i)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()  # on the stream the steps are launched on (torch's current stream)
    for i in range(args.steps):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)])
    ms_median = float(np.median(per_step))
    kv_bytes_step = kv_bytes_layer * base.layers
    value = kv_bytes_step / (ms_per_step * 1e-3) / 1e9

    # ---- timed region B: same steps, HIP events around the attention kernel of every layer
    n_ev = args.steps * base.layers
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_ev)]
    for a, b in evs:
        a.record()
        b.record()
    torch.cuda.synchronize()
    e = 0
    for i in range(args.steps):
        w, o = sets[i % copies], outs[i % copies]
        for l in range(base.layers):
            binding.kv_append(sh, w.k_new[l], w.v_new[l], w.k_pool[l], w.v_pool[l], bt, lens)
            binding.paged_decode(sh, w.q[l], w.k_pool[l], w.v_pool[l], bt, lens, o[l], ws,
                                 context_lens_host=host_lens, events=evs[e])
            e += 1
    torch.cuda.synchronize()
    kern = np.array([a.elapsed_time(b) for a, b in evs])
    kern_ms = float(kern.mean())
    achieved = kv_bytes_layer / (kern_ms * 1e-3) / 1e9
    waves = args.split_waves if args.split_waves > 0 else 1024
    if not full:  # a line of the `also` list: the whole step and the attention kernel
        return {
            "workload": base.name, "streams": base.num_streams, "layers": base.layers,
            "entry": "vox_decode_plan + vox_decode_layer per layer" if layerwise else "vox_decode_step",
            "kv_bytes_per_step": kv_bytes_step, "value": round(value, 1), "unit": "GB/s",
            "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
            "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
            "pct_hbm_peak_median": round(100.0 * kv_bytes_step / (ms_median * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
            "stream_steps_per_s": round(base.num_streams / (ms_per_step * 1e-3), 1),
            "kernel_ms": round(kern_ms, 4), "kernel_ms_median": round(float(np.median(kern)), 4),
            "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(base.name),
            "pool_copies": copies,
        }

    # ---- split-K balance: every wave's own start / end clock (100 MHz) in one more launch
    clocks = torch.full((2 * waves,), -1, dtype=torch.int64, device=dev)
    w0, o0 = sets[0], outs[0]
    binding.kv_append(sh, w0.k_new[0], w0.v_new[0], w0.k_pool[0], w0.v_pool[0], bt, lens)
    binding.paged_decode(sh, w0.q[0], w0.k_pool[0], w0.v_pool[0], bt, lens, o0[0], ws,
                         context_lens_host=host_lens, wave_clock=clocks)
    torch.cuda.synchronize()
    ck = clocks.cpu().numpy().reshape(waves, 2)
    ck = ck[ck[:, 0] >= 0]
    wave_spread = None
    if len(ck):
        dur = (ck[:, 1] - ck[:, 0]) * 1e-2  # ticks of 10 ns -> us
        end = (ck[:, 1] - ck[:, 0].min()) * 1e-2
        wave_spread = {"waves": int(len(ck)), "duration_us_min": round(float(dur.min()), 1),
                       "duration_us_median": round(float(np.median(dur)), 1),
                       "duration_us_max": round(float(dur.max()), 1),
                       "last_start_us": round(float((ck[:, 0].max() - ck[:, 0].min()) * 1e-2), 1),
                       "first_end_us": round(float(end.min()), 1),
                       "last_end_us": round(float(end.max()), 1)}

    # ---- the chip's streaming-read ceiling: 4 GiB read once, no arithmetic
    read_ceiling = None
    if not args.no_read_ceiling:
        probe = torch.empty(1 << 32, dtype=torch.uint8, device=dev).fill_(1)
        sink = torch.zeros(8192, dtype=torch.int32, device=dev)
        pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(5)]
        binding.read_probe(probe, sink)
        for a, b in pe:
            a.record()
            binding.read_probe(probe, sink)
            b.record()
        torch.cuda.synchronize()
        read_ceiling = round((1 << 32) / (min(a.elapsed_time(b) for a, b in pe) * 1e-3) / 1e9, 1)
        del probe
    # KV bytes plus everything else one layer's step has to move: queries, outputs, block
    # table reads, appended rows, partial records (written and read back)
    s_, hq_, hkv_, d_ = base.num_streams, base.num_q_heads, base.num_kv_heads, base.head_dim
    nb = int(((base.context_lens.astype(np.int64) + 15) // 16).sum())
    other_bytes = (s_ * hq_ * d_ * 2 + s_ * hq_ * d_ * 4 + nb * 4 * hkv_ + s_ * hkv_ * d_ * 4 +
                   2 * (waves + s_ * hkv_) * (hq_ // hkv_) * (d_ + 2) * 4)
    roofline = {
        "bound": "hbm",
        "kernel": "decode_kernel<ValuMath>" if path == binding.PATH_VALU else "decode_kernel<MfmaMath>",
        "achieved": round(achieved, 1),
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "kernel_ms": round(kern_ms, 4),
        "kernel_ms_median": round(float(np.median(kern)), 4),
        "bytes_per_launch": kv_bytes_layer,
        "traffic": measured_traffic(base.name) if path != binding.PATH_VALU else None,
        "read_ceiling_gbps": read_ceiling,
        "frac_of_read_ceiling": round(achieved / read_ceiling, 4) if read_ceiling else None,
        "other_algorithmic_bytes_per_launch": other_bytes,
    }

    # ---- CPU baseline: the oracle as it stands on a bounded sample of streams
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        def bits(t):
            return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

        qb, kp, vp = bits(base.q[0]), bits(base.k_pool[0]), bits(base.v_pool[0])
        per_tok = base.kv_bytes_per_token

        def run(n):
            t = time.perf_counter()
            oracle.paged_decode(qb, kp, vp, base.block_tables, base.context_lens, base.scale,
                                num_kv_heads=base.num_kv_heads, streams=(0, n))
            return time.perf_counter() - t

        probe_n = min(base.num_streams, 8)
        probe_t = run(probe_n)
        probe_tok = int(base.context_lens[:probe_n].astype(np.int64).sum())
        rate = probe_tok / max(probe_t, 1e-6)
        cum = np.cumsum(base.context_lens.astype(np.int64))
        n = int(np.searchsorted(cum, rate * args.cpu_seconds) + 1)
        n = max(probe_n, min(base.num_streams, n))
        toks = int(cum[n - 1])
        passes, secs = 0, 0.0
        while passes == 0 or (secs < args.cpu_seconds and passes < 64):
            secs += run(n)  # whole sample again: the oracle is fast on many-core hosts
            passes += 1
        threads = oracle.num_threads()
        oracle.set_num_threads(1)  # the same oracle on one core, on the probe's streams
        single = probe_tok * per_tok / max(run(probe_n), 1e-6) / 1e9
        oracle.set_num_threads(0)
        cpu = {
            "value": round(passes * toks * per_tok / secs / 1e9, 4),
            "unit": "GB/s",
            "cores": threads,
            "single_thread_value": round(single, 4),
            "kind": "oracle",
            "sample": f"fp64 oracle decode of streams [0,{n}) of {base.num_streams} "
                      f"({toks} tokens, layer 0), {passes} passes in {secs:.2f} s",
            "cpu_model": cpu_model(),
            "host_cpus": os.cpu_count(),
        }

    line = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(ms_median, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": base.name,
            "streams": base.num_streams,
            "q_heads": base.num_q_heads,
            "kv_heads": base.num_kv_heads,
            "head_dim": base.head_dim,
            "layers": base.layers,
            "total_tokens": base.total_tokens,
            "kv_bytes_per_step": kv_bytes_step,
            "pool_copies": copies,
            "path": args.path,
            "split_waves": args.split_waves,
            "host_lens": bool(args.host_lens),
            "hip_graph": bool(args.hip_graph),
            "rope_fused_append": bool(args.rope),
            "layerwise": bool(layerwise),
        },
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "stream_steps_per_s": round(base.num_streams / (ms_per_step * 1e-3), 1),
        "wave_spread": wave_spread,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    return line




def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3",
                    choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", *MULTI_WORKLOADS,
                             *SAMPLE_WORKLOADS],
                    help="cfg1..cfg5: decode step (cfg3 is the headline); the others are "
                         "multi-token steps (detokenizer chunks, prompts, admission mix)")
    ap.add_argument("--path", default="auto", choices=["auto", "mfma", "valu"])
    ap.add_argument("--split-waves", type=int, default=0)
    ap.add_argument("--layers", type=int, default=None, help="override the preset's layer count")
    ap.add_argument("--pool-copies", type=int, default=None,
                    help="distinct pool sets rotated across steps (default: enough to exceed 1 GiB)")
    ap.add_argument("--no-device-lens-only", dest="host_lens", action="store_true", default=True)
    ap.add_argument("--device-lens-only", dest="host_lens", action="store_false",
                    help="do not hand the host copy of context_lens to the library")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic for scaling HBM counters)")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture one step per pool set into a HIP graph and time the replays")
    ap.add_argument("--rope", action="store_true",
                    help="time vox_decode_step_rope: rotary embedding + Q/K/V split fused into "
                         "the append (inputs are packed QKV rows)")
    ap.add_argument("--no-read-ceiling", action="store_true",
                    help="skip the 4 GiB streaming-read probe that measures the chip's read ceiling")
    ap.add_argument("--layerwise", action="store_true",
                    help="time the step as one vox_decode_plan and a vox_decode_layer call per layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true",
                    help="headline workload only: skip the records of the other workloads in the default run")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the decode step shards by stream or by kv head with no exchange between GPUs)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2602_00269_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    binding.load()
    dev = torch.device("cuda:0")
    if args.workload in MULTI_WORKLOADS:
        return bench_multi(args, dev)
    if args.workload in SAMPLE_WORKLOADS:
        return bench_sample(args, dev)
    line = bench_decode(args, dev, args.workload, layerwise=args.layerwise)
    if args.workload == "cfg3" and not args.no_also:
        # the other decode presets in the same run: the 512-stream target config, the small
        # batch the paper's models run at, and the 28-layer full step
        import gc

        line["also"] = []
        for other in ("cfg4", "cfg2", "cfg5"):
            gc.collect()
            torch.cuda.empty_cache()
            line["also"].append(bench_decode(args, dev, other, full=False))
        gc.collect()
        torch.cuda.empty_cache()
        line["also"].append(bench_decode(args, dev, "cfg5", full=False, layerwise=True))
        # the steps next to the decode step (multi-token step, sampling), one short record each
        import copy

        for other in (*MULTI_WORKLOADS, *SAMPLE_WORKLOADS):
            gc.collect()
            torch.cuda.empty_cache()
            a = copy.copy(args)
            a.workload, a.no_cpu_baseline, a.copy_calibration = other, True, False
            r = (bench_multi if other in MULTI_WORKLOADS else bench_sample)(a, dev, emit=False)
            line["also"].append({
                "workload": r["config"]["workload"], "metric": r["metric"], "value": r["value"],
                "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                "kernel": r["roofline"]["kernel"], "kernel_ms": r["roofline"]["kernel_ms"],
                "bound": r["roofline"]["bound"], "frac": r["roofline"]["frac"],
                "traffic": r["roofline"]["traffic"]})
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
