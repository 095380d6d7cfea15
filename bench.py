#!/usr/bin/env python3
"""Benchmark of the Inf-MLLM streaming step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--sub cfg1,cfg2,cfg3,cfg4]

A step is one infmllm_step (append, chunk attention, column score + bias, top-r select,
compaction) over one chunk of a seeded synthetic stream whose inputs already sit in HBM.
Prints ONE JSON line.  Its headline (value, ms_per_step, roofline, cpu_baseline) is the largest
single-GPU workload, cfg5 (one layer of the long-text stress stream: 32 heads x 128, budget 8192, chunks
of 2048); the other workloads are carried as sub-records under "workloads", each with its own throughput,
roofline fractions and oracle timing.  Rooflines come from HIP events recorded around the kernels in
further passes over the same steps; the fp64 CPU oracle is timed on a bounded sample of each workload.
Before the W warm-up steps the same steps are run untimed for --spinup-ms (50 ms) so that the device has
reached its sustained clocks; the K timed steps follow the warm-up directly.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def algorithmic_work(cfg, L, t):
    """Per-launch algorithmic flops/bytes of each kernel in steady state (cache full)."""
    n, B, R = t + L, cfg.budget, cfg.recent
    d, Hq, Hkv = cfg.head_dim, cfg.heads, cfg.kv_heads
    elt = 2 if cfg.dtype == "bf16" else 4
    pairs = L * t + L * (L + 1) // 2                         # visible (query, key) pairs per head
    c, lq, r = n - R, min(R, L), B - R
    row = 2 * (2 * d * elt) + 16                            # K and V read + written, position and score
    # Rows an eviction actually moves in steady state: the retained rows that are not already inside physical
    # rows 0..B-1, i.e. the chunk's survivors.  With L <= R (all five workloads) every chunk row is inside the
    # recent window, so that is exactly L rows per kv-head; the r + R - L retained cached rows stay in place.
    moved = min(L, R)
    return {
        "attn": {"flops": 4.0 * d * pairs * Hq, "bytes": elt * d * (2 * n * Hkv + 2 * L * Hq)},
        "score": {"flops": 2.0 * d * lq * c * Hq, "bytes": elt * d * (c * Hkv + lq * Hq) + 4 * c * Hkv},
        "append": {"bytes": 2 * (2 * L * Hkv * d * elt) + 8 * L * Hkv},
        # selection launch: W' read, the index list written twice (stream scratch and the caller's), and the
        # placement plan: old row table read, rank / new row table / score written for the rows that stay
        "select": {"bytes": (4 * c + 8 * B + 16 * (B - moved) + 12 * moved) * Hkv},
        # placement launch: the moved rows' K and V read and written, their table entries
        "compact": {"bytes": (row + 12 + 12) * moved * Hkv, "rows_moved": moved * Hkv},
        # position-encoding pre-pass: every cached key, the chunk's keys and the queries read and written once
        "rope": {"bytes": 2 * elt * d * (n * Hkv + L * Hq)},
    }


def read_counters(name):
    """Figures that only a rocprofv3 --pmc run can give (HBM bytes per launch of the dominant kernel, the share
    of SIMD-cycles its matrix pipes were busy), from the committed summary of such runs of this same command,
    if there is one for the workload; None otherwise.  They are not measured in this process."""
    path = os.path.join(ROOT, "profiles", name)
    out = {"traffic": None, "mfma_busy": None, "source": None}
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                out["traffic"] = float(line.split(":", 1)[1])
                out["source"] = "profiles/" + name
            elif line.startswith("mfma_busy_frac:"):
                out["mfma_busy"] = float(line.split(":", 1)[1])
    except OSError:
        pass
    return out


def cpu_baseline(cfg, budget_seconds=12.0, policy="infmllm", rope_base=0.0, max_steps=48):
    """The oracle as it stands, timed on steady-state steps of the same workload."""
    import numpy as np
    import oracle
    from paper_2409_09086_amd.workloads import ChunkStream
    orc = oracle.OracleStream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, bias=cfg.bias,
                              policy=policy, rope_base=rope_base, rope_round=cfg.dtype if rope_base else None)
    rng = np.random.default_rng(cfg.seed)
    K = rng.standard_normal((cfg.kv_heads, cfg.budget, cfg.head_dim)) * cfg.sigma
    V = rng.standard_normal((cfg.kv_heads, cfg.budget, cfg.head_dim)) * cfg.sigma
    pos = np.tile(np.arange(cfg.budget), (cfg.kv_heads, 1))
    orc.load(K, V, pos, cfg.budget)                          # start from a full cache
    stream = ChunkStream(cfg, start_step=0) if cfg.ar_rho else ChunkStream(cfg, start_step=cfg.budget // cfg.chunk)
    tokens, steps, spent = 0, 0, 0.0
    while spent < budget_seconds and steps < max_steps:
        q, k, v = [x.double().numpy() for x in next(stream)]
        t0 = time.perf_counter()
        orc.step(q, k, v)
        spent += time.perf_counter() - t0
        tokens += q.shape[0]
        steps += 1
    return {"value": tokens / spent, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "%d steady-state steps of %s (cache full, n = %d), %.1f s of fp64 C + OpenMP" %
                      (steps, cfg.name, cfg.budget + cfg.chunk, spent),
            "ms_per_step": 1e3 * spent / steps}


def retention_leg(cfg, binding, dev, impl):
    """Sanity figure: what becomes of the keys the stream generator planted (cfg2: 1 % of the tokens carry a shared
    offset on every key dimension; cfg5: a bank of 128 keys recurs every 100 000 tokens).  A short untimed stream is
    run and the positions still cached are compared with the planted ones, counting only tokens that have left the
    recent window (inside it everything is kept).  None for workloads that plant nothing."""
    import numpy as np
    from paper_2409_09086_amd.workloads import ChunkStream
    if not (cfg.heavy_frac or cfg.recur_period):
        return None
    fill = -(-cfg.budget // cfg.chunk)
    if cfg.recur_period:
        hit_step = cfg.recur_period // cfg.chunk             # the step in which the bank arrives a second time
        stream, steps = ChunkStream(cfg, start_step=hit_step - fill), fill + 6
    else:
        stream, steps = ChunkStream(cfg), fill + 12
    first = stream.tokens
    s = binding.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=cfg.torch_dtype,
                       bias=cfg.bias, max_chunk=cfg.max_chunk, impl=impl, device=dev)
    planted = []
    for _ in range(steps):
        q, k, v = next(stream)
        planted.append(stream.last_planted)
        s.step(q.to(dev), k.to(dev), v.to(dev), report=False)
    planted = np.concatenate(planted)
    total = planted.shape[0]
    pos = s.positions().cpu().numpy()                        # [Hkv][B] stream positions, counted from this stream's start
    old = np.arange(total) < total - cfg.recent              # tokens outside the recent window
    kept = np.zeros((cfg.kv_heads, total), dtype=bool)
    for h in range(cfg.kv_heads):
        kept[h, pos[h]] = True
    n_pl = int((planted & old).sum())
    return {"steps": steps, "first_token": first, "planted_tokens_outside_recent_window": n_pl,
            "planted_kept_frac": round(float(kept[:, planted & old].mean()), 4) if n_pl else None,
            "all_kept_frac": round(float(kept[:, old].mean()), 4)}


def attn_kernel_name(cfg, L, mfma):
    """Which attention kernel the library's launch picks for this shape (the rule of launch_attn_mfma)."""
    if not mfma:
        return "attn_simple"
    wgs64 = (cfg.heads * (-(-L // 64)) + 3) // 4
    rounds = -(-wgs64 // 256)
    fills = wgs64 * 5 >= rounds * 256 * 4
    return "attn_fwd64" if cfg.head_dim == 128 and fills and cfg.budget + L >= 1024 else "attn_fwd"


def decode_leg(cfg, binding, chunks, dev, impl, ntok=64):
    """Secondary figure: decoding steps (one token, no eviction) on the same layer with the cache full."""
    import torch
    L = cfg.chunk
    s = binding.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=cfg.torch_dtype,
                       bias=cfg.bias, max_chunk=cfg.max_chunk, impl=impl, max_decode=ntok + 8, device=dev)
    for i in range(-(-cfg.budget // L) + 1):
        q, k, v = chunks[i % len(chunks)]
        s.step(q, k, v, report=False)
    toks = [(q[i:i + 1].contiguous(), k[i:i + 1].contiguous(), v[i:i + 1].contiguous())
            for q, k, v in chunks[:2] for i in range(ntok // 2)]
    out = torch.empty_like(toks[0][0])
    # the ntok tokens as one infmllm_decode_n call (one host call enqueues every token's launch)
    qn, kn, vn = [torch.cat([t[j] for t in toks]).contiguous() for j in range(3)]
    outn = torch.empty_like(qn)
    s.decode_n(qn[:8], kn[:8], vn[:8], out=outn[:8])         # untimed: the kernel's first launches
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    s.decode_n(qn, kn, vn, out=outn)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # same tokens again on a fresh full cache, with events around the decode kernels
    s2 = binding.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=cfg.torch_dtype,
                        bias=cfg.bias, max_chunk=cfg.max_chunk, impl=impl, max_decode=ntok, device=dev)
    for i in range(-(-cfg.budget // L) + 1):
        q, k, v = chunks[i % len(chunks)]
        s2.step(q, k, v, report=False)
    s2.profile(ntok)
    for q, k, v in toks:
        s2.decode(q, k, v, out=out)
    torch.cuda.synchronize()
    ms, cnt = s2.profile_read()["decode"]
    s2.profile(0)
    us = 1e3 * ms / cnt
    elt = 2 if cfg.dtype == "bf16" else 4
    n_avg = cfg.budget + (ntok + 1) / 2.0
    nbytes = 2 * n_avg * cfg.kv_heads * cfg.head_dim * elt          # every K and V row once
    gbs = nbytes / (us * 1e-6) / 1e9
    return {"tokens_per_s": round(ntok / elapsed, 1), "us_per_token": round(1e6 * elapsed / ntok, 3),
            "kernels_us": round(us, 3), "launches": cnt, "call": "infmllm_decode_n, %d tokens per call" % ntok,
            "hbm_frac_of_the_call": round(nbytes / (1e9 * elapsed / ntok) / PEAK_HBM_GBS, 4),
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(gbs / PEAK_HBM_GBS, 4), "algorithmic_bytes_per_token": nbytes}}


def layer_batched_leg(cfg, binding, chunks, dev, impl, n_layers, steps):
    """Secondary figure: n_layers streams of the workload's shape (the layers of a model) fed the same
    chunk per step, once with infmllm_step per layer and once with infmllm_step_attend per layer plus one
    infmllm_evict_batched per step.  Both in steady state (caches full); time per layer-step."""
    import torch
    L = cfg.chunk
    lib = binding.lib()
    P = ctypes.c_void_p
    cargs = [(P(q.data_ptr()), P(k.data_ptr()), P(v.data_ptr())) for q, k, v in chunks]
    outs = torch.empty((n_layers,) + tuple(chunks[0][0].shape), dtype=chunks[0][0].dtype, device=dev)
    po = [P(outs[i].data_ptr()) for i in range(n_layers)]
    fill = -(-cfg.budget // L) + 1
    res = {}
    for mode in ("per_layer", "batched"):
        ss = [binding.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=cfg.torch_dtype,
                             bias=cfg.bias, max_chunk=cfg.max_chunk, impl=impl, device=dev) for _ in range(n_layers)]
        hs = [s._h for s in ss]
        harr = (P * n_layers)(*hs)

        def run(count, first):
            for i in range(count):
                for li in range(n_layers):
                    a = cargs[(first + i + li) % len(cargs)]
                    if mode == "per_layer":
                        rc = lib.infmllm_step(hs[li], a[0], a[1], a[2], L, po[li], None, None)
                    else:
                        rc = lib.infmllm_step_attend(hs[li], a[0], a[1], a[2], L, po[li], None, None)
                    if rc != 0:
                        raise RuntimeError(binding.last_error())
                if mode == "batched" and lib.infmllm_stream_pending(hs[0]) == 1:
                    if lib.infmllm_evict_batched(harr, n_layers, None, None) != 0:
                        raise RuntimeError(binding.last_error())

        run(fill + 2, 0)
        torch.cuda.synchronize()
        assert all(len(s) == cfg.budget for s in ss)
        t0 = time.perf_counter()
        run(steps, fill + 2)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        res[mode] = {"us_per_layer_step": round(1e6 * el / (steps * n_layers), 3),
                     "tokens_per_s": round(L * steps * n_layers / el, 1)}
        del ss
    res["layers"] = n_layers
    res["steps"] = steps
    return res


def measure(cfg, args, binding, dev, steps, nchunks, full):
    """One workload: throughput pass, per-kernel event passes, (full only) single-step latencies and the decode
    and layer-batched legs.  Returns the record and the chunks kept in HBM."""
    import torch
    from paper_2409_09086_amd.workloads import ChunkStream
    L = cfg.chunk
    fill_steps = -(-cfg.budget // L)                         # steps until the cache is full
    warmup = max(args.warmup, fill_steps + 1)

    # inputs: seeded chunks of the configured stream, resident in HBM before any timing
    stream_in = ChunkStream(cfg)
    nchunks = min(max(nchunks, 2), cfg.steps)
    chunks = []
    for _ in range(nchunks):
        q, k, v = next(stream_in)
        if q.shape[0] != L:                                  # keep the timed loop at the ordinary chunk length
            q, k, v = q[:L].contiguous(), k[:L].contiguous(), v[:L].contiguous()
        chunks.append((q.to(dev), k.to(dev), v.to(dev)))
    out = torch.empty_like(chunks[0][0])
    retained = torch.empty((cfg.kv_heads, cfg.budget), dtype=torch.int32, device=dev)
    n_ret = torch.empty((1,), dtype=torch.int32, device=dev)

    s = binding.Stream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, dtype=cfg.torch_dtype,
                       bias=cfg.bias, max_chunk=cfg.max_chunk, impl=args.impl, policy=args.policy,
                       rope_base=args.rope or None, attn_tile=args.attn_tile, device=dev)
    lib = binding.lib()
    P = ctypes.c_void_p
    cargs = [(P(q.data_ptr()), P(k.data_ptr()), P(v.data_ptr())) for q, k, v in chunks]
    po, pr, pn = P(out.data_ptr()), P(retained.data_ptr()), P(n_ret.data_ptr())
    h = s._h

    def run(count, first):
        for i in range(count):
            a = cargs[(first + i) % nchunks]
            rc = lib.infmllm_step(h, a[0], a[1], a[2], L, po, pr, pn)
            if rc != 0:
                raise RuntimeError(binding.last_error())

    # Clock spin-up, untimed and before the warm-up steps: from idle the device takes some tens of milliseconds of
    # load to reach its sustained clocks (the first 1-2 ms of steps run ~8 % slower); the state of the stream
    # is the same steady state afterwards.
    spin_steps = 0
    t_spin = time.perf_counter()
    while (time.perf_counter() - t_spin) * 1e3 < args.spinup_ms:
        run(max(16, fill_steps + 1), 0)
        torch.cuda.synchronize()
        spin_steps += max(16, fill_steps + 1)
    run(warmup, 0)
    torch.cuda.synchronize()
    assert len(s) == cfg.budget and int(n_ret.item()) == cfg.budget

    # pass 1: whole-step throughput, no events inside the region
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps, warmup)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps

    # pass 2: the same steps with HIP events around every kernel, on the stream they run on
    prof_steps = min(steps, 256)
    s.profile(prof_steps)
    run(prof_steps, warmup + steps)
    torch.cuda.synchronize()
    prof = s.profile_read()
    # ... and once more with a single bracket around selection + placement (Alg. 1 l.5-8 as a whole)
    s.profile_select(["evict"])
    s.profile(prof_steps)
    run(prof_steps, warmup + steps)
    torch.cuda.synchronize()
    prof["evict"] = s.profile_read()["evict"]
    # ... and the dominant kernel on its own, so that no other event pair sits next to it in the stream
    s.profile_select(["attn"])
    s.profile(prof_steps)
    run(prof_steps, warmup + steps)
    torch.cuda.synchronize()
    prof["attn"] = s.profile_read()["attn"]
    s.profile_select(binding.KERNELS)
    s.profile(0)

    latency = None
    if full:
        # pass 3: latency of single steps (event pair around each call, on the stream the kernels run on)
        lat_steps = min(steps, 512)
        ts = torch.cuda.ExternalStream(s.hip_stream, device=dev) if s.hip_stream else torch.cuda.current_stream(dev)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(lat_steps)]
        for i, (e0, e1) in enumerate(evs):
            e0.record(ts)
            run(1, warmup + steps + prof_steps + i)
            e1.record(ts)
        torch.cuda.synchronize()
        lat = sorted(1e3 * e0.elapsed_time(e1) for e0, e1 in evs)
        latency = {"p50": round(lat[len(lat) // 2], 2), "p99": round(lat[min(len(lat) - 1, int(0.99 * len(lat)))], 2),
                   "max": round(lat[-1], 2), "steps": lat_steps}

    work = algorithmic_work(cfg, L, cfg.budget)
    kernels = {}
    for name, (ms, cnt) in prof.items():
        if not cnt:
            continue
        us = 1e3 * ms / cnt
        e = {"us": round(us, 3), "launches": cnt}
        w = work.get(name)
        if w is None:
            kernels[name] = e
            continue
        if "flops" in w:
            e["tflops"] = round(w["flops"] / (us * 1e-6) / 1e12, 2)
        e["gbs"] = round(w["bytes"] / (us * 1e-6) / 1e9, 1)
        kernels[name] = e
    attn = kernels["attn"]
    mfma = cfg.dtype == "bf16" and args.impl != 1
    peak = PEAK_BF16_TFLOPS if mfma else PEAK_FP32_TFLOPS
    ctr = read_counters("attn_fwd_%s_pmc.txt" % cfg.name)
    roofline = {"kernel": attn_kernel_name(cfg, L, mfma), "bound": "mfma" if mfma else "alu",
                "achieved": attn["tflops"], "peak": peak, "unit": "TFLOP/s", "frac": round(attn["tflops"] / peak, 4),
                "traffic": ctr["traffic"], "mfma_busy_counter": ctr["mfma_busy"], "counters_from": ctr["source"],
                "algorithmic_flops_per_launch": work["attn"]["flops"], "avg_us": attn["us"]}
    # selection + placement as one bracket (start of the selection launch to end of the last eviction launch)
    evict_us = kernels.get("evict", {}).get("us", 0.0)
    evict_bytes = work["select"]["bytes"] + work["compact"]["bytes"]
    evict = {"bound": "hbm", "achieved": round(evict_bytes / (evict_us * 1e-6) / 1e9, 1) if evict_us else None,
             "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(evict_bytes / (evict_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4) if evict_us else None,
             "algorithmic_bytes_per_step": evict_bytes, "avg_us": round(evict_us, 3)}
    rec = {
        "value": round(L * steps / elapsed, 1), "ms_per_step": round(ms_per_step, 5), "steps": steps, "warmup": warmup,
        "dtype": cfg.dtype,
        "config": {"workload": "%s: %d q-heads / %d kv-heads x %d, budget %d (recent %d), chunk %d, steady state n = %d"
                   % (cfg.name, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.budget, cfg.recent, L, cfg.budget + L),
                   "bias": cfg.bias, "seed": cfg.seed, "chunks_in_hbm": nchunks, "policy": args.policy,
                   "rope_base": args.rope, "spinup_ms": args.spinup_ms, "spinup_steps": spin_steps,
                   "kernels": "mfma" if mfma else "plain"},
        "roofline": roofline, "evict_roofline": evict, "kernels": kernels,
    }
    if latency:
        rec["step_latency_us"] = latency
    rec["decode"] = decode_leg(cfg, binding, chunks, dev, args.impl)
    del s
    if args.policy == "infmllm" and not args.rope:
        ret = retention_leg(cfg, binding, dev, args.impl)
        if ret:
            rec["planted_key_retention"] = ret
    if full and args.layers > 0:
        rec["layer_batched"] = layer_batched_leg(cfg, binding, chunks, dev, args.impl, args.layers,
                                                 max(4, min(steps, 2000 // args.layers)))
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--spinup-ms", type=float, default=50.0,
                    help="untimed steps run before the warm-up steps until this much time has passed: the GPU "
                         "raises its clocks only after some tens of milliseconds of load")
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="the headline workload (default: the largest single-GPU one)")
    ap.add_argument("--sub", default="cfg1,cfg2,cfg3,cfg4",
                    help="comma-separated workloads carried as sub-records under \"workloads\" (\"none\" = none)")
    ap.add_argument("--chunks", type=int, default=8, help="distinct chunks kept in HBM and cycled through")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--impl", type=int, default=None, help="debug: 1 = plain-arithmetic kernels")
    ap.add_argument("--attn-tile", type=int, default=None, help="debug: force a workgroup shape of the attention kernel")
    ap.add_argument("--policy", default="infmllm", choices=["infmllm", "window", "initial_recent", "cumulative"],
                    help="score the selection ranks (comparison policies); the default is the paper's method")
    ap.add_argument("--rope", type=float, default=0.0, metavar="BASE",
                    help="cache-relative rotary position encoding with this base (0 = off, the default)")
    ap.add_argument("--layers", type=int, default=8, help="streams in the layer-batched eviction leg (0 = skip)")
    ap.add_argument("--copy-calib", type=int, default=0, metavar="MIB",
                    help="also run an elementwise copy of this many MiB (reads MIB, writes MIB) three times, as "
                         "the known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this path runs on one GPU (heads would shard with no communication); "
                 "run it with --gpus 1")

    import torch
    from paper_2409_09086_amd import binding
    from paper_2409_09086_amd.workloads import CONFIGS

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calib:
        src = torch.ones(args.copy_calib << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    cfg = CONFIGS[args.workload]
    rec = measure(cfg, args, binding, dev, args.steps, args.chunks, full=True)
    result = {
        "metric": "streamed tokens/s per layer-step at budget B",
        "value": rec["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": rec["steps"], "warmup": rec["warmup"], "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": rec["dtype"], "data": "synthetic", "config": rec["config"],
        "roofline": rec["roofline"], "evict_roofline": rec["evict_roofline"], "kernels": rec["kernels"],
        "step_latency_us": rec.get("step_latency_us"), "decode": rec["decode"],
    }
    if "planted_key_retention" in rec:
        result["planted_key_retention"] = rec["planted_key_retention"]
    if "layer_batched" in rec:
        result["layer_batched"] = rec["layer_batched"]
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, budget_seconds=12.0, policy=args.policy, rope_base=args.rope)
    subs = {}
    for name in [x for x in args.sub.split(",") if x in CONFIGS and x != args.workload]:
        sc = CONFIGS[name]
        torch.cuda.empty_cache()
        r = measure(sc, args, binding, dev, max(4, min(args.steps, 200)), args.chunks, full=False)
        sub = {"tokens_per_s": r["value"], "us_per_step": round(1e3 * r["ms_per_step"], 3), "steps": r["steps"],
               "dtype": r["dtype"], "workload": r["config"]["workload"], "roofline": r["roofline"],
               "evict_roofline": r["evict_roofline"], "kernels": r["kernels"], "decode": r["decode"]}
        if "planted_key_retention" in r:
            sub["planted_key_retention"] = r["planted_key_retention"]
        if not args.no_cpu:
            sub["cpu_baseline"] = cpu_baseline(sc, budget_seconds=3.0, policy=args.policy, rope_base=args.rope, max_steps=16)
        subs[name] = sub
    if subs:
        result["workloads"] = subs
    print(json.dumps(result))


if __name__ == "__main__":
    main()
