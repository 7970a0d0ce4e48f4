#!/usr/bin/env python3
"""Benchmark of the hot path: multi-model paged GQA decode attention over one shared
KV page pool (plus balloon_resize latency), one MI355X.

One "step" = one decode step of the co-located models of the workload: one grouped
decode_attention_multi call (attention kernel + split-K merge) over every active
model's batch.  Inputs are resident in HBM before the timed region starts.  The
default workload is cfg 2 (two co-located models, lognormal context lengths); three
independently seeded replicas are rotated so that a step never re-reads what the
previous step left in the 256 MB Infinity Cache.

Prints ONE JSON line: the headline metric (KV bytes read per second by a decode step), `roofline`
(the attention kernel against the HBM peak, with its measured traffic), `cpu_baseline` (the CPU
oracle timed on the host cores), the measured read ceilings, and secondary legs: balloon_resize
latency (ordinary and elastic pools), kv_append, chunked-prefill attention, the host policies.

`--config 3` runs the bursty scenario instead (bookkeeping events between the decode launches,
a model mix that changes from step to step); `--frame-bytes` overrides a workload's frame size
(65536 = one or two blocks per frame: the most scattered pool).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

KERNEL_FORM_NAME = ("k_attention", "k_attention_deep")
HBM_PEAK_GBPS = 8000.0      # MI355X datasheet HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="3 = the bursty scenario: bookkeeping events and decode of the active models, step by step")
    ap.add_argument("--frame-bytes", type=int, default=0, help="override the workload's frame size (0 = as configured)")
    ap.add_argument("--layers", type=int, default=1,
                    help="layers per model sharing its block table; step i attends to layer i mod layers of every model")
    ap.add_argument("--size", default="full", choices=["full", "small"])
    ap.add_argument("--replicas", type=int, default=3)
    ap.add_argument("--items", type=int, default=0, help="work items (waves) per attention launch (0 = automatic)")
    ap.add_argument("--min-share", type=int, default=0, help="smallest share of pages per wave (0 = automatic)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample (0 = skip)")
    ap.add_argument("--no-balloon", action="store_true")
    ap.add_argument("--seg-cost", type=int, default=-1, help="allowance per segment in the work split, pages (-1 = default)")
    ap.add_argument("--condition-ms", type=int, default=1000,
                    help="untimed launches for this long before the warm-up, so that the clocks have settled (0 = none)")
    ap.add_argument("--kernel-form", type=int, default=-1, choices=[-1, 0, 1],
                    help="decode kernel: 0 = two waves per SIMD, 1 = one wave with a deeper ring, -1 = chosen by the launch")
    ap.add_argument("--tune", type=int, default=48, help="untimed launches that tune the per-XCD share weights before the warm-up (0 = equal weights)")
    ap.add_argument("--page-cost", type=int, default=-1, help="fixed cost of a page in the wave-sharing model, per mille (-1 = default)")
    ap.add_argument("--sweep-items", default="", help="comma list of work-item counts to time before the main run (stderr)")
    return ap.parse_args()


def condition(torch, fn, ms):
    """Keeps the GPU busy with fn(i) for about ms milliseconds: a GPU that has idled (set-up on the host,
    a previous leg's teardown) needs some hundred milliseconds of work before its clocks settle, and the
    first launches after an idle phase run 2-20 % slower than the steady state a serving loop is in."""
    t0, i = time.perf_counter(), 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(64):
            fn(i)
            i += 1
        torch.cuda.synchronize()
    return i


def profiled_traffic(kernel, workload, size):
    """HBM bytes per launch of the decode kernel from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE and WRITE_SIZE runs, scaled by kernels of known size); counters cannot
    be read from inside a timed run, so the figure is the stored one or None."""
    import re
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.md")
    if size != "full" or not os.path.exists(path):
        return None
    m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read())
    return int(m.group(1)) if m else None


def build_replicas(gpu, cfg_id, size, n, frame_bytes=0, layers=1):
    import copy
    from workloads.scenarios import Runner, make_config
    reps = []
    for r in range(n):
        cfg = copy.deepcopy(make_config(cfg_id, size))
        cfg.seed += 17 * r
        if frame_bytes:
            cfg.frame_bytes = frame_bytes
        for spec in cfg.models:
            spec.layers = layers
        t0 = time.time()
        reps.append(Runner(gpu, cfg).setup())
        print(f"[bench] replica {r}: pool {cfg.pool_bytes >> 20} MiB, KV {reps[-1].kv_bytes_step() / 1e9:.3f} GB, "
              f"set up in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    return reps


def device_inputs(torch, rep, step):
    import numpy as np
    mids = rep.active_models()
    qs = [torch.from_numpy(rep.queries(step, mi).view(np.int16)).cuda() for mi in mids]
    ctxs = [torch.from_numpy(rep.ctx[mi]).cuda() for mi in mids]
    outs = [torch.empty((rep.cfg.models[mi].batch, rep.cfg.models[mi].q_heads, rep.cfg.models[mi].head_dim),
                        dtype=torch.float32, device="cuda") for mi in mids]
    return [rep.models[mi] for mi in mids], qs, ctxs, outs


def balloon_latency(gpu, torch):
    """Wall-clock latency of balloon_resize (launch + kernel + result read-back) on a
    160 GB-class pool shape scaled to fit beside the benchmark pools: inflate to 176
    frames (one cfg-3 activation), fill, release, deflate to 0; median of 50 cycles."""
    import numpy as np
    pool = gpu.pool_create(8 << 30, 16, 2 << 20)
    m = gpu.model_register(pool, 32, 8, 128, 0, 32, 512)
    seqs = np.arange(32, dtype=np.int32)
    ctx = np.full(32, 2816, dtype=np.int32)        # 176 blocks each -> 5632 blocks = 176 frames
    t_inf, t_def, t_res, t_rel = [], [], [], []
    for _ in range(50):
        t0 = time.perf_counter(); assert gpu.balloon_resize(m, 176) == 176; t1 = time.perf_counter()
        assert gpu.seq_reserve_batch(m, seqs, ctx) == 5632; t2 = time.perf_counter()
        for s in range(32):
            gpu.seq_release(m, s)
        t3 = time.perf_counter(); assert gpu.balloon_resize(m, 0) == 0; t4 = time.perf_counter()
        t_inf.append(t1 - t0); t_res.append(t2 - t1); t_rel.append((t3 - t2) / 32); t_def.append(t4 - t3)
    gpu.model_unregister(m)
    gpu.pool_destroy(pool)
    med = lambda x: round(float(np.median(x) * 1e6), 2)
    res = {"inflate_176_frames_us": med(t_inf), "deflate_176_frames_us": med(t_def),
           "reserve_batch_5632_blocks_us": med(t_res), "release_176_blocks_us": med(t_rel),
           "kind": "host wall clock per call, median of 50"}
    # the same balloon on an elastic pool: frames are mapped when acquired and unmapped when given back
    for name, spare in (("elastic", 0), ("elastic_prealloc_176", 176)):
        pool = gpu.pool_create_elastic(8 << 30, 16, 2 << 20)
        assert pool >= 0, gpu.last_error()
        assert gpu.pool_set_prealloc(pool, spare) == spare
        m = gpu.model_register(pool, 32, 8, 128, 0, 32, 512)
        t_inf, t_def = [], []
        for _ in range(12):
            t0 = time.perf_counter(); assert gpu.balloon_resize(m, 176) == 176; t1 = time.perf_counter()
            assert gpu.balloon_resize(m, 0) == 0; t2 = time.perf_counter()
            t_inf.append(t1 - t0); t_def.append(t2 - t1)
        gpu.model_unregister(m)
        gpu.pool_destroy(pool)
        res[name + "_inflate_176_frames_us"] = med(t_inf[2:])
        res[name + "_deflate_176_frames_us"] = med(t_def[2:])
        res[name + "_first_inflate_us"] = round(t_inf[0] * 1e6, 2)
    return res


def append_latency(gpu, torch, rep, inputs):
    """The decode step's write path (kv_append) for the models of one replica: every sequence's
    last token is written again, 100 times; device time per call from events on the stream."""
    import numpy as np
    mids, qs, ctxs, outs = inputs
    res = {}
    for m, ctx, mi in zip(mids, ctxs, rep.active_models()):
        spec = rep.cfg.models[mi]
        g = torch.Generator(device="cpu"); g.manual_seed(1234 + mi)
        kx = torch.randn((spec.batch, spec.kv_heads, spec.head_dim), generator=g).to(torch.bfloat16).view(torch.int16).cuda()
        vx = torch.randn((spec.batch, spec.kv_heads, spec.head_dim), generator=g).to(torch.bfloat16).view(torch.int16).cuda()
        for _ in range(10):
            assert gpu.kv_append_dev(m, kx, vx, ctx) == spec.batch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(100):
            gpu.kv_append_dev(m, kx, vx, ctx)
        e1.record()
        torch.cuda.synchronize()
        res[f"model{mi}_batch{spec.batch}_{'e4m3' if spec.dtype else 'bf16'}_us"] = round(e0.elapsed_time(e1) * 10.0, 2)
    assert gpu.device_errors() == 0
    res["kind"] = "device time per kv_append call (one new token per sequence), mean of 100 back-to-back calls"
    return res


def prefill_leg(gpu, torch, condition_ms=1000):
    """Chunked prefill on one model of the headline workload's shape (32 q heads, 8 kv heads, head dim
    128, bf16 cache): 8 sequences with 2048 cached tokens each take a chunk of 512.  Reports device time
    per call and the rate of useful attention flops (4 * D * heads * visible (query, key) pairs)."""
    import numpy as np
    from workloads import gen
    hq, hkv, d, B, prefix, chunk = 32, 8, 128, 8, 2048, 512
    pool = gpu.pool_create(8 << 30, 16, 2 << 20)
    assert pool >= 0 and gpu.pool_seed_free_order(pool, gen.free_order((8 << 30) // (2 << 20), gen.generator(5))) == 0
    m = gpu.model_register(pool, hq, hkv, d, 0, B, 1024)
    ctx = prefix + chunk
    assert m >= 0 and gpu.balloon_resize(m, 1024) == 1024
    assert gpu.seq_reserve_batch(m, list(range(B)), [ctx] * B) >= 0
    for s in range(B):
        kv = gen.seq_kv((3, s), ctx, hkv, d, 0, 16)
        assert gpu.kv_write(m, s, 0, kv["k"], kv["v"]) == ctx
    g = torch.Generator(device="cpu"); g.manual_seed(1)
    q = torch.randn((B * chunk, hq, d), generator=g).to(torch.bfloat16).view(torch.int16).cuda()
    out = torch.empty((B * chunk, hq, d), dtype=torch.float32, device="cuda")
    ctxd = torch.full((B,), ctx, dtype=torch.int32, device="cuda")
    ql = np.full(B, chunk, dtype=np.int32)
    for _ in range(3):
        assert gpu.prefill_attention_dev(m, q, ql, ctxd, out) == 0
    torch.cuda.synchronize()
    condition(torch, lambda i: gpu.prefill_attention_dev(m, q, ql, ctxd, out), condition_ms)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        gpu.prefill_attention_dev(m, q, ql, ctxd, out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 20
    # the chunk's write path: the same 8 x 512 tokens appended to the cache (they overwrite themselves)
    kn = torch.randn((B * chunk, hkv, d), generator=g).to(torch.bfloat16).view(torch.int16).cuda()
    vn = torch.randn((B * chunk, hkv, d), generator=g).to(torch.bfloat16).view(torch.int16).cuda()
    for _ in range(2):
        assert gpu.kv_append_chunk_dev(m, kn, vn, ql, ctxd) == B * chunk
    torch.cuda.synchronize()
    e0.record()
    for _ in range(20):
        gpu.kv_append_chunk_dev(m, kn, vn, ql, ctxd)
    e1.record()
    torch.cuda.synchronize()
    append_us = e0.elapsed_time(e1) / 20 * 1e3
    assert gpu.device_errors() == 0
    pairs = B * sum(prefix + i + 1 for i in range(chunk))
    flops = 4.0 * d * hq * pairs
    for s in range(B):
        gpu.seq_release(m, s)
    gpu.balloon_resize(m, 0); gpu.model_unregister(m); gpu.pool_destroy(pool)
    tf = flops / ms / 1e9
    return {"workload": "8 sequences x (2048 cached + 512 new tokens), 32 q heads / 8 kv heads / head dim 128, bf16 cache",
            "us_per_call": round(ms * 1e3, 1), "useful_tflops": round(tf, 1), "gflop_per_call": round(flops / 1e9, 1),
            "kv_append_chunk_us": round(append_us, 1),
            "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0, "unit": "TFLOP/s", "frac": round(tf / 2500.0, 4)}}


def policy_leg():
    """Host time of the two policy calls at serving-loop sizes (no GPU work)."""
    import numpy as np
    from paper_2505_04021_amd import binding
    rng = np.random.default_rng(7)
    n = 1000
    arrival, slo = rng.uniform(0, 5, n), rng.choice([0.5, 1.0, 2.0, 4.0], n)
    p, c = rng.integers(1, 64, n) * 32.0, rng.choice([256.0, 512.0, 1024.0], n)
    t0 = time.perf_counter()
    for _ in range(50):
        acc = binding.arbitrate_requests(arrival, slo, p, c, 2.5)
    t1 = time.perf_counter()
    M = 64
    rate, size, s_, w = rng.uniform(1, 100, M), np.ones(M), rng.choice([0.05, 0.1], M), rng.uniform(1, 20, M)
    cur = rng.integers(-1, 8, M).astype(np.int32)
    for _ in range(50):
        binding.place_models(8, 288.0, 0.05, rate, size, s_, w, cur)
    t2 = time.perf_counter()
    return {"arbitrate_1000_requests_us": round((t1 - t0) / 50 * 1e6, 1), "accepted": len(acc),
            "place_64_models_8_gpus_us": round((t2 - t1) / 50 * 1e6, 1), "kind": "host wall clock per call through the binding"}


def cpu_baseline(rep, seconds):
    """The oracle, as it stands, on the same workload: the same bookkeeping calls and
    KV, decode attention of every model's batch on all host cores, repeated with the
    queries of successive steps until about `seconds` of CPU time have been spent."""
    import numpy as np
    from oracle import Oracle
    from workloads.scenarios import Runner
    orc = Oracle()
    r = Runner(orc, rep.cfg).setup()
    step_bytes = r.kv_bytes_step()
    t_total, n = 0.0, 0
    while t_total < seconds and n < 1000:
        for mi in r.active_models():
            q = r.queries(n, mi)
            t0 = time.perf_counter()
            rc, _ = orc.decode_attention(r.models[mi], q, r.ctx[mi])
            t_total += time.perf_counter() - t0
            assert rc == 0
        n += 1
    threads = orc.num_threads()
    # the same step on one thread (one step: a few seconds)
    orc.set_num_threads(1)
    t1 = 0.0
    for mi in r.active_models():
        q = r.queries(n, mi)
        t0 = time.perf_counter()
        rc, _ = orc.decode_attention(r.models[mi], q, r.ctx[mi])
        t1 += time.perf_counter() - t0
        assert rc == 0
    orc.set_num_threads(threads)
    r.teardown()
    return {"value": round(step_bytes * n / t_total / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle", "step_us": round(t_total / n * 1e6, 1),
            "one_thread_gbps": round(step_bytes / t1 / 1e9, 3), "one_thread_step_us": round(t1 * 1e6, 1),
            "sample": f"{n} full decode steps of replica 0 ({step_bytes / 1e6:.1f} MB of KV each, "
                      f"{t_total:.1f} s in total, fp64, {threads} OpenMP threads), then one step on one thread"}


def bursty_run(gpu, torch, args):
    """The bursty scenario (models switch on and off by a two-state Markov chain): each
    step first applies its bookkeeping events (release + deflate of a model that went idle,
    inflate + admission of one that woke up), then decodes every active model in one
    launch.  The KV cache keeps whatever the pool memory holds (the values do not change
    the time), queries are drawn once per model.  `value` counts the KV bytes of the
    decoded steps over the whole wall time, events included."""
    import numpy as np
    from workloads.scenarios import Runner, make_config
    cfg = make_config(3, args.size)
    if args.frame_bytes:
        cfg.frame_bytes = args.frame_bytes
    total = args.warmup + args.steps
    if total > cfg.steps:
        print(f"bench.py: the scenario has {cfg.steps} steps; --warmup + --steps is {total}", file=sys.stderr)
        sys.exit(2)
    r = Runner(gpu, cfg, write_kv=False).setup()
    qs = [torch.from_numpy(r.queries(0, mi).view(np.int16)).cuda() for mi in range(len(cfg.models))]
    outs = [torch.empty((s.batch, s.q_heads, s.head_dim), dtype=torch.float32, device="cuda") for s in cfg.models]
    ctxs = [torch.zeros(s.batch, dtype=torch.int32, device="cuda") for s in cfg.models]
    uids = [None] * len(cfg.models)

    def step(t):
        r.step(t)
        act = r.active_models()
        for mi in act:
            if uids[mi] is None or not np.array_equal(uids[mi], r.uid[mi]):    # a new batch was admitted
                ctxs[mi].copy_(torch.from_numpy(r.ctx[mi]))
                uids[mi] = r.uid[mi].copy()
        if act:
            rc = gpu.decode_attention_multi_dev([r.models[mi] for mi in act], [qs[mi] for mi in act],
                                                [ctxs[mi] for mi in act], [outs[mi] for mi in act])
            assert rc == 0, (rc, gpu.last_error())
            forms[gpu.last_kernel_form()] += 1
        return r.kv_bytes_step() if act else 0, len(act)

    forms = [0, 0]            # launches per kernel form (the library chooses per launch)
    gpu.tune_xcd(min(args.tune, args.warmup))
    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    n_events0 = len(r.log)
    gpu.timing_enable(1)
    forms[0] = forms[1] = 0
    kv, active, launches = 0, 0, 0
    t0 = time.perf_counter()
    for t in range(args.warmup, total):
        b, a = step(t)
        kv += b
        active += a
        launches += 1 if a else 0
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    n_rec, attn_ms = gpu.timing_read()
    gpu.timing_enable(False)
    assert gpu.device_errors() == 0 and n_rec == launches
    attn_gbps = kv / (attn_ms * 1e-3) / 1e9 if n_rec else 0.0
    result = {
        "metric": "kv_read_gbps_multi_model_paged_decode", "value": round(kv / wall / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "cfg": 3, "size": args.size, "frame_bytes": cfg.frame_bytes,
                   "pool_bytes": cfg.pool_bytes, "models": len(cfg.models),
                   "mean_active_models": round(active / args.steps, 2), "decode_launches": launches,
                   "bookkeeping_calls": len(r.log) - n_events0,
                   "kv_bytes_per_launch": int(kv / max(launches, 1))},
        "roofline": {"bound": "hbm", "kernel": KERNEL_FORM_NAME[0 if forms[0] >= forms[1] else 1], "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(attn_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "avg_launch_us": round(attn_ms / max(n_rec, 1) * 1e3, 2), "launches": n_rec,
                     "launches_by_kernel": dict(zip(KERNEL_FORM_NAME, forms))},
    }
    r.teardown()
    print(json.dumps(result), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2505_04021_amd import PrismKV

    gpu = PrismKV("cuda:0")
    gpu.set_split(args.items, args.min_share)
    if args.page_cost >= 0:
        gpu.set_page_cost(args.page_cost)
    gpu.set_segment_cost(args.seg_cost)
    assert gpu.set_kernel_form(args.kernel_form) == 0
    if args.config == 3:
        return bursty_run(gpu, torch, args)
    reps = build_replicas(gpu, args.config, args.size, args.replicas, args.frame_bytes, args.layers)
    inputs = [device_inputs(torch, rep, 0) for rep in reps]
    kv_per_rep = [rep.kv_bytes_step() for rep in reps]

    def step(i):
        mids, qs, ctxs, outs = inputs[i % len(reps)]
        if args.layers > 1:
            for m in mids:
                gpu.set_layer(m, (i // len(reps)) % args.layers)
        rc = gpu.decode_attention_multi_dev(mids, qs, ctxs, outs)
        assert rc == 0, (rc, gpu.last_error())

    for c in [int(x) for x in args.sweep_items.split(",") if x]:
        gpu.set_split(c, args.min_share)
        for i in range(10):
            step(i)
        torch.cuda.synchronize()
        gpu.timing_enable(True)
        t0 = time.perf_counter()
        for i in range(60):
            step(i)
        torch.cuda.synchronize()
        w = (time.perf_counter() - t0) / 60
        n_rec, a_ms = gpu.timing_read()
        gpu.timing_enable(False)
        print(f"[sweep] items {c:6d}: step {w * 1e6:7.1f} us  attention kernel {a_ms / n_rec * 1e3:7.1f} us",
              file=sys.stderr, flush=True)
    gpu.set_split(args.items, args.min_share)

    if args.tune > 0:             # part of the set-up, like any autotuning: never inside the timed region
        gpu.tune_xcd(args.tune)
        for i in range(args.tune):
            step(i)
        torch.cuda.synchronize()
    n_cond = condition(torch, step, args.condition_ms)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # The library launches on torch's current stream (PrismKV binds it), so these two events sit on the
    # kernel's own stream.  A step is exactly one k_attention launch: the events' span over the timed
    # region divided by the launches is the kernel's average duration, gaps between launches included.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert gpu.device_errors() == 0
    dev_ms = ev0.elapsed_time(ev1)

    total_bytes = sum(kv_per_rep[i % len(reps)] for i in range(args.steps))
    ms_per_step = wall * 1e3 / args.steps
    gbps = total_bytes / wall / 1e9
    attn_avg_ms = dev_ms / args.steps
    attn_gbps = total_bytes / (dev_ms * 1e-3) / 1e9

    # second opinion, outside the timed region: an event pair around single launches (the library
    # records them itself); each pair adds about 2 us of its own to what it brackets
    gpu.timing_enable(1)
    for i in range(min(args.steps, 64)):
        step(i)
    torch.cuda.synchronize()
    n_rec, br_ms = gpu.timing_read()
    gpu.timing_enable(False)

    result = {
        "metric": "kv_read_gbps_multi_model_paged_decode",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if args.config != 5 else "fp8_e4m3",
        "data": "synthetic",
        "config": {"workload": reps[0].cfg.name, "cfg": args.config, "size": args.size,
                   "frame_bytes": reps[0].cfg.frame_bytes, "layers": args.layers,
                   "replicas_rotated": len(reps), "kv_bytes_per_step": int(np.mean(kv_per_rep)),
                   "work_items": args.items or "auto", "xcd_tune_launches": args.tune,
                   "conditioning_launches": n_cond,
                   "xcd_weights": [round(x, 3) for x in gpu.get_xcd_weights()]},
        "step_us": round(ms_per_step * 1e3, 2),
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "device_ms_per_step": round(dev_ms / args.steps, 5),
        "roofline": {"bound": "hbm", "kernel": KERNEL_FORM_NAME[gpu.last_kernel_form()], "achieved": round(attn_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": None if args.frame_bytes or args.layers > 1 else profiled_traffic(KERNEL_FORM_NAME[gpu.last_kernel_form()], reps[0].cfg.name, args.size),
                     "avg_launch_us": round(attn_avg_ms * 1e3, 2), "launches": args.steps,
                     "bracketed_single_launch_us": round(br_ms / max(n_rec, 1) * 1e3, 2)},
    }
    result["read_ceiling_gbps"] = {"stream": round(gpu.stream_read_probe(4 << 30, 0, 10), 1),
                                   "scattered_8KiB": round(gpu.stream_read_probe(4 << 30, 8 << 10, 10), 1),
                                   "scattered_64KiB": round(gpu.stream_read_probe(4 << 30, 64 << 10, 10), 1)}
    if not args.no_balloon:
        result["balloon_resize"] = balloon_latency(gpu, torch)
        result["kv_append"] = append_latency(gpu, torch, reps[0], inputs[0])
        result["prefill_attention"] = prefill_leg(gpu, torch, min(args.condition_ms, 1000))
        result["policies"] = policy_leg()
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(reps[0], args.cpu_seconds)
    for rep in reps:
        rep.teardown()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
