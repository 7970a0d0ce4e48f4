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
                    help="decode kernel: 0 = two waves per SIMD, 1 = one wave per SIMD and as many waves as keep the memory busy, -1 = chosen by the launch")
    ap.add_argument("--tune", type=int, default=24,
                    help="weight updates the library's own tuning of the per-XCD shares may make (24 = what a process starts with; 0 = equal weights)")
    ap.add_argument("--no-legs", dest="legs", action="store_false", help="skip the secondary workloads (cfg 1, 3, 4, 5, cfg 2 on 64 KiB frames)")
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
    # the same calls enqueue-only: what a call costs the stream (events around 50 inflate / deflate pairs and
    # around 50 reserve / release pairs, back to back) and what it costs the host to issue
    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    e0.record()
    for _ in range(50):
        gpu.balloon_resize_enqueue(m, 176)
        gpu.balloon_resize_enqueue(m, 0)
    e1.record()
    h1 = time.perf_counter()
    last = gpu.balloon_resize_enqueue(m, 176)
    for _ in range(50):
        gpu.seq_reserve_batch_enqueue(m, seqs, ctx)
        last = gpu.seq_release_batch_enqueue(m, seqs)
    e2.record()
    assert gpu.ticket_result(last) == 5632
    torch.cuda.synchronize()
    assert gpu.balloon_resize(m, 0) == 0 and gpu.device_errors() == 0
    gpu.model_unregister(m)
    gpu.pool_destroy(pool)
    med = lambda x: round(float(np.median(x) * 1e6), 2)
    res = {"inflate_176_frames_us": med(t_inf), "deflate_176_frames_us": med(t_def),
           "inflate_us_per_frame": round(med(t_inf) / 176, 4), "deflate_us_per_frame": round(med(t_def) / 176, 4),
           "reserve_batch_5632_blocks_us": med(t_res), "release_176_blocks_us": med(t_rel),
           "kind": "host wall clock per call (launch + kernel + result read-back), median of 50",
           "enqueued_resize_176_frames_device_us": round(e0.elapsed_time(e1) * 1e3 / 100, 2),
           "enqueued_resize_device_us_per_frame": round(e0.elapsed_time(e1) * 1e3 / 100 / 176, 4),
           "enqueued_resize_host_us": round((h1 - h0) * 1e6 / 100, 2),
           "enqueued_reserve_plus_release_5632_blocks_device_us": round(e1.elapsed_time(e2) * 1e3 / 50, 2),
           "enqueued_kind": "enqueue-only forms: stream time per call from events around 100 back-to-back calls; host time to issue one"}
    # The same balloon on an elastic pool (frames have memory while owned, or while they wait in the
    # pre-allocation buffer on top of the free stack).  Without a buffer the call maps every frame itself;
    # with a buffer of 176 frames two models take turns, so that every inflate is a cold one (frames the
    # model never held) and finds its frames ready, refilled by the library's thread between the calls.
    for name, spare in (("elastic", 0), ("elastic_prealloc_176", 176)):
        pool = gpu.pool_create_elastic(8 << 30, 16, 2 << 20)
        assert pool >= 0, gpu.last_error()
        assert gpu.pool_set_prealloc(pool, spare) == spare
        ms = [gpu.model_register(pool, 32, 8, 128, 0, 32, 512), gpu.model_register(pool, 32, 8, 64, 0, 32, 512)]
        t_inf, t_def, t_settle = [], [], []
        for i in range(12):
            m = ms[i % 2]
            t0 = time.perf_counter(); assert gpu.balloon_resize(m, 176) == 176; t1 = time.perf_counter()
            gpu.pool_prealloc_wait(pool)
            t2 = time.perf_counter(); assert gpu.balloon_resize(m, 0) == 0; t3 = time.perf_counter()
            gpu.pool_prealloc_wait(pool); t4 = time.perf_counter()
            t_inf.append(t1 - t0); t_def.append(t3 - t2); t_settle.append(t4 - t3)
        st = gpu.pool_stats(pool)
        assert st["mapped_bytes"] == spare * (2 << 20), st
        for m in ms:
            gpu.model_unregister(m)
        gpu.pool_destroy(pool)
        res[name + "_inflate_176_frames_us"] = med(t_inf[2:])
        res[name + "_deflate_176_frames_us"] = med(t_def[2:])
        res[name + "_thread_catches_up_after_deflate_us"] = med(t_settle[2:])
        res[name + "_first_inflate_us"] = round(t_inf[0] * 1e6, 2)
    res["elastic_kind"] = ("host wall clock per balloon_resize call; two models take turns, so every inflate takes frames "
                           "its model never held; no call unmaps (the library's thread does, afterwards)")
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


def prefill_leg(gpu, torch, condition_ms=1000, dtype=0):
    """Chunked prefill on one model of the headline workload's shape (32 q heads, 8 kv heads, head dim
    128; dtype 0: bf16 cache, 1: e4m3 cache): 8 sequences with 2048 cached tokens each take a chunk of 512.
    Reports device time per call and the rate of useful attention flops (4 * D * heads * visible (query,
    key) pairs)."""
    import numpy as np
    from workloads import gen
    hq, hkv, d, B, prefix, chunk = 32, 8, 128, 8, 2048, 512
    pool = gpu.pool_create(8 << 30, 16, 2 << 20)
    assert pool >= 0 and gpu.pool_seed_free_order(pool, gen.free_order((8 << 30) // (2 << 20), gen.generator(5))) == 0
    m = gpu.model_register(pool, hq, hkv, d, dtype, B, 1024)
    ctx = prefix + chunk
    assert m >= 0 and gpu.balloon_resize(m, 1024) == 1024
    assert gpu.seq_reserve_batch(m, list(range(B)), [ctx] * B) >= 0
    for s in range(B):
        kv = gen.seq_kv((3, s), ctx, hkv, d, dtype, 16)
        assert gpu.kv_write(m, s, 0, kv["k"], kv["v"], kv["k_scale"], kv["v_scale"]) == ctx
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
    return {"workload": "8 sequences x (2048 cached + 512 new tokens), 32 q heads / 8 kv heads / head dim 128, "
                        + ("bf16" if dtype == 0 else "e4m3") + " cache",
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


def percentiles(us):
    import numpy as np
    a = np.asarray(us, dtype=np.float64)
    return {"median": round(float(np.median(a)), 2), "p10": round(float(np.percentile(a, 10)), 2),
            "p90": round(float(np.percentile(a, 90)), 2), "n": int(a.size)}


def per_step_times(torch, step, n):
    """Device time of n consecutive steps, one by one: an event behind every step on the library's
    stream; a step's time is the span to the event before it (the gap to the next launch included)."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(n):
        step(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    return [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n)]


LAUNCHES = [0]      # decode launches this process has issued (profiles slice their kernel trace by it)


def timed_decode(gpu, torch, step_fn, bytes_of_step, steps, warmup, condition_ms):
    """The timing protocol of a decode workload: conditioning, warm-up, `steps` timed steps between two
    events on the library's stream (and the host's clock around them), then the same steps once more
    with an event behind each for the spread."""
    def step(i):
        LAUNCHES[0] += 1
        step_fn(i)

    n_cond = condition(torch, step, condition_ms) if condition_ms > 0 else 0
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    first_timed = LAUNCHES[0]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = ev0.elapsed_time(ev1)
    total = sum(bytes_of_step(i) for i in range(steps))
    dist = percentiles(per_step_times(torch, step, min(steps, 200)))
    return {"wall_s": wall, "dev_ms": dev_ms, "bytes": total, "n_cond": n_cond, "dist": dist,
            "form": gpu.last_kernel_form(), "items": gpu.last_launch_items(), "timed_launches": [first_timed, first_timed + steps]}


def decode_summary(t, steps):
    """step time, GB/s and fraction of the HBM peak of a timed_decode() result, by the device's clock"""
    us = t["dev_ms"] * 1e3 / steps
    gbps = t["bytes"] / (t["dev_ms"] * 1e-3) / 1e9
    return {"step_us": round(us, 2), "step_us_wall": round(t["wall_s"] * 1e6 / steps, 2), "step_us_spread": t["dist"],
            "kv_gbps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "kernel": KERNEL_FORM_NAME[t["form"]], "work_items": t["items"], "steps": steps}


def static_leg(gpu, torch, cfg_id, steps, warmup, condition_ms, replicas, frame_bytes=0):
    """A secondary workload with a fixed batch (cfg 1, 2, 4, 5): set up, timed by the same protocol, torn down."""
    reps = build_replicas(gpu, cfg_id, "full", replicas, frame_bytes)
    inputs = [device_inputs(torch, rep, 0) for rep in reps]
    kv = [rep.kv_bytes_step() for rep in reps]

    def step(i):
        mids, qs, ctxs, outs = inputs[i % len(reps)]
        rc = gpu.decode_attention_multi_dev(mids, qs, ctxs, outs)
        assert rc == 0, (rc, gpu.last_error())

    t = timed_decode(gpu, torch, step, lambda i: kv[i % len(reps)], steps, warmup, condition_ms)
    assert gpu.device_errors() == 0
    res = decode_summary(t, steps)
    res.update({"workload": reps[0].cfg.name, "kv_bytes_per_step": int(sum(kv) / len(kv)), "replicas_rotated": len(reps),
                "frame_bytes": reps[0].cfg.frame_bytes, "ideal_us_at_hbm_peak": round(sum(kv) / len(kv) / HBM_PEAK_GBPS / 1e3, 1)})
    for rep in reps:
        rep.teardown()
    return res


def bursty_leg(gpu, torch, size, steps, warmup, frame_bytes=0):
    """The bursty scenario (cfg 3: models switch on and off by a two-state Markov chain): each step
    first issues its bookkeeping (release + deflate of a model that fell idle, inflate + admission of
    one that woke up: one enqueue-only call each, nothing waits), then decodes every active model in
    one launch.  The scenario is laid out as data beforehand, so the timed loop holds the library's
    calls and nothing of the harness; the calls' results are fetched one step late (they must all be
    successes) and never waited for.  The KV cache keeps whatever the pool memory holds (the values do
    not change the time), queries are drawn once per model.  The whole-step figure counts the KV bytes
    of the decoded steps over the whole wall time, bookkeeping included."""
    import numpy as np
    from workloads.scenarios import Runner, make_config
    cfg = make_config(3, size)
    if frame_bytes:
        cfg.frame_bytes = frame_bytes
    total = warmup + steps
    if total > cfg.steps:
        print(f"bench.py: the scenario has {cfg.steps} steps; --warmup + --steps is {total}", file=sys.stderr)
        sys.exit(2)
    r = Runner(gpu, cfg, write_kv=False, mode="enqueue").setup()
    tape = r.plan(0, total)
    n = len(cfg.models)
    qs = [torch.from_numpy(r.queries(0, mi).view(np.int16)).cuda() for mi in range(n)]
    outs = [torch.empty((s.batch, s.q_heads, s.head_dim), dtype=torch.float32, device="cuda") for s in cfg.models]
    ctxs = [torch.zeros(s.batch, dtype=torch.int32, device="cuda") for s in cfg.models]
    staged = [[torch.from_numpy(adm[mi]).pin_memory() if mi in adm else None for mi in range(n)] for _, _, adm, _ in tape]
    forms = [0, 0]
    tickets = []              # (step, ticket) of calls whose result has not been looked at yet

    def step(t):
        calls, act, adm, _ = tape[t]
        for name, mi, a in calls:
            tk = getattr(gpu, name)(r.models[mi], *a)
            assert tk >= 0, (name, tk)
            tickets.append((t, tk))
        for mi in adm:
            ctxs[mi].copy_(staged[t][mi], non_blocking=True)
        if act:
            rc = gpu.decode_attention_multi_dev([r.models[mi] for mi in act], [qs[mi] for mi in act],
                                                [ctxs[mi] for mi in act], [outs[mi] for mi in act])
            assert rc == 0, (rc, gpu.last_error())
            forms[gpu.last_kernel_form()] += 1
            LAUNCHES[0] += 1
        while tickets and tickets[0][0] < t:          # the previous steps' calls: done long ago
            res = gpu.ticket_result(tickets.pop(0)[1])
            assert res >= 0, res

    for t in range(warmup):
        step(t)
    torch.cuda.synchronize()
    gpu.timing_enable(1)
    forms[0] = forms[1] = 0
    first_timed = LAUNCHES[0]
    t0 = time.perf_counter()
    for t in range(warmup, total):
        step(t)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    n_rec, attn_ms = gpu.timing_read()
    gpu.timing_enable(False)
    while tickets:
        assert gpu.ticket_result(tickets.pop(0)[1]) >= 0
    kv = sum(tape[t][3] for t in range(warmup, total) if tape[t][1])
    launches = sum(1 for t in range(warmup, total) if tape[t][1])
    active = sum(len(tape[t][1]) for t in range(warmup, total))
    book = sum(len(tape[t][0]) for t in range(warmup, total))
    assert gpu.device_errors() == 0 and n_rec == launches
    # per-call cost of the enqueue-only bookkeeping on this pool, on the device: event spans around single calls
    attn_gbps = kv / (attn_ms * 1e-3) / 1e9 if n_rec else 0.0
    res = {"workload": cfg.name, "size": size, "frame_bytes": cfg.frame_bytes, "pool_bytes": cfg.pool_bytes, "models": n,
           "steps": steps, "mean_active_models": round(active / steps, 2), "decode_launches": launches,
           "bookkeeping_calls": book, "bookkeeping_calls_per_step": round(book / steps, 2),
           "kv_bytes_per_launch": int(kv / max(launches, 1)),
           "whole_step_us": round(wall * 1e6 / steps, 2), "whole_job_kv_gbps": round(kv / wall / 1e9, 1),
           "attention_avg_launch_us": round(attn_ms / max(n_rec, 1) * 1e3, 2), "attention_kv_gbps": round(attn_gbps, 1),
           "attention_frac_of_hbm_peak": round(attn_gbps / HBM_PEAK_GBPS, 4),
           "whole_step_over_attention": round((wall * 1e3 / steps) / (attn_ms / max(n_rec, 1)), 3) if n_rec else None,
           "launches_by_kernel": dict(zip(KERNEL_FORM_NAME, forms)), "timed_launches": [first_timed, LAUNCHES[0]],
           "ideal_us_at_hbm_peak": round(kv / max(launches, 1) / HBM_PEAK_GBPS / 1e3, 1),
           "kind": "attention: an event pair around every decode launch (each pair adds about 2 us); whole step: host clock "
                   "over all steps, enqueue-only bookkeeping included"}
    r.flush()
    r.teardown()
    return res


def bursty_run(gpu, torch, args):
    """--config 3 as the headline: the whole-job figure of the bursty scenario."""
    leg = bursty_leg(gpu, torch, args.size, args.steps, args.warmup, args.frame_bytes)
    result = {
        "metric": "kv_read_gbps_multi_model_paged_decode", "value": leg["whole_job_kv_gbps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(leg["whole_step_us"] / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": leg["workload"], "cfg": 3, "size": args.size, "frame_bytes": leg["frame_bytes"],
                   "pool_bytes": leg["pool_bytes"], "models": leg["models"], "mean_active_models": leg["mean_active_models"],
                   "decode_launches": leg["decode_launches"], "bookkeeping_calls": leg["bookkeeping_calls"],
                   "kv_bytes_per_launch": leg["kv_bytes_per_launch"]},
        "roofline": {"bound": "hbm", "kernel": max(leg["launches_by_kernel"], key=leg["launches_by_kernel"].get),
                     "achieved": leg["attention_kv_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": leg["attention_frac_of_hbm_peak"], "traffic": profiled_traffic("k_attention_deep", leg["workload"], args.size),
                     "avg_launch_us": leg["attention_avg_launch_us"], "launches": leg["decode_launches"],
                     "timed_launches": leg["timed_launches"], "launches_by_kernel": leg["launches_by_kernel"]},
        "bursty": leg,
    }
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

    bytes_of_step = lambda i: kv_per_rep[i % len(reps)]       # noqa: E731
    for c in [int(x) for x in args.sweep_items.split(",") if x]:
        gpu.set_split(c, args.min_share)
        t = timed_decode(gpu, torch, step, bytes_of_step, 60, 10, 0)
        print(f"[sweep] items {c:6d}: step {t['dev_ms'] / 60 * 1e3:7.1f} us", file=sys.stderr, flush=True)
    gpu.set_split(args.items, args.min_share)

    # First with equal weights and the library's tuning of them switched off: what a launch costs before
    # the library has learnt anything about this chip.
    gpu.tune_xcd(0)
    gpu.set_xcd_weights(None)
    untuned = timed_decode(gpu, torch, step, bytes_of_step, min(args.steps, 100), args.warmup, min(args.condition_ms, 300))
    # Then as any caller gets it: the library tunes the per-XCD weights by itself over its first launches
    # (here: the conditioning and warm-up launches), without any call from outside and without ever waiting.
    gpu.tune_xcd(args.tune)
    # The library launches on torch's current stream (PrismKV binds it), so the events of timed_decode sit
    # on the kernel's own stream.  A step is exactly one attention launch: the events' span over the timed
    # region divided by the launches is the kernel's average duration, gaps between launches included.
    t = timed_decode(gpu, torch, step, bytes_of_step, args.steps, args.warmup, args.condition_ms)
    assert gpu.device_errors() == 0
    wall, dev_ms, total_bytes = t["wall_s"], t["dev_ms"], t["bytes"]
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

    kernel = KERNEL_FORM_NAME[gpu.last_kernel_form()]
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
                   "work_items": t["items"], "work_items_chosen_by": "--items" if args.items else "the library, per launch", "xcd_weight_updates_allowed": args.tune,
                   "conditioning_launches": t["n_cond"],
                   "xcd_weights": [round(x, 3) for x in gpu.get_xcd_weights()],
                   "xcd_weights_found_by": "the library itself, during the conditioning and warm-up launches (no tuning call)"},
        "step_us": round(ms_per_step * 1e3, 2),
        "step_us_spread": t["dist"],
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "device_ms_per_step": round(dev_ms / args.steps, 5),
        "untuned": dict(decode_summary(untuned, min(args.steps, 100)), kind="equal XCD weights, the library's tuning switched off"),
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(attn_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": None if args.frame_bytes or args.layers > 1 else profiled_traffic(kernel, reps[0].cfg.name, args.size),
                     "traffic_kind": "stored figure of the committed rocprofv3 counter summary of this workload, not read in this run",
                     "avg_launch_us": round(attn_avg_ms * 1e3, 2), "launches": args.steps,
                     "timed_launches": t["timed_launches"],
                     "bracketed_single_launch_us": round(br_ms / max(n_rec, 1) * 1e3, 2)},
    }
    result["read_ceiling_gbps"] = {"stream": round(gpu.stream_read_probe(4 << 30, 0, 10), 1),
                                   "scattered_8KiB": round(gpu.stream_read_probe(4 << 30, 8 << 10, 10), 1),
                                   "scattered_64KiB": round(gpu.stream_read_probe(4 << 30, 64 << 10, 10), 1)}
    if not args.no_balloon:
        result["balloon_resize"] = balloon_latency(gpu, torch)
        result["kv_append"] = append_latency(gpu, torch, reps[0], inputs[0])
        result["prefill_attention"] = prefill_leg(gpu, torch, min(args.condition_ms, 1000))
        e4 = prefill_leg(gpu, torch, min(args.condition_ms, 500), dtype=1)
        result["prefill_attention"]["e4m3_cache"] = {k: e4[k] for k in ("us_per_call", "useful_tflops", "kv_append_chunk_us")}
        result["policies"] = policy_leg()
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(reps[0], args.cpu_seconds)
    for rep in reps:
        rep.teardown()
    if args.legs and args.config == 2 and args.size == "full" and not args.frame_bytes and args.layers == 1:
        # the other workloads, each by the same protocol (shorter), so that one run covers all five
        c = min(args.condition_ms, 300)
        legs = {}
        legs["cfg1"] = static_leg(gpu, torch, 1, 200, 20, c, 1)
        legs["cfg2_64KiB_frames"] = static_leg(gpu, torch, 2, 200, 20, c, 3, frame_bytes=65536)
        legs["cfg4"] = static_leg(gpu, torch, 4, 100, 10, c, 1)
        legs["cfg5"] = static_leg(gpu, torch, 5, 200, 20, c, 2)
        legs["cfg3"] = bursty_leg(gpu, torch, "full", 400, 30)
        result["configs"] = legs
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
