#!/usr/bin/env python3
"""Benchmark of the paged-KV attention hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workloads decode,cold,resume,mixed,merged]
  (merged: the scheduler's decode queue in one launch)
  further workloads, not in the default run: controller (the TPOT-driven loop on partitions), cushare
  (throughput against CU share), copycal (counter yardstick)

Prints ONE JSON line.  The headline metric is decode-attention HBM GB/s on the
decode-only configuration (64 sessions, contexts U[1024, 4096], 32/8 heads,
head_dim 128, page 16, bf16).  A step is one pass of the decode path over the
batch: ag_kv_append of the step's token for every session, then
ag_attn_decode.  (ag_decode_step, the same step in one launch, is timed beside
it.)  The same line carries the two prefill configurations
(TFLOP/s against the dense bf16 MFMA peak), the mixed-load decode-step
percentiles under CU-masked streams, and the fp64 oracle timed on the host.

All inputs are synthetic and seeded (paper_2603_10342_amd/inputs.py) and are
resident in HBM before any timed region starts.  Throughput figures count
ALGORITHMIC bytes / flops only (every cached K/V byte once; 4*D flop per
visible query-key pair and head).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic_pmc.txt")


def measured_traffic(key):
    """HBM bytes per launch (read + write) that rocprofv3's FETCH_SIZE / WRITE_SIZE counters showed for a kernel on a
    workload.  NOT measured in this run: counter runs cannot be taken inside this script, so the figure is read
    from the committed summary profiles/hbm_traffic_pmc.txt (see traffic_source())."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == key:
            return int(f[1]) + int(f[2])
    return None


def traffic_source():
    """Where `traffic` comes from: the summary file and the library commit it was taken at (its first line)."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None
    first = open(path).readline().strip().lstrip("# ")
    return f"{TRAFFIC_FILE} ({first}); a separate rocprofv3 --pmc run, not this run"


def roofline(bound, achieved, peak, unit, key, **extra):
    r = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
         "traffic": measured_traffic(key), "traffic_source": traffic_source()}
    r.update(extra)
    return r


def pct(xs, p):
    """Nearest-rank percentile."""
    s = sorted(xs)
    k = max(0, min(len(s) - 1, int(np.ceil(p / 100.0 * len(s))) - 1))
    return s[k]


class Dev:
    """A seeded Batch moved to the device once."""

    def __init__(self, b, torch, dev="cuda"):
        from paper_2603_10342_amd import inputs as I
        g = b.geom

        def t(a):
            if g.dtype == I.F32:
                return torch.from_numpy(np.ascontiguousarray(a)).to(dev)
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.bfloat16)

        def i32(a):
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)

        self.b, self.g = b, g
        self.q, self.k_new, self.v_new = t(b.q), t(b.k_new), t(b.v_new)
        self.bt, self.prefix, self.new, self.cu, self.ctx = (i32(b.block_tables), i32(b.prefix_lens), i32(b.new_lens),
                                                             i32(b.cu_new), i32(b.ctx_lens))
        self.total = b.total_new
        self.max_new = int(b.new_lens.max())
        self.max_ctx = int(b.ctx_lens.max())
        self.out = torch.zeros_like(self.q)
        self.i32 = i32


def settle(torch, step, seconds=0.3):
    """Untimed: run the step until the device has been busy for a while, so clocks and caches are in the state
    sustained serving sees (the first tens of milliseconds after an idle period run measurably slower)."""
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            step(i)
            i += 1
        torch.cuda.synchronize()


def time_steps(torch, step, steps, warmup, stream=None):
    """W untimed steps, then exactly K steps between two synchronisations.  Returns seconds per step."""
    settle(torch, step)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_time(B, torch, step, steps, warmup):
    """Mean duration (us) of the main attention kernel, from HIP events recorded around each launch on its stream."""
    B.ag_prof_enable(steps)
    try:
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        B.ag_prof_collect()
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        return B.ag_prof_collect()
    finally:
        B.ag_prof_disable()


# --------------------------------------------------------------------------- decode (config 2)
def bench_decode(args, torch, B, I):
    c = I.make_decode()
    g = c.geom
    nb = len(c.ctx_lens)
    fill, step = Dev(c.fill, torch), Dev(c.step, torch)
    ctx = step.ctx
    max_ctx = int(c.ctx_lens.max())
    sets = []
    for r in range(args.sets):
        bt = c.block_tables if r == 0 else I.deal_block_tables(I.rng_for(I.config_seed(2), 100 + r), c.ctx_lens,
                                                                g.page_size, g.num_pages, c.block_tables.shape[1])
        cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
        btd = fill.i32(bt)
        B.ag_kv_append(cache, fill.k_new, fill.v_new, btd, fill.prefix, fill.new, fill.cu, fill.total)
        sets.append((cache, btd))
    ws = torch.empty(B.ag_attn_decode_workspace_bytes(nb, g.num_q_heads, g.head_dim, max_ctx) // 4,
                     dtype=torch.float32, device="cuda")
    ws_step = torch.zeros(B.ag_decode_step_workspace_bytes(nb, g.num_q_heads, g.head_dim, max_ctx) // 4,
                          dtype=torch.float32, device="cuda")          # zeroed once; every call leaves its counters zero
    torch.cuda.synchronize()

    def one(i):
        cache, btd = sets[i % len(sets)]
        B.ag_kv_append(cache, step.k_new, step.v_new, btd, step.prefix, step.new, step.cu, step.total)
        B.ag_attn_decode(cache, step.q, step.out, btd, ctx, max_ctx, g.num_q_heads, g.scale, ws)

    def one_launch(i):
        cache, btd = sets[i % len(sets)]
        B.ag_decode_step(cache, step.k_new, step.v_new, step.q, step.out, btd, ctx, max_ctx, g.num_q_heads, g.scale, ws_step)

    sec = time_steps(torch, one, args.steps, args.warmup)
    prof = kernel_time(B, torch, one, args.steps, args.warmup)
    sec_one = time_steps(torch, one_launch, args.steps, args.warmup)
    prof_one = kernel_time(B, torch, one_launch, args.steps, args.warmup)
    # the same step recorded once per session set into a HIP graph and replayed
    graphs = []
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for r in range(len(sets)):
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=side):
            one(r)
        graphs.append(gr)
    torch.cuda.synchronize()
    sec_graph = time_steps(torch, lambda i: graphs[i % len(graphs)].replay(), args.steps, args.warmup)
    del graphs

    esz = 2
    kv_bytes = int(c.ctx_lens.astype(np.int64).sum()) * g.kv_bytes_per_token
    qo_bytes = 2 * nb * g.num_q_heads * g.head_dim * esz
    bt_bytes = int(((c.ctx_lens + g.page_size - 1) // g.page_size).sum()) * 4
    attn_bytes = kv_bytes + qo_bytes + bt_bytes
    append_bytes = 2 * nb * g.kv_bytes_per_token
    step_bytes = attn_bytes + append_bytes
    out = {
        "ms_per_step": sec * 1e3,
        "step_GBps": step_bytes / sec / 1e9,
        "attn_bytes": attn_bytes, "append_bytes": append_bytes, "kv_bytes": kv_bytes, "step_bytes": step_bytes,
        "entry_points": "ag_kv_append + ag_attn_decode (three launches)",
        "kernel": "decode_split_kernel + decode_merge_kernel (the whole ag_attn_decode call)",
        "kernel_us": prof["mean_us"], "kernel_us_min": prof["min_us"],
        "kernel_GBps": attn_bytes / (prof["mean_us"] * 1e-6) / 1e9,
        "graph_replay_ms_per_step": sec_graph * 1e3, "graph_replay_step_GBps": step_bytes / sec_graph / 1e9,
        "one_launch": {"entry_point": "ag_decode_step (append + attention + merge in one launch)",
                       "ms_per_step": sec_one * 1e3, "step_GBps": step_bytes / sec_one / 1e9,
                       "kernel_us": prof_one["mean_us"], "kernel_GBps": step_bytes / (prof_one["mean_us"] * 1e-6) / 1e9},
        "sets": len(sets), "sessions": nb, "mean_ctx": float(c.ctx_lens.mean()),
    }
    # the paper's own regime is a handful of agents (Sec. IV: 3-6 concurrent sessions): the step is then bound by
    # its launches, not by bytes - the same two ways on 4 sessions of about 1000 tokens
    gs = I.slm_geometry(1024)
    small = I.make_decode(batch=4, lo=1000, hi=1100, num_pages=1024, geom=gs, seed=I.config_seed(2) + 7)
    sf, ss = Dev(small.fill, torch), Dev(small.step, torch)
    cache0 = B.KVCache(gs.num_pages, gs.page_size, gs.num_kv_heads, gs.head_dim, gs.dtype, fill=0.0)
    B.ag_kv_append(cache0, sf.k_new, sf.v_new, sf.bt, sf.prefix, sf.new, sf.cu, sf.total)
    smax = int(small.ctx_lens.max())

    def small_two(i):
        B.ag_kv_append(cache0, ss.k_new, ss.v_new, ss.bt, ss.prefix, ss.new, ss.cu, ss.total)
        B.ag_attn_decode(cache0, ss.q, ss.out, ss.bt, ss.ctx, smax, g.num_q_heads, g.scale, ws)

    def small_one(i):
        B.ag_decode_step(cache0, ss.k_new, ss.v_new, ss.q, ss.out, ss.bt, ss.ctx, smax, g.num_q_heads, g.scale, ws_step)

    out["four_sessions_of_1000_tokens"] = {"two_calls_us": time_steps(torch, small_two, args.steps, args.warmup) * 1e6,
                                           "one_launch_us": time_steps(torch, small_one, args.steps, args.warmup) * 1e6}
    log("decode", json.dumps(out))

    if not args.no_cpu_baseline:
        from oracle import oracle as O       # cpu_baseline leg: the only use of the oracle in this file
        kp, vp = I.zero_pool(g.pool_shape, g.dtype), I.zero_pool(g.pool_shape, g.dtype)
        for b in (c.fill, c.step):
            O.kv_append(kp, vp, g.dtype, b.k_new, b.v_new, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new)
        reps, t_cpu, ref = 0, 0.0, None
        while t_cpu < 10.0 and reps < 400:
            t0 = time.perf_counter()
            ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cache, btd = sets[0]
        one(0)
        torch.cuda.synchronize()
        got = I.stored_to_f64(step.out.view(torch.int16).cpu().numpy().view(np.uint16), g.dtype)
        err = np.abs(got - ref)
        out["cpu_baseline"] = {"value": attn_bytes / (t_cpu / reps) / 1e9, "unit": "GB/s", "cores": O.num_threads(),
                               "kind": "oracle",
                               "sample": f"the whole decode batch (64 sessions), {reps} repetitions, {t_cpu:.1f} s"}
        out["check_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
                                  "rel_fro": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
        log("decode cpu", json.dumps(out["cpu_baseline"]), json.dumps(out["check_vs_oracle"]))
        del kp, vp
    return out


# --------------------------------------------------------------------------- prefill (configs 3, 4)
def bench_prefill(kind, args, torch, B, I):
    steps, warmup = max(5, args.steps // 4), max(2, args.warmup // 2)
    if kind == "cold":
        b = I.make_cold()
        g = b.geom
        cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
        d = Dev(b, torch)
    else:
        c = I.make_resume()
        b, g = c.chunk, c.geom
        cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
        f = Dev(c.fill, torch)
        B.ag_kv_append(cache, f.k_new, f.v_new, f.bt, f.prefix, f.new, f.cu, f.total)
        d = Dev(b, torch)
        del f
    torch.cuda.synchronize()

    def one(i):
        B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total)
        if kind == "cold":
            B.ag_attn_prefill(cache, d.q, d.out, d.bt, d.new, d.cu, d.total, d.max_new, g.num_q_heads, g.scale)
        else:
            B.ag_attn_resume(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx,
                             g.num_q_heads, g.scale)

    sec = time_steps(torch, one, steps, warmup)
    prof = kernel_time(B, torch, one, steps, warmup)
    flops = b.attn_flops()
    out = {
        "ms_per_step": sec * 1e3, "steps": steps, "warmup": warmup,
        "step_TFLOPs": flops / sec / 1e12, "tokens_per_s": b.total_new / sec,
        "flops": flops, "tokens": b.total_new, "sessions": b.batch,
        "kernel": "prefill_mfma_kernel", "kernel_us": prof["mean_us"], "kernel_us_min": prof["min_us"],
        "kernel_TFLOPs": flops / (prof["mean_us"] * 1e-6) / 1e12,
        "roofline": roofline("mfma", flops / (prof["mean_us"] * 1e-6) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s",
                             "prefill_mfma_kernel." + ("config3" if kind == "cold" else "config4"),
                             kernel="prefill_mfma_kernel", kernel_us=prof["mean_us"], algorithmic_flops=flops),
    }
    log(kind, json.dumps(out))

    if not args.no_cpu_baseline:
        # the oracle on a bounded, seeded sample of query rows (all 32 heads of each), timed; the same rows of the
        # GPU output are compared with it
        from oracle import oracle as O       # cpu_baseline leg
        kp, vp = I.zero_pool(g.pool_shape, g.dtype), I.zero_pool(g.pool_shape, g.dtype)
        fills = [b] if kind == "cold" else [c.fill, b]
        for x in fills:
            O.kv_append(kp, vp, g.dtype, x.k_new, x.v_new, x.block_tables, x.prefix_lens, x.new_lens, x.cu_new)
        rng = I.rng_for(I.config_seed(3 if kind == "cold" else 4), 77)
        n_rows = 8192 if kind == "cold" else 3072          # about 10 s of host time either way
        rs = rng.integers(0, b.batch, size=n_rows).astype(np.int32)
        ri = (rng.random(n_rows) * b.new_lens[rs]).astype(np.int32)
        t0 = time.perf_counter()
        ref = O.attn(kp, vp, g.dtype, b.q, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new, g.num_q_heads,
                     g.scale, rows=(rs, ri))
        t_cpu = time.perf_counter() - t0
        fl = 4 * g.head_dim * g.num_q_heads * int((b.prefix_lens[rs].astype(np.int64) + ri + 1).sum())
        one(0)
        torch.cuda.synchronize()
        rows = torch.from_numpy(b.cu_new[rs].astype(np.int64) + ri).to("cuda")
        got = I.stored_to_f64(d.out[rows].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), g.dtype)
        err = np.abs(got - ref)
        out["cpu_baseline"] = {"value": fl / t_cpu / 1e12, "unit": "TFLOP/s", "cores": O.num_threads(),
                               "kind": "oracle", "sample": f"{n_rows} random query rows x 32 heads, {t_cpu:.1f} s"}
        out["check_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
                                  "rel_fro": float(np.linalg.norm(got - ref) / np.linalg.norm(ref)), "rows": n_rows}
        log(kind + " cpu", json.dumps(out["cpu_baseline"]), json.dumps(out["check_vs_oracle"]))
        del kp, vp
    return out


# --------------------------------------------------------------------------- mixed load (config 5)
def placement(torch, B, stream, n_wg=4096):
    """Which (XCD, CU) pairs does a stream's work land on?"""
    ids = torch.zeros(n_wg, dtype=torch.int32, device="cuda")
    B.ag_probe_placement(ids, 20000, stream)
    torch.cuda.synchronize()
    v = ids.cpu().numpy().astype(np.int64)
    cu = (v & 0xFF) | (((v >> 8) & 0xF) << 8) | (((v >> 12) & 0xF) << 12)
    xcd = (v >> 16) & 0xF
    pairs = set(zip(xcd.tolist(), cu.tolist()))
    per_xcd = {}
    for x, _ in pairs:
        per_xcd[x] = per_xcd.get(x, 0) + 1
    return pairs, per_xcd


class MixedLoad:
    """Config 5's two request streams on one cache: a decode batch (stream A) and a loop of cold + resume
    prefills (stream B)."""

    def __init__(self, torch, B, I):
        m = I.make_mixed()
        g = m.geom
        self.B, self.g, self.m = B, g, m
        self.cache = cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
        self.cold, rfill, self.res, dfill, self.dec = (Dev(x, torch) for x in (m.cold, m.resume_fill, m.resume, m.decode_fill, m.decode))
        for f in (rfill, dfill):
            B.ag_kv_append(cache, f.k_new, f.v_new, f.bt, f.prefix, f.new, f.cu, f.total)
        self.max_ctx = self.dec.max_ctx
        self.ws = torch.zeros(B.ag_decode_step_workspace_bytes(self.dec.b.batch, g.num_q_heads, g.head_dim, self.max_ctx) // 4,
                              dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        self.prefill_tokens = self.cold.total + self.res.total
        self.prefill_flops = m.cold.attn_flops() + m.resume.attn_flops()
        self.kv_bytes = int(m.decode.ctx_lens.astype(np.int64).sum()) * g.kv_bytes_per_token

    def decode_step(self, st):
        """One decode step of the batch: the step's token appended, then attention, in one launch."""
        B, g, dec = self.B, self.g, self.dec
        B.ag_decode_step(self.cache, dec.k_new, dec.v_new, dec.q, dec.out, dec.bt, dec.ctx, self.max_ctx, g.num_q_heads,
                         g.scale, self.ws, stream=st)

    def prefill_loop(self, st):
        B, g, cold, res, cache = self.B, self.g, self.cold, self.res, self.cache
        B.ag_kv_append(cache, cold.k_new, cold.v_new, cold.bt, cold.prefix, cold.new, cold.cu, cold.total, stream=st)
        B.ag_attn_prefill(cache, cold.q, cold.out, cold.bt, cold.new, cold.cu, cold.total, cold.max_new,
                          g.num_q_heads, g.scale, stream=st)
        B.ag_kv_append(cache, res.k_new, res.v_new, res.bt, res.prefix, res.new, res.cu, res.total, stream=st)
        B.ag_attn_resume(cache, res.q, res.out, res.bt, res.prefix, res.new, res.cu, res.total, res.max_new,
                         res.max_ctx, g.num_q_heads, g.scale, stream=st)


def bench_mixed(args, torch, B, I, info):
    load = MixedLoad(torch, B, I)
    decode_step, prefill_loop = load.decode_step, load.prefill_loop
    prefill_tokens, prefill_flops, kv_bytes = load.prefill_tokens, load.prefill_flops, load.kv_bytes
    total_cus = info["num_cus"]
    n_xcd = info["num_xcd"] or 8
    per = total_cus // n_xcd

    def run(dstream, pstream, steps, warm=100):
        """Decode steps (one host sync each, as a real decode loop has) with an optional prefill loop beside."""
        ds = torch.cuda.ExternalStream(dstream) if dstream else torch.cuda.current_stream()
        stop = threading.Event()
        loops = [0]
        t_pref = [0.0]

        def pre():
            ps = torch.cuda.ExternalStream(pstream)
            t0 = time.perf_counter()
            while not stop.is_set():
                prefill_loop(pstream)
                ps.synchronize()
                loops[0] += 1
            t_pref[0] = time.perf_counter() - t0

        th = None
        if pstream is not None:
            th = threading.Thread(target=pre)
            th.start()
            time.sleep(0.05)
        lat = []
        for i in range(warm + steps):
            t0 = time.perf_counter()
            decode_step(dstream)
            ds.synchronize()
            if i >= warm:
                lat.append((time.perf_counter() - t0) * 1e6)
        stop.set()
        if th:
            th.join()
        r = {"p50_us": pct(lat, 50), "p99_us": pct(lat, 99), "mean_us": float(np.mean(lat)), "steps": steps}
        if th and t_pref[0] > 0:
            r["prefill_tokens_per_s"] = loops[0] * prefill_tokens / t_pref[0]
            r["prefill_TFLOPs"] = loops[0] * prefill_flops / t_pref[0] / 1e12
            r["prefill_loops"] = loops[0]
        return r

    def check_decode_while_prefill_runs(dstream, pstream):
        """The decode output of a step taken while the prefill loop runs on the other partition, against the
        oracle (every row)."""
        from oracle import oracle as O       # check leg
        m, g = load.m, load.g
        kp, vp = I.zero_pool(g.pool_shape, g.dtype), I.zero_pool(g.pool_shape, g.dtype)
        for b in (m.decode_fill, m.decode):
            O.kv_append(kp, vp, g.dtype, b.k_new, b.v_new, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new)
        ref = O.decode(kp, vp, g.dtype, m.decode.q, m.decode.block_tables, m.decode.ctx_lens, g.num_q_heads, g.scale)
        del kp, vp
        ds, ps = torch.cuda.ExternalStream(dstream), torch.cuda.ExternalStream(pstream)
        load.dec.out.fill_(float("nan"))
        torch.cuda.synchronize()
        for _ in range(3):                   # about 8 ms of prefill work queued on the other partition
            prefill_loop(pstream)
        for _ in range(4):                   # the steps run beside it; the last one's output is checked
            decode_step(dstream)
        ds.synchronize()
        busy = not ps.query()                # the prefill stream still had work when the last step finished
        got = I.stored_to_f64(load.dec.out.view(torch.int16).cpu().numpy().view(np.uint16), g.dtype)
        ps.synchronize()
        err = np.abs(got - ref)
        return {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
                "rel_fro": float(np.linalg.norm(got - ref) / np.linalg.norm(ref)), "rows": int(ref.shape[0]),
                "prefill_stream_busy_when_the_step_finished": bool(busy)}

    old_si = sys.getswitchinterval()
    sys.setswitchinterval(1e-5)
    out = {"decode_kv_bytes_per_step": kv_bytes, "prefill_tokens_per_loop": prefill_tokens,
           "prefill_flops_per_loop": prefill_flops, "decode_entry_point": "ag_decode_step",
           "p99_ratio_baseline": "decode alone on the same CU partition, prefill stream idle (isolates interference)",
           "p99_ratio_vs_full_gpu_baseline": "decode alone on the whole GPU (adds what the partition itself costs)",
           "splits": {}}
    try:
        full = out["decode_alone_full_gpu"] = run(None, None, args.mixed_steps)
        plain_a = B.ag_stream_create_cumask([0xFFFFFFFF] * ((total_cus + 31) // 32))
        plain_b = B.ag_stream_create_cumask([0xFFFFFFFF] * ((total_cus + 31) // 32))
        un = out["unmasked_two_streams"] = run(plain_a, plain_b, args.mixed_steps)
        un["p99_ratio_vs_full_gpu"] = un["p99_us"] / full["p99_us"]
        B.ag_stream_destroy(plain_a)
        B.ag_stream_destroy(plain_b)
        # the stated splits {32, 64, 96} and, beside them, larger decode shares
        for cus in (32, 64, 96, 128, 160):
            k = cus // n_xcd
            sd = B.ag_stream_create_cumask(B.ag_cumask_build(total_cus, n_xcd, 0, k))
            sp = B.ag_stream_create_cumask(B.ag_cumask_build(total_cus, n_xcd, k, per - k))
            pd, pxd = placement(torch, B, sd)
            pp, pxp = placement(torch, B, sp)
            alone = run(sd, None, args.mixed_steps)
            mixed = run(sd, sp, args.mixed_steps)
            e = {
                "decode_cus_seen": len(pd), "prefill_cus_seen": len(pp), "overlap": len(pd & pp),
                "decode_cus_per_xcd": sorted(pxd.values()), "prefill_cus_per_xcd": sorted(pxp.values()),
                "decode_alone": alone, "with_prefill": mixed,
                "p99_ratio": mixed["p99_us"] / alone["p99_us"], "p50_ratio": mixed["p50_us"] / alone["p50_us"],
                "p99_ratio_vs_full_gpu": mixed["p99_us"] / full["p99_us"],
                "p50_ratio_vs_full_gpu": mixed["p50_us"] / full["p50_us"],
                "within_1p5x_of_same_partition_alone": bool(mixed["p99_us"] <= 1.5 * alone["p99_us"]),
                "within_1p5x_of_full_gpu_alone": bool(mixed["p99_us"] <= 1.5 * full["p99_us"]),
            }
            if cus == 64 and not args.no_cpu_baseline:
                e["check_vs_oracle"] = check_decode_while_prefill_runs(sd, sp)
            out["splits"][str(cus)] = e
            log("mixed", cus, json.dumps(e))
            B.ag_stream_destroy(sd)
            B.ag_stream_destroy(sp)
    finally:
        sys.setswitchinterval(old_si)
    log("mixed", json.dumps({k: v for k, v in out.items() if k != "splits"}))
    return out


# --------------------------------------------------------------------------- decode queue in one launch
def bench_merged(args, torch, B, I):
    """The decode queue of a scheduling step (64 decodes + 8 short resume chunks) three ways: one merged launch
    (ag_attn_merged), the decode and resume entry points one after the other, and the resume entry point on
    everything."""
    lo, hi = (int(x) for x in args.merged_rows.split(","))
    c = I.make_decode_queue(n_lo=lo, n_hi=hi)
    g = c.geom
    fill, ch = Dev(c.fill, torch), Dev(c.chunk, torch)
    cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
    B.ag_kv_append(cache, fill.k_new, fill.v_new, fill.bt, fill.prefix, fill.new, fill.cu, fill.total)
    B.ag_kv_append(cache, ch.k_new, ch.v_new, ch.bt, ch.prefix, ch.new, ch.cu, ch.total)
    nd = int((c.chunk.new_lens == 1).sum())                # the decodes come first
    ws = torch.empty(B.ag_attn_merged_workspace_bytes(ch.total, g.num_q_heads, ch.max_ctx) // 4, dtype=torch.float32, device="cuda")
    wsd = torch.empty(B.ag_attn_decode_workspace_bytes(nd, g.num_q_heads, g.head_dim, ch.max_ctx) // 4, dtype=torch.float32, device="cuda")
    cu_r = (ch.cu[nd:] - nd).contiguous()
    max_new_r = int(c.chunk.new_lens[nd:].max())
    out_m, out_s, out_r = (torch.zeros_like(ch.q) for _ in range(3))
    torch.cuda.synchronize()

    def merged(i):
        B.ag_attn_merged(cache, ch.q, out_m, ch.bt, ch.prefix, ch.new, ch.cu, ch.total, ch.max_new, ch.max_ctx,
                         g.num_q_heads, g.scale, ws)

    def separate(i):
        B.ag_attn_decode(cache, ch.q[:nd], out_s[:nd], ch.bt[:nd], ch.ctx[:nd], ch.max_ctx, g.num_q_heads, g.scale, wsd)
        B.ag_attn_resume(cache, ch.q[nd:], out_s[nd:], ch.bt[nd:], ch.prefix[nd:], ch.new[nd:], cu_r, ch.total - nd,
                         max_new_r, ch.max_ctx, g.num_q_heads, g.scale)

    def resume_all(i):
        B.ag_attn_resume(cache, ch.q, out_r, ch.bt, ch.prefix, ch.new, ch.cu, ch.total, ch.max_new, ch.max_ctx,
                         g.num_q_heads, g.scale)

    steps, warmup = args.steps, args.warmup
    t_m = time_steps(torch, merged, steps, warmup)
    prof = kernel_time(B, torch, merged, steps, warmup)
    t_s = time_steps(torch, separate, steps, warmup)
    t_r = time_steps(torch, resume_all, max(5, steps // 4), 2)
    ctx = c.chunk.ctx_lens.astype(np.int64)
    kv_bytes = int(ctx.sum()) * g.kv_bytes_per_token
    qo_bytes = 2 * ch.total * g.num_q_heads * g.head_dim * 2
    bt_bytes = int(((ctx + g.page_size - 1) // g.page_size).sum()) * 4
    out = {
        "sessions_decoding": nd, "sessions_resuming": int(len(ctx) - nd), "rows": ch.total,
        "resume_rows": [int(x) for x in c.chunk.new_lens[nd:]],
        "merged_us": t_m * 1e6, "decode_then_resume_us": t_s * 1e6, "resume_entry_point_on_all_us": t_r * 1e6,
        "merged_split_kernel_us": prof["mean_us"],
        "kv_bytes_once": kv_bytes, "merged_GBps_of_kv_once": (kv_bytes + qo_bytes) / t_m / 1e9,
        # algorithmic bytes: the K/V of every session once + Q + O + 4 B per referenced page
        "roofline": roofline("hbm", (kv_bytes + qo_bytes + bt_bytes) / (prof["mean_us"] * 1e-6) / 1e9, HBM_PEAK_GBPS, "GB/s",
                             "merged_split_kernel.decode_queue", kernel="merged_split_kernel", kernel_us=prof["mean_us"],
                             algorithmic_bytes=kv_bytes + qo_bytes + bt_bytes,
                             whole_call_frac=(kv_bytes + qo_bytes + bt_bytes) / t_m / 1e9 / HBM_PEAK_GBPS),
        "flops": c.chunk.attn_flops(),
        "max_abs_merged_vs_separate": float((out_m.float() - out_s.float()).abs().max()),
        "max_abs_merged_vs_resume_all": float((out_m.float() - out_r.float()).abs().max()),
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as O       # check leg
        kp, vp = I.zero_pool(g.pool_shape, g.dtype), I.zero_pool(g.pool_shape, g.dtype)
        for b in (c.fill, c.chunk):
            O.kv_append(kp, vp, g.dtype, b.k_new, b.v_new, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new)
        b = c.chunk
        ref = O.attn(kp, vp, g.dtype, b.q, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new, g.num_q_heads, g.scale)
        got = I.stored_to_f64(out_m.view(torch.int16).cpu().numpy().view(np.uint16), g.dtype)
        err = np.abs(got - ref)
        out["check_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
                                  "rel_fro": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
    log("merged", json.dumps(out))
    return out


# --------------------------------------------------------------------------- closed loop (Algorithm 1)
class ServingLoad:
    """Config 5's sessions with resume chunks of mixed length on one cache, cut into the scheduler's two queues
    for every admission level (inputs.make_serving): the decode queue runs as one merged launch, the prefill
    queue as cold prefill + resume prefill of what was not admitted."""

    def __init__(self, torch, B, I, n_decode, levels):
        c = I.make_serving(n_decode=n_decode)
        g = c.geom
        self.B, self.g, self.c = B, g, c
        self.cache = cache = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
        for f in (c.resume_fill, c.decode_fill):
            d = Dev(f, torch)
            B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total)
        self.cold = Dev(c.cold, torch)
        self.qd = {a: Dev(c.queue_d[a], torch) for a in levels}
        self.qp = {a: (Dev(c.queue_p[a], torch) if c.queue_p[a] is not None else None) for a in levels}
        need = max(B.ag_attn_merged_workspace_bytes(d.total, g.num_q_heads, d.max_ctx) for d in self.qd.values())
        self.ws = torch.empty(need // 4, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        self.prefill_tokens = {a: self.cold.total + (self.qp[a].total if self.qp[a] is not None else 0) for a in levels}

    def level_for(self, b_prefill):
        return int((self.c.resume_lens <= b_prefill).sum())

    def decode_step(self, st, a):
        B, g, d = self.B, self.g, self.qd[a]
        B.ag_kv_append(self.cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total, stream=st)
        B.ag_attn_merged(self.cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx,
                         g.num_q_heads, g.scale, self.ws, stream=st)

    def prefill_loop(self, st, a):
        B, g, cold, res, cache = self.B, self.g, self.cold, self.qp[a], self.cache
        B.ag_kv_append(cache, cold.k_new, cold.v_new, cold.bt, cold.prefix, cold.new, cold.cu, cold.total, stream=st)
        B.ag_attn_prefill(cache, cold.q, cold.out, cold.bt, cold.new, cold.cu, cold.total, cold.max_new,
                          g.num_q_heads, g.scale, stream=st)
        if res is not None:
            B.ag_kv_append(cache, res.k_new, res.v_new, res.bt, res.prefix, res.new, res.cu, res.total, stream=st)
            B.ag_attn_resume(cache, res.q, res.out, res.bt, res.prefix, res.new, res.cu, res.total, res.max_new,
                             res.max_ctx, g.num_q_heads, g.scale, stream=st)


def bench_controller(args, torch, B, I, info):
    """The paper's loop on config 5's sessions (Sec. III-B, Algorithm 1; Sec. III-C): resume chunks no longer
    than B_prefill join the decodes in the decode queue, which a decode thread runs as one merged launch per
    step on the decode partition; cold prefills and the longer chunks form the prefill queue, which a prefill
    thread runs on the complementary partition; the scheduler closes a control interval every dt, moves
    R_min / B_prefill and rebinds.  Halfway three quarters of the decoding sessions leave.  Reports the
    trajectory, where it settles, and what a rebinding costs.  (Both threads re-run their queue at fixed
    positions, so latencies are stationary; while an admission level changes, the two threads may for one
    iteration both hold the same chunk: timing only, results are not checked here.)"""
    g_units = 4
    b_min, b_max, d_b = 64, 512, 64
    lens = np.asarray([16, 32, 64, 96, 128, 256, 384, 512])
    levels = sorted({int((lens <= b).sum()) for b in range(b_min, b_max + 1, d_b)} | {0})
    heavy = ServingLoad(torch, B, I, 64, levels)
    light = ServingLoad(torch, B, I, 16, levels)
    slots = B.Slots(g_units)
    S = slots.units()
    entries = [slots.get(i) for i in range(slots.count())]
    old_si = sys.getswitchinterval()
    sys.setswitchinterval(1e-5)
    out = {"g_units": g_units, "S": S, "entries": [e["decode_units"] for e in entries], "resume_chunk_rows": lens.tolist(),
           "admission_levels": levels}
    try:
        # reference: the decodes alone (no chunk admitted) on the whole device, same loop shape
        lat = []
        for i in range(300):
            t0 = time.perf_counter()
            heavy.decode_step(None, 0)
            torch.cuda.current_stream().synchronize()
            if i >= 100:
                lat.append((time.perf_counter() - t0) * 1e6)
        alone = pct(lat, 50)
        params = dict(S=S, r_base=g_units, r_init=g_units, b_init=b_max, delta_r=g_units, delta_b=d_b, b_min=b_min,
                      b_max=b_max, theta_low_us=1.3 * alone, theta_high_us=1.7 * alone)
        ctl = B.Controller(**params)
        dt = args.ctl_interval_ms / 1e3
        stop = threading.Event()
        cur = [slots.bind(params["r_init"])]
        adm = [heavy.level_for(params["b_init"])]
        load = [heavy]
        dec_lat, dec_after_rebind = [], []
        loops, held, ptok = [0], [0], [0]

        def decode_thread():
            last = -1
            while not stop.is_set():
                i = cur[0]
                st = entries[i]["decode_stream"]
                t0 = time.perf_counter()
                load[0].decode_step(st, adm[0])
                torch.cuda.ExternalStream(st).synchronize()
                us = (time.perf_counter() - t0) * 1e6
                ctl.record_decode(us)
                (dec_after_rebind if (i != last and last >= 0) else dec_lat).append((i, us))
                last = i

        def prefill_thread():
            while not stop.is_set():
                st = entries[cur[0]]["prefill_stream"]
                if not st:                          # the whole device is reserved for decode
                    held[0] += 1
                    time.sleep(dt / 4)
                    continue
                ld, a = load[0], adm[0]
                ld.prefill_loop(st, a)
                torch.cuda.ExternalStream(st).synchronize()
                loops[0] += 1
                ptok[0] += ld.prefill_tokens[a]

        td, tp = threading.Thread(target=decode_thread), threading.Thread(target=prefill_thread)
        t_start = time.perf_counter()
        td.start()
        tp.start()
        traj, bind_us = [], []
        n_int = args.ctl_intervals
        n_heavy_steps = 0
        for k in range(n_int):
            if k == n_int // 2:
                load[0] = light
                n_heavy_steps = len(dec_lat)
            time.sleep(dt)
            st = ctl.tick()
            t0 = time.perf_counter()
            i = slots.bind(st["r_min"])
            cur[0] = i
            bind_us.append((time.perf_counter() - t0) * 1e6)
            adm[0] = heavy.level_for(st["b_prefill"])
            traj.append({"t_ms": (time.perf_counter() - t_start) * 1e3, "tpot_us": st["tpot_us"], "r_min": st["r_min"],
                         "b_prefill": st["b_prefill"], "decode_units": entries[i]["decode_units"], "admitted": adm[0]})
        stop.set()
        td.join()
        tp.join()
        wall = time.perf_counter() - t_start
        torch.cuda.synchronize()

        def phase(tr, lats):
            tail = tr[len(tr) // 2:]                 # second half of the phase: after the transient
            ok = [x["tpot_us"] for x in tail if x["tpot_us"] == x["tpot_us"]]
            units = tail[-1]["decode_units"]
            steady = [us for (i, us) in lats[len(lats) // 2:] if entries[i]["decode_units"] == units]
            return {"settled_decode_units": units, "settled_b_prefill": tail[-1]["b_prefill"],
                    "settled_chunks_admitted": tail[-1]["admitted"],
                    "levels_seen_after_transient": sorted({x["decode_units"] for x in tail}),
                    "tpot_us_mean": float(np.mean(ok)) if ok else None,
                    "step_p50_us": pct(steady, 50) if steady else None, "step_p99_us": pct(steady, 99) if steady else None}

        out.update({
            "params": params, "interval_ms": args.ctl_interval_ms, "intervals": n_int,
            "decode_alone_p50_us": alone,
            "trajectory_r_min": [x["r_min"] for x in traj], "trajectory_b_prefill": [x["b_prefill"] for x in traj],
            "trajectory_tpot_us": [None if x["tpot_us"] != x["tpot_us"] else round(x["tpot_us"], 1) for x in traj],
            "phase_64_decoding_sessions": phase(traj[:n_int // 2], dec_lat[:n_heavy_steps]),
            "phase_16_decoding_sessions": phase(traj[n_int // 2:], dec_lat[n_heavy_steps:]),
            "decode_steps": len(dec_lat) + len(dec_after_rebind),
            "prefill_tokens_per_s": ptok[0] / wall, "prefill_loops": loops[0], "prefill_held_polls": held[0],
            "rebinds": len(dec_after_rebind),
            "rebind_host_us_mean": float(np.mean(bind_us)), "rebind_host_us_max": float(np.max(bind_us)),
            "first_step_after_rebind_us_median": pct([u for _, u in dec_after_rebind], 50) if dec_after_rebind else None,
            "epsilon_ctx_bound": float(np.max(bind_us)) / (args.ctl_interval_ms * 1e3),
        })
        ctl.close()
    finally:
        sys.setswitchinterval(old_si)
        torch.cuda.synchronize()
        slots.close()
    log("controller", json.dumps(out))
    return out


# --------------------------------------------------------------------------- CU-share profile (Fig. 3 analogue)
def bench_cushare(args, torch, B, I, info):
    """Throughput of the three request classes alone on R CUs per XCD, R = 1..32: the MI355X analogue of the
    paper's throughput-versus-SM-share profile (Sec. II-C, Fig. 3), the input of its allocation rule
    R* = min{R : mu_D(R) >= r_min} (Sec. III-B)."""
    total_cus, n_xcd = info["num_cus"], info["num_xcd"] or 8
    per = total_cus // n_xcd
    shares = [r for r in (1, 2, 4, 6, 8, 12, 16, 20, 24, 28, 32) if r <= per]

    dc = I.make_decode()
    g = dc.geom
    cache_d = B.KVCache(g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.dtype, fill=0.0)
    dfill, dstep = Dev(dc.fill, torch), Dev(dc.step, torch)
    B.ag_kv_append(cache_d, dfill.k_new, dfill.v_new, dfill.bt, dfill.prefix, dfill.new, dfill.cu, dfill.total)
    del dfill
    ws = torch.empty(B.ag_attn_decode_workspace_bytes(dstep.b.batch, g.num_q_heads, g.head_dim, dstep.max_ctx) // 4,
                     dtype=torch.float32, device="cuda")
    cold = Dev(I.make_cold(), torch)
    cache_c = B.KVCache(cold.g.num_pages, 16, 8, 128, I.BF16, fill=0.0)
    rc = I.make_resume()
    cache_r = B.KVCache(rc.geom.num_pages, 16, 8, 128, I.BF16, fill=0.0)
    rfill, res = Dev(rc.fill, torch), Dev(rc.chunk, torch)
    B.ag_kv_append(cache_r, rfill.k_new, rfill.v_new, rfill.bt, rfill.prefix, rfill.new, rfill.cu, rfill.total)
    del rfill
    torch.cuda.synchronize()

    def decode(st):
        B.ag_kv_append(cache_d, dstep.k_new, dstep.v_new, dstep.bt, dstep.prefix, dstep.new, dstep.cu, dstep.total, stream=st)
        B.ag_attn_decode(cache_d, dstep.q, dstep.out, dstep.bt, dstep.ctx, dstep.max_ctx, g.num_q_heads, g.scale, ws, stream=st)

    def coldp(st):
        B.ag_kv_append(cache_c, cold.k_new, cold.v_new, cold.bt, cold.prefix, cold.new, cold.cu, cold.total, stream=st)
        B.ag_attn_prefill(cache_c, cold.q, cold.out, cold.bt, cold.new, cold.cu, cold.total, cold.max_new, 32, cold.g.scale, stream=st)

    def resume(st):
        B.ag_kv_append(cache_r, res.k_new, res.v_new, res.bt, res.prefix, res.new, res.cu, res.total, stream=st)
        B.ag_attn_resume(cache_r, res.q, res.out, res.bt, res.prefix, res.new, res.cu, res.total, res.max_new,
                         res.max_ctx, 32, res.g.scale, stream=st)

    def rate(fn, st, n):
        ext = torch.cuda.ExternalStream(st)
        for _ in range(2):
            fn(st)
        ext.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn(st)
        ext.synchronize()
        return n / (time.perf_counter() - t0)

    out = {"cus_per_xcd": shares, "decode_steps_per_s": [], "cold_tokens_per_s": [], "resume_tokens_per_s": []}
    for r in shares:
        st = B.ag_stream_create_cumask(B.ag_cumask_build(total_cus, n_xcd, 0, r))
        out["decode_steps_per_s"].append(rate(decode, st, 40))
        out["cold_tokens_per_s"].append(rate(coldp, st, 3) * cold.total)
        out["resume_tokens_per_s"].append(rate(resume, st, 3) * res.total)
        B.ag_stream_destroy(st)
        log("cushare", r, out["decode_steps_per_s"][-1], out["cold_tokens_per_s"][-1], out["resume_tokens_per_s"][-1])
    for k in ("decode_steps_per_s", "cold_tokens_per_s", "resume_tokens_per_s"):
        out[k.split("_")[0] + "_normalised"] = [v / out[k][-1] for v in out[k]]
    # the paper's allocation rule on the measured decode profile: smallest share whose step rate meets a target
    # TPOT budget tau_max (ms): r_min = 1000 / tau_max steps per second
    out["min_share_for_tpot_ms"] = {str(tau): next((r for r, v in zip(shares, out["decode_steps_per_s"]) if v >= 1000.0 / tau), None)
                                    for tau in (0.25, 0.5, 1.0, 2.0)}
    # The paper's retention bound (Sec. III-B, Theorem 1) on the measured profiles, for the discrete allocation
    # set G = {g, 2g, ..., S} with g = 4 units: R_g* = min{R in G : mu_D(R) >= 1000 / tau_max}, overshoot delta = g
    # (one step of the allocation set), control overhead eps taken as 0 here (a rebinding is a table lookup, measured
    # by the controller workload): rho >= mu_P(S - R_g* - delta) / mu_P(S - R_g*), for an all-cold (eta = 1) and an
    # all-resume (eta = 0) prefill mix.
    gset = [r for r in shares if r % 4 == 0]
    mu = {k: dict(zip(shares, out[k])) for k in ("decode_steps_per_s", "cold_tokens_per_s", "resume_tokens_per_s")}
    bound = {}
    for tau in (0.2, 0.25, 0.3, 0.5, 1.0):
        rg = next((r for r in gset if mu["decode_steps_per_s"][r] >= 1000.0 / tau), None)
        e = {"R_g_star": rg}
        if rg is not None and per - rg - 4 in mu["cold_tokens_per_s"] and per - rg in mu["cold_tokens_per_s"] and per - rg - 4 > 0:
            e["rho_cold"] = mu["cold_tokens_per_s"][per - rg - 4] / mu["cold_tokens_per_s"][per - rg]
            e["rho_resume"] = mu["resume_tokens_per_s"][per - rg - 4] / mu["resume_tokens_per_s"][per - rg]
        bound[str(tau)] = e
    out["theorem1_bound_for_tpot_ms"] = bound
    return out


def bench_copycal(args, torch):
    """A plain device-to-device copy of known size: the yardstick the FETCH_SIZE / WRITE_SIZE counters of the
    attention kernels are scaled by (run this workload under `rocprofv3 --pmc`)."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    sec = time_steps(torch, lambda i: dst.copy_(src), 10, 2)
    out = {"bytes_read": n, "bytes_written": n, "ms": sec * 1e3, "GBps_read_plus_write": 2 * n / sec / 1e9}
    log("copycal", json.dumps(out))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workloads", default="decode,cold,resume,mixed,merged")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sets", type=int, default=4, help="disjoint session sets the decode step rotates over")
    ap.add_argument("--mixed-steps", type=int, default=2000)
    ap.add_argument("--merged-rows", default="16,64", help="range of the resume chunks' rows in the merged workload")
    ap.add_argument("--ctl-interval-ms", type=float, default=20.0, help="control interval of the closed-loop workload")
    ap.add_argument("--ctl-intervals", type=int, default=100)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1 (the path shards by session or "
              "by KV head with no exchange between GPUs, so a multi-GPU figure would be N independent copies)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_10342_amd import binding as B
    from paper_2603_10342_amd import inputs as I

    torch.cuda.set_device(0)
    info = B.ag_device_info()
    log("device", info, B.ag_version())
    want = [w for w in args.workloads.split(",") if w]
    res = {}
    if "decode" in want:
        res["decode"] = bench_decode(args, torch, B, I)
    if "cold" in want:
        res["cold_prefill"] = bench_prefill("cold", args, torch, B, I)
    if "resume" in want:
        res["resume_prefill"] = bench_prefill("resume", args, torch, B, I)
    if "mixed" in want:
        res["mixed"] = bench_mixed(args, torch, B, I, info)
    if "merged" in want:
        res["decode_queue_merged"] = bench_merged(args, torch, B, I)
    if "controller" in want:
        res["controller"] = bench_controller(args, torch, B, I, info)
    if "cushare" in want:
        res["cu_share_profile"] = bench_cushare(args, torch, B, I, info)
    if "copycal" in want:
        res["copycal"] = bench_copycal(args, torch)

    d = res.get("decode")
    line = {
        "metric": "decode_attn_hbm_GBps", "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode-only batch: 64 sessions, ctx ~ U[1024,4096], 32 q heads / 8 kv heads, "
                               "head_dim 128, page 16, 32768-page pool; step = ag_kv_append(1 token/session) + ag_attn_decode",
                   "sessions": 64, "num_q_heads": 32, "num_kv_heads": 8, "head_dim": 128, "page_size": 16,
                   "rotating_session_sets": args.sets},
        "device": info,
    }
    if d:
        line.update({
            "value": d["step_GBps"], "ms_per_step": d["ms_per_step"],
            "roofline": roofline("hbm", d["kernel_GBps"], HBM_PEAK_GBPS, "GB/s", "ag_attn_decode.config2",
                                 kernel=d["kernel"], kernel_us=d["kernel_us"], algorithmic_bytes=d["attn_bytes"]),
            "cpu_baseline": d.get("cpu_baseline"),
        })
    else:
        line.update({"value": None, "ms_per_step": None})
    line["workloads"] = res
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
