#!/usr/bin/env python3
"""Benchmark of the device-resident replay train step on one MI355X.

A "step" is one pass of the whole hot path: append the new experience(s), sample a
batch on the device, gather it, forward on s and s', TD target and loss, backward,
optimizer.  The headline value is train steps/s on the paper-shaped workload
(capacity 1,000,000, 27 floats per state, 30 actions, batch 128, MLP 27-256-256-30,
Adam) with every input already in HBM.  The same JSON line carries the gather kernel's
HBM roofline (measured live with events), the other workloads, and the CPU oracle
timed on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--legs p,pfull,phost,inram,gather,large,wide,cpu]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
FP32_VALU_PEAK_TFLOPS = 157.3

P_CFG = dict(capacity=1_000_000, D=27, A=30, B=128, H=256, burn_in=50_000, p_term=0.005,
             lr=1e-4, appends=1)
W_CFG = dict(capacity=4_000_000, D=27, A=30, B=4096, H=1024, p_term=0.005, lr=1e-4, appends=64)
L_CFG = dict(capacity=200_000, D=84 * 84 * 4, p_term=0.001)
GATHER_BATCHES = [32, 128, 512, 2048, 8192, 65536]
# HBM bytes per launch of sample_gather_pair_kernel<4, 2, 0> at batch 65,536 from rocprofv3 PMC runs
# (FETCH_SIZE 8,186.3 KiB x 2.000 + WRITE_SIZE 14,656.5 KiB x 1.000, the factors being what the
# same counters read for the 256 MiB plain copy of the copy_calibration leg); the runs and the
# table are in profiles/gather_kernels_hbm_traffic_pmc.txt.  Set to None when that kernel changes.
GATHER_65536_HBM_BYTES = (8186.3 * 2.000 + 14656.5 * 1.000) * 1024
GATHER_8M_65536_HBM_BYTES = (8215.9 * 2.000 + 14657.0 * 1.000) * 1024
GATHER_KERNEL = "sample_gather_pair_kernel<4, 2, 0>"
# the same for sample_gather_chain_kernel<1, 0> at batch 256
LARGE_256_HBM_BYTES = (7154.9 * 2.000 + 56461.1 * 1.000) * 1024
# and for append_pair_bulk_kernel<unsigned int> at 65,536 rows (profiles/append_bulk_kernel_hbm_traffic_pmc.txt)
APPEND_65536_HBM_BYTES = (7314.5 * 2.000 + 16384.0 * 1.000) * 1024
# and summed over the seven kernels of one wide step of a recorded run (profiles/wide_step_kernels_hbm_traffic_pmc.txt)
WIDE_STEP_HBM_BYTES = (90886.2 * 2.000 + 120684.0 * 1.000) * 1024


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def dev_rows(rows):
    import torch
    return {k: (None if v is None else
                torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda())
            for k, v in rows.items()}


def event_time_ms(fn, reps):
    """Average milliseconds per call of fn over `reps` back-to-back calls on the current stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for k in range(reps):
        fn(k)
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def graph_time_ms(fn, launches, replays):
    """Average milliseconds per launch when `launches` calls of fn are recorded into one graph
    and replayed back to back: kernel time plus the GPU's own inter-kernel gap, without the
    host's per-call cost."""
    import torch
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for k in range(launches):
            fn(k)
    graph.replay()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(replays):
        graph.replay()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / (launches * replays)


def prefill(ring, rows, n_total):
    """Append n_total experiences by cycling through the device copy of `rows` in large pieces."""
    d = dev_rows(rows)
    n = len(rows["a"])
    done = 0
    while done < n_total:
        m = min(n, n_total - done)
        ring.append(d["s"][:m], None if d["s_next"] is None else d["s_next"][:m], d["a"][:m],
                    d["r"][:m], d["term"][:m])
        done += m
    import torch
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- legs
def leg_paper_shaped(B, synth, steps, warmup, full_ring, host_payload=False, target_sync=0,
                     dueling=False, distinct=False, widths=None):
    """widths = (H, G): the two hidden widths instead of the workload's 256, 256."""
    import torch
    c = dict(P_CFG)
    H2 = 0
    if widths:
        c["H"], H2 = widths
    ring = B.Replay(c["capacity"], c["D"], burn_in=c["burn_in"], seed=0, max_append=4096,
                    distinct=distinct)
    base = synth.experiences(100_000, c["D"], c["A"], c["p_term"], seed=0)
    prefill(ring, base, c["capacity"] if full_ring else c["burn_in"])
    tr = B.Trainer(ring, c["H"], c["A"], c["B"], opt=B.RP_ADAM, loss=B.RP_HUBER, lr=c["lr"],
                   appends_per_step=c["appends"], target_sync=target_sync, dueling=dueling, hidden2=H2,
                   init_params=synth.init_params(c["D"], c["H"], c["A"] + (1 if dueling else 0), 0,
                                                 hidden2=H2 or None))
    stream_rows = synth.experiences(steps + warmup, c["D"], c["A"], c["p_term"], seed=1)
    src = stream_rows if host_payload else dev_rows(stream_rows)
    w = {k: v[:warmup] for k, v in src.items()}
    t = {k: v[warmup:] for k, v in src.items()}
    assert tr.steps(warmup, w["s"], w["s_next"], w["a"], w["r"], w["term"]) == warmup
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = tr.steps(steps, t["s"], t["s_next"], t["a"], t["r"], t["term"])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert done == steps
    loss = tr.last()["loss"]
    assert np.isfinite(loss)
    return {"steps_per_s": steps / dt, "ms_per_step": 1e3 * dt / steps,
            "kernels_per_step": tr.kernels_per_step(), "final_loss": loss,
            "ring_rows": ring.state()[1]}


def leg_gather_sweep(B, synth, reps, distinct=False, capacity=None, batches=None):
    """replay_sample_gather alone on a full ring (1M rows unless given); distinct = batches
    without duplicates.  Timed as a recorded graph of 100 calls with steps 0..99 (each launch
    draws other rows; one replay of the graph touches 100 x batch rows, 1.7 GB at batch 65,536,
    far more than the last-level cache holds, so rows do not survive from one use to the next)."""
    import torch
    c = P_CFG
    capacity = capacity or c["capacity"]
    ring = B.Replay(capacity, c["D"], seed=0, max_append=4096, distinct=distinct)
    prefill(ring, synth.experiences(100_000, c["D"], c["A"], c["p_term"], seed=0), capacity)
    out = []
    for batch in (batches or ([128, 2048, 8192, 65536] if distinct else GATHER_BATCHES)):
        bufs = ring.alloc_batch(batch)
        for k in range(10):
            ring.sample_gather(k, batch, out=bufs)
        ms_host = event_time_ms(lambda k: ring.sample_gather(k, batch, out=bufs), reps)
        ms = graph_time_ms(lambda k: ring.sample_gather(k, batch, out=bufs), 100, max(1, reps // 100))
        alg = batch * 2 * (2 * c["D"] + 3) * 4      # 228 B read + 228 B written per sampled row
        out.append({"batch": batch, "us_per_call": 1e3 * ms, "us_per_call_host_launched": 1e3 * ms_host,
                    "alg_bytes": alg, "GBps": alg / (ms * 1e-3) / 1e9})
    ring.close()
    return out


def leg_append_sweep(B, synth):
    """Time to add experiences as a function of the update size (the paper's update-size figure):
    n experiences per replay_append call, from device arrays (kernel time, events) and from host
    arrays (wall clock per call including the staging copies), on the paper-shaped ring."""
    import torch
    c = P_CFG
    ring = B.Replay(c["capacity"], c["D"], seed=0, max_append=65536)
    rows = synth.experiences(65536, c["D"], c["A"], c["p_term"], seed=3)
    d = dev_rows(rows)
    row_alg = 2 * (2 * c["D"] + 3) * 4          # 228 B read from the source arrays + 228 B written
    # the HIP runtime grows its pools during the first ~thousand launches of a process
    # (individual calls then take hundreds of microseconds): get past that before timing
    one = [rows[k][:1] for k in ("s", "s_next", "a", "r", "term")]
    for _ in range(2000):
        ring.append(*one)
    torch.cuda.synchronize()
    out = []
    for n in (1, 16, 256, 2000, 16384, 65536):
        dv = [d[k][:n] for k in ("s", "s_next", "a", "r", "term")]
        hv = [rows[k][:n] for k in ("s", "s_next", "a", "r", "term")]
        for _ in range(3):
            ring.append(*dv)
        reps = 200 if n <= 2000 else 50
        ms_dev = graph_time_ms(lambda k: ring.append(*dv), 20, max(1, reps // 20))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ring.append(*hv)
        torch.cuda.synchronize()
        ms_host = 1e3 * (time.perf_counter() - t0) / reps
        out.append({"update_size": n, "device_src_us_per_call": 1e3 * ms_dev,
                    "device_src_us_per_experience": 1e3 * ms_dev / n,
                    "device_src_GBps": n * row_alg / (ms_dev * 1e-3) / 1e9,
                    "host_src_us_per_call": 1e3 * ms_host,
                    "host_src_us_per_experience": 1e3 * ms_host / n})
    return out


def leg_copy_calibration(reps, n=64 * 1024 * 1024):
    """A plain device-to-device copy of known size (256 MiB read + 256 MiB written per launch):
    the "achievable" bandwidth next to the 8 TB/s peak, and the kernel whose FETCH_SIZE /
    WRITE_SIZE readings scale the HBM-traffic counters of the other kernels."""
    import torch
    a = torch.empty(n, dtype=torch.float32, device="cuda")
    b = torch.ones(n, dtype=torch.float32, device="cuda")
    for _ in range(3):
        a.copy_(b)
    ms = event_time_ms(lambda k: a.copy_(b), reps)
    return {"bytes_read": 4 * n, "bytes_written": 4 * n, "us_per_call": 1e3 * ms,
            "GBps": 8 * n / (ms * 1e-3) / 1e9}


def leg_copy_small(n, reps):
    """Plain copies of n floats each (4n bytes read + 4n written per launch), recorded in a graph
    like the gather sweep.  Every launch of a replay takes another slice of two 1 GiB buffers,
    so the data comes from HBM rather than from the 256 MB last-level cache."""
    import torch
    slices = max(2, (256 * 1024 * 1024) // n)
    a = torch.empty(slices * n, dtype=torch.float32, device="cuda")
    b = torch.ones(slices * n, dtype=torch.float32, device="cuda")

    def one(k):
        lo = (k % slices) * n
        a[lo:lo + n].copy_(b[lo:lo + n])
    launches = min(slices, 64)
    ms = graph_time_ms(one, launches, max(1, reps // launches))
    return {"bytes_read": 4 * n, "bytes_written": 4 * n, "us_per_call": 1e3 * ms,
            "GBps": 8 * n / (ms * 1e-3) / 1e9, "distinct_slices": slices}


def leg_large_state(B, reps):
    import torch
    c = L_CFG
    ring = B.Replay(c["capacity"], c["D"], B.RP_U8, B.RP_CHAIN, seed=0, max_append=64)
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    chunk = 10_000
    for lo in range(0, c["capacity"], chunk):
        s = torch.randint(0, 256, (chunk, c["D"]), dtype=torch.uint8, device="cuda", generator=g)
        a = torch.randint(0, 18, (chunk,), dtype=torch.int32, device="cuda", generator=g)
        r = torch.randn(chunk, device="cuda", generator=g)
        term = (torch.rand(chunk, device="cuda", generator=g) < c["p_term"]).to(torch.uint8)
        ring.append(s, None, a, r, term)
    torch.cuda.synchronize()
    out = []
    for batch in (32, 256):
        bufs = ring.alloc_batch(batch)
        for k in range(5):
            ring.sample_gather(k, batch, out=bufs)
        ms_host = event_time_ms(lambda k: ring.sample_gather(k, batch, out=bufs), reps)
        ms = graph_time_ms(lambda k: ring.sample_gather(k, batch, out=bufs), 50, max(1, reps // 50))
        alg = batch * (2 * c["D"] + 2 * c["D"] * 4)   # two u8 states read, two fp32 states written
        out.append({"batch": batch, "us_per_call": 1e3 * ms, "us_per_call_host_launched": 1e3 * ms_host,
                    "alg_bytes": alg, "GBps": alg / (ms * 1e-3) / 1e9})
    return out


def leg_wide(B, synth, steps, warmup):
    import torch
    c = W_CFG
    ring = B.Replay(c["capacity"], c["D"], B.RP_BF16, B.RP_PAIR, seed=0, max_append=64)
    prefill(ring, synth.experiences(250_000, c["D"], c["A"], c["p_term"], seed=0, state_dtype="bf16"),
            c["capacity"])
    tr = B.Trainer(ring, c["H"], c["A"], c["B"], param_dtype=B.RP_BF16, opt=B.RP_ADAM, lr=c["lr"],
                   appends_per_step=c["appends"],
                   init_params=synth.init_params(c["D"], c["H"], c["A"], 0))
    n = (steps + warmup) * c["appends"]
    pool = dev_rows(synth.experiences(n, c["D"], c["A"], c["p_term"], seed=1, state_dtype="bf16"))
    cut = warmup * c["appends"]
    w = {k: v[:cut] for k, v in pool.items()}
    t = {k: v[cut:] for k, v in pool.items()}
    tr.steps(warmup, w["s"], w["s_next"], w["a"], w["r"], w["term"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = tr.steps(steps, t["s"], t["s_next"], t["a"], t["r"], t["term"])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert done == steps and np.isfinite(tr.last()["loss"])
    D, H, A, Bt = c["D"], c["H"], c["A"], c["B"]
    flops = 4 * 2 * (D * H + H * H + H * A) * Bt    # forward on s and s', backward ~ 2 forwards on s
    return {"steps_per_s": steps / dt, "ms_per_step": 1e3 * dt / steps, "alg_flops": flops,
            "TFLOPs": flops * steps / dt / 1e12, "kernels_per_step": tr.kernels_per_step()}


def leg_device_vs_inram(B, synth, steps, warmup):
    """Train-step rate of the device-resident replay and of the in-RAM comparison system (host
    sampling and gather, one host-to-device copy of the batch per step) at the batch sizes of
    the paper's speed-up table, on the full 1M-row paper-shaped ring."""
    import torch
    c = P_CFG
    base = synth.experiences(100_000, c["D"], c["A"], c["p_term"], seed=0)
    stream_rows = synth.experiences(steps + warmup, c["D"], c["A"], c["p_term"], seed=1)
    fields = ("s", "s_next", "a", "r", "term")
    w = {k: stream_rows[k][:warmup] for k in fields}
    t = {k: stream_rows[k][warmup:] for k in fields}
    d_all = dev_rows(stream_rows)
    dw = {k: d_all[k][:warmup] for k in fields}
    dt_ = {k: d_all[k][warmup:] for k in fields}
    out = []
    for batch in (16, 32, 64, 128, 256):
        p0 = synth.init_params(c["D"], c["H"], c["A"], 0)
        # device-resident replay
        ring = B.Replay(c["capacity"], c["D"], burn_in=c["burn_in"], seed=0, max_append=4096)
        prefill(ring, base, c["capacity"])
        tr = B.Trainer(ring, c["H"], c["A"], batch, opt=B.RP_ADAM, loss=B.RP_HUBER, lr=c["lr"],
                       appends_per_step=1, init_params=p0)
        tr.steps(warmup, *[dw[k] for k in fields])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        assert tr.steps(steps, *[dt_[k] for k in fields]) == steps
        torch.cuda.synchronize()
        dev_rate = steps / (time.perf_counter() - t0)
        loss_dev = tr.last()["loss"]
        # in-RAM replay feeding the same step
        idle = B.Replay(8, c["D"], seed=0)
        tr2 = B.Trainer(idle, c["H"], c["A"], batch, opt=B.RP_ADAM, loss=B.RP_HUBER, lr=c["lr"],
                        appends_per_step=0, init_params=p0)
        ram = B.InRamReplay(c["capacity"], c["D"], batch, burn_in=c["burn_in"], seed=0)
        for lo in range(0, c["capacity"], 100_000):
            ram.append(*[base[k] for k in fields])
        ram.train_steps(tr2, warmup, 1, *[w[k] for k in fields])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        assert ram.train_steps(tr2, steps, 1, *[t[k] for k in fields]) == steps
        torch.cuda.synchronize()
        ram_rate = steps / (time.perf_counter() - t0)
        loss_ram = tr2.last()["loss"]
        out.append({"batch": batch, "device_steps_per_s": dev_rate, "inram_steps_per_s": ram_rate,
                    "speedup_pct": 100.0 * (dev_rate / ram_rate - 1.0),
                    "same_final_loss": bool(loss_dev == loss_ram)})
        for h in (tr, tr2, ram, ring, idle):
            h.close()
    return out


def leg_cpu_oracle(synth, seconds_budget):
    """The oracle's own append + sample + gather + train step on the paper-shaped workload."""
    import oracle
    c = P_CFG
    rows = synth.experiences(c["burn_in"] + 4096, c["D"], c["A"], c["p_term"], seed=0)
    cfg = oracle.make_cfg(c["D"], c["H"], c["A"], c["B"], loss=oracle.HUBER, opt=oracle.ADAM,
                          lr=c["lr"])
    res = {}
    for label, threads in (("all", os.cpu_count() if (os.cpu_count() or 1) <= 16 else 16), ("one", 1)):
        oracle.set_threads(threads)
        ring = oracle.Ring(c["capacity"], c["D"], burn_in=c["burn_in"])
        ring.append(rows["s"][:c["burn_in"] - 1], rows["s_next"][:c["burn_in"] - 1],
                    rows["a"][:c["burn_in"] - 1], rows["r"][:c["burn_in"] - 1],
                    rows["term"][:c["burn_in"] - 1])
        p = synth.init_params(c["D"], c["H"], c["A"], 0).astype(np.float64)
        m, v, t = np.zeros_like(p), np.zeros_like(p), 0
        k, t0 = 0, time.perf_counter()
        while True:
            j = c["burn_in"] - 1 + k
            ring.append(rows["s"][j:j + 1], rows["s_next"][j:j + 1], rows["a"][j:j + 1],
                        rows["r"][j:j + 1], rows["term"][j:j + 1])
            s, sn, a, r, term = ring.gather(ring.sample(0, k, c["B"]))
            o = oracle.train_step(cfg, p, m, v, t, s, sn, a, r, term)
            p, m, v, t = o.params, o.m, o.v, o.t
            k += 1
            if time.perf_counter() - t0 > seconds_budget / 2 or k >= 4096:
                break
        dt = time.perf_counter() - t0
        res[label] = {"steps": k, "steps_per_s": k / dt, "threads": oracle.get_threads()}
    oracle.set_threads(1)
    return res


def leg_cpu_oracle_extras(synth, threads):
    """The oracle on the other workloads: the gather sweep's six batch sizes on a full 1M-row
    ring, the Tiny workload's 100 train steps, and two steps of the wide workload."""
    import oracle
    oracle.set_threads(threads)
    res = {"threads": oracle.get_threads()}
    # gather sweep
    c = P_CFG
    rows = synth.experiences(100_000, c["D"], c["A"], c["p_term"], seed=0)
    ring = oracle.Ring(c["capacity"], c["D"])
    for _ in range(c["capacity"] // 100_000):
        ring.append(rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    g = []
    for batch in GATHER_BATCHES:
        reps, t0 = 0, time.perf_counter()
        while reps < 1000 and (reps < 3 or time.perf_counter() - t0 < 0.7):
            ring.gather(ring.sample(0, reps, batch))
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        alg = batch * 2 * (2 * c["D"] + 3) * 4
        g.append({"batch": batch, "reps": reps, "us_per_call": 1e6 * dt, "GBps": alg / dt / 1e9})
    res["gather_sweep"] = g
    del ring
    # Tiny: capacity 1024, 27-64-64-8, batch 32, SGD 1e-3, burn-in 256, one append per step, 100 steps
    rows = synth.experiences(400, 27, 8, 0.01, seed=0)
    ring = oracle.Ring(1024, 27, burn_in=256)
    ring.append(rows["s"][:255], rows["s_next"][:255], rows["a"][:255], rows["r"][:255], rows["term"][:255])
    cfg = oracle.make_cfg(27, 64, 8, 32, loss=oracle.HUBER, opt=oracle.SGD, lr=1e-3)
    p = synth.init_params(27, 64, 8, 0).astype(np.float64)
    t0 = time.perf_counter()
    for k in range(100):
        j = 255 + k
        ring.append(rows["s"][j:j + 1], rows["s_next"][j:j + 1], rows["a"][j:j + 1], rows["r"][j:j + 1],
                    rows["term"][j:j + 1])
        s_, sn, a, r, term = ring.gather(ring.sample(0, k, 32))
        p = oracle.train_step(cfg, p, None, None, 0, s_, sn, a, r, term).params
    res["tiny"] = {"steps": 100, "steps_per_s": 100 / (time.perf_counter() - t0)}
    # Wide: 27-1024-1024-30 with the bf16 rounding points, batch 4096, Adam, 64 appends per step
    w = W_CFG
    rows = synth.experiences(20_000, w["D"], w["A"], w["p_term"], seed=0, state_dtype="bf16")
    ring = oracle.Ring(20_000, w["D"], oracle.BF16)
    ring.append(rows["s"][:19_872], rows["s_next"][:19_872], rows["a"][:19_872], rows["r"][:19_872],
                rows["term"][:19_872])
    cfg = oracle.make_cfg(w["D"], w["H"], w["A"], w["B"], loss=oracle.HUBER, opt=oracle.ADAM, lr=w["lr"],
                          bf16=1)
    p = synth.init_params(w["D"], w["H"], w["A"], 0).astype(np.float64)
    m, v, t = np.zeros_like(p), np.zeros_like(p), 0
    t0 = time.perf_counter()
    for k in range(2):
        j = 19_872 + 64 * k
        ring.append(rows["s"][j:j + 64], rows["s_next"][j:j + 64], rows["a"][j:j + 64], rows["r"][j:j + 64],
                    rows["term"][j:j + 64])
        s_, sn, a, r, term = ring.gather(ring.sample(0, k, w["B"]))
        o = oracle.train_step(cfg, p, m, v, t, synth.bf16_bits_to_f32(s_), synth.bf16_bits_to_f32(sn), a, r, term)
        p, m, v, t = o.params, o.m, o.v, o.t
    res["wide"] = {"steps": 2, "steps_per_s": 2 / (time.perf_counter() - t0),
                   "note": "ring of 20,000 rows instead of 4,000,000 (the oracle's step does not depend on it)"}
    oracle.set_threads(1)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10_000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--legs", default="p,psteady,pfull,phost,pmodel,pnet,inram,gather,append,copy,large,wide,cpu")
    ap.add_argument("--gather-reps", type=int, default=1000)
    ap.add_argument("--wide-steps", type=int, default=2000)
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only; --gpus %d is not supported "
                 "(no collectives or multi-GPU sharding are part of it)" % args.gpus)
    legs = set(args.legs.split(","))

    import torch
    from paper_1801_03138_amd import binding as B
    from paper_1801_03138_amd import synth
    B.lib()   # raises if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    out = {}
    log("[bench] paper-shaped train steps (burn-in ring) ...")
    p = leg_paper_shaped(B, synth, args.steps, args.warmup, full_ring=False)
    log("[bench]   %.0f steps/s, %d kernels/step" % (p["steps_per_s"], p["kernels_per_step"]))
    if "psteady" in legs:
        # a fixed-length run whatever --steps says, so that the steady-state rate is on record
        log("[bench] paper-shaped train steps, fixed 10,000-step run ...")
        out["paper_shaped_steady_state"] = leg_paper_shaped(B, synth, 10_000, 500, full_ring=False)
        out["paper_shaped_steady_state"]["steps"] = 10_000
        out["paper_shaped_steady_state"]["warmup"] = 500
        log("[bench]   %.0f steps/s" % out["paper_shaped_steady_state"]["steps_per_s"])
    if "pfull" in legs:
        log("[bench] paper-shaped train steps (full 1M-row ring) ...")
        out["paper_shaped_full_ring"] = leg_paper_shaped(B, synth, args.steps, args.warmup, True)
        log("[bench]   %.0f steps/s" % out["paper_shaped_full_ring"]["steps_per_s"])
    if "phost" in legs:
        log("[bench] paper-shaped train steps, append payload from host memory ...")
        out["paper_shaped_host_payload"] = leg_paper_shaped(B, synth, args.steps, args.warmup,
                                                            False, host_payload=True)
        log("[bench]   %.0f steps/s" % out["paper_shaped_host_payload"]["steps_per_s"])
    if "pmodel" in legs:
        log("[bench] paper-shaped train steps with the paper's model options (frozen target network "
            "synced every 10,000 updates; dueling head) ...")
        out["paper_shaped_target_network"] = leg_paper_shaped(B, synth, args.steps, args.warmup, False,
                                                              target_sync=10_000)
        out["paper_shaped_dueling"] = leg_paper_shaped(B, synth, args.steps, args.warmup, False, dueling=True)
        out["paper_shaped_dueling_target_network"] = leg_paper_shaped(
            B, synth, args.steps, args.warmup, False, target_sync=10_000, dueling=True)
        out["paper_shaped_without_duplicates"] = leg_paper_shaped(B, synth, args.steps, args.warmup, False,
                                                                  distinct=True)
        for k in ("paper_shaped_target_network", "paper_shaped_dueling", "paper_shaped_dueling_target_network",
                  "paper_shaped_without_duplicates"):
            log("[bench]   %-42s %8.0f steps/s, %d kernels/step" %
                (k, out[k]["steps_per_s"], out[k]["kernels_per_step"]))
    if "pnet" in legs:
        # the paper's own network: shared layer 128, value and advantage stream 512 each, dueling
        # head, frozen target network synced every 10,000 updates (Deep Q-Network Model), fp32
        log("[bench] paper-shaped replay with the paper's own network 27-128-(512+512)-(1+30) ...")
        k = "paper_network_27_128_1024_dueling_target"
        out[k] = leg_paper_shaped(B, synth, args.steps, args.warmup, False, target_sync=10_000,
                                  dueling=True, widths=(128, 1024))
        out[k]["network"] = "27-128-(512+512)-(1+30), fp32, dueling head, target network"
        log("[bench]   %.0f steps/s, %d kernels/step" % (out[k]["steps_per_s"], out[k]["kernels_per_step"]))
    if "inram" in legs:
        log("[bench] device-resident replay vs in-RAM replay with a per-step batch copy ...")
        out["device_vs_inram"] = leg_device_vs_inram(B, synth, min(args.steps, 4000), 200)
        for g in out["device_vs_inram"]:
            log("[bench]   B=%-4d device %8.0f steps/s   in-RAM %8.0f steps/s   %+6.1f %%" %
                (g["batch"], g["device_steps_per_s"], g["inram_steps_per_s"], g["speedup_pct"]))
    roofline = None
    rooflines = []
    if "gather" in legs:
        log("[bench] gather sweep on the full 1M-row ring ...")
        out["gather_sweep"] = leg_gather_sweep(B, synth, args.gather_reps)
        for g in out["gather_sweep"]:
            log("[bench]   B=%-6d %8.2f us  %8.1f GB/s" % (g["batch"], g["us_per_call"], g["GBps"]))
        g = out["gather_sweep"][-1]
        roofline = {"kernel": GATHER_KERNEL, "workload": "gather sweep, batch %d, "
                    "capacity 1,000,000, 27 fp32 per state" % g["batch"], "bound": "hbm",
                    "achieved": g["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": g["GBps"] / HBM_PEAK_GBS, "traffic": GATHER_65536_HBM_BYTES,
                    "alg_bytes_per_launch": g["alg_bytes"], "us_per_launch": g["us_per_call"],
                    "note": "the 256 MB ring is about the size of the last-level cache: a cache / HBM mix; "
                            "see rooflines for a 2 GB ring and the 5.6 GB large-state ring"}
        rooflines.append(dict(roofline))
        # the same kernel on a ring eight times the size of the last-level cache
        big = leg_gather_sweep(B, synth, max(100, args.gather_reps // 4), capacity=8_000_000,
                               batches=[65536])[0]
        out["gather_8M_row_ring"] = big
        log("[bench]   8M-row ring (2 GB) B=65536 %8.2f us  %8.1f GB/s" % (big["us_per_call"], big["GBps"]))
        rooflines.append({"kernel": GATHER_KERNEL, "workload": "gather, batch 65536, capacity 8,000,000 "
                          "(2 GB ring, eight times the last-level cache), 27 fp32 per state",
                          "bound": "hbm", "achieved": big["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": big["GBps"] / HBM_PEAK_GBS, "traffic": GATHER_8M_65536_HBM_BYTES,
                          "alg_bytes_per_launch": big["alg_bytes"], "us_per_launch": big["us_per_call"]})
    if "gather" in legs:
        out["gather_sweep_without_duplicates"] = leg_gather_sweep(B, synth, max(100, args.gather_reps // 4),
                                                                  distinct=True)
        for g in out["gather_sweep_without_duplicates"]:
            log("[bench]   without duplicates B=%-6d %8.2f us  %8.1f GB/s" %
                (g["batch"], g["us_per_call"], g["GBps"]))
    if "append" in legs:
        log("[bench] append: time per experience against the update size ...")
        out["append_sweep"] = leg_append_sweep(B, synth)
        for g in out["append_sweep"]:
            log("[bench]   n=%-6d device src %8.2f us/call %9.4f us/exp %7.1f GB/s | host src %9.2f us/call "
                "%9.4f us/exp" % (g["update_size"], g["device_src_us_per_call"],
                                  g["device_src_us_per_experience"], g["device_src_GBps"],
                                  g["host_src_us_per_call"], g["host_src_us_per_experience"]))
        g = out["append_sweep"][-1]
        rooflines.append({"kernel": "append_pair_bulk_kernel<unsigned int>", "workload": "append %d experiences "
                          "from device arrays into the 1M-row ring, 27 fp32 per state" % g["update_size"],
                          "bound": "hbm", "achieved": g["device_src_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": g["device_src_GBps"] / HBM_PEAK_GBS, "traffic": APPEND_65536_HBM_BYTES,
                          "alg_bytes_per_launch": g["update_size"] * 2 * (2 * P_CFG["D"] + 3) * 4,
                          "us_per_launch": g["device_src_us_per_call"]})
    if "copy" in legs:
        log("[bench] plain device-to-device copy, 256 MiB ...")
        out["copy_calibration"] = leg_copy_calibration(20)
        log("[bench]   %.1f GB/s" % out["copy_calibration"]["GBps"])
        if roofline is not None:
            roofline["frac_of_copy_bandwidth"] = roofline["achieved"] / out["copy_calibration"]["GBps"]
            # a plain copy that moves as many bytes as the roofline launch (half read, half written)
            small = leg_copy_small(roofline["alg_bytes_per_launch"] // 8, 640)
            out["copy_same_bytes_as_gather"] = small
            roofline["frac_of_same_size_copy"] = roofline["achieved"] / small["GBps"]
            log("[bench]   same-size copy (%.1f MB): %.2f us, %.1f GB/s" %
                (8 * (roofline["alg_bytes_per_launch"] // 8) / 1e6, small["us_per_call"], small["GBps"]))
    if "large" in legs:
        log("[bench] large-state gather (200,000 x 84x84x4 uint8, one state per slot) ...")
        out["large_state_gather"] = leg_large_state(B, max(50, args.gather_reps // 5))
        for g in out["large_state_gather"]:
            g["frac_hbm"] = g["GBps"] / HBM_PEAK_GBS
            log("[bench]   B=%-6d %8.2f us  %8.1f GB/s" % (g["batch"], g["us_per_call"], g["GBps"]))
        g = out["large_state_gather"][-1]
        rooflines.append({"kernel": "sample_gather_chain_kernel<1, 0>", "workload": "large-state gather, batch "
                          "%d, 200,000 x 84x84x4 uint8 (5.6 GB ring), uint8 -> fp32 / 255" % g["batch"],
                          "bound": "hbm", "achieved": g["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": g["GBps"] / HBM_PEAK_GBS, "traffic": LARGE_256_HBM_BYTES,
                          "alg_bytes_per_launch": g["alg_bytes"], "us_per_launch": g["us_per_call"]})
    if "wide" in legs:
        log("[bench] wide fused step (bf16, batch 4096, 27-1024-1024-30) ...")
        w = leg_wide(B, synth, args.wide_steps, 10)
        w["frac_mfma"] = w["TFLOPs"] / BF16_MFMA_PEAK_TFLOPS
        out["wide_step"] = w
        log("[bench]   %.1f steps/s, %.1f TFLOP/s" % (w["steps_per_s"], w["TFLOPs"]))
        rooflines.append({"kernel": "whole wide step (%d kernels step by step, one fewer in the recorded runs "
                                    "timed here; the dense products are gemm_nt_kernel)" % w["kernels_per_step"],
                          "workload": "wide fused step: batch 4096, 27-1024-1024-30, bf16 operands, fp32 "
                                      "accumulation, Adam, 64 appends per step", "bound": "mfma",
                          "achieved": w["TFLOPs"], "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": w["frac_mfma"], "traffic": WIDE_STEP_HBM_BYTES, "alg_flops_per_step": w["alg_flops"],
                          "us_per_step": 1e3 * w["ms_per_step"]})
    cpu = None
    if "cpu" in legs:
        log("[bench] CPU oracle on the paper-shaped workload ...")
        o = leg_cpu_oracle(synth, args.cpu_seconds)
        cpu = {"value": o["all"]["steps_per_s"], "unit": "steps/s", "cores": o["all"]["threads"],
               "kind": "oracle",
               "sample": "%d paper-shaped train steps (append 1, sample+gather 128, 27-256-256-30 "
                         "step, Adam) after a 50,000-row burn-in" % o["all"]["steps"],
               "value_1thread": o["one"]["steps_per_s"], "host_cpus": os.cpu_count()}
        log("[bench]   %.1f steps/s on %d threads, %.1f on one" %
            (cpu["value"], cpu["cores"], cpu["value_1thread"]))
        log("[bench] CPU oracle on the gather sweep, the Tiny workload and the wide workload ...")
        x = leg_cpu_oracle_extras(synth, cpu["cores"])
        cpu["gather_sweep"] = x["gather_sweep"]
        cpu["tiny"] = x["tiny"]
        cpu["wide"] = x["wide"]
        for g in x["gather_sweep"]:
            log("[bench]   gather B=%-6d %10.1f us  %6.2f GB/s" % (g["batch"], g["us_per_call"], g["GBps"]))
        log("[bench]   Tiny %.0f steps/s; wide %.3f steps/s" % (x["tiny"]["steps_per_s"], x["wide"]["steps_per_s"]))

    line = {
        "metric": "replay train steps/sec at B=128, cap 1M; gather GB/s vs HBM peak",
        "value": p["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": p["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "paper-shaped: capacity 1,000,000, state 27 fp32, 30 actions, "
                               "burn-in 50,000, 1 append/step from HBM, batch 128, MLP 27-256-256-30, "
                               "Huber, Adam 1e-4, one HIP graph per step",
                   "kernels_per_step": p["kernels_per_step"]},
        "roofline": roofline, "rooflines": rooflines, "cpu_baseline": cpu,
        # context only: another machine, another framework, the paper's own dueling network
        "paper_context": {"speedup_in_gpu_vs_in_ram_pct": {"16": 30.54, "32": 54.87, "64": 67.08,
                                                           "128": 114.41, "256": 114.35},
                          "at_batch_128_pct": 114.41,
                          "hardware": "one NVIDIA TITAN X (Pascal) 12 GB, TensorFlow, fp32",
                          "source": "the paper's Table 1 (Results)",
                          "compare_with": "device_vs_inram[batch 128].speedup_pct"},
    }
    line.update(out)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
