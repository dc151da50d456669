#!/usr/bin/env python3
"""Benchmark of the MixKVQ decode hot path on one MI355X.

A step = one pass of the whole hot path for one batch: mixkvq_quantize_append of
one new token per sequence (with the block flush, channel re-selection and
quantize-and-pack whenever the residual window is full) followed by
mixkvq_decode_attention with |q| accumulation.  Inputs are synthetic and already
resident in HBM when the timed region starts.

Before the W counted warm-up steps every cache copy is stepped once and the GPU is kept busy with uncounted steps
for about 20 ms; then exactly K steps are timed between two synchronisations.  With no --config the headline is
configuration 1 (the metric's workload); configurations 2, 3 (decode) and 4 (prefill) are timed in the same run and
reported under "other_workloads".

Prints ONE JSON line (see the fields below).  `value` is effective bandwidth:
algorithmic bytes of a decode step (minimal representation of the method: packed
codes, fp16 scale/zero per group, fp16-tier values, index bytes, the fp16 residual
window, q in and out) divided by the measured time per step.
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
LLC_BYTES = 256 << 20   # last-level (Infinity) cache

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE in KiB per
    dispatch, each scaled by what the same counter read for a plain device copy of known size in the same run), as
    listed in profiles/hbm_traffic.txt beside the commands that measured them.  None when the table has no such row
    (the counters are not read while the benchmark runs)."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                col = line.split()
                if len(col) >= 6 and not line.startswith("#") and col[0] == workload and col[1] == kernel:
                    fetch_kib, write_kib, fetch_scale, write_scale = (float(x) for x in col[2:6])
                    return round(fetch_kib * 1024 * fetch_scale + write_kib * 1024 * write_scale, 1)
    except OSError:
        pass
    return None


def copy_kernel_gbs():
    """Bandwidth of a plain device copy (512 MiB read + 512 MiB written per call), the practical reference
    beside the nominal 8 TB/s: GB/s of read + written bytes."""
    import torch
    n = 512 << 20
    x = torch.empty(n, dtype=torch.uint8, device="cuda")
    y = torch.empty_like(x)
    for _ in range(3):
        y.copy_(x)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        y.copy_(x)
    b.record()
    torch.cuda.synchronize()
    gbs = 10 * 2 * n / (a.elapsed_time(b) * 1e-3) / 1e9
    del x, y
    return gbs


def algorithmic_bytes_thresholds(w, gc, r):
    """The same count under the threshold policy, where every block has its own tier sizes: they are read from
    the channel lists of the cache's block records (entries other than 255)."""
    lay, k16, ks = gc.layout, w.k16, w.k4 + w.k16
    nb = gc.state()[0] // w.R
    idx = gc.block_records()[:, :nb, lay.off_idx:lay.off_idx + ks]
    n16 = (idx[..., :k16] != 255).sum(dim=-1).double()
    n4 = (idx[..., k16:] != 255).sum(dim=-1).double()
    D, R, ng, g = w.D, w.R, w.R // w.Gk, w.Hq // w.Hkv
    nlo = D - n16 - n4
    per_block = R * nlo / 4 + ng * nlo * 4 + R * n4 / 2 + ng * n4 * 4 + R * n16 * 2 + (n16 + n4) \
        + R * D // 4 + R * (D // w.Gv) * 4
    total = float(per_block.sum()) + w.B * w.Hkv * (r * D * 4 + g * D * 4)
    return int(total), float(n16.mean()), float(n4.mean())


def algorithmic_bytes(w, n_q, r):
    """Bytes one decode step must move, all (batch, KV head) pairs."""
    D, ks, g = w.D, w.k4 + w.k16, w.Hq // w.Hkv
    nb, ng = n_q // w.R, n_q // w.Gk
    per_pair = (n_q * (D - ks) // 4 + ng * (D - ks) * 4 + n_q * w.k4 // 2 + ng * w.k4 * 4 + n_q * w.k16 * 2
                + nb * ks + n_q * D // 4 + n_q * (D // w.Gv) * 4 + r * D * 4 + g * D * 4)
    return per_pair * w.B * w.Hkv


class HipEvents:
    """hipEvent pairs straight from the HIP runtime (they must be recorded on the
    stream the kernel runs on, inside the library call)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0 and self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            ms = ctypes.c_float()
            assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            out.append(ms.value)
        return out

    def destroy(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def build_inputs(cfg_id, w, host_batch):
    """K, V [B, Hkv, T, D], prompt queries and per-step tensors on the device.
    `host_batch` batch entries are drawn on the host; the others are device-side
    copies with the channel order rolled (so that channel selection differs)."""
    import numpy as np
    import torch
    import synth_inputs as S
    hb = min(host_batch, w.B)
    K, V, _ = S.heavy_tailed_kv(cfg_id, hb, w.Hkv, w.T)
    Qp = S.outlier_queries(cfg_id, hb, w.Hq, 256)
    qs = S.outlier_queries(cfg_id, hb, w.Hq, 8, stream=3)
    dk = torch.empty((w.B, w.Hkv, w.T, w.D), dtype=torch.float16, device="cuda")
    dv = torch.empty_like(dk)
    dqp = torch.empty((w.B, w.Hq, 256, w.D), dtype=torch.float16, device="cuda")
    dq = torch.empty((8, w.B, w.Hq, w.D), dtype=torch.float16, device="cuda")
    hk, hv, hq, hs = (torch.from_numpy(a).cuda() for a in (K, V, Qp, qs))
    for b in range(w.B):
        src, roll = b % hb, 7 * (b // hb)
        dk[b] = torch.roll(hk[src], roll, dims=-1)
        dv[b] = torch.roll(hv[src], roll, dims=-1)
        dqp[b] = torch.roll(hq[src], roll, dims=-1)
        dq[:, b] = torch.roll(hs[src], roll, dims=-1).permute(1, 0, 2)
    host = dict(K=K, V=V, Qp=Qp, qs=qs)
    return dk, dv, dqp, dq, host


def cpu_baseline(cfg_id, w, host, budget_s=20.0):
    """The oracle's decode step (append one token, attention) timed on the host for
    one batch entry at full context."""
    import numpy as np
    from oracle import mixkvq_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    cfg = O.OracleConfig(B=1, Hq=w.Hq, Hkv=w.Hkv, D=w.D, T_max=w.T + w.R, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    oc = O.OracleCache(cfg)
    K, V, Qp, qs = host["K"][:1], host["V"][:1], host["Qp"][:1], host["qs"][:1]
    sel = oc.select_channels(Qp, K)
    oc.append(K, V, sel)                       # prefill: not timed
    n, t0 = 0, time.perf_counter()
    while True:
        q1 = np.ascontiguousarray(qs[:, :, n % qs.shape[2]])
        oc.append(K[:, :, n:n + 1], V[:, :, n:n + 1])
        oc.decode_attention(q1, accumulate_q=True)
        n += 1
        el = time.perf_counter() - t0
        if el > budget_s or n >= 8:
            break
    import dataclasses
    w1 = dataclasses.replace(w, B=1)
    nbytes = algorithmic_bytes(w1, oc.n_quant, oc.n_res)
    return {"value": round(nbytes * n / el / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} decode steps of 1 of {w.B} batch entries (all {w.Hkv} KV heads, {w.T} tokens), "
                      f"{el / n * 1e3:.0f} ms per step"}


def build_prefill_inputs(cfg_id, w, Lq):
    """K, V [B, Hkv, T, D] and the prompt queries [B, Hq, Lq, D] of the prefill workload on the device: one batch
    entry is drawn on the host, the others are device-side copies with the channel order rolled by 7 per entry."""
    import torch
    import synth_inputs as S
    K, V, _ = S.heavy_tailed_kv(cfg_id, 1, w.Hkv, w.T)
    Q = S.outlier_queries(cfg_id, 1, w.Hq, Lq)
    dk = torch.empty((w.B, w.Hkv, w.T, w.D), dtype=torch.float16, device="cuda")
    dv = torch.empty_like(dk)
    dq = torch.empty((w.B, w.Hq, Lq, w.D), dtype=torch.float16, device="cuda")
    hk, hv, hq = (torch.from_numpy(a).cuda() for a in (K, V, Q))
    for b in range(w.B):
        dk[b] = torch.roll(hk[0], 7 * b, dims=-1)
        dv[b] = torch.roll(hv[0], 7 * b, dims=-1)
        dq[b] = torch.roll(hq[0], 7 * b, dims=-1)
    del hk, hv, hq
    return dk, dv, dq, dict(K=K, V=V, Q=Q)


def prefill_bytes(w, Lq):
    """(fp16 input bytes, bytes written) of one prefill pass: K, V and the prompt queries in; block records and the
    residual window out."""
    P = w.B * w.Hkv
    kv = 2 * P * w.T * w.D * 2
    qb = w.B * w.Hq * Lq * w.D * 2
    n_q = w.R * (-(-w.T // w.R) - 1)
    out = algorithmic_bytes(w, n_q, 0) - P * (w.Hq // w.Hkv) * w.D * 4 + P * (w.T - n_q) * w.D * 4
    return kv + qb, out


def bench_prefill(args, w, cfg_id):
    """Configuration 4: full-prompt channel scoring + top-k + mixed-precision pack.  A step = cache reset and
    mixkvq_prefill(Q, K, V) (= mixkvq_select_channels(Q, K), then mixkvq_quantize_append(K, V, sel)) over the whole batch."""
    import torch
    import paper_2512_19206_amd as M
    import synth_inputs as S
    Lq = w.T
    dk, dv, dq, _ = build_prefill_inputs(cfg_id, w, Lq)
    kw = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, D=w.D, T_max=-(-w.T // w.R) * w.R, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16)
    gc = M.Cache(M.make_config(**kw))
    sel = torch.empty((w.B, w.Hkv, w.k4 + w.k16), dtype=torch.uint8, device="cuda")

    def step(with_q=True, per_block=False):
        gc.reset()
        if per_block:
            M.mixkvq_select_channels(gc, dq if with_q else None, dk, sel=sel)
            M.mixkvq_quantize_append(gc, dk, dv, sel=None)
        else:
            M.mixkvq_prefill(gc, dq if with_q else None, dk, dv, sel=sel)

    def timed(n, **kws):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step(**kws)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    n_steps, n_warm = min(args.steps, 8), min(args.warmup, 2)
    for _ in range(n_warm):
        step()
    el = timed(n_steps)
    el_noq = timed(n_steps, with_q=False)
    el_pb = timed(n_steps, per_block=True)
    in_b, out_b = prefill_bytes(w, Lq)
    in_noq = in_b - w.B * w.Hq * Lq * w.D * 2
    value = in_b / el / 1e9
    # measured HBM bytes of the step's three streaming kernels (the full-size workload only: that is what was profiled)
    traffic = None
    if w == S.WORKLOADS[cfg_id]:
        parts = [measured_traffic(w.name, k) for k in ("qabs_accumulate_kernel", "key_range_kernel", "flush_block_fast_kernel")]
        if all(x is not None for x in parts):
            traffic = round(sum(parts), 1)
    result = {
        "metric": "prefill quantization: GB/s of fp16 input consumed (K, V, prompt queries)", "value": round(value, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": n_steps, "warmup": n_warm, "ms_per_step": round(el * 1e3, 4),
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "T": w.T, "Lq": Lq, "Gk": w.Gk,
                   "Gv": w.Gv, "R": w.R, "k4": w.k4, "k16": w.k16, "input_bytes": in_b, "written_bytes": out_b,
                   "step": "cache_reset + mixkvq_prefill(Q, K, V) = select_channels(Q, K) + quantize_append(K, V, sel)"},
        "without_prompt_queries": {"ms_per_step": round(el_noq * 1e3, 4), "value": round(in_noq / el_noq / 1e9, 2),
                                   "unit": "GB/s", "input_bytes": in_noq},
        "per_block_selection": {"ms_per_step": round(el_pb * 1e3, 4), "value": round(in_b / el_pb / 1e9, 2), "unit": "GB/s",
                                "note": "same calls, but every block is scored on its own tokens inside the pack kernel "
                                        "(sel = NULL) instead of using the selection made over the whole prompt"},
        "roofline": {"bound": "hbm", "kernel": "whole step (qabs_accumulate, key_range, flush_block: streaming kernels)",
                     "achieved": round((in_b + out_b) / el / 1e9, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round((in_b + out_b) / el / 1e9 / HBM_PEAK_GBS, 4), "traffic": traffic},
    }
    del dq
    copy_gbs = copy_kernel_gbs()
    result["copy_kernel"] = {"value": round(copy_gbs, 1), "unit": "GB/s read+write, 512 MiB device copy on this box",
                             "pct_of_copy_kernel": round(100 * (in_b + out_b) / el / 1e9 / copy_gbs, 2)}
    return result


def bench_decode(args, cfg_id, steps, warmup, with_cpu_baseline):
    """Decode configurations 1-3: a step = mixkvq_decode_step (append one token per sequence, with the block flush and
    channel re-selection whenever the window is full, then attention with |q| accumulation).  Returns the result dict."""
    import torch
    import paper_2512_19206_amd as M
    import synth_inputs as S
    import dataclasses

    w = S.WORKLOADS[cfg_id]
    if args.tokens:
        w = S.scaled_workload(cfg_id, T=args.tokens)
    policy_kw = {}
    if args.group_size:
        w = dataclasses.replace(w, name=w.name + "_g%d" % args.group_size, Gk=args.group_size, Gv=args.group_size)
        with_cpu_baseline = False
    if args.residual_length:
        R = args.residual_length
        # key groups must divide a record: 32 tokens for R = 32 and R = 96 (stored as three records of 32)
        w = dataclasses.replace(w, name=w.name + "_r%d" % R, R=R, Gk=32 if R % 64 else min(w.Gk, R, 128))
        with_cpu_baseline = False
    if args.thresholds:
        tau16, tau4 = (float(x) for x in args.thresholds.split(","))
        w = dataclasses.replace(w, name=w.name + "_thresholds", k4=16, k16=8)
        policy_kw = dict(policy=1, tau16=tau16, tau4=tau4)
        with_cpu_baseline = False
    n_q0 = w.R * (-(-w.T // w.R) - 1)
    step_bytes = algorithmic_bytes(w, n_q0, w.T - n_q0)     # with thresholds: the capacity, refined below
    copies = args.copies or max(1, math.ceil(2 * LLC_BYTES / step_bytes))
    n_ev = min(steps, 512)
    n_ps = min(steps, 512)
    n_settle = int(0.02 / (step_bytes / 6e12)) + 64      # steps the 20 ms settling phase can take at most (6 TB/s)
    total_steps = steps + warmup + n_ev + n_ps + copies + n_settle
    per_copy = -(-total_steps // copies)
    T_max = (w.T + per_copy + 272 + 2 * w.R) // w.R * w.R     # + the single-copy pass on copy 0

    dk, dv, dqp, dq, host = build_inputs(cfg_id, w, args.host_batch)
    kw = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, D=w.D, T_max=T_max, Gk=w.Gk, Gv=w.Gv, R=w.R, k4=w.k4, k16=w.k16, **policy_kw)
    caches = []
    for c in range(copies):
        gc = M.Cache(M.make_config(**kw))
        sel = M.mixkvq_select_channels(gc, dqp, dk)
        M.mixkvq_quantize_append(gc, dk, dv, sel=None if (args.thresholds or args.per_block_selection) else sel)
        caches.append(gc)
    torch.cuda.synchronize()
    tiers = None
    if args.thresholds:
        step_bytes, n16_mean, n4_mean = algorithmic_bytes_thresholds(w, caches[0], w.T - n_q0)
        tiers = {"tau16": tau16, "tau4": tau4, "mean_fp16_channels_per_block": round(n16_mean, 2),
                 "mean_4bit_channels_per_block": round(n4_mean, 2),
                 "key_bits_per_channel": round((16 * n16_mean + 4 * n4_mean + 2 * (w.D - n16_mean - n4_mean)) / w.D, 3)}
    k1 = dk[:, :, :64]   # new tokens are drawn from the prompt tensors (same distribution)
    v1 = dv[:, :, :64]
    out = torch.empty((w.B, w.Hq, w.D), dtype=torch.float16, device="cuda")
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda")

    if args.calibration_copy_mib:
        src = torch.full((args.calibration_copy_mib << 20,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(i):
        gc = caches[i % copies]
        t = i % 64
        M.mixkvq_decode_step(gc, k1[:, :, t:t + 1], v1[:, :, t:t + 1], dq[i % 8], out=out, lse=lse, accumulate_q=True)

    # every cache copy is stepped once before anything is counted (a full prompt window is flushed by its first
    # step, and a copy's first touch would otherwise land wherever the rotation first reaches it)
    i = 0
    for _ in range(copies):
        step(i)
        i += 1
    # ... and the GPU is kept busy for about 20 ms (uncounted steps of the same kind), so that a short run
    # (--steps 20 --warmup 5) is not timed on clocks that are still ramping up
    torch.cuda.synchronize()
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.02:
        for _ in range(8):
            step(i)
            i += 1
        torch.cuda.synchronize()
    for _ in range(warmup):
        step(i)
        i += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(i)
        i += 1
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    ms_per_step = el / steps * 1e3
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # second pass over the same kind of steps with HIP events around the split-K attention kernel
    ev = HipEvents(n_ev)
    for n in range(n_ev):
        gc = caches[i % copies]
        gc.set_timing_events(*ev.pairs[n])
        step(i)
        gc.set_timing_events(None, None)
        i += 1
    torch.cuda.synchronize()
    k_ms = ev.elapsed_ms()
    ev.destroy()
    k_avg_ms = sum(k_ms) / len(k_ms)

    # third pass: every step between its own pair of events (whole step, flush steps included), for the
    # mean / worst step and the share of the block flushes
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ps)]
    flushed = []
    for n in range(n_ps):
        nq_before = caches[i % copies].state()[0]
        evs[n][0].record()
        step(i)
        evs[n][1].record()
        flushed.append(caches[i % copies].state()[0] != nq_before)
        i += 1
    torch.cuda.synchronize()
    ps = [a.elapsed_time(b) * 1e3 for a, b in evs]

    # fourth pass: one cache copy only (when it fits the last-level cache this is the cache-warm figure)
    n_cw = min(steps, 256)
    for n in range(16):
        M.mixkvq_decode_step(caches[0], k1[:, :, :1], v1[:, :, :1], dq[n % 8], out=out, lse=lse, accumulate_q=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for n in range(n_cw):
        M.mixkvq_decode_step(caches[0], k1[:, :, :1], v1[:, :, :1], dq[n % 8], out=out, lse=lse, accumulate_q=True)
    torch.cuda.synchronize()
    single_copy_us = (time.perf_counter() - t0) / n_cw * 1e6
    ps_flush = [t for t, f in zip(ps, flushed) if f]
    ps_plain = [t for t, f in zip(ps, flushed) if not f]
    achieved = step_bytes / (k_avg_ms * 1e-3) / 1e9
    on_matrix_cores = M.mixkvq_decode_path(caches[0]) == M.PATH_MATRIX

    result = {
        "metric": "quantized-KV decode attention: effective HBM GB/s at %dK ctx" % (w.T // 1024), "value": round(value, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "T": w.T, "Gk": w.Gk, "Gv": w.Gv,
                   "R": w.R, "k4": w.k4, "k16": w.k16, "cache_copies": copies,
                   "algorithmic_bytes_per_step": step_bytes,
                   "step": "decode_step = quantize_append(1 token, flush every R) + decode_attention(accumulate_q)"},
        "roofline": {"bound": "hbm",
                     "kernel": "decode_fused_kernel" if on_matrix_cores
                     else "decode_split_kernel (vector-ALU fallback: no matrix-core variant for this configuration)",
                     "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "kernel_avg_us": round(k_avg_ms * 1e3, 2), "kernel_min_us": round(min(k_ms) * 1e3, 2),
                     "launches_timed": n_ev,
                     "traffic": measured_traffic(w.name, "decode_fused_kernel") if (on_matrix_cores and w == S.WORKLOADS[cfg_id]) else None,
                     "traffic_unit": "bytes per launch (profiles/hbm_traffic.txt)",
                     "algorithmic_bytes_per_launch": step_bytes},
    }
    result["single_copy"] = {"us_per_step": round(single_copy_us, 2), "steps": n_cw,
                             "value": round(step_bytes / single_copy_us / 1e3, 2), "unit": "GB/s",
                             "note": "one cache copy (%.0f MB) reused every step: %s" % (
                                 step_bytes / 1e6, "fits the 256 MB last-level cache (cache-warm)"
                                 if step_bytes < LLC_BYTES else "larger than the 256 MB last-level cache")}
    result["per_step_us"] = {
        "steps": n_ps, "mean": round(sum(ps) / len(ps), 2), "worst": round(max(ps), 2),
        "plain_steps_mean": round(sum(ps_plain) / max(1, len(ps_plain)), 2),
        "flush_steps": len(ps_flush), "flush_steps_mean": round(sum(ps_flush) / max(1, len(ps_flush)), 2),
        "amortised_with_flush_every_R": round((sum(ps_plain) / max(1, len(ps_plain)) * (w.R - 1)
                                               + (sum(ps_flush) / len(ps_flush) if ps_flush else 0.0)) / w.R, 2),
        "note": "each step between its own event pair (adds event overhead to every step)"}
    if tiers:
        result["config"]["threshold_policy"] = tiers
    result["config"]["selection"] = "per block" if (args.thresholds or args.per_block_selection) else "one per prompt"
    del caches, dk, dv, dqp, dq, k1, v1
    torch.cuda.empty_cache()
    copy_gbs = copy_kernel_gbs()
    result["copy_kernel"] = {"value": round(copy_gbs, 1), "unit": "GB/s read+write, 512 MiB device copy on this box",
                             "pct_of_copy_kernel": round(100 * value / copy_gbs, 2),
                             "kernel_pct_of_copy_kernel": round(100 * achieved / copy_gbs, 2)}
    if with_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg_id, w, host)
    return result


def summary_of(r):
    """The figures of one more workload that ride along in the default run's JSON line."""
    keep = {k: r[k] for k in ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "pct_of_hbm_peak") if k in r}
    keep["workload"] = r["config"]["workload"]
    rf = r["roofline"]
    keep["roofline"] = {k: rf[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "kernel_avg_us", "traffic")
                        if k in rf}
    for k in ("per_step_us", "without_prompt_queries"):
        if k in r:
            keep[k] = r[k]
    return keep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--config", type=int, default=0,
                    help="time one workload configuration only (1, 2, 3: decode step; 4: prefill); default: configuration 1 "
                         "as the headline, then 2, 3 and 4 under 'other_workloads'")
    ap.add_argument("--copies", type=int, default=0, help="independent cache copies rotated over (0 = enough for 2x LLC)")
    ap.add_argument("--host-batch", type=int, default=2)
    ap.add_argument("--tokens", type=int, default=0, help="override the context length of the configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--group-size", type=int, default=0,
                    help="override the key and value group size of the configuration (32: the paper's accuracy setting)")
    ap.add_argument("--residual-length", type=int, default=0,
                    help="override the residual length R of the configuration (32, 64, 96, 128 or 256); key groups larger "
                         "than a record are cut to it")
    ap.add_argument("--per-block-selection", action="store_true",
                    help="fill the cache with every block scored on its own tokens (as blocks flushed during decoding "
                         "are) instead of one selection for the whole prompt")
    ap.add_argument("--thresholds", type=str, default="",
                    help="'tau16,tau4': the three-tier threshold policy with room for 8 fp16 and 16 four-bit channels per "
                         "block instead of the configuration's top-k budget (every block scored on its own tokens)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run 4 plain device copies of this many MiB (reference reading for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the hot path has no collective); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_19206_amd as M
    import synth_inputs as S
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    M.load_library()

    def prefill(cfg_id):
        w = S.WORKLOADS[cfg_id]
        if args.tokens:
            w = S.scaled_workload(cfg_id, T=args.tokens)
        if args.group_size:
            import dataclasses
            w = dataclasses.replace(w, name=w.name + "_g%d" % args.group_size, Gk=args.group_size, Gv=args.group_size)
        return bench_prefill(args, w, cfg_id)

    if args.config == 4:
        print(json.dumps(prefill(4)))
        return
    if args.config:
        print(json.dumps(bench_decode(args, args.config, args.steps, args.warmup, not args.no_cpu_baseline)))
        return
    # default: the metric's workload (configuration 1) is the line's headline; the other configurations follow under
    # one extra key, each timed the same way (configuration 3 always over its 512 consecutive steps)
    result = bench_decode(args, 1, args.steps, args.warmup, not args.no_cpu_baseline)
    others = {}
    for cfg_id in (2, 3):
        r = bench_decode(args, cfg_id, 512 if cfg_id == 3 else args.steps, args.warmup, False)
        others[r["config"]["workload"]] = summary_of(r)
    r = prefill(4)
    others[r["config"]["workload"]] = summary_of(r)
    result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
