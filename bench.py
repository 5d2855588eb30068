#!/usr/bin/env python3
"""Benchmark of the middle-submodel forward on one MI355X.

Metric: middle-submodel hidden tokens/s on the 7B-shaped single-device workload
(30 decoder layers, d 4096, 32 heads x 128, FFN 11008, bf16; a 2048-row prompt fed
as 8 chunks of 256 against the growing paged KV cache).  One "step" = one
hat_mid_forward over one 256-row chunk (all kernels of the path, all 30 layers);
steps cycle through the 8 chunk positions, releasing the device after the 8th.
Inputs are resident in HBM before the timed region.

Besides the contract line it reports, in the same JSON object:
  roofline      the dominant kernel class of that workload (by GPU time), timed
                with HIP events on the launch stream inside the library
  kernels       every kernel class of the step: average duration and roofline
  legs          (tree-verify step included) chunk-attention MFMA fraction on a mixed-batch step and verify-
                attention HBM GB/s on a verify-heavy step (30 devices)
  chunk_size_sweep  13B-shaped model, 8192-row prompts, chunk sizes 64..1024, with the 8 devices batched
                per step and with one device per step: GPU time per step against chunk size and prefix
                (the cost profile g(.)), chunk-attention MFMA / min-roofline fraction per chunk size,
                and the chunk sizes the library's scheduler (Eq. 3) derives for a few uplinks
  measured_peaks  microbenchmarks built into the library (streaming read / copy, matrix-core loop, direct-to-LDS
                load path): the measured ceilings next to the published peaks
  cpu_baseline  the CPU oracle timed on this host on a bounded sample
  host_fed      the same workload with hidden states in pinned host memory (PCIe-inclusive; not the metric)
  paper_context end-to-end numbers the paper reports on other hardware
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import hat_inputs as hi  # noqa: E402

PEAK_MFMA_BF16 = 2.5e15   # FLOP/s, dense (same figure for fp16 and bf16 operands)
PEAK_HBM = 8.0e12         # B/s
SEED = 2000


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gen_weights(cfg, seed, n_layers):
    workers = min(16, os.cpu_count() or 8)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(lambda l: hi.layer_weights(cfg, l, seed), range(n_layers)))


def to_dev_bf16(x):
    import torch
    return torch.from_numpy(hi.bf16_bits(np.ascontiguousarray(x, np.float32)).view(np.int16)).view(torch.bfloat16).cuda()


def upload(weights):
    return [{k: to_dev_bf16(v) for k, v in w.items()} for w in weights]


# ---------------------------------------------------------------- algorithmic work per kernel class
def gemm_work(T, d, F):
    """(flops, bytes) per launch of the four GEMM classes."""
    w = {}
    for name, N, K, out_b in (("gemm_qkv", 3 * d, d, 2), ("gemm_o", d, d, 8), ("gemm_gateup", 2 * F, d, 1),
                              ("gemm_down", d, F, 8)):
        flops = 2.0 * T * N * K
        # weights once + activations in (bf16) + result out (bf16; fp32 read+write for the residual;
        # gate/up writes T*F bf16 = half of its N columns)
        byts = 2.0 * N * K + 2.0 * T * K + T * N * out_b
        w[name] = (flops, byts)
    return w


def attn_work(segs, d):
    """segs: list of (start, n).  Causal half not counted; K and V read once."""
    flops = sum(4.0 * d * (n * s + n * (n + 1) / 2.0) for s, n in segs)
    byts = sum(2.0 * (s + n) * d * 2 + 2.0 * n * d * 2 for s, n in segs)
    return flops, byts


def roof(flops, byts, sec):
    """Binding roofline of one launch."""
    t_m, t_h = flops / PEAK_MFMA_BF16, byts / PEAK_HBM
    if t_m >= t_h:
        a = flops / sec / 1e12
        return {"bound": "mfma", "achieved": a, "peak": PEAK_MFMA_BF16 / 1e12, "unit": "TFLOP/s",
                "frac": a / (PEAK_MFMA_BF16 / 1e12)}
    a = byts / sec / 1e9
    return {"bound": "hbm", "achieved": a, "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": a / (PEAK_HBM / 1e9)}


# ---------------------------------------------------------------- main workload
def prepare_cfg2(m, cfg, n_chunks=8, chunk=256):
    import torch
    from paper_2503_18989_amd.binding import CSegment
    xs, outs, arrs = [], [], []
    for i in range(n_chunks):
        x = to_dev_bf16(hi.hidden_rows(chunk, cfg["d_model"], SEED, i))
        o = torch.empty_like(x)
        arr = (CSegment * 1)()
        arr[0] = CSegment(0, hi.CHUNK, chunk, i * chunk, x.data_ptr(), o.data_ptr())
        xs.append(x); outs.append(o); arrs.append(arr)
    return xs, outs, arrs


def run_cfg2(m, arrs, steps, warmup):
    import torch
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    n = len(arrs)

    def one(i):
        j = i % n
        if j == 0:
            m.release(0)
        m.forward_raw(arrs[j], 1, sp)
    for i in range(warmup):
        one(i)
    # continue the cycle where the warmup left it so that chunk positions stay consistent
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(warmup, warmup + steps):
        one(i)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) / 1e3


def run_cfg2_host(m, cfg, steps, warmup, n_chunks=8, chunk=256):
    """The same cfg-2 step fed from pinned host memory through hat_mid_forward_host (upload of the next
    chunk overlaps the current step; results copied back to host): the PCIe-inclusive rate."""
    import torch
    from paper_2503_18989_amd.binding import CSegment
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    xs, outs, arrs = [], [], []
    for i in range(n_chunks):
        x = torch.from_numpy(hi.bf16_bits(hi.hidden_rows(chunk, cfg["d_model"], SEED, i)).view(np.int16)).view(torch.bfloat16).pin_memory()
        o = torch.empty_like(x).pin_memory()
        arr = (CSegment * 1)()
        arr[0] = CSegment(0, hi.CHUNK, chunk, i * chunk, x.data_ptr(), o.data_ptr())
        xs.append(x); outs.append(o); arrs.append(arr)

    def one(i):
        j = i % n_chunks
        if j == 0:
            m.release(0)
        rc = m.lib.hat_mid_forward_host(m._handle, arrs[j], 1, sp)
        if rc != 0:
            m._check(rc)
    for i in range(warmup):
        one(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup, warmup + steps):
        one(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return {"value": chunk * steps / wall, "unit": "hidden tokens/s", "ms_per_step": wall / steps * 1e3,
            "bytes_per_step_each_way": chunk * cfg["d_model"] * 2,
            "note": "hidden states start and end in pinned host memory (hat_mid_forward_host); never the headline value"}


def uplink_emulation(m, cfg, step_ms, n_chunks=8, chunk=256):
    """Time to the last deep hidden state of a 2048-row prompt (the cloud's share of the time to first token)
    when the device's hidden states arrive over an uplink of beta_up bytes/s (Sec. 3.3): with the paper's prompt
    chunking -- a chunk is uploaded (PCIe) and processed as soon as it has arrived, while the next one is still
    on the air -- against the plain U-shaped order, where the whole prompt has to arrive first.  The uplink is
    emulated on the host: chunk j is handed to hat_mid_forward_host at (j + 1) * chunk * A / beta_up after the
    start, A = 2 d bytes per row; everything from there on (H2D on the library's copy stream, the step, D2H) is
    real.  Rates: the paper's WiFi (10 MB/s), 100 MB/s, the rate at which a chunk takes as long to arrive as to
    process (where Eq. 3 puts the chunk size), and 1 GB/s."""
    import torch
    from paper_2503_18989_amd.binding import CSegment
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    A = 2 * cfg["d_model"]
    xs, outs, arrs = [], [], []
    for i in range(n_chunks):
        x = torch.from_numpy(hi.bf16_bits(hi.hidden_rows(chunk, cfg["d_model"], SEED, i)).view(np.int16)).view(torch.bfloat16).pin_memory()
        o = torch.empty_like(x).pin_memory()
        arr = (CSegment * 1)()
        arr[0] = CSegment(0, hi.CHUNK, chunk, i * chunk, x.data_ptr(), o.data_ptr())
        xs.append(x); outs.append(o); arrs.append(arr)

    def run(beta, overlap):
        m.release(0)
        torch.cuda.synchronize()
        per_chunk = chunk * A / beta
        t0 = time.perf_counter()

        def wait_until(t):
            while True:
                dt = t0 + t - time.perf_counter()
                if dt <= 0:
                    return
                time.sleep(dt if dt > 2e-3 else 0)      # sleep, then spin over the last 2 ms
        if overlap:
            for j in range(n_chunks):
                wait_until((j + 1) * per_chunk)
                rc = m.lib.hat_mid_forward_host(m._handle, arrs[j], 1, sp)
                if rc != 0:
                    m._check(rc)
        else:
            wait_until(n_chunks * per_chunk)
            for j in range(n_chunks):
                rc = m.lib.hat_mid_forward_host(m._handle, arrs[j], 1, sp)
                if rc != 0:
                    m._check(rc)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    balanced = chunk * A / (step_ms * 1e-3)
    rows = []
    for name, beta in (("10 MB/s (the paper's WiFi)", 10e6), ("100 MB/s", 100e6), ("balanced: chunk arrives in one step time", balanced),
                       ("1 GB/s", 1e9)):
        run(beta if beta > 50e6 else 1e9, True)      # warm
        a = min(run(beta, True) for _ in range(2))
        b = min(run(beta, False) for _ in range(2))
        rows.append({"uplink": name, "beta_up_MB_per_s": beta / 1e6, "upload_ms_whole_prompt": n_chunks * chunk * A / beta * 1e3,
                     "ms_with_overlap": a, "ms_without_overlap": b, "saved_ms": b - a})
    return {"workload": "2048-row prompt as %d chunks of %d, 7B-shaped, %d layers; A = %d bytes per row" % (n_chunks, chunk, cfg["n_layers"], A),
            "what": "time from the start of the upload to the last chunk's deep hidden states back in host memory", "by_uplink": rows}


def profile_classes(m, run_steps):
    """Per kernel class: (avg seconds per launch, launches) with event bracketing on."""
    import torch
    m.set_profiling(True)
    m.kernel_times()
    run_steps()
    torch.cuda.synchronize()
    t = m.kernel_times()
    m.set_profiling(False)
    return {k: (ms / 1e3 / max(cnt, 1), cnt) for k, (ms, cnt) in t.items() if cnt}


def timed_steps(step, n):
    """Mean GPU milliseconds of n consecutive calls of step(), between two events on the current stream."""
    import torch
    st = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(st)
    for _ in range(n):
        step()
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


# ---------------------------------------------------------------- legs for the attention kernels
def attention_legs(cfg7, dev_layers):
    """The verify-heavy step (config-4 shape: 30 devices, 5 draft rows each, cache lengths uniform in
    [1024, 8192]), the same devices submitting trees of 8, and the mixed step (config-3 shape: 10 chunks
    + 20 verify segments over prefixes U[256, 4096]), each at the model's full depth: step time,
    per-class kernel times, verify-attention HBM GB/s, chunk-attention and GEMM MFMA fractions."""
    import torch
    from paper_2503_18989_amd import HatMid, Segment
    cfg = dict(cfg7)
    n_layers = cfg["n_layers"]
    d, H, hd = cfg["d_model"], cfg["n_heads"], cfg["head_dim"]
    out = {}
    kbig = (torch.randn((8192, H, hd), device="cuda", dtype=torch.float32) * 1.28).to(torch.bfloat16)
    vbig = (torch.randn((8192, H, hd), device="cuda", dtype=torch.float32) * 1.28).to(torch.bfloat16)

    def install(m, lengths):
        for dev, ln in enumerate(lengths):
            for l in range(n_layers):
                m.kv_import(dev, l, 0, kbig[:ln], vbig[:ln])

    # --- verify-heavy step
    lengths = hi.verify_lengths(SEED + 4)
    pages = sum((ln + 5 * 8 + 15) // 16 for ln in lengths) + 64
    m = HatMid(cfg, dev_layers[:n_layers], n_pages=pages, max_devices=32, max_step_tokens=256, max_pos=8192 + 64)
    install(m, lengths)
    xs = [to_dev_bf16(hi.hidden_rows(5, d, SEED + 4, dev)) for dev in range(30)]

    def vstep():
        segs = [Segment(dev, hi.VERIFY, lengths[dev], xs[dev]) for dev in range(30)]   # re-verify in place
        m.forward(segs)
    for _ in range(3):
        vstep()
    prof = profile_classes(m, lambda: [vstep() for _ in range(8)])
    fl, by = attn_work([(ln, 5) for ln in lengths], d)
    sec = prof["attn_verify"][0]
    out["verify_attn"] = dict(roof(fl, by, sec), us_per_launch=sec * 1e6, algorithmic_bytes=by,
                              traffic=recorded_leg_traffic("attn_verify_kernel<128, false>"),
                              traffic_source="profiles/traffic_attention_legs.txt (recorded rocprofv3 --pmc runs, not measured in this run)",
                              workload="30 devices x 5 rows, cache lengths U[1024,8192], 7B-shaped layer")
    out["verify_step_classes_us"] = {k: round(v[0] * 1e6, 2) for k, v in prof.items()}
    # the same launch with the kernel's arithmetic taken out (hat_mid_debug_set_verify_probe): what this
    # access order -- head-major pool, page-list walk, one register stage per wave -- can reach here
    m.set_verify_probe(True)
    sec_p = profile_classes(m, lambda: [vstep() for _ in range(8)])["attn_verify"][0]
    m.set_verify_probe(False)
    out["verify_attn"]["loads_only"] = {"us_per_launch": sec_p * 1e6, "GBps": by / sec_p / 1e9, "frac_of_peak": by / sec_p / PEAK_HBM,
                                        "kernel_vs_loads_only": sec_p / sec}
    vstep()     # a real step again: the probe leaves the verify rows' attention output unwritten
    ms = timed_steps(vstep, 8)
    out["verify_step"] = {"tokens": 150, "layers": n_layers, "gpu_ms": ms, "hidden_tokens_per_s": 150 / (ms * 1e-3),
                          "roofline": out["verify_attn"]}

    # --- the same devices submitting a tree of 8 candidates each (the tree-verifying comparison
    # system's step, Sec. 4.1) instead of a chain of 5: what the larger step costs on this engine
    xt = [to_dev_bf16(hi.hidden_rows(8, d, SEED + 5, dev)) for dev in range(30)]
    masks = hi.tree_masks(hi.MEDUSA_LIKE_TREE)

    def tstep():
        m.forward([Segment(dev, hi.VERIFY, lengths[dev], xt[dev], tree_mask=masks) for dev in range(30)])
    for _ in range(3):
        tstep()
    prof_t = profile_classes(m, lambda: [tstep() for _ in range(8)])
    fl, by = attn_work([(ln, 8) for ln in lengths], d)
    sec = prof_t["attn_verify"][0]
    ms_t = timed_steps(tstep, 8)
    out["tree_verify_attn"] = dict(roof(fl, by, sec), us_per_launch=sec * 1e6, algorithmic_bytes=by,
                                   workload="30 devices x tree of 8, same caches")
    out["tree_verify_step"] = {"tokens": 240, "layers": n_layers, "gpu_ms": ms_t, "hidden_tokens_per_s": 240 / (ms_t * 1e-3),
                               "ms_ratio_to_chain_of_5": ms_t / ms, "roofline": out["tree_verify_attn"]}
    m.close()
    del m
    torch.cuda.empty_cache()

    # --- mixed step: 10 chunks + 20 verifies over prefixes U[256,4096]
    pref = hi.mixed_prefixes(SEED + 3)
    segs_desc = hi.mixed_step(SEED + 3, 0, pref)
    pages = sum((p + n + 15) // 16 for (_, _, p, n) in segs_desc) + 64
    T = sum(n for (_, _, _, n) in segs_desc)
    m = HatMid(cfg, dev_layers[:n_layers], n_pages=pages, max_devices=32, max_step_tokens=max(T, 256), max_pos=8192)
    install(m, pref)
    xin = [to_dev_bf16(hi.hidden_rows(n, d, SEED + 3, dev)) for (dev, _, _, n) in segs_desc]

    def mstep():
        m.forward([Segment(dev, kind, p, x) for (dev, kind, p, n), x in zip(segs_desc, xin)])
    for _ in range(3):
        mstep()
    prof = profile_classes(m, lambda: [mstep() for _ in range(8)])
    chunks = [(p, n) for (_, kind, p, n) in segs_desc if kind == hi.CHUNK]
    fl, by = attn_work(chunks, d)
    sec = prof["attn_chunk"][0]
    r = roof(fl, by, sec)
    out["chunk_attn"] = dict(r, us_per_launch=sec * 1e6, mfma_frac=fl / sec / PEAK_MFMA_BF16,
                             workload="10 chunks %s over prefixes U[256,4096] (+20 verify segments in the same step)"
                             % sorted(n for _, n in chunks))
    gw = gemm_work(T, d, cfg["d_ffn"])
    out["mixed_step_classes_us"] = {k: round(v[0] * 1e6, 2) for k, v in prof.items()}
    out["mixed_step_gemm_mfma_frac"] = {k: gw[k][0] / prof[k][0] / PEAK_MFMA_BF16 for k in gw}
    ms = timed_steps(mstep, 8)
    m.close()
    del m
    torch.cuda.empty_cache()
    # the same step over an fp16 cache (cache rows are matrix-core operands as they are: no widening)
    m = HatMid(cfg, dev_layers[:n_layers], n_pages=pages, max_devices=32, max_step_tokens=max(T, 256), max_pos=8192, kv_dtype="f16")
    install(m, pref)
    for _ in range(3):
        mstep()
    prof16 = profile_classes(m, lambda: [mstep() for _ in range(8)])
    sec16 = prof16["attn_chunk"][0]
    out["chunk_attn_fp16_cache"] = dict(roof(fl, by, sec16), us_per_launch=sec16 * 1e6, mfma_frac=fl / sec16 / PEAK_MFMA_BF16)
    out["mixed_step_fp16_cache"] = {"tokens": T, "layers": n_layers, "gpu_ms": timed_steps(mstep, 8)}
    dom = max(gw, key=lambda k: prof[k][0])
    out["mixed_step"] = {"tokens": T, "layers": n_layers, "gpu_ms": ms, "hidden_tokens_per_s": T / (ms * 1e-3),
                         "roofline": dict(roof(gw[dom][0], gw[dom][1], prof[dom][0]), kernel=dom,
                                          us_per_launch=prof[dom][0] * 1e6)}
    m.close()
    return out


# ---------------------------------------------------------------- chunk-size sweep (cost profile)
def chunk_sweep(n_layers, chunks=(64, 128, 256, 512, 1024), n_devices=8, prompt=8192):
    """13B-shaped middle submodel, 8 devices with 8192-row prompts fed in chunks of c, all
    devices batched per step (T = 8c rows): GPU time per step against (c, prefix) -- the
    per-chunk-size cost profile g(.) that the paper's chunk-size rule (Sec. 3.3, Eq. 3) consumes."""
    import torch
    from paper_2503_18989_amd import HatMid
    from paper_2503_18989_amd.binding import CSegment
    cfg = hi.with_layers(hi.MID13B, n_layers)
    d = cfg["d_model"]
    t0 = time.time()
    weights = gen_weights(cfg, SEED + 5, n_layers)
    dev_layers = upload(weights)
    del weights
    log("13B-shaped weights (%d layers) ready in %.1f s" % (n_layers, time.time() - t0))
    # fp16 cache: a bf16 cache puts this 38-layer model's first chunks above the 2e-2 parity bar (tests/test_gpu_depth.py)
    m = HatMid(cfg, dev_layers, n_pages=n_devices * prompt // 16 + 16, max_devices=n_devices,
               max_step_tokens=n_devices * max(chunks), max_pos=prompt, kv_dtype="f16")
    del dev_layers
    torch.cuda.empty_cache()
    sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    x = to_dev_bf16(hi.hidden_rows(max(chunks), d, SEED + 5, 0))      # the same rows for every device and step
    out = torch.empty((n_devices, max(chunks), d), dtype=torch.bfloat16, device="cuda")
    def feed(c, ndev):
        """All chunks of size c of `ndev` prompts, one step per chunk position; returns the sweep point."""
        for dev in range(n_devices):
            m.release(dev)
        steps = prompt // c
        arr = (CSegment * ndev)()
        ms, attn = [], None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        extra = 0.0
        for j in range(steps):
            for dev in range(ndev):
                arr[dev] = CSegment(dev, hi.CHUNK, c, j * c, x.data_ptr(), out[dev].data_ptr())
            if j == steps // 2:            # the middle step again under per-kernel events: attention figures
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                m.set_profiling(True); m.kernel_times()
                m.forward_raw(arr, ndev, sp)
                torch.cuda.synchronize()
                kt = m.kernel_times(); m.set_profiling(False)
                for dev in range(ndev):    # undo: the timed step below appends the same rows again
                    arr[dev] = CSegment(dev, hi.CHUNK, c, j * c, x.data_ptr(), out[dev].data_ptr())
                sec_a = kt["attn_chunk"][0] / max(kt["attn_chunk"][1], 1) / 1e3
                fl, by = attn_work([(j * c, c)] * ndev, d)
                attn = {"us_per_launch": sec_a * 1e6, "mfma_frac": fl / sec_a / PEAK_MFMA_BF16,
                        "min_roofline_frac": max(fl / PEAK_MFMA_BF16, by / PEAK_HBM) / sec_a, "prefix": j * c}
                extra += time.perf_counter() - t1
            m.forward_raw(arr, ndev, sp)
            if j in (0, steps // 2, steps - 1):
                ms.append(m.last_step_stats()[1])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0 - extra
        return {"chunk": c, "rows_per_step": ndev * c, "steps": steps, "ms_first_step": ms[0],
                "ms_middle_step": ms[1], "ms_last_step": ms[2], "ms_mean_step": dt / steps * 1e3,
                "hidden_tokens_per_s": ndev * prompt / dt, "chunk_attention_middle_step": attn}

    res, res1 = [], []
    for c in chunks:
        res.append(feed(c, n_devices))
        log("sweep c=%d: %.2f ms/step mean (first %.2f, last %.2f), %.0f tokens/s" % (c, res[-1]["ms_mean_step"], res[-1]["ms_first_step"], res[-1]["ms_last_step"], res[-1]["hidden_tokens_per_s"]))
    for c in chunks:
        res1.append(feed(c, 1))
        log("sweep c=%d, one device per step: %.2f ms/step mean, %.0f tokens/s" % (c, res1[-1]["ms_mean_step"], res1[-1]["hidden_tokens_per_s"]))
    m.close()
    return {"workload": "13B-shaped (%d layers, d 5120, 40x128 heads, FFN 13824), %d devices x %d-row prompts, "
                        "all devices batched per step; fp16 KV cache" % (n_layers, n_devices, prompt), "kv_cache": "fp16", "points": res,
            "points_one_device_per_step": res1,
            "chunk_size_rule": chunk_size_rule(res, d)}


def chunk_size_rule(points, d):
    """The consumer of the sweep: the library's state monitor (hat_sched_*, Sec. 3.2) is fed the
    measured (rows per step, ms per step) pairs and the chunk-size rule (Sec. 3.3, Eq. 3) is solved for
    a few uplinks and pipeline lengths.  A = 2 d bytes per token (fp16 hidden state); the standing
    load mu is the smallest measured batch (observed last, alpha = 0: the table is the sweep itself)."""
    from paper_2503_18989_amd import HatSched
    sched = HatSched([p["rows_per_step"] for p in points], alpha=0.0)
    for p in sorted(points, key=lambda p: -p["rows_per_step"]):
        sched.observe(p["rows_per_step"], p["ms_mean_step"])
    A = 2.0 * d
    rows = []
    for mb_s in (1, 10, 100, 1000):
        beta = mb_s * 1e6 / 1e3                       # bytes per ms
        rows.append({"uplink_MB_per_s": mb_s,
                     "chunk_size_P1": sched.chunk_size(A, beta, 1, 16, 8192),
                     "chunk_size_P4": sched.chunk_size(A, beta, 4, 16, 8192),
                     "parallel_draft_steps": sched.parallel_draft_steps(5, A, beta, 2 * beta, 20.0)})
    out = {"mu_rows": sched.mu, "g_ms_at_mu": sched.predict(sched.mu), "bytes_per_token": A,
           "note": "chunk sizes clamped to [16, 8192]; drafting delay 20 ms per step, downlink = 2 x uplink, draft length 5",
           "by_uplink": rows}
    sched.close()
    return out


# ---------------------------------------------------------------- GEMM classes beside the vendor BLAS (context)
def gemm_reference(rows=(150, 256, 1024, 3556, 4096), model="7b"):
    """The four GEMM classes of one layer as this library runs them (event-bracketed, inside a 2-layer
    model; QKV, gate/up with SwiGLU applied, O and down with the fp32 residual update) beside a plain
    `x @ w.T` of the same shapes through the vendor BLAS that PyTorch-ROCm links (fp16 in, fp16 out, no
    epilogue).  A reference point for reading the MFMA fractions: nothing in the product path calls it."""
    import torch
    from paper_2503_18989_amd import HatMid, Segment
    base = hi.MID13B if model == "13b" else hi.MID7B
    cfg = hi.with_layers(base, 2)
    d, F = cfg["d_model"], cfg["d_ffn"]
    dev = upload(gen_weights(cfg, SEED, 2))
    out = {"model": model, "rows": {}}
    for T in rows:
        m = HatMid(cfg, dev, n_pages=2 * T // 16 + 8, max_devices=2, max_step_tokens=max(T, 256), max_pos=2 * T)
        x = to_dev_bf16(hi.hidden_rows(T, d, SEED, 0))

        def run(n):
            for _ in range(n):
                m.release(0)
                m.forward([Segment(0, hi.CHUNK, 0, x)])
        run(3)
        prof = profile_classes(m, lambda: run(10))
        row = {}
        for name, N, K in (("gemm_qkv", 3 * d, d), ("gemm_o", d, d), ("gemm_gateup", 2 * F, d), ("gemm_down", d, F)):
            a16 = torch.randn(T, K, device="cuda", dtype=torch.float16)
            w16 = torch.randn(N, K, device="cuda", dtype=torch.float16)
            for _ in range(3):
                a16 @ w16.t()
            ms = timed_steps(lambda: a16 @ w16.t(), 20)
            fl = 2.0 * T * N * K
            ours = prof[name][0]
            row[name] = {"us": round(ours * 1e6, 1), "mfma_frac": round(fl / ours / PEAK_MFMA_BF16, 3),
                         "vendor_us": round(ms * 1e3, 1), "vendor_mfma_frac": round(fl / (ms * 1e-3) / PEAK_MFMA_BF16, 3)}
            del a16, w16
        out["rows"][str(T)] = row
        log("gemm reference, %s, T=%d: %s" % (model, T, row))
        m.close()
    return out


# ---------------------------------------------------------------- measured peaks (microbenchmarks in the library)
def measured_peaks():
    """hat_mid_debug_peak: what the chip delivers through the instruction mixes of this library's kernels."""
    from paper_2503_18989_amd.binding import measure_peak
    out = {}
    for kind, unit, peak in (("stream_read", "GB/s", PEAK_HBM), ("stream_read_nt", "GB/s", PEAK_HBM), ("copy", "GB/s", PEAK_HBM),
                             ("mfma_f16", "TFLOP/s", PEAK_MFMA_BF16), ("lds_load", "GB/s", None)):
        r = measure_peak(kind, nbytes=(1 << 30) if kind != "copy" else (2 << 30), iters=20)
        e = {"value": r / (1e12 if unit == "TFLOP/s" else 1e9), "unit": unit}
        if peak:
            e["frac_of_published_peak"] = r / peak
        if kind == "mfma_f16":
            e["implied_clock_GHz"] = r / (256 * 4 * 1024.0) / 1e9    # 4 SIMDs x 1024 FLOP per clock per CU
        if kind == "lds_load":
            e["bytes_per_clock_per_cu_at_2.4GHz"] = r / 256 / 2.4e9
        out[kind] = e
    out["note"] = ("stream_read*: 1 GiB read once per launch, every wave a contiguous span in 16 KB steps (16 loads of 16 bytes per "
                   "lane in flight, 32 waves per CU); copy: 1 GiB read + 1 GiB written; mfma_f16: 32x32x16 fp16 matrix instructions only, two waves per SIMD; lds_load: direct-to-LDS "
                   "loads of a cache-resident 1 MiB region, one 4-wave workgroup per CU, 16 loads in flight per wave")
    return out


# ---------------------------------------------------------------- measured HBM traffic (from profiles/)
def recorded_traffic(kernel):
    """HBM bytes per launch of a kernel class as measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this benchmark (separate passes; the summary and the commands are in profiles/traffic_cfg2.txt)."""
    path = os.path.join(ROOT, "profiles", "traffic_cfg2.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel + "_hbm_bytes_per_launch":
            return float(parts[1])
    return None


# ---------------------------------------------------------------- CPU baseline (oracle)
def recorded_leg_traffic(kernel):
    """HBM bytes per launch of an attention kernel in the legs (the first, i.e. largest, row of that kernel in
    profiles/traffic_attention_legs.txt: fetched + written bytes, counters scaled by the copy calibration)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "traffic_attention_legs.txt")
    try:
        for line in open(path):
            if line.startswith(kernel):
                f = dict(kv.split("=") for kv in line[len(kernel):].split())   # (the kernel name itself contains a space)
                return float(f["fetch_bytes"]) + float(f["write_bytes"])
    except OSError:
        pass
    return None


def cpu_baseline(cfg7, weights, n_layers=6, n_chunks=8, chunk=256):
    from oracle import OracleMiddle
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    cfg = hi.with_layers(cfg7, n_layers)
    m = OracleMiddle(cfg, weights[:n_layers])
    t0 = time.perf_counter()
    for i in range(n_chunks):
        m.forward([(0, i * chunk, hi.hidden_rows(chunk, cfg["d_model"], SEED, i))])
    dt = time.perf_counter() - t0
    scale = cfg7["n_layers"] / n_layers
    return {"value": n_chunks * chunk / (dt * scale), "unit": "hidden tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of 8 chunks (%d rows) through %d of %d layers in %.1f s, numpy float64; "
                      "extrapolated linearly in layers" % (n_chunks, n_chunks * chunk, n_layers, cfg7["n_layers"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-legs", action="store_true", help="skip the attention legs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--layers", type=int, default=0, help="override depth (for profiling runs; the line is then not the metric)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the 13B-shaped chunk-size sweep")
    ap.add_argument("--sweep-layers", type=int, default=38, help="depth of the chunk-size sweep model")
    ap.add_argument("--host-fed-only", action="store_true", help="only the headline workload, device-fed and host-fed, and the uplink emulation")
    ap.add_argument("--peaks", action="store_true", help="only the machine microbenchmarks (hat_mid_debug_peak): prints them as JSON and exits")
    ap.add_argument("--gemm-reference", action="store_true",
                    help="only the GEMM classes beside the vendor BLAS on the same shapes (7B and 13B shapes): prints JSON and exits")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling FETCH_SIZE/WRITE_SIZE counters)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the middle-submodel forward on ONE GPU; --gpus %d is not supported "
              "(no sharding, no collectives)" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_18989_amd import HatMid
    if a.peaks:
        print(json.dumps({"measured_peaks": measured_peaks()}))
        return
    if a.gemm_reference:
        print(json.dumps({"gemm_reference": [gemm_reference(model="7b"), gemm_reference(rows=(1024, 4096, 8192), model="13b")]}))
        return
    cfg = dict(hi.MID7B)
    if a.layers:
        cfg = hi.with_layers(cfg, a.layers)
    L, d, F = cfg["n_layers"], cfg["d_model"], cfg["d_ffn"]
    t0 = time.time()
    weights = gen_weights(cfg, SEED, L)
    log("weights generated in %.1f s" % (time.time() - t0))
    dev_layers = upload(weights)
    m = HatMid(cfg, dev_layers, n_pages=2048 // 16 + 8, max_devices=4, max_step_tokens=256, max_pos=2048)
    xs, outs, arrs = prepare_cfg2(m, cfg)
    wall, gpu_s = run_cfg2(m, arrs, a.steps, a.warmup)
    sec = max(wall, gpu_s)
    T = 256
    value = T * a.steps / sec
    log("cfg2: %.3f ms/step, %.0f hidden tokens/s" % (sec / a.steps * 1e3, value))
    host_fed = run_cfg2_host(m, cfg, a.steps, a.warmup)
    log("cfg2 from host memory: %.3f ms/step, %.0f hidden tokens/s" % (host_fed["ms_per_step"], host_fed["value"]))
    host_fed["uplink_emulation"] = uplink_emulation(m, cfg, sec / a.steps * 1e3)
    for r in host_fed["uplink_emulation"]["by_uplink"]:
        log("uplink %s: %.1f ms with overlap, %.1f ms without" % (r["uplink"], r["ms_with_overlap"], r["ms_without_overlap"]))
    if a.host_fed_only:
        print(json.dumps({"value": value, "ms_per_step": sec / a.steps * 1e3, "host_fed": host_fed}))
        return

    # per-class timing (separate pass, events around every launch)
    def cyc():
        sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        for i in range(16):
            if i % 8 == 0:
                m.release(0)
            m.forward_raw(arrs[i % 8], 1, sp)
    prof = profile_classes(m, cyc)
    gw = gemm_work(T, d, F)
    kernels = {}
    for k, (s, cnt) in prof.items():
        entry = {"us_per_launch": round(s * 1e6, 2), "launches_per_step": cnt / 16.0}
        if k in gw:
            entry.update(roof(gw[k][0], gw[k][1], s))
            entry["mfma_frac"] = gw[k][0] / s / PEAK_MFMA_BF16
        elif k == "attn_chunk":
            # average over the 8 chunk positions
            fl = np.mean([attn_work([(i * 256, 256)], d)[0] for i in range(8)])
            by = np.mean([attn_work([(i * 256, 256)], d)[1] for i in range(8)])
            entry.update(roof(fl, by, s))
            entry["mfma_frac"] = fl / s / PEAK_MFMA_BF16
        kernels[k] = entry
    per_step = {k: v["us_per_launch"] * v["launches_per_step"] for k, v in kernels.items()}
    dom = max((k for k in per_step if "bound" in kernels[k]), key=lambda k: per_step[k])
    roofline = {k: kernels[dom][k] for k in ("bound", "achieved", "peak", "unit", "frac")}
    roofline.update(kernel=dom, traffic=recorded_traffic(dom),
                    traffic_source="profiles/traffic_cfg2.txt (recorded rocprofv3 --pmc runs of this workload, not measured in this run)",
                    us_per_launch=kernels[dom]["us_per_launch"],
                    algorithmic_bytes=gw[dom][1] if dom in gw else None,
                    algorithmic_flops=gw[dom][0] if dom in gw else None)
    # whole-step roofline: sum over classes of max(flop/peak, bytes/peak), matrix kernels only
    ideal = L * sum(max(f / PEAK_MFMA_BF16, b / PEAK_HBM) for f, b in gw.values())
    m.close()
    del m
    torch.cuda.empty_cache()
    # the same workload over an fp16 cache (reported beside the headline, which keeps the workload's bf16 cache)
    m = HatMid(cfg, dev_layers, n_pages=2048 // 16 + 8, max_devices=4, max_step_tokens=256, max_pos=2048, kv_dtype="f16")
    wall16, gpu16 = run_cfg2(m, arrs, a.steps, a.warmup)
    fp16_cache = {"value": T * a.steps / max(wall16, gpu16), "unit": "hidden tokens/s", "ms_per_step": max(wall16, gpu16) / a.steps * 1e3}
    log("cfg2 with an fp16 cache: %.3f ms/step" % fp16_cache["ms_per_step"])
    m.close()
    del m
    torch.cuda.empty_cache()

    peaks = measured_peaks()
    legs = None
    if not a.no_legs:
        legs = attention_legs(cfg, dev_layers)
    if a.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    del dev_layers
    torch.cuda.empty_cache()
    sweep = None
    if not a.no_sweep:
        sweep = chunk_sweep(a.sweep_layers)
    cpu = None
    if not a.no_cpu:
        cpu = cpu_baseline(cfg, weights)

    line = {
        "metric": "middle-submodel hidden tokens/s; chunk-attn MFMA % peak; verify-attn HBM GB/s",
        "value": value, "unit": "hidden tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec / a.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "7B-shaped middle submodel (%d layers, d 4096, 32x128 heads, FFN 11008), one device, "
                               "2048-row prompt as 8 chunks of 256, bf16 KV in 16-token pages" % L,
                   "rows_per_step": T, "io_dtype": "bf16", "weights": "bf16 values", "kv_cache": "bf16",
                   "mfma_operands": "fp16 (fp32 accumulate)"},
        "gpu_event_ms_per_step": gpu_s / a.steps * 1e3, "host_wall_ms_per_step": wall / a.steps * 1e3,
        "step_roofline_ms": ideal * 1e3, "step_roofline_frac": ideal / (sec / a.steps),
        "roofline": roofline, "kernels": kernels, "measured_peaks": peaks, "legs": legs, "chunk_size_sweep": sweep, "cpu_baseline": cpu,
        "host_fed": host_fed, "same_workload_fp16_cache": fp16_cache,
        "paper_context": "paper reports end-to-end TTFT -41..54% / TBT -41..77% on 30 Jetson devices + 8xA6000 "
                         "(other hardware, whole system): context only, not a target",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
