#!/usr/bin/env python3
"""Benchmark of the KV-cache hot path on one MI355X.

A step is one decode step of the whole model-shaped cache: for every layer, append the
step's new token (fp16 window copy, plus the quantize-and-pack flush of 32 tokens every
32 steps) and run the fused dequantize-and-attend kernel over the whole context.  The
cache (seeded synthetic fp16 K/V shaped like the paper's models) is quantized and resident
in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  `value` is decode tokens/s (batch tokens per step / step time) of the
3.25-bit mixed schedule; the same shape with uniform K8V8 is timed in the same run and
reported under `kv8`.  `roofline` describes the dominant kernel, `cpu_baseline` the CPU oracle.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


SCALE_BYTES = 4                 # 2 with --meta fp16 (scales stored and used as fp16)
KEYS_PER_TOKEN = False          # True with --keys per-token (keys grouped like values)
FUSED_STEP = True               # False with --separate-calls (kvq_quantize_append + kvq_decode_attention per layer)


def layer_bytes(w, kb, vb, n_packed, n_res):
    """Algorithmic HBM bytes of one decode_attention launch on one layer: codes, fp32 scales and fp16 zero-points of the
    packed tokens of both tensors, the fp16 window rows, the queries and the outputs."""
    from paper_2502_04420_amd import bytes_per_token

    per_tok = bytes_per_token(kb, vb, w.head_dim, w.group, scale_bytes=SCALE_BYTES)
    bh = w.batch * w.n_kv_heads
    return bh * (n_packed * per_tok + n_res * 4 * w.head_dim) + 2 * w.batch * w.n_q_heads * w.head_dim * 2


class HipEvents:
    """Raw HIP events through the runtime library (the one torch has already loaded), for the library's timing hook."""

    def __init__(self):
        import ctypes

        self.ct = ctypes
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self):
        ev = self.ct.c_void_p()
        rc = self.lib.hipEventCreate(self.ct.byref(ev))
        if rc:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev

    def elapsed_ms(self, a, b):
        ms = self.ct.c_float()
        rc = self.lib.hipEventElapsedTime(self.ct.byref(ms), a, b)
        if rc:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return ms.value

    def destroy(self, ev):
        self.lib.hipEventDestroy(ev)


def build_cache(torch, pkg, W, w, extra_tokens, variant=0, splits=0):
    """Configure the library for workload w and prefill it layer by layer (inputs generated on the GPU)."""
    dev = "cuda:0"
    cache = pkg.KVQ(w.n_layers, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context + extra_tokens, w.kbits,
                    w.vbits, group=w.group, residual=w.residual, device=dev,
                    meta_dtype=pkg.META_FP16 if SCALE_BYTES == 2 else pkg.META_FP32,
                    key_mode=pkg.KEYS_PER_TOKEN if KEYS_PER_TOKEN else pkg.KEYS_PER_CHANNEL)
    cache.set_decode_options(variant, splits)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    q_ms = 0.0
    # the seeded generator works on 64-bit integers: draw the context in token chunks (multiples of the group) that keep
    # its temporaries near 2 GiB each, and append chunk by chunk (chunked appends give the same cache as one bulk append)
    chunk = max(w.group, ((1 << 28) // (w.batch * w.n_kv_heads * w.head_dim)) // w.group * w.group)
    # the first launch of a kernel instantiation pays for loading its code: one small append per precision pair first
    pairs = sorted(set(zip(w.kbits, w.vbits)))
    tiny = pkg.KVQ(len(pairs), 1, w.n_q_heads, w.n_kv_heads, w.head_dim, 128, [p[0] for p in pairs], [p[1] for p in pairs],
                   group=w.group, residual=w.residual, device=dev,
                   meta_dtype=pkg.META_FP16 if SCALE_BYTES == 2 else pkg.META_FP32,
                   key_mode=pkg.KEYS_PER_TOKEN if KEYS_PER_TOKEN else pkg.KEYS_PER_CHANNEL)
    kv = torch.randn(1, w.n_kv_heads, 96, w.head_dim, device=dev).to(torch.float16)
    for i in range(len(pairs)):
        tiny.quantize_append(i, kv, kv)
    torch.cuda.synchronize()
    tiny.close()
    del tiny, kv
    # A fill of 256 MB is queued in front of every timed append: while the GPU is busy with it the host enqueues the
    # append, so the two events bracket the GPU's work on it and not the host's launch latency on an idle GPU (and the
    # fill leaves none of the inputs in the last-level cache).
    pad = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    for layer in range(w.n_layers):
        for t0 in range(0, w.context, chunk):
            t1 = min(w.context, t0 + chunk)
            K, V = W.kv_tokens(w, layer, t0, t1, device=dev)
            pad.zero_()
            ev0.record()
            cache.quantize_append(layer, K, V)
            ev1.record()
            torch.cuda.synchronize()
            q_ms += ev0.elapsed_time(ev1)
            del K, V
    del pad
    return cache, q_ms


def step_inputs(torch, W, w, n_steps):
    """Per layer: queries [S,B,Hq,D] and new tokens [S,B,Hkv,1,D] for S decode steps, on the GPU."""
    dev = "cuda:0"
    qs, ks, vs = [], [], []
    for layer in range(w.n_layers):
        qs.append(torch.stack([W.query(w, layer, s, device=dev) for s in range(n_steps)]))
        K, V = W.kv_tokens(w, layer, 0, n_steps, device=dev, stream=1, total=n_steps)
        ks.append(K.permute(2, 0, 1, 3).contiguous().unsqueeze(3))
        vs.append(V.permute(2, 0, 1, 3).contiguous().unsqueeze(3))
    return qs, ks, vs


def run_steps(torch, cache, w, qs, ks, vs, outs, s0, s1, probes=None):
    """Decode steps s0..s1-1 through the C ABI with pre-resolved pointers (no per-call Python checks).

    probes = {layer: [(begin, end) HIP event pair per step]}: on those layers the main decode kernel of step s stamps
    its pair with its own start and end (the live measurement inside the timed region)."""
    from ctypes import c_void_p

    lib, h = cache._lib, cache._h
    L = w.n_layers
    hooked = False
    for s in range(s0, s1):
        for layer in range(L):
            if probes is not None and layer in probes:
                lib.kvq_set_kernel_events(h, probes[layer][s - s0][0], probes[layer][s - s0][1])
                hooked = True
            elif hooked:
                lib.kvq_set_kernel_events(h, None, None)
                hooked = False
            if FUSED_STEP:
                rc = lib.kvq_append_decode_attention(h, layer, c_void_p(ks[layer][s].data_ptr()), c_void_p(vs[layer][s].data_ptr()),
                                                     c_void_p(qs[layer][s].data_ptr()), c_void_p(outs[layer].data_ptr()))
                if rc:
                    raise RuntimeError("kvq_append_decode_attention failed: %d" % rc)
                continue
            rc = lib.kvq_quantize_append(h, layer, c_void_p(ks[layer][s].data_ptr()), c_void_p(vs[layer][s].data_ptr()), 1)
            if rc:
                raise RuntimeError("kvq_quantize_append failed: %d" % rc)
            rc = lib.kvq_decode_attention(h, layer, c_void_p(qs[layer][s].data_ptr()), c_void_p(outs[layer].data_ptr()))
            if rc:
                raise RuntimeError("kvq_decode_attention failed: %d" % rc)
        if hooked:
            lib.kvq_set_kernel_events(h, None, None)
            hooked = False


def time_workload(torch, pkg, W, w, steps, warmup, variant=0, splits=0, per_kernel=True):
    """Returns a dict with step time, tokens/s, algorithmic GB/s and per-layer-type decode timings."""
    total_steps = warmup + steps
    cache, prefill_ms = build_cache(torch, pkg, W, w, total_steps + 8, variant, splits)
    qs, ks, vs = step_inputs(torch, W, w, total_steps)
    outs = [torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.float16, device="cuda:0") for _ in range(w.n_layers)]
    run_steps(torch, cache, w, qs, ks, vs, outs, 0, warmup)
    torch.cuda.synchronize()
    # One layer of every precision pair is timed live inside the timed region: its main decode kernel stamps a HIP
    # event pair with its own start and end, one pair per step (kvq_set_kernel_events).
    hip = HipEvents()
    by_pair = {}
    for l in range(w.n_layers):
        by_pair.setdefault((w.kbits[l], w.vbits[l]), []).append(l)
    probes = {ls[len(ls) // 2]: [(hip.create(), hip.create()) for _ in range(steps)] for ls in by_pair.values()}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    run_steps(torch, cache, w, qs, ks, vs, outs, warmup, total_steps, probes if per_kernel else None)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(wall_ms, gpu_ms) / steps
    cache.set_kernel_events(None, None)
    t_mid = w.context + warmup + steps // 2
    np_mid = w.group * (max(t_mid - w.residual, 0) // w.group)
    per_pair = {}
    for layer, evs in probes.items():
        key = (w.kbits[layer], w.vbits[layer])
        if per_kernel:
            ms = [hip.elapsed_ms(a, b) for a, b in evs]
            nbytes = layer_bytes(w, key[0], key[1], np_mid, t_mid - np_mid)
            per_pair["K%dV%d" % key] = {"layers": len(by_pair[key]), "probed_layer": layer, "launches": len(ms),
                                        "kernel_ms": sum(ms) / len(ms), "bytes": nbytes,
                                        "kernel_gbps": nbytes / (sum(ms) / len(ms) * 1e-3) / 1e9}
        for a, b in evs:
            hip.destroy(a)
            hip.destroy(b)

    # bytes of one step at the middle of the timed region
    T_mid = w.context + warmup + steps // 2
    n_p = w.group * (max(T_mid - w.residual, 0) // w.group)
    step_bytes = sum(layer_bytes(w, w.kbits[l], w.vbits[l], n_p, T_mid - n_p) for l in range(w.n_layers))
    res = {
        "workload": w.name, "ms_per_step": ms_per_step, "gpu_ms_per_step": gpu_ms / steps, "wall_ms_per_step": wall_ms / steps,
        "tokens_per_s": w.batch / (ms_per_step * 1e-3), "step_bytes": step_bytes,
        "algorithmic_gbps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "prefill_quantize_ms": prefill_ms, "per_pair": per_pair,
        "prefill_quantize_input_gbps": (w.n_layers * w.batch * w.n_kv_heads * w.context * w.head_dim * 4) / (prefill_ms * 1e-3) / 1e9,
    }
    cache.close()
    del cache, qs, ks, vs, outs
    torch.cuda.empty_cache()
    return res


MFMA_F16_PEAK_TFLOPS = 2500.0     # MI355X dense fp16 matrix-core peak


def time_prefill_attention(torch, pkg, W, w, layer, reps=3, meta=None, keys=None, reference=True):
    """The prompt's own causal attention over the dequantized cache of one layer (every position a query), timed
    between HIP events stamped by the kernel's own dispatch.  Algorithmic flops: 4 * head_dim per (query, visible
    token) pair and query head."""
    T = w.context
    kw = {}
    if meta is not None:
        kw["meta_dtype"] = meta
    if keys is not None:
        kw["key_mode"] = keys
    cache = pkg.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, T + w.group, [w.kbits[layer]], [w.vbits[layer]],
                    group=w.group, residual=w.residual, **kw)
    chunk = max(w.group, ((1 << 28) // (w.batch * w.n_kv_heads * w.head_dim)) // w.group * w.group)
    for t0 in range(0, T, chunk):
        K, V = W.kv_tokens(w, layer, t0, min(T, t0 + chunk), device="cuda:0")
        cache.quantize_append(0, K, V)
    del K, V
    gq = w.n_q_heads // w.n_kv_heads
    q = torch.empty(w.batch, w.n_q_heads, T, w.head_dim, dtype=torch.float16, device="cuda:0")
    for h0 in range(0, w.n_q_heads, gq):
        q[:, h0:h0 + gq] = W.prefill_queries(w, layer, T, device="cuda:0", heads=(h0, gq))
    out = torch.empty_like(q)
    cache.prefill_attention(0, q, out)
    torch.cuda.synchronize()
    hip = HipEvents()

    def timed_calls(n):
        evs = [(hip.create(), hip.create()) for _ in range(n)]
        for a, b in evs:
            cache.set_kernel_events(a, b)
            cache.prefill_attention(0, q, out)
        cache.set_kernel_events(None, None)
        torch.cuda.synchronize()
        ms = [hip.elapsed_ms(a, b) for a, b in evs]
        for a, b in evs:
            hip.destroy(a)
            hip.destroy(b)
        return sum(ms) / len(ms)

    avg = timed_calls(reps)
    # for reference, the same call with the per-cache choice of the key channels that keep their second fp16 number
    # switched off (every channel keeps it): one call, not part of the figure
    all_channels_ms = None
    if reference:
        cache.set_prefill_options(1)
        cache.prefill_attention(0, q, out)
        all_channels_ms = timed_calls(1)
        cache.set_prefill_options(0)
    flops = 4.0 * w.head_dim * (T * (T + 1) // 2) * w.batch * w.n_q_heads
    res = {"kernel": "prefill_attention<K%dV%d>" % (w.kbits[layer], w.vbits[layer]), "layer": layer, "queries": T,
           "launches_timed": reps, "avg_launch_ms": avg, "flops_per_launch": flops,
           "roofline": {"bound": "mfma", "achieved": flops / (avg * 1e-3) / 1e12, "peak": MFMA_F16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": flops / (avg * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, "traffic": None},
           "prompt_tokens_per_s_per_layer": w.batch * T / (avg * 1e-3),
           "low_parts": "dequantized keys centred per channel; their second fp16 number kept per cache for all channels or for "
                        "the 32 that need it (chosen on the GPU from the stored metadata and a sample of the queries)",
           "ms_with_low_parts_of_all_channels": all_channels_ms}
    cache.close()
    del cache, q, out
    torch.cuda.empty_cache()
    return res


def cpu_baseline(W, w, budget_s=20.0):
    """The CPU oracle as it stands on a bounded sample: one layer per distinct precision pair, a slice of
    the batch, the full context; one decode step (append + attention) each, extrapolated linearly."""
    import numpy as np
    import oracle
    import torch

    pairs = {}
    for l in range(w.n_layers):
        pairs.setdefault((w.kbits[l], w.vbits[l]), []).append(l)
    b_s = min(w.batch, 2)
    ws = W.Workload(w.name + "-sample", w.n_layers, b_s, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context, w.kbits, w.vbits,
                    seed=w.seed, group=w.group, residual=w.residual, outlier_channels=w.outlier_channels,
                    outlier_scale=w.outlier_scale, key_bias_std=w.key_bias_std)
    step_s = 0.0
    t_start = time.perf_counter()
    for (kb, vb), layers in pairs.items():
        layer = layers[0]
        oc = oracle.OracleCache(1, b_s, w.n_q_heads, w.n_kv_heads, w.head_dim, [kb], [vb], group=w.group, residual=w.residual,
                                scale_fp16=SCALE_BYTES == 2, key_per_token=KEYS_PER_TOKEN)
        K, V = W.kv_tokens(ws, layer, 0, w.context)
        oc.quantize_append(0, K.numpy(), V.numpy())
        kn, vn = W.kv_tokens(ws, layer, 0, 1, stream=1, total=1)
        q = W.query(ws, layer, 0).numpy()
        reps, t_pair = 0, 0.0
        while reps < 1 or t_pair < budget_s / len(pairs):
            t0 = time.perf_counter()
            oc.quantize_append(0, kn.numpy(), vn.numpy())
            oc.decode_attention(0, q)
            t_pair += time.perf_counter() - t0
            reps += 1
        step_s += (t_pair / reps) * len(layers) * (w.batch / b_s)
        oc.close()
    return {
        "value": w.batch / step_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "one layer per precision pair (%s), %d of %d sequences, full %d-token context, append + decode; "
                  "extrapolated linearly to %d layers x batch %d (sampled in %.1f s)" % (
                      ", ".join("K%dV%d" % p for p in pairs), b_s, w.batch, w.context, w.n_layers, w.batch,
                      time.perf_counter() - t_start),
    }


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "decode_traffic.json")
KERNEL_SOURCES = ("kvq_decode_mfma.hip", "kvq_layout.h", "kvq_internal.h")
PREFILL_SOURCES = ("kvq_prefill_attn.hip", "kvq_layout.h", "kvq_internal.h")


def kernel_source_hash(name=""):
    """Hash of the sources of the kernel a traffic record belongs to (records named prefill_attention:... belong to the
    prefill-stage attention kernels, all others to the decode kernel): a counter record taken with other sources is
    not this kernel's."""
    import hashlib

    h = hashlib.sha256()
    for src in (PREFILL_SOURCES if name.startswith("prefill_attention:") else KERNEL_SOURCES):
        with open(os.path.join(ROOT, "paper_2502_04420_amd", "csrc", src), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def summary(res, w):
    """The figures of one timed workload that the extra objects of the line carry."""
    counts = {}
    for l in range(w.n_layers):
        k = "K%dV%d" % (w.kbits[l], w.vbits[l])
        counts[k] = counts.get(k, 0) + 1
    pairs = {}
    for k, v in res["per_pair"].items():
        rec = read_traffic(w.name + ":" + k)
        pairs[k] = {"layers": counts[k], "kernel_us": v["kernel_ms"] * 1e3, "bytes_per_launch": v["bytes"],
                    "kernel_gbps": v["kernel_gbps"], "frac_of_hbm_peak": v["kernel_gbps"] / HBM_PEAK_GBPS,
                    "traffic": rec["total_bytes"] if rec else None}
    return {"workload": w.name, "tokens_per_s": res["tokens_per_s"], "ms_per_step": res["ms_per_step"],
            "hbm_gbps": res["algorithmic_gbps"], "hbm_frac_of_peak": res["algorithmic_gbps"] / HBM_PEAK_GBPS, "per_pair": pairs}


def extra_configs(torch, pkg, W, args):
    """The benchmark's other single-GPU configurations, each a decode loop like the main one (fewer steps):
    the Qwen2.5-7B shape (28 layers, 28 q / 4 kv heads, biased keys) at batch 8 and 32768 tokens with the 4.0-bit
    schedule (even layers K8V2, odd K4V2) against uniform K8V8, and uniform K8V8 on the Llama shape at batch 16 and
    4096 tokens."""
    out = {}
    wq, wq8 = W.named("qwen7b", "mix4.0", 8, 32768), W.named("qwen7b", "K8V8", 8, 32768)
    rq = time_workload(torch, pkg, W, wq, 16, 2, args.variant, args.splits)
    rq8 = time_workload(torch, pkg, W, wq8, 16, 2, args.variant, args.splits)
    out["qwen7b-B8-T32768"] = dict(summary(rq, wq), steps=16, warmup=2, kv8=summary(rq8, wq8),
                                   speedup_vs_kv8=rq["tokens_per_s"] / rq8["tokens_per_s"])
    if not args.no_prefill_attn:
        # the prompt's own attention on this shape (keys with a large offset on every channel), one K4V2 layer
        out["qwen7b-B8-T32768"]["prefill_attention"] = time_prefill_attention(torch, pkg, W, wq, 1, reps=2,
                                                                              reference=not args.no_prefill_reference)
    w2 = W.config2(16, 4096)
    r2 = time_workload(torch, pkg, W, w2, 32, 4, args.variant, args.splits)
    out["llama8b-B16-T4096-K8V8"] = dict(summary(r2, w2), steps=32, warmup=4)
    return out


def read_traffic(name):
    """HBM bytes per launch of a decode kernel from the committed rocprofv3 counter record (FETCH_SIZE / WRITE_SIZE
    runs, see profiles/), or None when there is none for this configuration or when it was taken with other kernel
    sources than the ones in the tree (the record carries their hash)."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(name)
    except (OSError, ValueError):
        return None
    if rec is None or rec.get("kernel_sources") != kernel_source_hash(name):
        return None
    return rec


def record_traffic(args):
    """--record-traffic NAME FETCH_KIB WRITE_KIB FETCH_SCALE WRITE_SCALE SOURCE: store the counter means of one decode
    kernel (per dispatch, from two rocprofv3 --pmc runs) together with the hash of the kernel sources they belong to."""
    name, fetch_kib, write_kib, fscale, wscale, source = args
    try:
        with open(TRAFFIC_FILE) as f:
            data = json.load(f)
    except (OSError, ValueError):
        data = {}
    fb, wb = float(fetch_kib) * 1024.0 * float(fscale), float(write_kib) * 1024.0 * float(wscale)
    data[name] = {"fetch_bytes": fb, "write_bytes": wb, "total_bytes": fb + wb, "source": source,
                  "kernel_sources": kernel_source_hash(name), "recorded": time.strftime("%Y-%m-%d")}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(data, f, indent=1)
    print("recorded", name, data[name])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama8b-B16-T8192",
                    help="llama8b-B<batch>-T<context> (3.25-bit mix vs K8V8) or qwen7b-B<batch>-T<context> (4.0-bit mix vs K8V8)")
    ap.add_argument("--schedule", default="",
                    help="layer-wise schedule: llama8b: mix3.25 (default, the benchmark's), kivi-c3.25, kivi-c4.90 (the paper's "
                         "searched ones); qwen7b: mix4.0 (default), kivi-c3.92 (the paper's); or a uniform pair like K4V2")
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 vector-ALU kernel, 2 matrix-core kernel")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--meta", choices=["fp32", "fp16"], default="fp32",
                    help="precision of the stored scales (fp16 = the narrow-metadata variant; zero-points are exact either way)")
    ap.add_argument("--keys", choices=["per-channel", "per-token"], default="per-channel",
                    help="key grouping: per channel over 32 tokens (KIVI mode, default) or per token over 32 channels")
    ap.add_argument("--separate-calls", action="store_true",
                    help="per layer and step call kvq_quantize_append and kvq_decode_attention instead of the one-call "
                         "step kvq_append_decode_attention (same work, one more launch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kv8", action="store_true")
    ap.add_argument("--no-32k", action="store_true",
                    help="skip the extra point at 32768 tokens of context (same family and schedule, batch 32, 16 steps: "
                         "enough bytes per launch for the kernels' steady state)")
    ap.add_argument("--no-prefill-attn", action="store_true",
                    help="skip the extra measurement of the prefill-stage attention kernel (one layer of the dominant pair)")
    ap.add_argument("--no-prefill-reference", action="store_true",
                    help="prefill attention: skip the extra call with the per-cache treatment of the keys switched off "
                         "(used for profiling runs, whose per-kernel means would mix the two)")
    ap.add_argument("--only", default="", help="time just 'mix' or 'kv8' (used for profiling runs)")
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="skip the two further benchmark configurations timed after the main one: the Qwen2.5-7B shape "
                         "(28 q / 4 kv heads, batch 8, 32768 tokens, 4.0-bit mix vs K8V8) and uniform K8V8 at 4096 tokens")
    ap.add_argument("--record-traffic", nargs=6, metavar=("NAME", "FETCH_KIB", "WRITE_KIB", "FETCH_SCALE", "WRITE_SCALE", "SOURCE"),
                    help="no benchmark: store rocprofv3 FETCH_SIZE / WRITE_SIZE means of a decode kernel in profiles/decode_traffic.json")
    ap.add_argument("--copy-calib", action="store_true",
                    help="first run 5 plain streaming kernels that read 1 GiB and write 1 GiB (torch.neg on fp32; "
                         "a known-size reference for hardware counters)")
    args = ap.parse_args()
    if args.record_traffic:
        record_traffic(args.record_traffic)
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import kvq_workloads as W
    import paper_2502_04420_amd as pkg

    global SCALE_BYTES, KEYS_PER_TOKEN, FUSED_STEP
    FUSED_STEP = not args.separate_calls
    SCALE_BYTES = 2 if args.meta == "fp16" else 4
    KEYS_PER_TOKEN = args.keys == "per-token"
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    pkg.load_library()
    if args.copy_calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.neg(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    fam, bpart, tpart = args.workload.split("-")
    batch, context = int(bpart[1:]), int(tpart[1:])
    if fam not in W.SCHEDULES:
        raise SystemExit("unknown workload family %r (have %s)" % (fam, ", ".join(W.SCHEDULES)))
    schedule = args.schedule or {"llama8b": "mix3.25", "qwen7b": "mix4.0"}[fam]
    w_mix = W.named(fam, schedule, batch, context)
    w_kv8 = W.named(fam, "K8V8", batch, context)

    mix = None if args.only == "kv8" else time_workload(torch, pkg, W, w_mix, args.steps, args.warmup, args.variant, args.splits)
    kv8 = None
    if not args.no_kv8 and args.only != "mix":
        kv8 = time_workload(torch, pkg, W, w_kv8, args.steps, args.warmup, args.variant, args.splits)
    main_res = mix if mix is not None else kv8
    w_main = w_mix if mix is not None else w_kv8

    # dominant kernel = the decode kernel of the precision pair that carries the most layers
    counts = {}
    for l in range(w_main.n_layers):
        k = "K%dV%d" % (w_main.kbits[l], w_main.vbits[l])
        counts[k] = counts.get(k, 0) + 1
    dom = max(counts, key=counts.get)
    pk = main_res["per_pair"][dom]
    roofline = {
        "bound": "hbm", "kernel": "decode_mfma<%s> (%d of %d layers)" % (dom, counts[dom], w_main.n_layers),
        "achieved": pk["kernel_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": pk["kernel_gbps"] / HBM_PEAK_GBPS,
        "avg_launch_ms": pk["kernel_ms"], "bytes_per_launch": pk["bytes"], "launches_timed": pk["launches"],
        "timed": "inside the timed region, layer %d of every step, between HIP events stamped by the kernel's own dispatch" % pk["probed_layer"],
    }
    # HBM bytes per launch measured with the counters (fetch + write), or null when this configuration was not profiled
    detail = read_traffic(w_main.name + ":" + dom + (":scales-fp16" if args.meta == "fp16" else "") + (":keys-per-token" if KEYS_PER_TOKEN else ""))
    roofline["traffic"] = detail["total_bytes"] if detail else None
    roofline["traffic_detail"] = detail if detail else (
        "no counter record for this configuration taken with the kernel sources in the tree (profiles/decode_traffic.json)")
    from paper_2502_04420_amd import equivalent_precision

    eq_bits = equivalent_precision(w_main.kbits, w_main.vbits)
    metric_name = ("fused dequant decode-attn tokens/s + HBM GB/s, 3.25-bit mix vs KV8, 1 GPU" if fam == "llama8b" and schedule == "mix3.25"
                   else "fused dequant decode-attn tokens/s + HBM GB/s, %s %.2f-bit schedule vs KV8, 1 GPU" % (schedule, eq_bits))

    out = {
        "metric": metric_name, "value": main_res["tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp16 MFMA operands (codes exact, q*s and p*s as hi + lo fp16 pairs), fp32 accumulate", "data": "synthetic",
        "config": {"workload": w_main.name, "layers": w_main.n_layers, "batch": w_main.batch, "q_heads": w_main.n_q_heads,
                   "kv_heads": w_main.n_kv_heads, "head_dim": w_main.head_dim, "context": w_main.context,
                   "equivalent_bits": equivalent_precision(w_main.kbits, w_main.vbits), "group": 32, "residual": 32,
                   "scales": args.meta, "zero_points": "fp16 (exact)", "key_grouping": args.keys,
                   "step": "per layer: append 1 token (+ flush of 32 every 32 steps) + fused decode attention, "
                           + ("two calls" if args.separate_calls else "one call (kvq_append_decode_attention)")},
        "hbm_gbps": main_res["algorithmic_gbps"], "hbm_frac_of_peak": main_res["algorithmic_gbps"] / HBM_PEAK_GBPS,
        "step_bytes": main_res["step_bytes"], "gpu_ms_per_step": main_res["gpu_ms_per_step"],
        "prefill_quantize_input_gbps": main_res["prefill_quantize_input_gbps"],
        "per_pair": main_res["per_pair"], "roofline": roofline,
    }
    if kv8 is not None and mix is not None:
        out["kv8"] = {"workload": w_kv8.name, "tokens_per_s": kv8["tokens_per_s"], "ms_per_step": kv8["ms_per_step"],
                      "hbm_gbps": kv8["algorithmic_gbps"], "hbm_frac_of_peak": kv8["algorithmic_gbps"] / HBM_PEAK_GBPS,
                      "per_pair": kv8["per_pair"]}
        out["speedup_vs_kv8"] = mix["tokens_per_s"] / kv8["tokens_per_s"]
    if not args.no_32k and not args.only and context < 32768:
        # the same schedule against uniform K8V8 at 32K context: enough bytes per launch for the kernels' steady state
        b32 = 32 if fam == "llama8b" else 8
        wl, w8 = W.named(fam, schedule, b32, 32768), W.named(fam, "K8V8", b32, 32768)
        r_mix = time_workload(torch, pkg, W, wl, 16, 2, args.variant, args.splits)
        r_kv8 = time_workload(torch, pkg, W, w8, 16, 2, args.variant, args.splits)
        out["at_32k_context"] = {
            "workload": wl.name, "steps": 16, "warmup": 2, "tokens_per_s": r_mix["tokens_per_s"], "ms_per_step": r_mix["ms_per_step"],
            "hbm_gbps": r_mix["algorithmic_gbps"], "hbm_frac_of_peak": r_mix["algorithmic_gbps"] / HBM_PEAK_GBPS,
            "per_pair": r_mix["per_pair"],
            "kv8": {"workload": w8.name, "tokens_per_s": r_kv8["tokens_per_s"], "ms_per_step": r_kv8["ms_per_step"],
                    "hbm_frac_of_peak": r_kv8["algorithmic_gbps"] / HBM_PEAK_GBPS, "per_pair": r_kv8["per_pair"]},
            "speedup_vs_kv8": r_mix["tokens_per_s"] / r_kv8["tokens_per_s"]}
    if not args.no_extra_configs and not args.only and fam == "llama8b" and not args.schedule:
        out["extra_configs"] = extra_configs(torch, pkg, W, args)
    if not args.no_prefill_attn and not args.only:
        dom_layers = [l for l in range(w_main.n_layers) if "K%dV%d" % (w_main.kbits[l], w_main.vbits[l]) == dom]
        out["prefill_attention"] = time_prefill_attention(
            torch, pkg, W, w_main, dom_layers[len(dom_layers) // 2],
            meta=pkg.META_FP16 if args.meta == "fp16" else None, keys=pkg.KEYS_PER_TOKEN if KEYS_PER_TOKEN else None,
            reference=not args.no_prefill_reference)
        # HBM bytes of one call (all its launches: dequantization passes and attention passes), from the counter record
        rec = read_traffic("prefill_attention:" + w_main.name + ":" + dom + (":scales-fp16" if args.meta == "fp16" else "") +
                           (":keys-per-token" if KEYS_PER_TOKEN else ""))
        out["prefill_attention"]["roofline"]["traffic"] = rec["total_bytes"] if rec else None
        if rec:
            out["prefill_attention"]["roofline"]["traffic_detail"] = rec
    out["paper_context"] = "paper reports +16.79%..+21.25% end-to-end tokens/s for its 3.25-bit schedule over KIVI-KV8 (GPU not named)"
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, w_main)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
