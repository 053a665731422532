#!/usr/bin/env python3
"""Benchmark of the rotate-and-quantize hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one rq_rotate_quantize call (load, zero-pad, rotate, absmax, scale, round/clip, pack)
over one batch of the Llama-shaped configuration: X bf16 [2048 x 4096], H_4096, b = 4,
clip = 0.9.  Batches live in a ring of distinct HBM buffers larger than the last-level cache,
so every step reads cold data; the K steps are replayed from one HIP graph so the timed region
is kernel work, not Python launch overhead (the eager per-call rate is reported next to it).
The last line printed is one JSON object: metric / value / unit, the roofline of the dominant
kernel, the sustained rate on a large launch, a per-configuration table and the CPU oracle's rate.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
RING_BYTES = 1536 << 20         # ring of batches: well above the 256 MB last-level cache
# HBM bytes per timed launch measured with rocprofv3 PMC counters (FETCH_SIZE, WRITE_SIZE, each scaled
# by what the same counter reads for a 256 MiB copy); it does not depend on timing, so it is recorded
# here from profiles/hbm_traffic_wave_sylvester_llama_hidden_b4.txt rather than re-measured per run
TRAFFIC_BYTES_PER_LAUNCH = {"wave_sylvester": 21_160_770}


def algorithmic_bytes_per_row(d: int, n: int, bits: int, elem: int = 2) -> int:
    """Bytes in + out per row: the input row, the packed codes, one fp32 scale."""
    return elem * d + n * bits // 8 + 4


def bytes_view(t):
    return t.numel() * t.element_size()


def time_steady_state(torch, binding, h, base, bits, clip, rows_total):
    """One large launch (input >= 1 GiB): the kernel's sustained rate without launch effects."""
    reps = rows_total // base.shape[0]
    x = base.repeat(reps, 1)
    codes = torch.empty((x.shape[0], h.n * bits // 8), dtype=torch.uint8, device="cuda")
    scales = torch.empty((x.shape[0],), dtype=torch.float32, device="cuda")
    for _ in range(2):
        binding.rotate_quantize(h, x, bits, clip, codes=codes, scales=scales)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_it = 5
    e0.record()
    for _ in range(n_it):
        binding.rotate_quantize(h, x, bits, clip, codes=codes, scales=scales)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / n_it
    nbytes = x.shape[0] * algorithmic_bytes_per_row(x.shape[1], h.n, bits)
    return {"rows": int(x.shape[0]), "ms_per_launch": ms, "GBps": nbytes / ms / 1e6,
            "frac_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBPS,
            "tokens_per_s": x.shape[0] / ms * 1e3}


VALU_PEAK_TLANEOPS = 39.3       # 256 CUs x 64 lanes x 2.4 GHz, packed fp32 excluded (T lane-ops/s)


def _min_ms(torch, fn, n=6, rounds=8):
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / n)
    return best


def _graph_ms(torch, fn, n=20, rounds=8):
    """Short calls: n of them captured in one HIP graph and replayed, so that what is timed is the GPU's
    launch-to-launch rate and not how fast Python can issue calls.  Best of `rounds` replays, HIP events."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(n):
            fn()
    g.replay()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / n)
    return best


def time_all_configs(torch, binding, wl):
    """Every configuration's rotate_quantize at its own row count and at a steady-state row count
    (input >= 1 GiB, rows tiled from a 2048-row seeded sample), plus quant_error on the
    calibration tensor.  Best of 8 rounds of 6 launches, HIP events, inputs resident and reused
    (warm caches for the small shapes): context next to the cold-ring headline figure."""
    res = {}
    for name in ("llama_hidden", "qwen_hidden", "ffn_expand", "ffn_down", "kv_k"):
        w = wl.WORKLOADS[name]
        base_rows = min(w.rows, 2048)
        xb = wl.generate(w.with_rows(base_rows))
        x0 = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        h = binding.hadamard_build(w.n)
        steady_rows = w.rows if name.startswith("kv") else max(w.rows, ((1 << 30) // (2 * w.d)) // base_rows * base_rows)
        for b in w.bits:
            row_bytes = algorithmic_bytes_per_row(w.d, w.n, b)
            entry = {"n": w.n, "d": w.d, "bits": b}
            for label, rows in (("config_rows", w.rows), ("steady_rows", steady_rows)):
                x = x0.repeat(max(1, rows // base_rows), 1)
                codes = torch.empty((x.shape[0], w.n * b // 8), dtype=torch.uint8, device="cuda")
                scales = torch.empty((x.shape[0],), dtype=torch.float32, device="cuda")
                call = lambda: binding.rotate_quantize(h, x, b, w.clip, codes=codes, scales=scales)
                # the config-exact launches are a few microseconds long: graph replay, inputs warm
                ms = _graph_ms(torch, call) if label == "config_rows" and not name.startswith("kv") else _min_ms(torch, call)
                gbps = x.shape[0] * row_bytes / ms / 1e6
                entry[label] = {"rows": int(x.shape[0]), "us": ms * 1e3, "GBps": gbps,
                                "frac_hbm_peak": gbps / HBM_PEAK_GBPS}
                entry["kernel"] = h.last_kernel
                del x, codes, scales
            res[f"{name}_b{b}"] = entry
        del x0
        torch.cuda.empty_cache()
    # widened entry points: asymmetric group-128 on the key cache, rotation-free quantizer
    w = wl.WORKLOADS["kv_k"]
    x = torch.from_numpy(wl.generate(w.with_rows(2048)).view(np.int16)).cuda().view(torch.bfloat16)
    x = x.repeat(w.rows // 2048, 1)
    h = binding.hadamard_build(w.n)
    b = w.bits[0]
    codes = torch.empty((x.shape[0], w.n * b // 8), dtype=torch.uint8, device="cuda")
    scales = torch.empty((x.shape[0], 1), dtype=torch.float32, device="cuda")
    mins = torch.empty((x.shape[0], 1), dtype=torch.float32, device="cuda")
    ms = _min_ms(torch, lambda: binding.rotate_quantize_asym(h, x, b, w.clip, codes=codes, scales=scales, mins=mins))
    gbps = x.shape[0] * (2 * w.d + w.n * b / 8 + 8) / ms / 1e6
    res[f"kv_k_asym_b{b}"] = {"n": w.n, "d": w.d, "bits": b, "rows": int(x.shape[0]), "us": ms * 1e3,
                              "GBps": gbps, "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
    del x, codes, scales, mins
    # asymmetric group-128 quantizer without a rotation (the value cache: its rotation is fused upstream)
    w = wl.WORKLOADS["kv_v"]
    x = torch.from_numpy(wl.generate(w.with_rows(2048)).view(np.int16)).cuda().view(torch.bfloat16)
    x = x.repeat(w.rows // 2048, 1)
    b = w.bits[0]
    codes = torch.empty((x.shape[0], w.d * b // 8), dtype=torch.uint8, device="cuda")
    scales = torch.empty((x.shape[0], 1), dtype=torch.float32, device="cuda")
    mins = torch.empty((x.shape[0], 1), dtype=torch.float32, device="cuda")
    ms = _min_ms(torch, lambda: binding.quantize_asym(x, b, w.clip, codes=codes, scales=scales, mins=mins))
    gbps = x.shape[0] * (2 * w.d + w.d * b / 8 + 8) / ms / 1e6
    res[f"kv_v_plain_asym_b{b}"] = {"d": w.d, "bits": b, "rows": int(x.shape[0]), "us": ms * 1e3, "GBps": gbps,
                                    "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": "plain_quantize_asym"}
    # the same rows through the per-token symmetric quantizer without a rotation (several rows per wave)
    codes = torch.empty((x.shape[0], w.d * b // 8), dtype=torch.uint8, device="cuda")
    ms = _min_ms(torch, lambda: binding.quantize(x, b, w.clip, codes=codes, scales=scales))
    gbps = x.shape[0] * (2 * w.d + w.d * b / 8 + 4) / ms / 1e6
    res[f"kv_v_plain_sym_b{b}"] = {"d": w.d, "bits": b, "rows": int(x.shape[0]), "us": ms * 1e3, "GBps": gbps,
                                   "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": "plain_quantize_short"}
    del x, codes, scales, mins
    # rotation alone (the query heads carry the same per-head H_128 as the keys): bf16 in, bf16 out
    w = wl.WORKLOADS["kv_k"]
    x = torch.from_numpy(wl.generate(w.with_rows(2048)).view(np.int16)).cuda().view(torch.bfloat16)
    x = x.repeat(w.rows // 2048, 1)
    h = binding.hadamard_build(w.n)
    y = torch.empty_like(x)
    ms = _min_ms(torch, lambda: binding.rotate(h, x, out=y))
    gbps = x.shape[0] * 4 * w.d / ms / 1e6
    res["rotate_heads_bf16"] = {"n": w.n, "rows": int(x.shape[0]), "us": ms * 1e3, "GBps": gbps,
                                "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
    # the way back for the key cache as the paper quantizes it (section 5.1: asymmetric groups of 128, 3 bits):
    # packed codes + Delta + lo -> bf16 head rows in the original basis
    codes, scales, mins = binding.rotate_quantize_asym(h, x, 3, w.clip)
    ms = _min_ms(torch, lambda: binding.dequantize_rotate(h, codes, scales, 3, mins=mins, out=y))
    gbps = x.shape[0] * (w.n * 3 // 8 + 8 + 2 * w.d) / ms / 1e6
    res["dequantize_rotate_kv_asym_b3"] = {"n": w.n, "rows": int(x.shape[0]), "out": "bf16", "us": ms * 1e3, "GBps": gbps,
                                           "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
    del x, y, codes, scales, mins
    # the way back for hidden-state rows (codes + scale -> rows in the original basis), bf16 and fp32 out
    w = wl.WORKLOADS["llama_hidden"]
    x = torch.from_numpy(wl.generate(w).view(np.int16)).cuda().view(torch.bfloat16).repeat(32, 1)
    h = binding.hadamard_build(w.n)
    codes, scales = binding.rotate_quantize(h, x, 4, w.clip)
    for dt, key, esz in ((torch.bfloat16, "bf16", 2), (torch.float32, "f32", 4)):
        y = torch.empty((x.shape[0], w.n), dtype=dt, device="cuda")
        ms = _min_ms(torch, lambda: binding.dequantize_rotate(h, codes, scales, 4, out=y))
        gbps = x.shape[0] * (w.n * 4 // 8 + 4 + esz * w.n) / ms / 1e6
        res[f"dequantize_rotate_llama_b4_{key}"] = {"n": w.n, "rows": int(x.shape[0]), "out": key, "us": ms * 1e3, "GBps": gbps,
                                                    "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
        del y
    # codes + scale -> values in the rotated domain (section 2.1's X^ = round(X / Delta) * Delta), fp32 out
    y = torch.empty((x.shape[0], w.n), dtype=torch.float32, device="cuda")
    ms = _min_ms(torch, lambda: binding.dequantize(h, codes, scales, 4, out=y))
    gbps = x.shape[0] * (w.n * 4 // 8 + 4 + 4 * w.n) / ms / 1e6
    res["dequantize_llama_b4_f32"] = {"n": w.n, "rows": int(x.shape[0]), "out": "f32", "us": ms * 1e3, "GBps": gbps,
                                      "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
    del x, y, codes, scales
    # rotation alone on a Paley-block order (H_28 (x) H_128): bf16 in, bf16 out, H and H^T
    w = wl.WORKLOADS["qwen_hidden"]
    x = torch.from_numpy(wl.generate(w.with_rows(2048)).view(np.int16)).cuda().view(torch.bfloat16).repeat(36, 1)
    h = binding.hadamard_build(w.n)
    y = torch.empty_like(x)
    for tr, key in ((False, "rotate_qwen_bf16"), (True, "rotate_qwen_bf16_transposed")):
        ms = _min_ms(torch, lambda: binding.rotate(h, x, transpose=tr, out=y))
        gbps = x.shape[0] * 4 * w.d / ms / 1e6
        res[key] = {"n": w.n, "rows": int(x.shape[0]), "us": ms * 1e3, "GBps": gbps,
                    "frac_hbm_peak": gbps / HBM_PEAK_GBPS, "kernel": h.last_kernel}
    del x, y
    w = wl.WORKLOADS["llama_hidden"]
    x = torch.from_numpy(wl.generate(w).view(np.int16)).cuda().view(torch.bfloat16).repeat(64, 1)
    codes = torch.empty((x.shape[0], w.d * 4 // 8), dtype=torch.uint8, device="cuda")
    scales = torch.empty((x.shape[0],), dtype=torch.float32, device="cuda")
    ms = _min_ms(torch, lambda: binding.quantize(x, 4, w.clip, codes=codes, scales=scales))
    gbps = x.shape[0] * algorithmic_bytes_per_row(w.d, w.d, 4) / ms / 1e6
    res["plain_quantize_llama_b4"] = {"d": w.d, "bits": 4, "rows": int(x.shape[0]), "us": ms * 1e3,
                                      "GBps": gbps, "frac_hbm_peak": gbps / HBM_PEAK_GBPS,
                                      "kernel": "plain_quantize"}
    del x, codes, scales
    torch.cuda.empty_cache()
    # whole-dimension Paley block (1536 + 8 = 1544 = 1543 + 1): a dense contraction on the matrix cores
    w = wl.WORKLOADS["llama_hidden"]
    xs = wl.generate(w)[:, :1544].copy()
    for rows in (2048, 16384):
        x = torch.from_numpy(xs.view(np.int16)).cuda().view(torch.bfloat16).repeat(rows // 2048, 1)
        h = binding.hadamard_build(1544)
        codes = torch.empty((rows, 1544 * 4 // 8), dtype=torch.uint8, device="cuda")
        scales = torch.empty((rows,), dtype=torch.float32, device="cuda")
        ms = _graph_ms(torch, lambda: binding.rotate_quantize(h, x, 4, w.clip, codes=codes, scales=scales), n=5, rounds=4)
        flops = 2.0 * 1544 * 1544 * rows
        res[f"dense_1544_b4_rows{rows}"] = {
            "n": 1544, "bits": 4, "rows": rows, "us": ms * 1e3, "kernel": h.last_kernel,
            "GBps": rows * algorithmic_bytes_per_row(1544, 1544, 4) / ms / 1e6,
            "roofline": {"bound": "mfma", "unit": "TFLOP/s", "achieved": flops / ms / 1e9, "peak": 2500.0,
                         "frac": flops / ms / 1e9 / 2500.0,
                         "note": "2 n^2 flops per row (dense +-1 matrix, bf16 operands); limited by the "
                                 "n^2/8 bytes of operand table each workgroup (16 or 32 rows) reads"}}
        del x, codes, scales
    # quant_error on the other projections a clip search visits (512 rows each; 65536 KV head rows)
    clips = wl.clip_grid()
    for name, rows in (("qwen_hidden", 512), ("ffn_expand", 512), ("ffn_down", 512), ("kv_k", 65536)):
        w = wl.WORKLOADS[name].with_rows(rows)
        x = torch.from_numpy(wl.generate(w).view(np.int16)).cuda().view(torch.bfloat16)
        h = binding.hadamard_build(w.n)
        mse = torch.empty(len(clips), dtype=torch.float32, device="cuda")
        ws = torch.empty(binding.quant_error_workspace(rows, len(clips)) // 8, dtype=torch.float64, device="cuda")
        ms = _graph_ms(torch, lambda: binding.quant_error(h, x, 3, clips, mse=mse, workspace=ws), n=10, rounds=4)
        ec = rows * w.n * len(clips)
        res[f"quant_error_{name}_b3"] = {"rows": rows, "n": w.n, "clips": len(clips), "us": ms * 1e3,
                                         "kernel": h.last_kernel, "element_candidates_per_s": ec / ms * 1e3,
                                         "alu_frac": 5 * ec / ms / 1e9 / VALU_PEAK_TLANEOPS}
        del x, mse, ws
    w = wl.WORKLOADS["calib"]
    x = torch.from_numpy(wl.generate(w).view(np.int16)).cuda().view(torch.bfloat16)
    h = binding.hadamard_build(w.n)
    mse = torch.empty(len(clips), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.quant_error_workspace(w.rows, len(clips)) // 8, dtype=torch.float64, device="cuda")
    ms = _graph_ms(torch, lambda: binding.quant_error(h, x, 3, clips, mse=mse, workspace=ws))
    ec = w.rows * w.n * len(clips)
    res["quant_error_calib_b3"] = {
        "rows": w.rows, "n": w.n, "clips": len(clips), "us": ms * 1e3, "kernel": h.last_kernel,
        "element_candidates_per_s": ec / ms * 1e3,
        "roofline": {"bound": "alu", "unit": "T lane-ops/s", "achieved": 5 * ec / ms / 1e9,
                     "peak": VALU_PEAK_TLANEOPS, "frac": 5 * ec / ms / 1e9 / VALU_PEAK_TLANEOPS,
                     "frac_of_published_fp32_vector_peak": 5 * ec / ms / 1e9 / 78.6,
                     "note": "5 VALU lane-ops per element-candidate; two launches (row sums, reduction); peak = "
                             "256 CUs x 64 lanes x 2.4 GHz without packed fp32 (compiled out), the published "
                             "78.6 T lane-ops/s counts packed issue"}}
    ms = _graph_ms(torch, lambda: binding.quant_error_noalloc(h, x, 3, clips, mse))
    res["quant_error_noalloc_calib_b3"] = {"rows": w.rows, "n": w.n, "clips": len(clips), "us": ms * 1e3,
                                           "kernel": h.last_kernel, "note": "static device scratch instead of a workspace"}
    # Algorithm 1 on the calibration tensor with quant_error as the objective (host loop, batched probes)
    t0 = time.perf_counter()
    n_search = 20
    for _ in range(n_search):
        clip_found, _, trace = binding.gbs_search(h, x, 3, 1.0 / 256)
    res["gbs_search_calib_b3"] = {"rows": w.rows, "n": w.n, "eps": 1.0 / 256, "probes": len(trace), "clip": clip_found,
                                  "ms_per_search": (time.perf_counter() - t0) * 1e3 / n_search}
    # hidden and FFN widths of the model families the paper evaluates (section 5), b = 4, bf16 and
    # fp16 rows, N(0, 1/4) entries, 512 MiB of input per launch; a width without a Hadamard order is
    # zero-padded to the next one (section 4.2)
    widths = {}
    for d in (896, 1536, 2048, 3584, 4096, 5120, 8192, 4864, 8960, 11008, 13824, 14336, 18944, 28672):
        n = binding.next_order(d)
        h = binding.hadamard_build(n)
        rows = max(256, (1 << 29) // (2 * d) // 256 * 256)
        entry = {"n": n, "p": h.p, "rows": rows}
        for dt, key in ((torch.bfloat16, "bf16"), (torch.float16, "f16")):
            x = (torch.randn(rows, d, device="cuda") * 0.5).to(dt)
            codes = torch.empty((rows, n * 4 // 8), dtype=torch.uint8, device="cuda")
            scales = torch.empty((rows,), dtype=torch.float32, device="cuda")
            ms = _min_ms(torch, lambda: binding.rotate_quantize(h, x, 4, 0.9, codes=codes, scales=scales), n=4, rounds=6)
            entry[key] = {"us": ms * 1e3, "frac_hbm_peak": rows * algorithmic_bytes_per_row(d, n, 4) / ms / 1e6 / HBM_PEAK_GBPS,
                          "kernel": h.last_kernel}
            del x, codes, scales
        widths[str(d)] = entry
    res["model_widths_b4"] = widths
    torch.cuda.empty_cache()
    return res


def cpu_baseline(x_bits, n, bits, clip):
    """The oracle as it stands, timed on the host cores on the same batch."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import rotq_oracle as oracle
    threads = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        nt = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        if nt:
            threads = max(nt)
    except Exception:
        pass
    try:
        threads = min(threads, len(os.sched_getaffinity(0)))
    except Exception:
        pass
    # whole batches until about 10 s of CPU work have been done (at most 30 batches)
    reps = 0
    t0 = time.perf_counter()
    while True:
        q, _, _, _ = oracle.rotate_quantize(x_bits, n, bits, clip)
        oracle.pack_codes(q, bits)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 30:
            break
    rows, d = x_bits.shape
    nbytes = reps * rows * algorithmic_bytes_per_row(d, n, bits)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} passes over one full batch [{rows} x {d}] bf16, fp64 dense H_{n} product + "
                      f"quantize + pack, {dt:.2f} s", "tokens_per_s": reps * rows / dt}


def parity_stats(torch, binding, wl):
    """Part of the cpu_baseline leg (the only place bench.py touches the oracle): one checked launch per
    configuration on a bounded sample of its rows, outside every timed region.  Per configuration: code
    mismatches against the oracle, how many of them lie inside the 1e-6 band around a rounding boundary
    (the others would be errors), the size of that band's population, the largest relative scale error."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import rotq_oracle as oracle
    out = {}
    for name, rows in (("tiny", 64), ("llama_hidden", 256), ("qwen_hidden", 256), ("ffn_expand", 256),
                       ("ffn_down", 16), ("kv_k", 4096), ("kv_v", 4096)):
        w = wl.WORKLOADS[name].with_rows(rows)
        x = wl.generate(w)
        xt = (torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16) if x.dtype == np.uint16
              else torch.from_numpy(x).cuda())
        h = binding.hadamard_build(w.n)
        for b in w.bits:
            codes, scales = binding.rotate_quantize(h, xt, b, w.clip)
            torch.cuda.synchronize()
            q, delta, t, _ = oracle.rotate_quantize(x, w.n, b, w.clip)
            qg = oracle.unpack_codes(codes.cpu().numpy(), b, w.n)
            mism = qg != q
            exempt = oracle.boundary_exempt(t, b, 1e-6)
            sg = scales.cpu().numpy().astype(np.float64)
            nz = delta > 0
            rel = np.abs(sg[nz] - delta[nz]) / delta[nz]
            out[f"{name}_b{b}"] = {"rows": rows, "elements": int(q.size), "kernel": h.last_kernel,
                                   "mismatches": int(mism.sum()),
                                   "mismatches_off_boundary": int((mism & ~exempt).sum()),
                                   "exempt_fraction": float(exempt.mean()),
                                   "max_rel_scale_err": float(rel.max()) if rel.size else 0.0}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--repeats", type=int, default=7,
                    help="the timed region (one replay of K steps) is run this many times; the median is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-steady-state", action="store_true")
    ap.add_argument("--no-stream-reference", action="store_true",
                    help="skip the traffic-only reference kernel (practical floor of the launch)")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table")
    ap.add_argument("--variant", type=int, default=0,
                    help="rq_hadamard_set_variant value for the timed step (0 = automatic kernel choice)")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run one 256 MiB device-to-device copy, the known-size reference that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (rows are independent, "
              "so N GPUs would each run this same kernel on their share of the rows); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_13989_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    w = wl.WORKLOADS["llama_hidden"]
    bits, clip = 4, w.clip
    x_bits = wl.generate(w)
    base = torch.from_numpy(x_bits.view(np.int16)).cuda().view(torch.bfloat16)
    h = binding.hadamard_build(w.n)
    h.set_variant(args.variant)

    row_bytes = algorithmic_bytes_per_row(w.d, w.n, bits)
    batch_bytes = w.rows * row_bytes
    ring = max(2, RING_BYTES // batch_bytes)
    # same rows in every slot, rolled so that slots differ; only the addresses need to be distinct
    xs = [torch.roll(base, shifts=i, dims=0).contiguous() for i in range(ring)]
    codes = [torch.empty((w.rows, w.n * bits // 8), dtype=torch.uint8, device="cuda") for _ in range(ring)]
    scales = [torch.empty((w.rows,), dtype=torch.float32, device="cuda") for _ in range(ring)]

    def step(i):
        s = i % ring
        binding.rotate_quantize(h, xs[s], bits, clip, codes=codes[s], scales=scales[s])

    # eager: one C-ABI call per step from Python
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # graph: the same K steps captured once, replayed inside the timed region
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(args.steps):
            step(i)
    for _ in range(max(1, args.warmup // max(1, args.steps)) + 1):
        graph.replay()
    torch.cuda.synchronize()
    # the timed region is one replay = exactly K steps, bracketed by synchronisation on both sides; it is
    # repeated and the median taken, so that a short run (K = 20: 0.15 ms) is not at the mercy of one
    # scheduling hiccup of the host
    walls, kerns = [], []
    for _ in range(args.repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        walls.append((time.perf_counter() - t0) * 1e3)
        kerns.append(e0.elapsed_time(e1))
    wall_ms = float(np.median(walls))
    kernel_ms = float(np.median(kerns)) / args.steps       # average launch duration, HIP events
    ms_per_step = wall_ms / args.steps
    kernel_name = h.last_kernel

    value = batch_bytes / ms_per_step / 1e6                # GB/s over the timed region
    achieved = batch_bytes / kernel_ms / 1e6
    out = {
        "metric": "rotate+quantize GB/s (bytes in+out)",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_min": min(walls) / args.steps,
        "ms_per_step_events": kernel_ms,
        "timed_region_repeats": args.repeats,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "llama_hidden: X bf16 [2048 x 4096], H_4096, b=4, clip=0.9, "
                               "Student-t(3) + 8 outlier channels x50 + 2 massive tokens x500, seed 100",
                   "rows": w.rows, "d": w.d, "n": w.n, "bits": bits, "clip": clip,
                   "ring_buffers": ring, "launch": "hip graph replay of K steps"},
        "tokens_per_s": w.rows / ms_per_step * 1e3,
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "eager_ms_per_step": eager_ms,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(kernel_name), "kernel": kernel_name,
                     "kernel_ms": kernel_ms, "algorithmic_bytes_per_launch": batch_bytes,
                     "traffic_source": "rocprofv3 FETCH_SIZE / WRITE_SIZE of this launch shape, profiles/"
                                       "hbm_traffic_wave_sylvester_llama_hidden_b4.txt (independent of timing)"},
    }
    if not args.no_stream_reference:
        # the same ring and graph with the traffic-only kernel: the practical floor of this launch shape
        def ref_step(i):
            sl = i % ring
            binding.stream_reference(xs[sl], bits, codes=codes[sl], scales=scales[sl])
        with torch.cuda.stream(side):
            ref_step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        ref_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(ref_graph):
            for i in range(args.steps):
                ref_step(i)
        ref_graph.replay()
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record()
        ref_graph.replay()
        r1.record()
        torch.cuda.synchronize()
        ref_ms = r0.elapsed_time(r1) / args.steps
        xl = base.repeat(131072 // base.shape[0], 1)
        cl = torch.empty((xl.shape[0], w.n * bits // 8), dtype=torch.uint8, device="cuda")
        sl_ = torch.empty((xl.shape[0],), dtype=torch.float32, device="cuda")
        ref_long = _min_ms(torch, lambda: binding.stream_reference(xl, bits, codes=cl, scales=sl_))
        out["stream_reference"] = {
            "what": "kernel with the same loads and stores and no arithmetic (rq_stream_reference), same ring and graph",
            "kernel_ms": ref_ms, "GBps": batch_bytes / ref_ms / 1e6,
            "frac_hbm_peak": batch_bytes / ref_ms / 1e6 / HBM_PEAK_GBPS,
            "rotate_quantize_over_reference": kernel_ms / ref_ms,
            "steady_rows": int(xl.shape[0]), "steady_ms": ref_long,
            "steady_frac_hbm_peak": xl.shape[0] * row_bytes / ref_long / 1e6 / HBM_PEAK_GBPS}
        del xl, cl, sl_
    if args.pmc_calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(7)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_steady_state:
        st = time_steady_state(torch, binding, h, base, bits, clip, 131072)
        out["steady_state"] = st
        # the same kernel on a launch long enough to leave launch latency behind (1 GiB of input)
        out["roofline_steady"] = {"bound": "hbm", "achieved": st["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                  "frac": st["frac_hbm_peak"], "kernel": kernel_name, "rows": st["rows"],
                                  "kernel_ms": st["ms_per_launch"],
                                  "algorithmic_bytes_per_launch": st["rows"] * row_bytes}
    if not args.no_configs:
        del xs, codes, scales
        torch.cuda.empty_cache()
        out["configs"] = time_all_configs(torch, binding, wl)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x_bits, w.n, bits, clip)
        out["cpu_baseline"]["parity"] = parity_stats(torch, binding, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
