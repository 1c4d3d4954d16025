#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

One "step" = one xattn_decode call (partition + split-KV decode kernel + merge kernel) over one batch
of synthetic input that is already resident in HBM.  Prints ONE JSON line:

  metric/value/unit   KV-read GB/s of the whole call on the headline workload (BASELINE config 2):
                      sum_b kv_len[b] * n_kv_heads * 128 * 2 (K and V) * 2 B, divided by the mean
                      time of one step (EXACTLY --steps steps back to back on one stream, bracketed
                      by device synchronisation, after --warmup untimed steps)
  timing              median and minimum per step (one event per step, second pass), latency of one
                      call issued on an idle device and waited for
  roofline            the split-KV decode kernel alone against the 8 TB/s HBM peak: algorithmic
                      bytes / its mean duration, from HIP events the library records around the
                      kernel on the stream it is launched on (third pass); `traffic` = HBM bytes per
                      launch from profiles/traffic.json, which profile_summary.py writes from
                      rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script
  cpu_baseline        the fp64 CPU oracle, as it stands, timed on this machine's host cores
  parity              GPU result against the oracle on the benchmarked inputs, EVERY sequence
  workloads           the same figures (timing, roofline, parity, cpu_baseline) for the other three
                      large GQA workloads and the two latent-KV workloads (each with at least 200
                      timed steps after 50 warm-up steps, stated per entry), plus `tiny` as latency
  xtensor_vs_plain    configs 2 and 5 with the same bytes in xTensor ranges and in plain allocations
  graph_vs_eager      the headline step replayed from a HIP graph against eager launches
  xtensor_page_ops    host cost of the page operations of the xTensor pool
  decode_loop         a decode loop whose sequences keep crossing page boundaries: mapping in the
                      step, pre-mapping in the background, and everything mapped beforehand

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only]
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
KERNEL_SOURCES = ["xattn_kernels.hip", "xattn_mla.hip", "xattn_device.h", "xattn_plan.h", "xattn_kernels.h"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash():
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2510_14686_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch of the workload's decode kernel, from the tracked file that
    profile_summary.py writes out of rocprofv3 counter runs (null if none is recorded)."""
    try:
        with open(TRAFFIC_JSON) as fh:
            t = json.load(fh)
    except (OSError, ValueError):
        return None, None
    e = t.get("workloads", {}).get(workload)
    if not e:
        return None, None
    info = {"file": "profiles/traffic.json", "profile": e.get("profile"), "bytes_read": e["bytes_read"],
            "bytes_written": e["bytes_written"],
            "kernel_sources_changed_since": t.get("kernel_source_hash") != kernel_source_hash()}
    return e["bytes_read"] + e["bytes_written"], info


def time_steps(step, steps, warmup):
    """The timing protocol: `warmup` untimed steps; exactly `steps` steps back to back between two
    events, bracketed by synchronisation (mean); the same again with an event after every step (median,
    min); single calls on an idle device, each waited for (latency)."""
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t_wall
    mean_ms = e0.elapsed_time(e1) / steps
    n = min(steps, 2000)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record(stream)
    for i in range(n):
        step()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]
    lat = []
    for _ in range(min(max(steps, 5), 30)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - t0) * 1e3)
    return {"ms_per_step": mean_ms, "ms_per_step_wall": t_wall * 1e3 / steps,
            "ms_per_step_median": statistics.median(per), "ms_per_step_min": min(per),
            "single_call_latency_ms_median": statistics.median(lat), "single_call_latency_ms_min": min(lat)}


def kernel_timing(step, n):
    """Mean durations of the decode kernel and the merge kernel: HIP events recorded by the library
    on the launch stream around each kernel."""
    import torch

    import paper_2510_14686_amd as xa
    xa.xattn_configure(xa.XATTN_CFG_TIMING, 1)
    xa.xattn_timing_read()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    got, dec_ms, mrg_ms = xa.xattn_timing_read()
    xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
    return dec_ms / max(got, 1), mrg_ms / max(got, 1), got


def parity_and_cpu_baseline(oracle_call, compare, sel_desc, work_units, unit, min_seconds):
    """Runs the oracle over the benchmarked inputs (all sequences), compares, and reports the
    oracle's own speed as the CPU baseline.  The first pass is the verification; it is repeated until
    min_seconds of CPU work have been timed."""
    import oracle
    t0 = time.time()
    ref = oracle_call()
    t_first = time.time() - t0
    parity = compare(ref)
    reps, t_total = 1, t_first
    while t_total < min_seconds and reps < 200:
        t0 = time.time()
        oracle_call()
        t_total += time.time() - t0
        reps += 1
    t_cpu = t_total / reps
    base = {"value": work_units / t_cpu, "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s, %d pass(es) of %.2f s each" % (sel_desc, reps, t_cpu), "seconds_per_pass": t_cpu}
    return parity, base


def parity_dict(out_h, lse_h, ref_out, ref_lse, n_seq):
    from gpu_util import errors
    max_abs, rel_rows, rel_all, lse_err = errors(out_h, lse_h, ref_out, ref_lse)
    return {"sequences_checked": n_seq, "max_abs": max_abs, "max_row_rel_l2": rel_rows, "rel_l2": rel_all,
            "lse_max_abs": lse_err, "pass": bool(max_abs <= 1e-2 and rel_rows <= 5e-3 and lse_err <= 1e-3)}


def run_workload(w, steps, warmup, cpu_seconds, also_plain=False, also_graph=False):
    """One GQA workload: timing, kernel roofline, parity on every sequence, CPU baseline; optionally the
    same bytes in plain allocations (A/B of the xTensor placement) and a HIP-graph replay."""
    import numpy as np
    import torch

    import oracle
    import paper_2510_14686_amd as xa
    t0 = time.time()
    lens = w.kv_lens()
    q = w.make_q()
    ks, vs = w.make_kv(lens)
    kv_bytes = w.kv_bytes(lens)
    log("[%s] generated %.2f GB of K/V for %d sequences in %.1f s" % (w.name, kv_bytes / 1e9, w.batch, time.time() - t0))
    B, T, Hq, Hkv, D = w.batch, w.q_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    res = {"workload": w.name, "batch": B, "q_len": T, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D,
           "kv_tokens": int(lens.sum()), "kv_bytes": kv_bytes, "kv_placement":
           "xtensor: per-sequence virtual ranges, 2 MiB chunks in seeded random order" if w.xtensor else "plain allocations"}
    qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
    lens_d = torch.from_numpy(lens).cuda()
    out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
    lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def timed_on(store):
        def step():
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, stream)
        return step, time_steps(step, steps, warmup)

    def rates(t):
        gbs = kv_bytes / (t["ms_per_step"] * 1e-3) / 1e9
        return dict(t, kv_read_GBps=gbs, pct_of_hbm_peak=100.0 * gbs / HBM_PEAK_GBS,
                    token_steps_per_s=B * T / (t["ms_per_step"] * 1e-3))

    xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
    t0 = time.time()
    store = xa.KVStore(ks, vs, device=0, xtensor=w.xtensor, seed=w.seed)
    log("[%s] placed K/V in %.1f s (%d chunks)" % (w.name, time.time() - t0, store.n_chunks))
    try:
        step, t = timed_on(store)
        res.update(rates(t))
        res["launch"] = "eager"
        dec_ms, mrg_ms, n = kernel_timing(step, min(steps, 2000))
        achieved = kv_bytes / (dec_ms * 1e-3) / 1e9
        traffic, traffic_info = measured_traffic(w.name)
        res["roofline"] = {"kernel": "split_decode_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                           "traffic_source": traffic_info,
                           "timing": "HIP events recorded by the library on the launch stream around the kernel, "
                                     "mean over timed_launches (they bracket the launch: a few us above rocprofv3's kernel time)",
                           "algorithmic_bytes_per_launch": kv_bytes, "kernel_ms": dec_ms,
                           "merge_kernel_ms": mrg_ms, "timed_launches": n}
        if also_graph:
            # one step recorded into a HIP graph (after an eager call on the capture stream, which sizes
            # that stream's workspace); a timed step is one replay
            side = torch.cuda.Stream()
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, side)
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, side)
            tg = time_steps(graph.replay, steps, warmup)
            te = time_steps(step, steps, warmup)
            res["graph_vs_eager"] = {"graph_replay": {k: tg[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min", "single_call_latency_ms_median")},
                                     "eager": {k: te[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min", "single_call_latency_ms_median")}}
            del graph
        # parity on the benchmarked inputs, every sequence, and the oracle's speed
        out.zero_()
        step()
        torch.cuda.synchronize()
        out_h = out.cpu().numpy().view(np.uint16)
        lse_h = lse.cpu().numpy()
        res["parity"], res["cpu_baseline"] = parity_and_cpu_baseline(
            lambda: oracle.attn(q, ks, vs, lens, w.scale),
            lambda ref: parity_dict(out_h, lse_h, ref[0], ref[1], B),
            "all %d sequences (%d KV tokens)" % (B, int(lens.sum())), kv_bytes / 1e9, "GB/s", cpu_seconds)
        res["cpu_baseline"]["token_steps_per_s"] = B * T / res["cpu_baseline"]["seconds_per_pass"]
    finally:
        store.close()
    if also_plain:
        # A/B of the placement: the same kernel on the same bytes in ordinary allocations
        other = xa.KVStore(ks, vs, device=0, xtensor=not w.xtensor, seed=w.seed)
        try:
            step2, t2 = timed_on(other)
            dec2, mrg2, _ = kernel_timing(step2, min(steps, 2000))
            a = {k: res[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min", "kv_read_GBps")}
            a["kernel_ms"] = dec_ms
            b = {k: rates(t2)[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min", "kv_read_GBps")}
            b["kernel_ms"] = dec2
            res["xtensor_vs_plain"] = {"xtensor" if w.xtensor else "plain": a, "plain" if w.xtensor else "xtensor": b}
        finally:
            other.close()
    log("[%s] %.1f us/step (median %.1f, min %.1f)  %.0f GB/s (%.1f%% of peak)  kernel %.1f us -> %.0f GB/s  merge %.1f us  parity %s  oracle %.2f s"
        % (w.name, res["ms_per_step"] * 1e3, res["ms_per_step_median"] * 1e3, res["ms_per_step_min"] * 1e3,
           res["kv_read_GBps"], res["pct_of_hbm_peak"], dec_ms * 1e3, achieved, mrg_ms * 1e3, res["parity"],
           res["cpu_baseline"]["seconds_per_pass"]))
    return res


def run_mla_workload(w, steps, warmup, cpu_seconds):
    """Latent-KV (MLA-shaped) decode: same protocol; the roofline is the bf16 matrix peak."""
    import numpy as np
    import torch

    import oracle
    import paper_2510_14686_amd as xa
    t0 = time.time()
    lens = w.kv_lens()
    q = w.make_q()
    cs = w.make_cache(lens)
    kv_bytes, flops = w.kv_bytes(lens), w.flops(lens)
    log("[%s] generated %.2f GB of latent cache for %d sequences in %.1f s" % (w.name, kv_bytes / 1e9, w.batch, time.time() - t0))
    B, T, H = w.batch, w.q_len, w.n_heads
    res = {"workload": w.name, "batch": B, "q_len": T, "n_heads": H, "d_latent": w.d_latent, "d_rope": w.d_rope,
           "kv_tokens": int(lens.sum()), "kv_bytes": kv_bytes, "flops": flops,
           "kv_placement": "xtensor: per-sequence virtual ranges, 2 MiB chunks in seeded random order"}
    store = xa.KVStore(cs, cs, device=0, xtensor=w.xtensor, seed=w.seed)
    try:
        qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
        lens_d = torch.from_numpy(lens).cuda()
        out = torch.zeros((B, T, H, w.d_latent), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, H), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()

        def step():
            xa.xattn_mla_decode(qd, store.k_ptrs, lens_d, B, T, H, w.d_latent, w.d_rope, w.scale, out, lse, stream)

        xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
        t = time_steps(step, steps, warmup)
        res.update(t)
        ms_step = t["ms_per_step"]
        res["kv_read_GBps"] = kv_bytes / (ms_step * 1e-3) / 1e9
        res["pct_of_hbm_peak"] = 100.0 * res["kv_read_GBps"] / HBM_PEAK_GBS
        res["tflops"] = flops / (ms_step * 1e-3) / 1e12
        res["token_steps_per_s"] = B * T / (ms_step * 1e-3)
        dec_ms, mrg_ms, n = kernel_timing(step, min(steps, 1000))
        achieved = flops / (dec_ms * 1e-3) / 1e12
        traffic, traffic_info = measured_traffic(w.name)
        res["roofline"] = {"kernel": "mla_decode_kernel", "bound": "mfma", "achieved": achieved,
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                           "traffic": traffic, "traffic_source": traffic_info,
                           "timing": "HIP events recorded by the library on the launch stream around the kernel",
                           "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": kv_bytes,
                           "kernel_ms": dec_ms, "merge_kernel_ms": mrg_ms, "timed_launches": n,
                           "hbm_GBps_of_kernel": kv_bytes / (dec_ms * 1e-3) / 1e9}
        out.zero_()
        step()
        torch.cuda.synchronize()
        out_h = out.cpu().numpy().view(np.uint16)
        lse_h = lse.cpu().numpy()
        res["parity"], res["cpu_baseline"] = parity_and_cpu_baseline(
            lambda: oracle.mla(q, cs, lens, w.d_latent, w.scale),
            lambda ref: parity_dict(out_h, lse_h, ref[0], ref[1], B),
            "all %d sequences (%d cached tokens)" % (B, int(lens.sum())), flops / 1e12, "TFLOP/s", cpu_seconds)
        log("[%s] %.1f us/step (median %.1f, min %.1f)  %.0f GB/s (%.1f%% of HBM peak)  %.0f TFLOP/s  kernel %.1f us -> %.0f TFLOP/s (%.1f%% of bf16 MFMA peak)  merge %.1f us  parity %s  oracle %.1f s"
            % (w.name, ms_step * 1e3, t["ms_per_step_median"] * 1e3, t["ms_per_step_min"] * 1e3, res["kv_read_GBps"],
               res["pct_of_hbm_peak"], res["tflops"], dec_ms * 1e3, achieved, 100 * achieved / MFMA_BF16_PEAK_TFLOPS,
               mrg_ms * 1e3, res["parity"], res["cpu_baseline"]["seconds_per_pass"]))
    finally:
        store.close()
    return res


def tiny_latency(steps):
    """Config 1 (0.45 MB of K/V, far below the last-level cache): reported as latency only."""
    import numpy as np
    import torch

    import oracle
    import paper_2510_14686_amd as xa
    import workloads
    w = workloads.CONFIGS["tiny"]
    lens, q = w.kv_lens(), w.make_q()
    ks, vs = w.make_kv(lens)
    B, T, Hq, Hkv, D = w.batch, w.q_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    with xa.KVStore(ks, vs, device=0, xtensor=False) as store:
        qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
        lens_d = torch.from_numpy(lens).cuda()
        out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()

        def step():
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, stream)

        t = time_steps(step, steps, 10)
        torch.cuda.synchronize()
        ref_out, ref_lse = oracle.attn(q, ks, vs, lens, w.scale)
        par = parity_dict(out.cpu().numpy().view(np.uint16), lse.cpu().numpy(), ref_out, ref_lse, B)
    return {"workload": "tiny", "note": "latency only: the inputs fit the caches", "us_per_call_back_to_back": t["ms_per_step"] * 1e3,
            "us_per_call_median": t["ms_per_step_median"] * 1e3, "us_per_call_min": t["ms_per_step_min"] * 1e3,
            "us_single_call_with_sync_median": t["single_call_latency_ms_median"] * 1e3,
            "us_single_call_with_sync_min": t["single_call_latency_ms_min"] * 1e3, "parity": par}


def beam_search_bench():
    """Host beam-search selection (section 4.5.1): the library's heap with early exit, the same entry
    point sorting all candidates, and the numpy oracle, on the synthetic request batches; one thread."""
    import numpy as np

    import oracle
    import paper_2510_14686_amd as xa
    import workloads
    res = {}
    for name in sorted(workloads.BEAM_CONFIGS):
        w = workloads.BEAM_CONFIGS[name]
        beam, cand, tok = w.make()
        want = oracle.beam_select(beam, cand, tok)
        out = xa.xbeam_select(beam, cand, tok)
        ok = all(np.array_equal(a, b) for a, b in zip(out[:3], want))

        def timed(fn, min_s=0.3):
            fn()
            n, t0 = 0, time.perf_counter()
            while time.perf_counter() - t0 < min_s:
                fn()
                n += 1
            return (time.perf_counter() - t0) / n

        t_heap = timed(lambda: xa.xbeam_select(beam, cand, tok, out_lp=out[0], out_parent=out[1], out_tok=out[2], visited=out[3]))
        t_sort = timed(lambda: xa.xbeam_select(beam, cand, tok, flags=xa.XBEAM_FULL_SORT, out_lp=out[0], out_parent=out[1], out_tok=out[2], visited=out[3]))
        out = xa.xbeam_select(beam, cand, tok)
        t_orc = timed(lambda: oracle.beam_select(beam, cand, tok))
        R, W, K = cand.shape
        res[name] = {"n_req": R, "beam_width": W, "top_k": K, "matches_oracle": bool(ok),
                     "us_per_request_heap_early_exit": 1e6 * t_heap / R, "us_per_request_full_sort": 1e6 * t_sort / R,
                     "us_per_request_numpy_oracle": 1e6 * t_orc / R, "speedup_vs_full_sort": t_sort / t_heap,
                     "candidates_examined_fraction": float(out[3].sum()) / (R * W * K)}
        log("[%s] W=%d K=%d: heap+early exit %.1f us/request, full sort %.1f us/request (x%.1f), numpy oracle %.1f us/request, examined %.1f%% of the candidates, matches oracle: %s"
            % (name, W, K, 1e6 * t_heap / R, 1e6 * t_sort / R, t_sort / t_heap, 1e6 * t_orc / R,
               100 * res[name]["candidates_examined_fraction"], ok))
    return res


def xtensor_page_ops(n_pages=256, reps=3):
    """Host-side cost of the page operations of the xTensor pool, microseconds per 2 MiB page
    (the paper's "Low Overhead Allocation": Map/Unmap are expensive, reuse and pre-mapping hide them)."""
    import paper_2510_14686_amd as xa
    page = xa.XTENSOR_CHUNK_BYTES
    t = {"create_pool": [], "map_on_demand": [], "unmap": [], "reuse_open": [], "close_reusable": [],
         "standalone_map": [], "standalone_unmap": []}
    for _ in range(reps):
        t0 = time.perf_counter()
        pool = xa.xtensor_pool_create(0, n_pages, 1)
        t["create_pool"].append((time.perf_counter() - t0) / n_pages)
        base, rng, _ = xa.xtensor_open(pool, 1, n_pages * page, 0)
        t0 = time.perf_counter()
        xa.xtensor_grow(rng, n_pages * page)
        t["map_on_demand"].append((time.perf_counter() - t0) / n_pages)
        t0 = time.perf_counter()
        xa.xtensor_close(rng, True)
        t["close_reusable"].append((time.perf_counter() - t0) / n_pages)
        t0 = time.perf_counter()
        base, rng, reused = xa.xtensor_open(pool, 2, n_pages * page, n_pages * page)
        t["reuse_open"].append((time.perf_counter() - t0) / n_pages)
        assert reused
        t0 = time.perf_counter()
        xa.xtensor_close(rng, False)
        t["unmap"].append((time.perf_counter() - t0) / n_pages)
        xa.xtensor_pool_destroy(pool)
        t0 = time.perf_counter()
        base, h = xa.xtensor_map(n_pages * page, n_pages * page, 7, 0)
        t["standalone_map"].append((time.perf_counter() - t0) / n_pages)
        t0 = time.perf_counter()
        xa.xtensor_unmap(h)
        t["standalone_unmap"].append((time.perf_counter() - t0) / n_pages)
    return {k + "_us_per_page": round(1e6 * min(v), 3) for k, v in t.items()} | {"pages": n_pages, "page_bytes": page}


def decode_loop_bench(n_steps=64):
    """Section 4.3, "Low Overhead Allocation": does pre-mapping hide the map?  A decode loop of 64
    Qwen3-8B-shaped sequences (append one token with write_kvcache, attend, wait for the result as a
    sampler would) in which every step one sequence crosses a page boundary of its K and of its V
    range (the lengths are staggered so), run three ways on the same pool:
      map_in_step     the step itself calls xtensor_grow for the pages it is about to write
      premap_async    the pages of step i + 1 are requested from the pool's background thread right
                      after step i has been enqueued, i.e. while the GPU runs step i
      mapped_before   every page of the run is mapped before the loop (no map in any step)
    Reported: mean wall time per step; the difference to mapped_before is the map's exposed cost."""
    import numpy as np
    import torch

    import paper_2510_14686_amd as xa
    B, T, Hq, Hkv, D = 64, 1, 32, 8, 128
    row = Hkv * D * 2
    page = xa.XTENSOR_CHUNK_BYTES
    tok_per_page = page // row                                   # 1024
    scale = float(np.float32(1.0 / np.sqrt(D)))
    # Sequence b starts with 2 * tok_per_page - b tokens (two pages mapped); the append of step s writes
    # its row start[b] + s, which is the first row of its third page exactly in step s = b.
    start = np.array([2 * tok_per_page - b for b in range(B)], np.int64)
    max_len = int(start.max()) + n_steps + 1
    reserve = -(-max_len * row // page) * page + page
    stream = torch.cuda.current_stream()
    qd = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
    kn = torch.zeros((B, T, Hkv, D), dtype=torch.int16, device="cuda")
    out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
    res = {}
    for mode in ("mapped_before", "map_in_step", "premap_async", "mapped_before_again"):
        pool = xa.xtensor_pool_create(0, 2 * B * (reserve // page), 5)
        ranges = []
        try:
            for b in range(B):
                for _ in range(2):
                    mapped = reserve if mode.startswith("mapped_before") else int(start[b]) * row
                    base, rng, _ = xa.xtensor_open(pool, b, reserve, mapped)
                    ranges.append((base, rng))
            k_ptrs = torch.tensor([ranges[2 * b][0] for b in range(B)], dtype=torch.int64).cuda()
            v_ptrs = torch.tensor([ranges[2 * b + 1][0] for b in range(B)], dtype=torch.int64).cuda()
            lens_all = torch.from_numpy(np.stack([(start + s + 1) for s in range(n_steps)]).astype(np.int32)).cuda()

            def pages_for_step(s):
                """(range handle, bytes that must be backed) for the appends of step s."""
                need = []
                for b in range(B):
                    new_len = int(start[b]) + s + 1
                    if (new_len - 1) % tok_per_page == 0:           # the appended row is the first of a page
                        for r in (ranges[2 * b][1], ranges[2 * b + 1][1]):
                            need.append((r, new_len * row))
                return need

            maps = 0
            if mode == "premap_async":                          # the pages of step 0, requested before the loop
                for r, nbytes in pages_for_step(0):
                    xa.xtensor_premap_async(r, nbytes)
                    maps += 1
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(n_steps):
                lens_d = lens_all[s]
                if mode == "map_in_step":
                    for r, nbytes in pages_for_step(s):
                        maps += xa.xtensor_grow(r, nbytes)
                elif mode == "premap_async":
                    for r, _ in pages_for_step(s):
                        xa.xtensor_premap_wait(r)               # requested during the previous step
                xa.xattn_write_kvcache(kn, kn, k_ptrs, v_ptrs, lens_d, B, T, Hkv, D, stream)
                xa.xattn_decode(qd, k_ptrs, v_ptrs, lens_d, B, T, Hq, Hkv, D, scale, out, None, stream)
                if mode == "premap_async" and s + 1 < n_steps:
                    for r, nbytes in pages_for_step(s + 1):
                        xa.xtensor_premap_async(r, nbytes)
                        maps += 1
                torch.cuda.synchronize()                        # the sampled token is needed before the next step
            dt = (time.perf_counter() - t0) / n_steps
            res[mode] = {"us_per_step": dt * 1e6, "pages_mapped_in_loop": maps}
        finally:
            torch.cuda.synchronize()
            for _, rng in ranges:
                xa.xtensor_close(rng, False)
            xa.xtensor_pool_destroy(pool)
    res["config"] = {"batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "steps": n_steps, "tokens_per_page": int(tok_per_page),
                     "start_lengths": "2048 - b (sequence b crosses a page boundary of K and of V in step b)"}
    base = min(res["mapped_before"]["us_per_step"], res["mapped_before_again"]["us_per_step"])
    res["exposed_map_cost_us_per_step"] = {"map_in_step": res["map_in_step"]["us_per_step"] - base,
                                           "premap_async": res["premap_async"]["us_per_step"] - base}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="qwen3_8b_decode")
    ap.add_argument("--only", action="store_true", help="measure only --workload: no other workloads, A/B rows or host-side measurements")
    ap.add_argument("--cpu-seconds", type=float, default=None,
                    help="CPU seconds the oracle is timed for per workload (default: 10 for the headline, one pass for the others; 0 = one pass)")
    ap.add_argument("--pieces", type=int, default=0, help="override the number of pieces of the partition (0 = automatic)")
    ap.add_argument("--min-piece-tokens", type=int, default=0, help="override the minimum piece size (0 = default)")
    ap.add_argument("--path", type=int, default=0, help="inner loop: 0 automatic, 1 vector, 2 matrix cores")
    ap.add_argument("--beam", action="store_true", help="host-only: time the beam-search selection step (heap with early exit vs sorting everything)")
    ap.add_argument("--mla-layout", type=int, default=0, help="latent-KV kernel: 0 automatic, 1 one 16-row tile per wave, 2 two tiles per wave")
    ap.add_argument("--pv-mode", type=int, default=0, help="precision of the softmax weights in the value product, see XATTN_CFG_PV_MODE")
    ap.add_argument("--xcd-skew", type=int, default=0, help="XATTN_CFG_XCD_SKEW: 0 default, n = (n - 1) per mille moved from the odd XCDs' parts to the even ones'")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB ten times (reads 1 GiB, writes 1 GiB per launch): "
                         "the known-size kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--xtensor", action="store_true", help="only the xTensor page operations and the decode loop with page crossings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.beam:
        print(json.dumps({"beam_search": beam_search_bench()}), flush=True)
        return

    import torch

    import workloads
    from paper_2510_14686_amd import build as xbuild
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(xbuild.LIB_PATH):
        xbuild.build()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"launches": 10, "bytes_read_per_launch": 1 << 30,
                                             "bytes_written_per_launch": 1 << 30}}))
        return

    import paper_2510_14686_amd as xa
    xa.xattn_configure(xa.XATTN_CFG_PIECES, args.pieces)
    xa.xattn_configure(xa.XATTN_CFG_MIN_PIECE_TOKENS, args.min_piece_tokens)
    xa.xattn_configure(xa.XATTN_CFG_PATH, args.path)
    xa.xattn_configure(xa.XATTN_CFG_PV_MODE, args.pv_mode)
    xa.xattn_configure(xa.XATTN_CFG_MLA_LAYOUT, args.mla_layout)
    xa.xattn_configure(xa.XATTN_CFG_XCD_SKEW, args.xcd_skew)
    if args.xtensor:
        print(json.dumps({"xtensor_page_ops": xtensor_page_ops(), "decode_loop": decode_loop_bench()}), flush=True)
        return
    head_cpu = 10.0 if args.cpu_seconds is None else args.cpu_seconds
    other_cpu = 0.0 if args.cpu_seconds is None else args.cpu_seconds
    common = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "bf16 in/out, fp32 accumulate",
              "data": "synthetic (seeded N(0,1) bf16, seeded lengths)"}
    if args.workload in workloads.MLA_CONFIGS:
        r = run_mla_workload(workloads.MLA_CONFIGS[args.workload], args.steps, args.warmup, head_cpu)
        line = {"metric": "latent-KV decode attention: TFLOP/s (bf16 MFMA) + KV-read GB/s, 1 MI355X",
                "value": r["tflops"], "unit": "TFLOP/s", "ms_per_step": r["ms_per_step"],
                "config": {k: r[k] for k in ("workload", "batch", "q_len", "n_heads", "d_latent", "d_rope", "kv_tokens",
                                             "kv_bytes", "flops", "kv_placement")},
                "timing": {k: r[k] for k in ("ms_per_step_median", "ms_per_step_min", "single_call_latency_ms_median")},
                "kv_read_GBps": r["kv_read_GBps"], "token_steps_per_s": r["token_steps_per_s"],
                "roofline": r["roofline"], "cpu_baseline": r["cpu_baseline"], "parity": r["parity"]}
        line.update(common)
        print(json.dumps(line), flush=True)
        return

    full = not args.only
    head = workloads.CONFIGS[args.workload]
    main_res = run_workload(head, args.steps, args.warmup, head_cpu, also_plain=full, also_graph=full)
    others, ab, extra = {}, {}, {}
    if "xtensor_vs_plain" in main_res:
        ab[main_res["workload"]] = main_res["xtensor_vs_plain"]
    if full:
        # The other workloads are measured with at least 200 timed steps after at least 50 warm-up steps
        # (stated in each entry): 20 steps on cold clocks say little about a 0.1-0.4 ms kernel, and the
        # matrix-bound latent-KV kernel in particular follows the clock the box sustains.
        o_steps, o_warmup = max(args.steps, 200), max(args.warmup, 50)
        keep = ("steps", "warmup", "ms_per_step", "ms_per_step_median", "ms_per_step_min", "single_call_latency_ms_median", "kv_read_GBps",
                "pct_of_hbm_peak", "token_steps_per_s", "kv_bytes", "kv_tokens", "batch", "q_len", "kv_placement",
                "roofline", "parity", "cpu_baseline")
        for name in workloads.CONFIG_ORDER:
            if name in ("tiny", args.workload):
                continue
            r = run_workload(workloads.CONFIGS[name], o_steps, o_warmup, other_cpu, also_plain=(name == "skewed_xtensor"))
            r["steps"], r["warmup"] = o_steps, o_warmup
            others[name] = {k: r[k] for k in keep}
            if "xtensor_vs_plain" in r:
                ab[name] = r["xtensor_vs_plain"]
        for name in sorted(workloads.MLA_CONFIGS):
            r = run_mla_workload(workloads.MLA_CONFIGS[name], o_steps, o_warmup, other_cpu)
            r["steps"], r["warmup"] = o_steps, o_warmup
            others[name] = {k: r[k] for k in keep + ("tflops", "flops", "n_heads")}
        others["tiny"] = tiny_latency(max(args.steps, 50))
        extra["xtensor_page_ops"] = xtensor_page_ops()
        extra["decode_loop"] = decode_loop_bench()

    line = {
        "metric": "KV-read HBM GB/s (% of 8 TB/s) + attention token-steps/s, 1 MI355X",
        "value": main_res["kv_read_GBps"], "unit": "GB/s",
        "pct_of_hbm_peak": main_res["pct_of_hbm_peak"], "token_steps_per_s": main_res["token_steps_per_s"],
        "ms_per_step": main_res["ms_per_step"],
        "timing": {k: main_res[k] for k in ("ms_per_step_median", "ms_per_step_min", "ms_per_step_wall",
                                            "single_call_latency_ms_median", "single_call_latency_ms_min")},
        "config": {"workload": main_res["workload"], "batch": main_res["batch"], "q_len": main_res["q_len"],
                   "n_q_heads": main_res["n_q_heads"], "n_kv_heads": main_res["n_kv_heads"],
                   "head_dim": main_res["head_dim"], "kv_tokens": main_res["kv_tokens"],
                   "kv_bytes": main_res["kv_bytes"], "kv_placement": main_res["kv_placement"],
                   "launch": main_res["launch"]},
        "roofline": main_res["roofline"], "cpu_baseline": main_res.get("cpu_baseline"),
        "parity": main_res["parity"], "workloads": others, "xtensor_vs_plain": ab,
        "graph_vs_eager": main_res.get("graph_vs_eager"),
    }
    line.update(common)
    line.update(extra)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
