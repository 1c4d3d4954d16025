#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

One "step" = one xattn_decode call (partition + split-KV decode kernel + merge kernel) over one batch
of synthetic input that is already resident in HBM.  Prints ONE JSON line:

  metric/value/unit   KV-read GB/s of the whole call: sum_b kv_len[b] * n_kv_heads * 128 * 2 (K and V)
                      * 2 B, divided by the time of one step (K steps back to back on one stream)
  token_steps_per_s   batch * q_len / time of one step
  roofline            the split-KV decode kernel alone against the 8 TB/s HBM peak; its duration is
                      measured in a second pass with HIP events around each kernel
  cpu_baseline        the fp64 CPU oracle, as it stands, timed on this machine's host cores
  workloads           the same figures for the other large synthetic workloads
  parity              GPU result against the oracle on the benchmarked inputs (all or sampled rows)

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
# HBM bytes per decode-kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (summaries under profiles/), scaled by the factor a plain copy kernel of known size gives.
# None until measured for the workload.
MEASURED_TRAFFIC_BYTES = {
    # profiles/<kernel>__<workload>.txt: FETCH_SIZE x 2.0000 + WRITE_SIZE x 1.0000 of the decode kernel
    "qwen3_8b_decode": 646547269,
    "long_context": 1628809212,
    "spec_verify": 2459629508,
    "skewed_xtensor": 2154417468,
    "mla_decode": 375470448,       # of which 47.0 MB are the partial results written
    "mla_verify": 454308238,       # of which 92.2 MB written
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def run_workload(w, steps, warmup, check_rows, cpu_baseline, use_graph=False):
    import numpy as np
    import torch

    import paper_2510_14686_amd as xa
    from workloads import bf16_to_f32

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

    t0 = time.time()
    store = xa.KVStore(ks, vs, device=0, xtensor=w.xtensor, seed=w.seed)
    log("[%s] placed K/V in %.1f s (%d chunks)" % (w.name, time.time() - t0, store.n_chunks))
    try:
        qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
        lens_d = torch.from_numpy(lens).cuda()
        out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()

        def step():
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, stream)

        xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        eager_step = step
        if use_graph:
            # one step recorded into a HIP graph; a timed step is one replay
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, w.scale, out, lse, side)
            step = graph.replay
            for _ in range(warmup):
                step()
            torch.cuda.synchronize()
        res["launch"] = "hip graph replay" if use_graph else "eager"
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_wall = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        t_wall = time.perf_counter() - t_wall
        ms_step = e0.elapsed_time(e1) / steps
        res["ms_per_step"] = ms_step
        res["ms_per_step_wall"] = t_wall * 1e3 / steps
        res["kv_read_GBps"] = kv_bytes / (ms_step * 1e-3) / 1e9
        res["pct_of_hbm_peak"] = 100.0 * res["kv_read_GBps"] / HBM_PEAK_GBS
        res["token_steps_per_s"] = B * T / (ms_step * 1e-3)

        # second pass: per-kernel durations from events recorded inside the library, on the same stream
        xa.xattn_configure(xa.XATTN_CFG_TIMING, 1)
        xa.xattn_timing_read()
        n_timed = min(steps, 2000)
        for _ in range(n_timed):
            eager_step()
        torch.cuda.synchronize()
        n, dec_ms, mrg_ms = xa.xattn_timing_read()
        xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
        dec_ms_avg, mrg_ms_avg = dec_ms / max(n, 1), mrg_ms / max(n, 1)
        achieved = kv_bytes / (dec_ms_avg * 1e-3) / 1e9
        res["roofline"] = {"kernel": "split_decode_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                           "algorithmic_bytes_per_launch": kv_bytes, "kernel_ms": dec_ms_avg,
                           "merge_kernel_ms": mrg_ms_avg, "timed_launches": n}

        # parity on the benchmarked inputs
        import oracle
        from gpu_util import errors
        torch.cuda.synchronize()
        out_h = out.cpu().numpy().view(np.uint16)
        lse_h = lse.cpu().numpy()
        sel = list(range(B)) if check_rows is None or check_rows >= B else \
            sorted(set(np.linspace(0, B - 1, check_rows).astype(int).tolist() + [int(np.argmax(lens)), int(np.argmin(lens))]))
        t0 = time.time()
        ref_out, ref_lse = oracle.attn(q[sel], [ks[b] for b in sel], [vs[b] for b in sel], lens[sel], w.scale)
        t_or = time.time() - t0
        max_abs, rel_rows, rel_all, lse_err = errors(out_h[sel], lse_h[sel], ref_out, ref_lse)
        res["parity"] = {"sequences_checked": len(sel), "max_abs": max_abs, "max_row_rel_l2": rel_rows,
                         "rel_l2": rel_all, "lse_max_abs": lse_err,
                         "pass": bool(max_abs <= 1e-2 and rel_rows <= 5e-3 and lse_err <= 1e-3)}
        log("[%s] %.1f us/step  %.0f GB/s (%.1f%% of peak)  kernel %.1f us -> %.0f GB/s  merge %.1f us  parity %s"
            % (w.name, ms_step * 1e3, res["kv_read_GBps"], res["pct_of_hbm_peak"], dec_ms_avg * 1e3, achieved,
               mrg_ms_avg * 1e3, res["parity"]))

        if cpu_baseline:
            # The oracle as it stands on the host cores, over the sequences just checked.
            sel_tokens = int(lens[sel].sum())
            # repeated until about 10 s of CPU work have been timed
            reps = 0
            t0 = time.time()
            while reps < 3 or (time.time() - t0 < 10.0 and reps < 1000):
                oracle.attn(q[sel], [ks[b] for b in sel], [vs[b] for b in sel], lens[sel], w.scale)
                reps += 1
            t_cpu = (time.time() - t0) / reps
            sel_bytes = sel_tokens * Hkv * D * 4
            res["cpu_baseline"] = {"value": sel_bytes / t_cpu / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
                                   "kind": "oracle",
                                   "sample": "%d of %d sequences (%d KV tokens), %d repetitions, %.2f s each"
                                             % (len(sel), B, sel_tokens, reps, t_cpu),
                                   "token_steps_per_s": len(sel) * T / t_cpu}
    finally:
        store.close()
    return res


MFMA_BF16_PEAK_TFLOPS = 2500.0


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


def run_mla_workload(w, steps, warmup, check_rows):
    """Latent-KV (MLA-shaped) decode: same protocol as run_workload; the roofline is the bf16 matrix peak."""
    import numpy as np
    import torch

    import oracle
    import paper_2510_14686_amd as xa
    from gpu_util import errors
    t0 = time.time()
    lens = w.kv_lens()
    q = w.make_q()
    cs = w.make_cache(lens)
    kv_bytes, flops = w.kv_bytes(lens), w.flops(lens)
    log("[%s] generated %.2f GB of latent cache for %d sequences in %.1f s" % (w.name, kv_bytes / 1e9, w.batch, time.time() - t0))
    B, T, H = w.batch, w.q_len, w.n_heads
    res = {"workload": w.name, "batch": B, "q_len": T, "n_heads": H, "d_latent": w.d_latent, "d_rope": w.d_rope,
           "kv_tokens": int(lens.sum()), "kv_bytes": kv_bytes, "flops": flops}
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
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        ms_step = e0.elapsed_time(e1) / steps
        res["ms_per_step"] = ms_step
        res["kv_read_GBps"] = kv_bytes / (ms_step * 1e-3) / 1e9
        res["pct_of_hbm_peak"] = 100.0 * res["kv_read_GBps"] / HBM_PEAK_GBS
        res["tflops"] = flops / (ms_step * 1e-3) / 1e12
        res["token_steps_per_s"] = B * T / (ms_step * 1e-3)
        xa.xattn_configure(xa.XATTN_CFG_TIMING, 1)
        xa.xattn_timing_read()
        for _ in range(min(steps, 1000)):
            step()
        torch.cuda.synchronize()
        n, dec_ms, mrg_ms = xa.xattn_timing_read()
        xa.xattn_configure(xa.XATTN_CFG_TIMING, 0)
        dec_ms_avg, mrg_ms_avg = dec_ms / max(n, 1), mrg_ms / max(n, 1)
        achieved = flops / (dec_ms_avg * 1e-3) / 1e12
        res["roofline"] = {"kernel": "mla_decode_kernel", "bound": "mfma", "achieved": achieved,
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                           "traffic": MEASURED_TRAFFIC_BYTES.get(w.name), "algorithmic_flops_per_launch": flops,
                           "algorithmic_bytes_per_launch": kv_bytes, "kernel_ms": dec_ms_avg,
                           "merge_kernel_ms": mrg_ms_avg, "timed_launches": n,
                           "hbm_GBps_of_kernel": kv_bytes / (dec_ms_avg * 1e-3) / 1e9}
        out_h = out.cpu().numpy().view(np.uint16)
        lse_h = lse.cpu().numpy()
        sel = list(range(B)) if check_rows is None or check_rows >= B else \
            sorted(set(np.linspace(0, B - 1, check_rows).astype(int).tolist() + [int(np.argmax(lens)), int(np.argmin(lens))]))
        t0 = time.time()
        ref_out, ref_lse = oracle.mla(q[sel], [cs[b] for b in sel], lens[sel], w.d_latent, w.scale)
        t_cpu = time.time() - t0
        sel_tokens = int(lens[sel].sum())
        sel_flops = sel_tokens * T * H * 2 * (w.d_qk + w.d_latent)
        res["cpu_baseline"] = {"value": sel_flops / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "%d of %d sequences (%d cached tokens), one pass, %.2f s"
                                                           % (len(sel), B, sel_tokens, t_cpu)}
        max_abs, rel_rows, rel_all, lse_err = errors(out_h[sel], lse_h[sel], ref_out, ref_lse)
        res["parity"] = {"sequences_checked": len(sel), "max_abs": max_abs, "max_row_rel_l2": rel_rows,
                         "rel_l2": rel_all, "lse_max_abs": lse_err,
                         "pass": bool(max_abs <= 1e-2 and rel_rows <= 5e-3 and lse_err <= 1e-3)}
        log("[%s] %.1f us/step  %.0f GB/s (%.1f%% of HBM peak)  %.0f TFLOP/s  kernel %.1f us -> %.0f TFLOP/s (%.1f%% of bf16 MFMA peak)  merge %.1f us  parity %s"
            % (w.name, ms_step * 1e3, res["kv_read_GBps"], res["pct_of_hbm_peak"], res["tflops"], dec_ms_avg * 1e3,
               achieved, 100 * achieved / MFMA_BF16_PEAK_TFLOPS, mrg_ms_avg * 1e3, res["parity"]))
    finally:
        store.close()
    return res


def xtensor_page_ops(n_pages=256, reps=5):
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="qwen3_8b_decode")
    ap.add_argument("--only", action="store_true", help="measure only --workload, not the other large workloads")
    ap.add_argument("--pieces", type=int, default=0, help="override the number of pieces of the partition (0 = automatic)")
    ap.add_argument("--min-piece-tokens", type=int, default=0, help="override the minimum piece size (0 = default)")
    ap.add_argument("--path", type=int, default=0, help="inner loop: 0 automatic, 1 vector, 2 matrix cores")
    ap.add_argument("--beam", action="store_true", help="host-only: time the beam-search selection step (heap with early exit vs sorting everything)")
    ap.add_argument("--mla-layout", type=int, default=0, help="latent-KV kernel: 0 automatic, 1 one 16-row tile per wave, 2 two tiles per wave")
    ap.add_argument("--pv-mode", type=int, default=0, help="matrix path p.V product: 0 default (bf16 MFMA, hi+lo parts), 1 fp32 MFMA, 2 single bf16 MFMA")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB ten times (reads 1 GiB, writes 1 GiB per launch): "
                         "the known-size kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--graph", action="store_true", help="time replays of one HIP graph holding the call instead of eager calls")
    ap.add_argument("--xtensor", action="store_true",
                    help="only time the xTensor page operations (map, unmap, reuse, pre-mapping) and print them")
    ap.add_argument("--check-sequences", type=int, default=None, help="sequences verified against the oracle (default all)")
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
    if args.xtensor:
        print(json.dumps({"xtensor_page_ops": xtensor_page_ops()}), flush=True)
        return
    if args.workload in workloads.MLA_CONFIGS:
        r = run_mla_workload(workloads.MLA_CONFIGS[args.workload], args.steps, args.warmup, args.check_sequences or 8)
        print(json.dumps({"metric": "latent-KV decode attention: TFLOP/s (bf16 MFMA) + KV-read GB/s, 1 MI355X",
                          "value": r["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                          "dtype": "bf16 in/out, fp32 accumulate", "data": "synthetic (seeded N(0,1) bf16, seeded lengths)",
                          "config": {k: r[k] for k in ("workload", "batch", "q_len", "n_heads", "d_latent", "d_rope",
                                                       "kv_tokens", "kv_bytes", "flops")},
                          "kv_read_GBps": r["kv_read_GBps"], "token_steps_per_s": r["token_steps_per_s"],
                          "roofline": r["roofline"], "cpu_baseline": r["cpu_baseline"], "parity": r["parity"]}), flush=True)
        return
    head = workloads.CONFIGS[args.workload]
    main_res = run_workload(head, args.steps, args.warmup, args.check_sequences, cpu_baseline=True, use_graph=args.graph)
    others = {}
    if not args.only:
        for name in workloads.CONFIG_ORDER:
            if name in ("tiny", args.workload):
                continue
            r = run_workload(workloads.CONFIGS[name], args.steps, args.warmup, 24, cpu_baseline=False, use_graph=args.graph)
            others[name] = {k: r[k] for k in ("ms_per_step", "kv_read_GBps", "pct_of_hbm_peak", "token_steps_per_s",
                                              "kv_bytes", "kv_tokens", "batch", "q_len", "kv_placement", "parity")}
            others[name]["roofline"] = r["roofline"]

    line = {
        "metric": "KV-read HBM GB/s (% of 8 TB/s) + attention token-steps/s, 1 MI355X",
        "value": main_res["kv_read_GBps"], "unit": "GB/s",
        "pct_of_hbm_peak": main_res["pct_of_hbm_peak"], "token_steps_per_s": main_res["token_steps_per_s"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 in/out, fp32 accumulate", "data": "synthetic (seeded N(0,1) bf16, seeded lengths)",
        "config": {"workload": main_res["workload"], "batch": main_res["batch"], "q_len": main_res["q_len"],
                   "n_q_heads": main_res["n_q_heads"], "n_kv_heads": main_res["n_kv_heads"],
                   "head_dim": main_res["head_dim"], "kv_tokens": main_res["kv_tokens"],
                   "kv_bytes": main_res["kv_bytes"], "kv_placement": main_res["kv_placement"],
                   "launch": main_res["launch"]},
        "roofline": main_res["roofline"], "cpu_baseline": main_res.get("cpu_baseline"),
        "parity": main_res["parity"], "workloads": others,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
