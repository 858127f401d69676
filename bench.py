#!/usr/bin/env python3
"""Throughput benchmark of the KV compress + decompress hot path on one MI355X.

A step = kvp_quantize(K), kvp_quantize(V), kvp_dequantize_paged(K), kvp_dequantize_paged(V) on the
Llama-3-8B-shaped cache (32 layers x 8 KV heads x 128 x 32768 tokens, bf16, int4 group 64, 16-token
pages, scattered block table), inputs resident in HBM.  value = input KV bytes (K+V, bf16) per
second over the timed steps.  The same JSON line carries the roofline of the dominant kernel
(measured with HIP events on the launch stream inside the timed region), the CPU oracle timed on a
bounded sample, and per-operation figures for the other entry points on their own workloads.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
VALU_FP32_PEAK_TFLOPS = 78.6    # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz, no packed fp32
VALU_FP32_PUBLISHED_TFLOPS = 157.3   # published fp32 vector peak (packed fp32)
VALU_DOT2_PEAK_TFLOPS = 157.3        # v_dot2_f32_f16: two multiply-adds per lane and cycle


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=None, help="override the layer count (debugging only)")
    ap.add_argument("--no-ops", action="store_true", help="skip the per-operation side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only", default=None,
                    help="profiling aid: run only one operation in a loop "
                         "(quantize|dequantize|dequantize_identity|copy|score|select|select_many|select_long|eval)")
    return ap.parse_args()


def ensure_built():
    from paper_2512_14946_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()


def event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def profile_figures(name: str):
    """Figures recorded in a committed rocprofv3 summary: HBM bytes per launch (two --pmc runs, scaled by the copy
    kernel's reading) and the kernel's average launch time under --kernel-trace."""
    path = os.path.join(ROOT, "profiles", name)
    out = {}
    if os.path.exists(path):
        text = open(path).read()
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
        if m:
            out["traffic"] = float(m.group(1))
        m = re.search(r"avg_launch_us:\s*([0-9.eE+]+)", text)
        if m:
            out["launch_ms"] = float(m.group(1)) * 1e-3
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every box here has one); --gpus N with N > 1 is not "
              "supported. The path shards by context / layer / KV head with no exchange between GPUs.",
              file=sys.stderr)
        sys.exit(2)
    ensure_built()
    import torch
    import paper_2512_14946_amd as kvp
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kvp_* operations have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    cfg = dict(workloads.CONFIGS["llama3_8b_int4_paged"])
    if args.layers:
        cfg["L"] = args.layers
    L, T, H, D, bits, group, bs = cfg["L"], cfg["T"], cfg["H"], cfg["D"], cfg["bits"], cfg["group"], cfg["bs"]
    K, V = workloads.make_kv(L, T, H, D, seed=0, outlier_scale=cfg["outlier_scale"], device=dev)
    bt, nb = workloads.make_block_table(T, bs, seed=0, device=dev)
    qK = kvp.alloc_qplane(L, T, H, D, bits, group, dev, page=bs)
    qV = kvp.alloc_qplane(L, T, H, D, bits, group, dev, page=bs)
    pK = kvp.alloc_paged(L, T, H, D, bt, nb, bs)
    pV = kvp.alloc_paged(L, T, H, D, bt, nb, bs)
    plane_bytes = K.numel() * 2
    input_bytes = 2 * plane_bytes
    comp_bytes = qK.nbytes()
    alg_bytes_per_launch = plane_bytes + comp_bytes   # one quantize (or dequantize) launch over one plane

    def ev():
        return torch.cuda.Event(enable_timing=True)

    if args.only:
        return profile_only(args, kvp, workloads, torch, dev, K, V, qK, pK, bt, nb)

    def step(marks=None):
        if marks is not None:
            e = [ev() for _ in range(5)]
            e[0].record(stream)
        kvp.kvp_quantize(K, qK)
        if marks is not None:
            e[1].record(stream)
        kvp.kvp_quantize(V, qV)
        if marks is not None:
            e[2].record(stream)
        kvp.kvp_dequantize_paged(qK, pK)
        if marks is not None:
            e[3].record(stream)
        kvp.kvp_dequantize_paged(qV, pV)
        if marks is not None:
            e[4].record(stream)
            marks.append(e)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    value = input_bytes / (wall / args.steps) / 1e9

    q_ms = [m for e in marks for m in event_ms([(e[0], e[1]), (e[1], e[2])])]
    d_ms = [m for e in marks for m in event_ms([(e[2], e[3]), (e[3], e[4])])]
    q_avg, d_avg = sum(q_ms) / len(q_ms), sum(d_ms) / len(d_ms)

    def kernel_entry(name, avg_ms, profile):
        """Roofline figures of one kernel of the step: algorithmic bytes over the launch time measured with events
        inside the timed steps; HBM traffic and the profiler's own launch time come from the committed rocprofv3
        summary of the same command (they are not re-measured by this run, and the entry says so)."""
        got = alg_bytes_per_launch / (avg_ms * 1e-3) / 1e9
        prof = profile_figures(profile)
        e = {"kernel": name, "avg_launch_ms": round(avg_ms, 4), "achieved": round(got, 1),
             "frac": round(got / HBM_PEAK_GBS, 4), "share_of_step": round(2 * avg_ms / ms_per_step, 3),
             "traffic": prof.get("traffic"), "traffic_source": f"rocprofv3 --pmc, offline: profiles/{profile}",
             "profile_avg_launch_ms": prof.get("launch_ms")}
        if prof.get("launch_ms") and abs(avg_ms - prof["launch_ms"]) > 0.05 * prof["launch_ms"]:
            e["warning"] = ("launch time differs by more than 5 % from the profiled one: the traffic figure may "
                            "describe an older build of this kernel")
        return e

    sym = "symmetric"
    q_entry = kernel_entry(f"quantize_kernel<{bits},{group},{sym},linear>", q_avg, "quantize_int4g64_llama3_8b_pmc.md")
    d_entry = kernel_entry(f"dequantize_paged_kernel<{bits},{group},{sym},paged>", d_avg,
                           "dequantize_paged_int4g64_llama3_8b_pmc.md")
    # the kernel with the larger share of the step is the headline; the other one rides along
    first, second = (d_entry, q_entry) if d_avg >= q_avg else (q_entry, d_entry)
    roofline = {"bound": "hbm", "kernel": first["kernel"], "achieved": first["achieved"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": first["frac"], "traffic": first["traffic"],
                "traffic_source": first["traffic_source"], "algorithmic_bytes_per_launch": alg_bytes_per_launch,
                "avg_launch_ms": first["avg_launch_ms"], "profile_avg_launch_ms": first["profile_avg_launch_ms"],
                "share_of_step": first["share_of_step"], "secondary": second}
    if "warning" in first:
        roofline["warning"] = first["warning"]
    achieved = first["achieved"]

    # plain copy of the same plane: the practical ceiling of a streaming kernel on this part
    tmp = torch.empty_like(K)
    for _ in range(2):
        kvp.kvp_copy_bytes(tmp, K)
    a, b = ev(), ev()
    a.record(stream)
    for _ in range(10):
        kvp.kvp_copy_bytes(tmp, K)
    b.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 2 * plane_bytes / (a.elapsed_time(b) / 10 * 1e-3) / 1e9
    roofline["copy_kernel_GBs"] = round(copy_gbs, 1)
    roofline["frac_of_copy"] = round(achieved / copy_gbs, 4)
    del tmp

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(K, V, bt, nb, cfg, workloads)

    ops = None
    if not args.no_ops:
        del qK, qV, pK, pV
        torch.cuda.empty_cache()
        ops = side_measurements(kvp, workloads, torch, dev, K, V)

    out = {
        "metric": "KV compress+decompress GB/s (input KV bytes), 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "llama3_8b_int4_paged", "shape": f"{L}x{H}x{D}x{T} bf16 K and V",
                   "codec": f"int{bits} group {group}", "page_tokens": bs, "input_bytes": input_bytes,
                   "step": "quantize(K), quantize(V), dequantize_paged(K), dequantize_paged(V)"},
        "pct_of_hbm_peak_per_op": {"quantize": round(100 * q_entry["frac"], 1),
                                   "dequantize": round(100 * d_entry["frac"], 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "ops": ops,
    }
    print(json.dumps(out))


def cpu_baseline(K, V, bt, nb, cfg, workloads):
    """The CPU oracle, as it stands, on bounded samples of the same workloads: quantize + dequantize_paged of the
    headline configuration on all host threads (`value`) and on one core, then measured slices of the score,
    select and proxy oracles with their full-configuration times extrapolated linearly (and labelled so)."""
    import numpy as np
    import torch
    import oracle
    oracle.build()
    sample_layers = min(32, K.shape[0])
    cores = min(os.cpu_count() or 1, 16)
    T, bs, bits, group = cfg["T"], cfg["bs"], cfg["bits"], cfg["group"]
    kb = K[:sample_layers].cpu().view(torch.int16).numpy().view(np.uint16)
    vb = V[:sample_layers].cpu().view(torch.int16).numpy().view(np.uint16)
    # split every layer in token slabs so that all threads have work; each slab is a whole number of pages
    slabs = max(1, cores * 2 // sample_layers)
    slab_tokens = (T // slabs) // bs * bs
    jobs = []
    for plane in (kb, vb):
        for l in range(sample_layers):
            for s in range(slabs):
                t0 = s * slab_tokens
                t1 = T if s == slabs - 1 else t0 + slab_tokens
                jobs.append((plane, l, t0, t1))

    def run(job):
        plane, l, t0, t1 = job
        x = plane[l:l + 1, t0:t1]
        codes, scales = oracle.quantize(x, bits, group)
        n = t1 - t0
        oracle.dequantize_paged(codes, scales, bits, group, n, np.arange((n + bs - 1) // bs, dtype=np.int32),
                                (n + bs - 1) // bs, bs)
        return x.nbytes

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        done = sum(ex.map(run, jobs))
    dt = time.perf_counter() - t0
    # the same work on ONE core: two layers of K
    t0 = time.perf_counter()
    one = sum(run((kb, l, 0, T)) for l in range(min(2, sample_layers)))
    dt1 = time.perf_counter() - t0

    def bits_of(t):
        return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    slices = {}
    # scores: one (layer, kv head) of the 70B-shaped configuration (M = 512 rows x 16384 keys)
    c = workloads.CONFIGS["llama3_70b_drop_int4"]
    Ks, _ = workloads.make_kv(1, c["T"], 1, c["D"], seed=0)
    Qs = workloads.make_q(1, c["W"], c["G"], c["D"], seed=0)
    t0 = time.perf_counter()
    sc = oracle.score_tokens(bits_of(Qs), bits_of(Ks))
    ds = time.perf_counter() - t0
    cells = c["L"] * c["H"]
    slices["score_tokens"] = {"sample": f"1 of {cells} (layer, kv head) cells of llama3_70b_drop_int4, one core",
                              "seconds": round(ds, 3), "full_config_seconds_one_core": round(ds * cells, 1),
                              "extrapolated": True}
    # select: 8 of the 640 score rows
    rows = np.ascontiguousarray(np.tile(np.where(np.isfinite(sc[0]), sc[0], 0.0).astype(np.float32), (8, 1)))
    k = oracle.keep_count(c["keep_ratio"], c["T"])
    t0 = time.perf_counter()
    oracle.select_topk(rows, k)
    dsel = time.perf_counter() - t0
    slices["select_topk"] = {"sample": f"8 of {cells} rows of {c['T']} scores, k = {k}, one core", "seconds": round(dsel, 4),
                             "full_config_seconds_one_core": round(dsel * cells / 8, 2), "extrapolated": True}
    # proxy: one (layer, kv head) cell of one context of the sweep, 4 of the 40 configurations
    c = workloads.CONFIGS["utility_sweep"]
    Ke, Ve = workloads.make_kv(1, c["T"], 1, c["D"], seed=0)
    Qe = workloads.make_q(1, c["W"], c["G"], c["D"], seed=0)
    sub = [(16, 0, c["T"]), (8, 128, c["T"]), (4, 64, c["T"] // 2), (2, 32, c["T"] // 4)]
    t0 = time.perf_counter()
    oracle.eval_configs(bits_of(Qe), bits_of(Ke), bits_of(Ve), sub)
    de = time.perf_counter() - t0
    n_cfg = (1 + len(c["bits_set"]) * len(c["group_set"])) * (len(c["keep_ratios"]) + 1)
    cells = c["L"] * c["H"]
    slices["eval_configs"] = {"sample": f"1 of {cells} cells of one context of utility_sweep, {len(sub)} of {n_cfg} "
                                        "configurations, one core", "seconds": round(de, 3),
                              "one_context_seconds_one_core": round(de * cells * n_cfg / len(sub), 1),
                              "full_config_seconds_one_core": round(de * cells * n_cfg / len(sub) * c["n_ctx"], 0),
                              "extrapolated": True, "note": "the oracle recomputes every configuration from scratch; "
                              "its cost is taken as linear in cells, configurations and contexts"}
    return {"value": round(done / dt / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{sample_layers} of {K.shape[0]} layers of the same K and V ({done / 2**20:.0f} MiB of input), "
                      f"quantize + dequantize_paged, {len(jobs)} token slabs over {cores} threads",
            "seconds": round(dt, 2),
            "one_core": {"value": round(one / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                         "sample": f"{min(2, sample_layers)} layers of K ({one / 2**20:.0f} MiB)", "seconds": round(dt1, 2)},
            "slices": slices}


def _time_loop(torch, fn, iters, warm=3, batches=3):
    """Median over `batches` event-timed batches of `iters` calls, after `warm` untimed calls (the clocks of an
    idle GPU take a few milliseconds of load to settle)."""
    for _ in range(warm):
        fn()
    times = []
    for _ in range(batches):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / iters * 1e-3)
    return sorted(times)[len(times) // 2]


def side_measurements(kvp, workloads, torch, dev, K8, V8):
    """Per-operation figures on the other benchmark configurations (outside the timed steps)."""
    ops = {}
    # --- int8 g128 and int2 g32 codecs on the resident 8B-shaped planes (beyond the last-level cache) ---
    L, T, H, D = K8.shape
    bt, nb = workloads.make_block_table(T, 16, seed=0, device=dev)
    for name, bits, group in [("int8_g128", 8, 128), ("int2_g32", 2, 32), ("int4_g32", 4, 32),
                              ("asymmetric_int4_g64", 4, 64), ("asymmetric_int2_g32", 2, 32),
                              ("per_channel_int4_g32", 4, 32), ("per_channel_int4_g128", 4, 128),
                              ("per_channel_asymmetric_int2_g32", 2, 32), ("per_channel_asymmetric_int2_g128", 2, 128)]:
        qp = kvp.alloc_qplane(L, T, H, D, bits, group, dev, asymmetric="asymmetric" in name,
                              per_channel=name.startswith("per_channel"))
        pg = kvp.alloc_paged(L, T, H, D, bt, nb, 16)
        tq = _time_loop(torch, lambda: kvp.kvp_quantize(K8, qp), 10, warm=2)
        td = _time_loop(torch, lambda: kvp.kvp_dequantize_paged(qp, pg), 10, warm=2)
        alg = K8.numel() * 2 + qp.nbytes()
        if name == "int4_g32":
            ident = kvp.PagedKV(pg.pool, torch.arange(nb, dtype=torch.int32, device=dev), T)
            ti = _time_loop(torch, lambda: kvp.kvp_dequantize_paged(qp, ident), 5)
            ops["dequantize_contiguous_pages_int4_g32"] = {
                "workload": "same plane, identity block table (pages not scattered)",
                "dequantize_GBs_alg": round(alg / ti / 1e9, 1), "dequantize_frac_hbm": round(alg / ti / 1e9 / HBM_PEAK_GBS, 4)}
        ops[name] = {"workload": f"{L}x{H}x{D}x{T} plane", "quantize_GBs_alg": round(alg / tq / 1e9, 1),
                     "dequantize_GBs_alg": round(alg / td / 1e9, 1),
                     "quantize_frac_hbm": round(alg / tq / 1e9 / HBM_PEAK_GBS, 4),
                     "dequantize_frac_hbm": round(alg / td / 1e9 / HBM_PEAK_GBS, 4)}
        del qp, pg
    # --- single-layer int8 config: 8 MiB planes are cache-resident and launch-bound; a rotating set of
    #     64 independent copies (512 MiB per plane set) defeats the 256 MB last-level cache ---
    c1 = workloads.CONFIGS["single_layer_int8"]
    n_rot = 64
    K1, _ = workloads.make_kv(n_rot, c1["T"], c1["H"], c1["D"], seed=0, device=dev)   # n_rot independent "layers"
    bt1, nb1 = workloads.make_block_table(c1["T"], 16, seed=0, device=dev)
    q1 = [kvp.alloc_qplane(1, c1["T"], c1["H"], c1["D"], 8, 128, dev) for _ in range(n_rot)]
    p1 = [kvp.alloc_paged(1, c1["T"], c1["H"], c1["D"], bt1, nb1, 16) for _ in range(n_rot)]
    views = [K1[i:i + 1] for i in range(n_rot)]
    alg1 = views[0].numel() * 2 + q1[0].nbytes()

    def rot_q():
        for i in range(n_rot):
            kvp.kvp_quantize(views[i], q1[i])

    def rot_d():
        for i in range(n_rot):
            kvp.kvp_dequantize_paged(q1[i], p1[i])
    t_same_q = _time_loop(torch, lambda: kvp.kvp_quantize(views[0], q1[0]), 50, warm=5)
    t_same_d = _time_loop(torch, lambda: kvp.kvp_dequantize_paged(q1[0], p1[0]), 50, warm=5)
    t_rot_q = _time_loop(torch, rot_q, 3) / n_rot
    t_rot_d = _time_loop(torch, rot_d, 3) / n_rot
    # the same 64 launches replayed from a HIP graph (the library neither allocates nor synchronizes,
    # so a caller can capture it): what is left is the device-side launch cost
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        rot_q()
        rot_d()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gq, gd = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(gq):
        rot_q()
    with torch.cuda.graph(gd):
        rot_d()
    t_graph_q = _time_loop(torch, gq.replay, 5) / n_rot
    t_graph_d = _time_loop(torch, gd.replay, 5) / n_rot
    # scores and keep-set of the same single layer (M = G*W = 128 window rows, k = half the tokens)
    Q1 = workloads.make_q(n_rot, c1["W"], c1["G"] * c1["H"], c1["D"], seed=0, device=dev)
    qviews = [Q1[i:i + 1] for i in range(n_rot)]
    sc1 = torch.empty(1, c1["H"], c1["T"], dtype=torch.float32, device=dev)
    ws1 = torch.empty(kvp.kvp_score_workspace_bytes(1, c1["H"], c1["G"] * c1["H"], c1["W"], c1["T"]) + 16,
                      dtype=torch.uint8, device=dev)
    k1 = kvp.kvp_keep_count(c1["keep_ratio"], c1["T"])
    idx1 = torch.empty(c1["H"], k1, dtype=torch.int32, device=dev)

    def rot_s():
        for i in range(n_rot):
            kvp.kvp_score_tokens(qviews[i], views[i], sc1, ws=ws1)
    t_rot_s = _time_loop(torch, rot_s, 3) / n_rot
    t_sel1 = _time_loop(torch, lambda: kvp.kvp_select_topk(sc1.view(c1["H"], c1["T"]), k1, idx1), 50, warm=5)
    ops["single_layer_int8"] = {
        "workload": f"1x{c1['H']}x{c1['D']}x{c1['T']} plane (8 MiB), int8 g128; 'rotating' = {n_rot} independent copies in turn",
        "quantize_us_cache_resident": round(t_same_q * 1e6, 1), "dequantize_us_cache_resident": round(t_same_d * 1e6, 1),
        "quantize_us_rotating": round(t_rot_q * 1e6, 1), "dequantize_us_rotating": round(t_rot_d * 1e6, 1),
        "quantize_GBs_alg_rotating": round(alg1 / t_rot_q / 1e9, 1), "dequantize_GBs_alg_rotating": round(alg1 / t_rot_d / 1e9, 1),
        "quantize_us_rotating_hip_graph": round(t_graph_q * 1e6, 1), "dequantize_us_rotating_hip_graph": round(t_graph_d * 1e6, 1),
        "quantize_GBs_alg_hip_graph": round(alg1 / t_graph_q / 1e9, 1), "dequantize_GBs_alg_hip_graph": round(alg1 / t_graph_d / 1e9, 1),
        "score_us_rotating": round(t_rot_s * 1e6, 1), "select_us": round(t_sel1 * 1e6, 1), "select_k": k1,
        "note": "launch-bound: one quantize call moves 16.3 MB (2 us at peak); times include the per-call launch path; "
                "a score call is two launches"}
    del gq, gd, K1, q1, p1, views, Q1, qviews
    # --- long-context int2 config at its true shape (4 KV heads: 16 KiB pages, outlier channels x16) ---
    c5 = workloads.CONFIGS["long_context_int2"]
    K5, _ = workloads.make_kv(c5["L"], c5["T"], c5["H"], c5["D"], seed=0, outlier_scale=c5["outlier_scale"], device=dev)
    bt5, nb5 = workloads.make_block_table(c5["T"], 16, seed=0, device=dev)
    q5 = kvp.alloc_qplane(c5["L"], c5["T"], c5["H"], c5["D"], 2, 32, dev)
    p5 = kvp.alloc_paged(c5["L"], c5["T"], c5["H"], c5["D"], bt5, nb5, 16)
    t5q = _time_loop(torch, lambda: kvp.kvp_quantize(K5, q5), 5)
    t5d = _time_loop(torch, lambda: kvp.kvp_dequantize_paged(q5, p5), 5)
    alg5 = K5.numel() * 2 + q5.nbytes()
    ops["long_context_int2"] = {"workload": f"{c5['L']}x{c5['H']}x{c5['D']}x{c5['T']} plane (3.5 GiB), int2 g32",
                                "quantize_ms": round(t5q * 1e3, 3), "dequantize_ms": round(t5d * 1e3, 3),
                                "quantize_frac_hbm": round(alg5 / t5q / 1e9 / HBM_PEAK_GBS, 4),
                                "dequantize_frac_hbm": round(alg5 / t5d / 1e9 / HBM_PEAK_GBS, 4),
                                "compress_decompress_input_GBs": round(K5.numel() * 2 / (t5q + t5d) / 1e9, 1)}
    del q5, p5
    # attention scores at this shape (M = G*W = 224 window rows: the regime where the K reads count), then the
    # keep-set from those scores
    Q5 = workloads.make_q(c5["L"], c5["W"], c5["G"] * c5["H"], c5["D"], seed=0, device=dev)
    sc5 = torch.empty(c5["L"], c5["H"], c5["T"], dtype=torch.float32, device=dev)
    ws5 = torch.empty(kvp.kvp_score_workspace_bytes(c5["L"], c5["H"], c5["G"] * c5["H"], c5["W"], c5["T"]) + 16,
                      dtype=torch.uint8, device=dev)
    t5s = _time_loop(torch, lambda: kvp.kvp_score_tokens(Q5, K5, sc5, ws=ws5), 5)
    rows5 = c5["L"] * c5["H"]
    k5 = kvp.kvp_keep_count(c5["keep_ratio"], c5["T"])
    idx5 = torch.empty(rows5, k5, dtype=torch.int32, device=dev)
    wsel5 = torch.empty(kvp.kvp_select_workspace_bytes(rows5, c5["T"], k5), dtype=torch.uint8, device=dev)
    t5sel = _time_loop(torch, lambda: kvp.kvp_select_topk(sc5.view(rows5, c5["T"]), k5, idx5, ws=wsel5), 100, warm=20)
    M5 = c5["G"] * c5["W"]
    flops5 = 2 * 2.0 * rows5 * M5 * c5["T"] * c5["D"]
    ops["long_context_score_select"] = {
        "workload": f"{c5['L']}x{c5['H']}x{c5['D']}x{c5['T']} K plane, G={c5['G']}, W={c5['W']} (M={M5}), keep {k5}",
        "score_ms": round(t5s * 1e3, 3), "score_TFLOPs": round(flops5 / t5s / 1e12, 1),
        "score_frac_mfma": round(flops5 / t5s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "score_K_read_GBs": round(2 * K5.numel() * 2 / t5s / 1e9, 1),
        "score_K_read_frac_hbm": round(2 * K5.numel() * 2 / t5s / 1e9 / HBM_PEAK_GBS, 4),
        "select_us": round(t5sel * 1e6, 1), "select_GBs_alg": round(rows5 * (c5["T"] + k5) * 4 / t5sel / 1e9, 1),
        "note": "scores come from kvp_score_tokens (two passes over K: both counted in score_K_read)"}
    del K5, Q5, sc5, ws5, idx5, wsel5
    # --- key-only importance scores (knorm, keydiff) on the resident K plane ---
    sc8 = torch.empty(L, H, T, dtype=torch.float32, device=dev)
    wsk = torch.empty(kvp.kvp_score_keys_workspace_bytes(L, H, T, kvp.KVP_SCORE_KEYDIFF) + 16, dtype=torch.uint8, device=dev)
    tn = _time_loop(torch, lambda: kvp.kvp_score_keys(K8, kvp.KVP_SCORE_KNORM, sc8), 5)
    tk = _time_loop(torch, lambda: kvp.kvp_score_keys(K8, kvp.KVP_SCORE_KEYDIFF, sc8, ws=wsk), 5)
    kb = K8.numel() * 2
    ops["key_scores"] = {"workload": f"{L}x{H}x{D}x{T} K plane",
                         "knorm_ms": round(tn * 1e3, 3), "knorm_GBs_alg": round((kb + sc8.numel() * 4) / tn / 1e9, 1),
                         "knorm_frac_hbm": round((kb + sc8.numel() * 4) / tn / 1e9 / HBM_PEAK_GBS, 4),
                         "keydiff_ms": round(tk * 1e3, 3), "keydiff_GBs_alg": round((2 * kb + sc8.numel() * 4) / tk / 1e9, 1),
                         "keydiff_frac_hbm": round((2 * kb + sc8.numel() * 4) / tk / 1e9 / HBM_PEAK_GBS, 4)}
    del sc8, wsk
    # --- 70B-shaped drop + quantize pipeline at its true shape (80 layers, 5 GiB of K and V) ---
    c = workloads.CONFIGS["llama3_70b_drop_int4"]
    Ls = c["L"]
    Kc, Vc = workloads.make_kv(Ls, c["T"], c["H"], c["D"], seed=0, device=dev)
    Qc = workloads.make_q(Ls, c["W"], c["G"] * c["H"], c["D"], seed=0, device=dev)
    k = kvp.kvp_keep_count(c["keep_ratio"], c["T"])
    sc = torch.empty(Ls, c["H"], c["T"], dtype=torch.float32, device=dev)
    ws = torch.empty(kvp.kvp_score_workspace_bytes(Ls, c["H"], c["G"] * c["H"], c["W"], c["T"]) + 16,
                     dtype=torch.uint8, device=dev)
    idx = torch.empty(Ls * c["H"], k, dtype=torch.int32, device=dev)
    qk = kvp.alloc_qplane(Ls, k, c["H"], c["D"], c["bits"], c["group"], dev)
    t_score = _time_loop(torch, lambda: kvp.kvp_score_tokens(Qc, Kc, sc, ws=ws), 5)
    sv = sc.view(Ls * c["H"], c["T"])
    t_sel = _time_loop(torch, lambda: kvp.kvp_select_topk(sv, k, idx), 100, warm=20)   # tens of us per call: long batches
    sm = torch.empty(Ls * c["H"], c["T"], dtype=torch.float32, device=dev)
    t_smooth = _time_loop(torch, lambda: kvp.kvp_smooth_scores(sv, c["W"], 7, "max", out=sm), 100, warm=20)
    keep = idx.view(Ls, c["H"], k)
    t_gq = _time_loop(torch, lambda: kvp.kvp_quantize(Kc, qk, keep_idx=keep), 5)
    # restore of the dropped+quantized plane: compact (k-slot pool) and at the original positions (T-token pool)
    btk, nbk = workloads.make_block_table(k, 16, seed=0, device=dev)
    btT, nbT = workloads.make_block_table(c["T"], 16, seed=0, device=dev)
    pk = kvp.alloc_paged(Ls, k, c["H"], c["D"], btk, nbk, 16)
    pT = kvp.alloc_paged(Ls, c["T"], c["H"], c["D"], btT, nbT, 16)
    t_rc = _time_loop(torch, lambda: kvp.kvp_dequantize_paged(qk, pk), 5)
    t_rs = _time_loop(torch, lambda: kvp.kvp_dequantize_paged_scatter(qk, keep, pT), 5)
    restore_bytes = qk.nbytes() + Ls * k * c["H"] * c["D"] * 2
    M = c["G"] * c["W"]
    flops = 2 * 2.0 * Ls * c["H"] * M * c["T"] * c["D"]
    sel_bytes = Ls * c["H"] * (c["T"] + k) * 4
    gq_bytes = Ls * k * c["H"] * c["D"] * 2 + qk.nbytes() + idx.numel() * 4
    ops["llama3_70b_drop_int4"] = {
        "workload": f"{Ls} x {c['H']} x {c['D']} x {c['T']}, G={c['G']}, W={c['W']}, keep {k}",
        "score_ms": round(t_score * 1e3, 3), "score_TFLOPs": round(flops / t_score / 1e12, 1),
        "score_frac_mfma": round(flops / t_score / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "select_us": round(t_sel * 1e6, 1), "select_GBs_alg": round(sel_bytes / t_sel / 1e9, 1),
        "select_frac_hbm": round(sel_bytes / t_sel / 1e9 / HBM_PEAK_GBS, 4),
        "smooth_k7_us": round(t_smooth * 1e6, 1), "smooth_GBs_alg": round(2 * sc.numel() * 4 / t_smooth / 1e9, 1),
        "gather_quantize_ms_per_plane": round(t_gq * 1e3, 3), "gather_quantize_GBs_alg": round(gq_bytes / t_gq / 1e9, 1),
        "restore_compact_ms_per_plane": round(t_rc * 1e3, 3), "restore_compact_GBs_alg": round(restore_bytes / t_rc / 1e9, 1),
        "restore_scatter_ms_per_plane": round(t_rs * 1e3, 3),
        "restore_scatter_GBs_alg": round((restore_bytes + idx.numel() * 4) / t_rs / 1e9, 1),
        "pipeline_input_GBs": round(2 * Kc.numel() * 2 / (t_score + t_sel + 2 * t_gq) / 1e9, 1)}
    del Kc, Vc, Qc, sc, sm, ws, idx, qk, pk, pT
    # --- long-context select: 112 rows of 131072 scores ---
    c = workloads.CONFIGS["long_context_int2"]
    rows = c["L"] * c["H"]
    k = kvp.kvp_keep_count(c["keep_ratio"], c["T"])
    s = workloads.make_scores(rows, c["T"], seed=0, device=dev)
    idx = torch.empty(rows, k, dtype=torch.int32, device=dev)
    wsel = torch.empty(kvp.kvp_select_workspace_bytes(rows, c["T"], k), dtype=torch.uint8, device=dev)
    t_sel = _time_loop(torch, lambda: kvp.kvp_select_topk(s, k, idx, ws=wsel), 100, warm=20)
    ops["long_context_select"] = {"workload": f"{rows} rows x {c['T']} squared-normal stand-in scores, k={k}",
                                  "select_us": round(t_sel * 1e6, 1),
                                  "select_GBs_alg": round(rows * (c["T"] + k) * 4 / t_sel / 1e9, 1)}
    del s, idx, wsel
    # --- utility-table sweep: the 64 contexts of the configuration, context i from seed i, generated on the
    #     device; one kvp_eval_configs call per context, all enqueued on one stream with one shared workspace ---
    c = workloads.CONFIGS["utility_sweep"]
    n_ctx = c["n_ctx"]
    ctxs = []
    for i in range(n_ctx):
        Ke, Ve = workloads.make_kv(c["L"], c["T"], c["H"], c["D"], seed=i, device=dev)
        Qe = workloads.make_q(c["L"], c["W"], c["G"] * c["H"], c["D"], seed=i, device=dev)
        ctxs.append((Qe, Ke, Ve))
    ks = [kvp.kvp_keep_count(r, c["T"]) for r in c["keep_ratios"]] + [c["T"]]
    variants = [(16, 0)] + [(b, g) for b in c["bits_set"] for g in c["group_set"]]
    cfgs = [(b, g, kk) for (b, g) in variants for kk in ks]
    ws = torch.empty(kvp.kvp_eval_workspace_bytes(c["L"], c["H"], c["G"] * c["H"], c["W"], c["T"], len(cfgs)),
                     dtype=torch.uint8, device=dev)
    loss = torch.empty(n_ctx, len(cfgs), dtype=torch.float32, device=dev)
    Qe, Ke, Ve = ctxs[0]
    t_ev = _time_loop(torch, lambda: kvp.kvp_eval_configs(Qe, Ke, Ve, cfgs, loss=loss[0], ws=ws), 2)
    t_ev_mx = _time_loop(torch, lambda: kvp.kvp_eval_configs(Qe, Ke, Ve, cfgs, loss=loss[0], ws=ws, pv_matrix_cores=True), 2)
    t_ev_32 = _time_loop(torch, lambda: kvp.kvp_eval_configs(Qe, Ke, Ve, cfgs, loss=loss[0], ws=ws, pv_fp32=True), 2)

    def sweep():
        for i, (q_, k_, v_) in enumerate(ctxs):
            kvp.kvp_eval_configs(q_, k_, v_, cfgs, loss=loss[i], ws=ws)
    t_sweep = _time_loop(torch, sweep, 1, warm=1, batches=2)
    M = c["G"] * c["W"]
    # work actually done: one stream per codec, each over the largest keep-set (here all T tokens); the
    # 16-bit stream doubles as the reference
    tokens = len(variants) * max(ks)
    pv_flops = 2.0 * c["L"] * c["H"] * M * c["D"] * tokens
    pv_rate = pv_flops * n_ctx / t_sweep / 1e12
    ops["utility_sweep"] = {"workload": f"{n_ctx} contexts (seed i for context i) of {c['L']}x{c['H']}x{c['D']}x{c['T']}, "
                                        f"{len(cfgs)} configs each, one call per context on one stream",
                            "sweep_ms": round(t_sweep * 1e3, 1), "eval_ms_per_context": round(t_sweep * 1e3 / n_ctx, 2),
                            "eval_ms_one_context_alone": round(t_ev * 1e3, 2),
                            "configs_per_s": round(len(cfgs) * n_ctx / t_sweep, 1),
                            "input_GBs": round(n_ctx * 2 * Ke.numel() * 2 / t_sweep / 1e9, 1),
                            "bound": "alu", "pv_TFLOPs": round(pv_rate, 2),
                            "pv_operands": "fp16 pairs (v_dot2_f32_f16), fp32 accumulation",
                            "pv_frac_valu_dot2_peak": round(pv_rate / VALU_DOT2_PEAK_TFLOPS, 4),
                            "peaks_TFLOPs": {"v_dot2_f32_f16 (256 CU x 4 SIMD x 16 lanes x 4 flop x 2.4 GHz)": VALU_DOT2_PEAK_TFLOPS,
                                             "fp32 fma, no packed fp32 (x 2 flop)": VALU_FP32_PEAK_TFLOPS,
                                             "published fp32 vector (packed fp32, not used by this library)": VALU_FP32_PUBLISHED_TFLOPS},
                            "opt_in_pv_fp32": {"eval_ms_one_context_alone": round(t_ev_32 * 1e3, 2),
                                               "pv_TFLOPs_fp32": round(pv_flops / t_ev_32 / 1e12, 2),
                                               "pv_frac_valu_peak_no_packed_fp32": round(pv_flops / t_ev_32 / 1e12 / VALU_FP32_PEAK_TFLOPS, 4),
                                               "pv_frac_published_fp32_vector_peak": round(pv_flops / t_ev_32 / 1e12 / VALU_FP32_PUBLISHED_TFLOPS, 4)},
                            "opt_in_pv_matrix_cores": {"eval_ms_one_context_alone": round(t_ev_mx * 1e3, 2),
                                                       "configs_per_s": round(len(cfgs) / t_ev_mx, 1),
                                                       "mfma_TFLOPs": round(3 * pv_flops / t_ev_mx / 1e12, 1)}}
    return ops


def profile_only(args, kvp, workloads, torch, dev, K, V, qK, pK, bt, nb):
    """Loop one operation so that a profiler sees only it (used for the summaries under profiles/)."""
    n = args.steps
    if args.only == "quantize":
        for _ in range(n):
            kvp.kvp_quantize(K, qK)
    elif args.only in ("dequantize", "dequantize_identity"):
        kvp.kvp_quantize(K, qK)
        if args.only == "dequantize_identity":   # pages in token order instead of the scattered table
            pK = kvp.PagedKV(pK.pool, torch.arange(nb, dtype=torch.int32, device=dev), pK.T)
        for _ in range(n):
            kvp.kvp_dequantize_paged(qK, pK)
    elif args.only == "copy":
        tmp = torch.empty_like(K)
        for _ in range(n):
            kvp.kvp_copy_bytes(tmp, K)
    elif args.only in ("score", "select"):
        c = workloads.CONFIGS["llama3_70b_drop_int4"]
        Ls = 16
        Kc, _ = workloads.make_kv(Ls, c["T"], c["H"], c["D"], seed=0, device=dev)
        Qc = workloads.make_q(Ls, c["W"], c["G"] * c["H"], c["D"], seed=0, device=dev)
        sc = torch.empty(Ls, c["H"], c["T"], dtype=torch.float32, device=dev)
        ws = torch.empty(kvp.kvp_score_workspace_bytes(Ls, c["H"], c["G"] * c["H"], c["W"], c["T"]) + 16,
                         dtype=torch.uint8, device=dev)
        k = kvp.kvp_keep_count(c["keep_ratio"], c["T"])
        idx = torch.empty(Ls * c["H"], k, dtype=torch.int32, device=dev)
        kvp.kvp_score_tokens(Qc, Kc, sc, ws=ws)
        for _ in range(n):
            if args.only == "score":
                kvp.kvp_score_tokens(Qc, Kc, sc, ws=ws)
            else:
                kvp.kvp_select_topk(sc.view(Ls * c["H"], c["T"]), k, idx)
    elif args.only in ("select_many", "select_long"):
        # 2560 rows x 16384 (more rows than block slots) or the long-context shape (112 rows x 131072)
        rows, T = (2560, 16384) if args.only == "select_many" else (112, 131072)
        s = workloads.make_scores(rows, T, seed=0, device=dev)
        k = kvp.kvp_keep_count(0.3 if args.only == "select_many" else 0.1, T)
        idx = torch.empty(rows, k, dtype=torch.int32, device=dev)
        wsel = torch.empty(max(kvp.kvp_select_workspace_bytes(rows, T, k), 16), dtype=torch.uint8, device=dev)
        for _ in range(n):
            kvp.kvp_select_topk(s, k, idx, ws=wsel)
    elif args.only == "eval":
        c = workloads.CONFIGS["utility_sweep"]
        Ke, Ve = workloads.make_kv(c["L"], c["T"], c["H"], c["D"], seed=0, device=dev)
        Qe = workloads.make_q(c["L"], c["W"], c["G"] * c["H"], c["D"], seed=0, device=dev)
        ks = [kvp.kvp_keep_count(r, c["T"]) for r in c["keep_ratios"]] + [c["T"]]
        variants = [(16, 0)] + [(b, g) for b in c["bits_set"] for g in c["group_set"]]
        cfgs = [(b, g, kk) for (b, g) in variants for kk in ks]
        for _ in range(n):
            kvp.kvp_eval_configs(Qe, Ke, Ve, cfgs)
    else:
        raise SystemExit(f"unknown --only {args.only}")
    torch.cuda.synchronize()
    print(json.dumps({"only": args.only, "launches": n, "plane_bytes": K.numel() * 2, "compressed_bytes": qK.nbytes()}))


if __name__ == "__main__":
    main()
