#!/usr/bin/env python3
"""Benchmark of the per-layer KV object hot path on ONE MI355X.

A step is one pass of the whole path over the Llama-3-8B-shaped 32K-token workload (config 2):
for every layer, save (tutti_layer_save: extents + WRITE entries + pack in one launch), then for every
layer, restore (tutti_layer_restore: extents + READ entries + unpack in one launch).  Every layer
has its own K/V planes and its own staging buffer, so each launch touches memory no earlier launch
left in the 256 MB Infinity Cache.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line on stdout; progress goes to stderr.
  value            payload GB/s of the per-layer RESTORE of config 2 (the metric's quantity; 1 GB = 1e9 B)
  roofline         the dominant kernel (k_layer<unpack>: the fused restore) against the 8 TB/s HBM peak,
                   timed with events on the launch stream inside the timed region
  cpu_baseline     the CPU oracle, as it stands, on a bounded sample of configs 1-4 (1 thread and every core
                   of the affinity mask)
Further legs of the same line (all on by default; --quick leaves them out): the save, the copy kernels alone,
copy ceilings and the scattered-copy floor, entries built per second, configs 3 and 4 at their real pool sizes,
config 5 (CU budgets and a CU-masked I/O domain beside two GEMMs) with the slack table it yields, the ring
path, and a sweep of the prefix length from 1K to 128K tokens (eager launches and a HIP-graph replay).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(xs):
    return float(np.median(np.asarray(xs, dtype=np.float64)))


def read_traffic_note():
    """HBM bytes per restore launch measured with rocprofv3 --pmc (profiles/), if recorded."""
    path = os.path.join(ROOT, "profiles", "k_restore_llama8b_32k_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="layers resident (0 = all 32 if memory allows)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="config 2's step only: none of the further legs")
    ap.add_argument("--no-extra", action="store_true", help="skip the copy-ceiling / entry-rate legs")
    ap.add_argument("--no-corun", action="store_true", help="skip config 5 (CU budgets beside a GEMM) and the slack table")
    ap.add_argument("--no-rings", action="store_true", help="skip the ring path (IOCBs, issue_io, retrieve/store_layer)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip configs 3 and 4")
    ap.add_argument("--no-length-sweep", action="store_true", help="skip the 1K..128K-token prefix-length sweep")
    ap.add_argument("--scatter-sweep", action="store_true",
                    help="also sweep the granularity, the order and the launch shape of tutti_scatter_baseline")
    ap.add_argument("--hnd-sweep", action="store_true",
                    help="also time head-major pools of four row sizes, moved 16 bytes per lane and through LDS tiles")
    ap.add_argument("--pinned-stage", action="store_true",
                    help="also time the restore with the staging buffer in pinned host memory (host-link bound)")
    ap.add_argument("--write-lut", default="", help="also write the slack table (JSON) to this path")
    ap.add_argument("--no-placement", action="store_true",
                    help="take the pool's planes as the allocator hands them out instead of putting every layer's K "
                         "and V plane in different HBM regions")
    ap.add_argument("--region-matrix", action="store_true",
                    help="instead of the benchmark: restore and save of config 2's layer for every combination of HBM "
                         "region of the K plane, the V plane and the staging buffer; prints its own JSON line")
    ap.add_argument("--region-map", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark: classify candidates of MIB mebibytes (at least 128) covering the free "
                         "HBM by region, in allocation order; prints its own JSON line")
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--plain-loads", action="store_true", help="disable non-temporal loads/stores")
    args = ap.parse_args()
    if args.quick:
        args.no_extra = args.no_corun = args.no_rings = args.no_other_configs = args.no_length_sweep = True
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no collective and no cross-GPU step; "
              "run it with --gpus 1 (each GPU of a larger job would run exactly this on its own shard)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_03375_amd import binding as B
    from paper_2605_03375_amd import workloads as W

    B.product_lib()  # no fallback: raises if libtutti.so is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    tuned = bool(args.wgs_per_cu or args.unroll or args.plain_loads)
    if tuned:   # an experiment: the same kernels in another launch shape, from the measurement library
        B.use_bench_library(True)
        B.tutti_set_tuning(args.wgs_per_cu, args.unroll)
        B.tutti_set_nontemporal(0 if args.plain_loads else 3)

    if args.region_map:
        print(json.dumps(region_map(torch, dev, args.region_map)), flush=True)
        return
    if args.region_matrix:
        print(json.dumps(region_matrix(torch, B, W.llama8b_32k(), dev)), flush=True)
        return

    w = W.llama8b_32k()
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    plane_bytes = s.num_blocks * bb
    n_tab = int(w.block_table.size)
    payload_layer = 2 * n_tab * bb                       # K + V bytes of one layer's hit blocks
    n_sqe_layer = 2 * ((n_tab * bb + w.chunk_bytes - 1) // w.chunk_bytes)
    free, total = torch.cuda.mem_get_info()
    per_layer = 2 * plane_bytes + payload_layer
    fit = int((free - (6 << 30)) // per_layer)
    L = min(s.num_layers, fit) if args.layers == 0 else min(args.layers, s.num_layers, fit)
    if L < 1:
        raise SystemExit("not enough free HBM for even one layer of the pool")
    log(f"[bench] {w.name}: {L}/{s.num_layers} layers resident, {plane_bytes >> 20} MiB per plane, "
        f"{payload_layer >> 20} MiB payload per layer, free HBM {free >> 30} GiB")

    geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                head_dim=s.head_dim, elt_bytes=s.elt_bytes)
    cfg = B.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    t0 = time.time()
    # where the planes sit: every layer's K plane and V plane in different regions of the HBM (set-up, untimed)
    planes, planes_same, placement_info, placed_stages = placed_planes(
        torch, L, plane_bytes, dev, reserve_bytes=(L * payload_layer) + (12 << 30), place=not args.no_placement,
        stage_bytes=payload_layer)
    log(f"[bench] placement ({time.time() - t0:.1f} s): {placement_info}")
    td = {"fp16": torch.float16, "bf16": torch.bfloat16}[s.dtype]
    for l in range(L):
        W.device_values(W.seed_for(2, l), plane_bytes // 2, s.dtype, dev, out=planes[l][0].view(td))
        W.device_values(W.seed_for(2, l) + 500, plane_bytes // 2, s.dtype, dev, out=planes[l][1].view(td))
        if l % 8 == 7 or l == L - 1:
            torch.cuda.synchronize()
            log(f"[bench] filled {l + 1}/{L} layers ({time.time() - t0:.1f} s)")
    pools = [B.make_pool(k, v, **geom) for k, v in planes]
    pools_same = [B.make_pool(k, v, **geom) for k, v in planes_same]
    if placed_stages is not None:
        stages = placed_stages[:L]
        for st in stages:
            st.zero_()
    else:
        stages = [torch.zeros(payload_layer, dtype=torch.uint8, device=dev) for _ in range(L)]
    d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
    d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
    d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
    ext_w = torch.zeros(L, 32, dtype=torch.uint8, device=dev)
    ext_r = torch.zeros(L, 32, dtype=torch.uint8, device=dev)
    tot_w = torch.zeros(L, 2, dtype=torch.int64, device=dev)
    tot_r = torch.zeros(L, 2, dtype=torch.int64, device=dev)
    wsqe = torch.zeros(L, n_sqe_layer * 64, dtype=torch.uint8, device=dev)
    rsqe = torch.zeros(L, n_sqe_layer * 64, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    sgl_id = 1
    stream = torch.cuda.current_stream()

    def save_layers():
        for l in range(L):
            B.tutti_layer_save(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload_layer,
                               stages[l].data_ptr(), sgl_id, ext_w[l], tot_w[l], wsqe[l], n_sqe_layer, 0, status,
                               stream)

    def save_layers_unfused():
        for l in range(L):
            B.tutti_obj_layout(pools[l], cfg, d_n, 1, ext_w[l], tot_w[l], stream)
            B.tutti_obj_pack(pools[l], cfg, ext_w[l], 1, d_tab, n_tab, stages[l], payload_layer, 0, status, stream)
            B.tutti_sqe_build(pools[l], cfg, ext_w[l], 1, d_fid, l, B.OP_WRITE, stages[l].data_ptr(), sgl_id,
                              wsqe[l], n_sqe_layer, status, stream)

    def restore_layers(budget=0, on=None):
        for l in range(L):
            B.tutti_layer_restore(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload_layer,
                                  stages[l].data_ptr(), sgl_id, ext_r[l], tot_r[l], rsqe[l], n_sqe_layer, budget,
                                  status, stream if on is None else on)

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731  (events of torch's current stream = launch stream)

    # host copy of layer 0 as generated, before any kernel of the library has touched it: what the oracle
    # works from in the cpu_baseline leg, and what the pool must still hold after save + restore
    pristine = None if args.no_cpu_baseline else (planes[0][0].cpu().numpy(), planes[0][1].cpu().numpy())

    for _ in range(args.warmup):
        save_layers()
        restore_layers()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    marks = []
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record(stream)
        save_layers()
        e1.record(stream)
        restore_layers()
        e2.record(stream)
        marks.append((e0, e1, e2))
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_begin) * 1e3 / args.steps
    save_ms = [a.elapsed_time(b) for a, b, _ in marks]
    rest_ms = [b.elapsed_time(c) for _, b, c in marks]
    assert int(status.item()) == 0, f"device status word {int(status.item())}: a block or capacity check tripped"

    restore_us = float(np.mean(rest_ms)) * 1e3 / L       # average restore launch, launch gaps included
    value = payload_layer / (restore_us * 1e-6) / 1e9    # the metric: payload GB/s of the per-layer restore
    save_us = float(np.mean(save_ms)) * 1e3 / L
    # algorithmic bytes of one restore launch: payload read + payload written, the block table,
    # the request counts and file ids, the entries and extents it writes
    restore_alg_bytes = 2 * payload_layer + 4 * n_tab + 4 * w.n_req * 2 + 64 * n_sqe_layer + 32 * w.n_req + 16
    achieved = restore_alg_bytes / (restore_us * 1e-6) / 1e9

    out = {
        "metric": "per-layer KV restore payload GB/s (and % of HBM peak in roofline.frac), Llama-3-8B shape, 32K-token "
                  "prefix, one launch per layer, the pool's planes placed across the HBM regions (config.placement; the same "
                  "planes without that in restore_K_and_V_in_one_region); the step also saves every layer (see save); "
                  "SQEs built/sec in sqe",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config 2: llama8b_32k (bf16 KV, block 16, 8 KV heads x 128, 65536-block pool per "
                               "layer, one 32K-token prefix = 2048 shuffled blocks, 2 MiB chunks)",
                   "layers_resident": L, "layers_model": s.num_layers, "payload_bytes_per_layer": payload_layer,
                   "step": "per layer: layer_save (extents + WRITE entries + pack); then per layer: layer_restore "
                           "(extents + READ entries + unpack); one launch each",
                   "library": "libtutti_bench.so (tuned launch shape: an experiment)" if tuned else "libtutti.so",
                   "wgs_per_cu": args.wgs_per_cu, "unroll": args.unroll, "nontemporal": not args.plain_loads},
        "roofline": {"bound": "hbm", "kernel": "k_layer<unpack> (tutti_layer_restore)", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic_note(),
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs recorded in "
                                       "profiles/k_restore_llama8b_32k_pmc.txt, not measured in this run",
                     "north_star_bar": 0.70, "bar_met": bool(achieved / HBM_PEAK_GBPS >= 0.70),
                     "algorithmic_bytes_per_launch": restore_alg_bytes, "avg_launch_us": round(restore_us, 2)},
        "restore": {"us_per_layer": round(restore_us, 2),
                    "payload_GBps": round(payload_layer / (restore_us * 1e-6) / 1e9, 1),
                    "traffic_GBps": round(2 * payload_layer / (restore_us * 1e-6) / 1e9, 1),
                    "pct_hbm_peak": round(100 * 2 * payload_layer / (restore_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
                    "median_train_ms": round(median(rest_ms), 4), "min_train_ms": round(min(rest_ms), 4),
                    "p95_train_ms": round(float(np.percentile(rest_ms, 95)), 4)},
        "save": {"us_per_layer": round(save_us, 2),
                 "payload_GBps": round(payload_layer / (save_us * 1e-6) / 1e9, 1),
                 "traffic_GBps": round(2 * payload_layer / (save_us * 1e-6) / 1e9, 1),
                 "pct_hbm_peak": round(100 * 2 * payload_layer / (save_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
                 "launches_per_layer": 1},
    }
    out["config"]["placement"] = placement_info
    out["restore"]["host_us_per_call"] = host_us_per_call(torch, restore_layers, L)
    out["restore"]["blocks_per_call"] = n_tab
    # the same without the Python binding in between: the loop runs in C (measurement library, same source)
    c_ns = []
    for _ in range(7):
        torch.cuda.synchronize()
        c_ns.append(B.tutti_host_cost_of_restore(pools[0], cfg, d_n, 1, d_tab, n_tab, d_fid, 0, stages[0], payload_layer,
                                                 stages[0].data_ptr(), sgl_id, ext_r[0], tot_r[0], rsqe[0], n_sqe_layer,
                                                 L, 0, status, stream))
    torch.cuda.synchronize()
    out["restore"]["host_us_per_call_from_c"] = round(median(c_ns) / 1e3, 2)
    if pools_same:
        # the same planes paired within one region (what an allocator that knows nothing of the regions mostly gives)
        def same_train():
            for l, p in enumerate(pools_same):
                B.tutti_layer_restore(p, cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload_layer,
                                      stages[l].data_ptr(), sgl_id, ext_r[l], tot_r[l], rsqe[l], n_sqe_layer, 0,
                                      status, stream)
        same_train()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            a, b = ev(), ev()
            a.record(stream)
            same_train()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / len(pools_same))
        us_same = median(ts)
        out["restore_K_and_V_in_one_region"] = {
            "layers": len(pools_same), "us_per_layer": round(us_same, 2),
            "pct_hbm_peak": round(100 * 2 * payload_layer / (us_same * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
            "note": "the same planes, paired so that a layer's K and V plane lie in one HBM region (contents differ "
                    "from the seeded pool after this leg: it runs after the timed region and the CPU-baseline copy)"}
        # put the seeded contents back where this leg overwrote them: restore every layer once more from its stage
        restore_layers()
        torch.cuda.synchronize()
    if not args.no_extra:
        # the same restore train with an event between every two launches (adds a gap of a microsecond or two to
        # each): the layers differ only in where the driver placed their planes, and so does their time
        per = np.zeros((3, L))
        for rep in range(3):
            evs = [ev() for _ in range(L + 1)]
            for l in range(L):
                evs[l].record(stream)
                B.tutti_layer_restore(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload_layer,
                                      stages[l].data_ptr(), sgl_id, ext_r[l], tot_r[l], rsqe[l], n_sqe_layer, 0,
                                      status, stream)
            evs[L].record(stream)
            torch.cuda.synchronize()
            per[rep] = [evs[l].elapsed_time(evs[l + 1]) * 1e3 for l in range(L)]
        by_layer = np.median(per, axis=0)[1:]            # the first launch of a train also pays for the idle queue
        out["restore"]["by_layer_with_event_gaps_us"] = {
            "min": round(float(by_layer.min()), 1), "median": round(float(np.median(by_layer)), 1),
            "max": round(float(by_layer.max()), 1),
            "layers_under_49us": int((by_layer < 49.0).sum()), "layers": int(by_layer.size),
            "sorted": [round(float(x), 1) for x in np.sort(by_layer)]}
    log(f"[bench] step {ms_per_step:.3f} ms, restore {restore_us:.1f} us/layer "
        f"({out['restore']['traffic_GBps']} GB/s traffic, {out['restore']['pct_hbm_peak']} % of peak), "
        f"save {save_us:.1f} us/layer")

    if not args.no_extra:
        ts = []
        for _ in range(3):
            a, b = ev(), ev()
            a.record(stream)
            save_layers_unfused()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / L)
        out["save_unfused_3_launches"] = {"us_per_layer": round(median(ts), 2)}
        # the copy kernels on their own (extents already on the device): tutti_obj_unpack / tutti_obj_pack
        alone = {}
        for label, fn in (("unpack_alone", B.tutti_obj_unpack), ("pack_alone", B.tutti_obj_pack)):
            ts = []
            for rep in range(4):
                a, b = ev(), ev()
                a.record(stream)
                for l in range(L):
                    fn(pools[l], cfg, ext_r[l], 1, d_tab, n_tab, stages[l], payload_layer, 0, status, stream)
                b.record(stream)
                torch.cuda.synchronize()
                if rep:
                    ts.append(a.elapsed_time(b) * 1e3 / L)
            alone[label] = {"us_per_layer": round(median(ts), 2),
                            "pct_hbm_peak": round(100 * 2 * payload_layer / (median(ts) * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)}
        out["copy_kernels_alone"] = alone
        out["copy_ceiling"] = copy_ceiling(torch, B, stages, payload_layer, dev)
        out["copy_ceiling"]["restore_vs_copy"] = round(out["restore"]["traffic_GBps"] /
                                                       out["copy_ceiling"]["traffic_GBps"], 4)
        out["chip_stream_ceilings"] = per_cu_limits(torch, B, dev, budgets=(0,))["0"]
        out["scatter_floor"] = scatter_floor(torch, B, w, stages, payload_layer, dev)
        out["scatter_floor"]["restore_vs_floor"] = round(out["scatter_floor"]["scattered_writes"]["us"] /
                                                         out["restore"]["us_per_layer"], 4)
        out["scatter_floor"]["pack_vs_floor"] = round(out["scatter_floor"]["scattered_reads"]["us"] /
                                                      out["save"]["us_per_layer"], 4)
        out["sqe"] = sqe_rate(torch, B, W, dev)
        out["sqe"]["direct_to_block"] = direct_rate(torch, B, W, dev)
        out["sqe"]["direct_to_block_2M_entries"] = big_entry_rate(torch, B, dev)
        log(f"[bench] copy ceiling {out['copy_ceiling']}; entries {out['sqe']}")
    cpu2 = None
    if not args.no_cpu_baseline:   # needs layer 0 as saved and restored: before the legs below overwrite the pool
        cpu2 = cpu_baseline(torch, W, w, planes[0], pristine, stages[0], geom, payload_layer)
    if not args.no_extra and placement_info.get("placed"):
        # the plain copy again, from a layer's K plane to its V plane (different HBM regions): does the ceiling move?
        def across():
            for l in range(L):
                B.tutti_copy_baseline(planes[l][1][:payload_layer], planes[l][0][:payload_layer], payload_layer)
        across()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            a, b = ev(), ev()
            a.record(stream)
            across()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / L)
        out["copy_ceiling"]["us_per_copy_between_two_regions"] = round(median(ts), 2)
    if not args.no_corun:
        out["per_cu_limits"] = per_cu_limits(torch, B, dev)
        out["corun"] = {
            "note": "config 5: the restore of config 2 on one stream beside a bf16 GEMM looping on another, each "
                    "timed while the other outlasts it; budget = cu_budget argument, domain = a CU-masked stream "
                    "from tutti_io_domain_create with cu_budget 0",
            "gemm_4096x4096x4096 (256 tiles of 256x256: one per CU)":
                corun_sweep(torch, B, restore_layers, L, payload_layer, dev),
            "gemm_4096x5120x4096 (320 tiles: not a multiple of the CU count)":
                corun_sweep(torch, B, restore_layers, L, payload_layer, dev, gemm_n=(4096, 5120, 4096)),
            "gemm_8192x8192x8192 (1024 tiles)":
                corun_sweep(torch, B, restore_layers, L, payload_layer, dev, gemm_iters=12, reps=2,
                            gemm_n=(8192, 8192, 8192), budgets=(8, 32, 0), domains=(32,)),
        }
        out["slack_lut"] = slack_lut(torch, B, w, pools, planes, cfg, d_tab, d_fid, dev)
        if args.write_lut:
            with open(args.write_lut, "w") as f:
                json.dump(out["slack_lut"], f, indent=1)
    if not args.no_rings:
        out["rings_direct_to_block"] = ring_leg(torch, B, w, pools, planes, cfg, d_n, d_tab, n_tab, d_fid,
                                                payload_layer, dev)
    if not args.no_length_sweep:
        out["length_sweep"] = length_sweep(torch, B, W, pools, cfg, dev)
    if args.scatter_sweep:
        out["scatter_sweep"] = scatter_sweep(torch, B, stages, payload_layer, dev)
        out["scatter_orders_32KiB"] = scatter_orders(torch, B, stages, payload_layer, dev)
        out["scatter_shapes_32KiB"] = scatter_shapes(torch, B, w, stages, payload_layer, dev)
        out["visit_order"] = visit_order(torch, B, W, dev)
    if args.hnd_sweep:
        out["head_major_rows"] = hnd_rows(torch, B, w, planes, stages, dev)
    if args.pinned_stage:
        out["pinned_host_stage"] = pinned_leg(torch, B, pools, cfg, d_n, d_tab, n_tab, d_fid, payload_layer,
                                              n_sqe_layer, dev)
    if not args.no_extra:
        out["restore_address_order"] = ordered_restore(torch, B, s.num_blocks, pools, cfg, d_n, d_tab, n_tab, d_fid,
                                                       stages, payload_layer, n_sqe_layer, dev)
    if not args.no_other_configs:
        del pools, planes, pools_same, planes_same, stages, restore_layers, save_layers, save_layers_unfused
        torch.cuda.empty_cache()
        out["other_configs"] = {
            "config3_batch64_zipf": restore_leg(torch, B, W.batch64_zipf(), dev, max_layers=8,
                                                place=not args.no_placement),
            "config4_llama70b_128k": restore_leg(torch, B, W.llama70b_128k(), dev, max_layers=80,
                                                 place=not args.no_placement),
        }
        # what one rank of a tensor-parallel group of 8 runs on config 4: one KV head of every block, so 4 KiB blocks
        # (the paper keeps one instance of the store beside every GPU process: sec. 3.4 "Support for Multi-GPUs")
        w4 = W.llama70b_128k()
        w_tp = dataclasses.replace(w4, name="llama70b_128k_tp8_rank",
                                   shape=dataclasses.replace(w4.shape, num_kv_heads=w4.shape.num_kv_heads // 8))
        out["other_configs"]["config4_one_rank_of_tp8"] = restore_leg(torch, B, w_tp, dev, max_layers=80,
                                                                      place=not args.no_placement)
    if cpu2 is not None:
        out["cpu_baseline"] = cpu2
        out["cpu_baseline"]["other_configs"] = cpu_baseline_others(W)
    print(json.dumps(out), flush=True)


def placed_planes(torch, n_layers, plane_bytes, dev, reserve_bytes, place=True, stage_bytes=0, stage_rotation=0):
    """K and V planes for n_layers layers.  place: candidates covering about 200 GiB are allocated, told apart by
    HBM region with paper_2605_03375_amd.placement (a timing probe with the real restore call), every layer gets a K
    plane and a V plane from different regions, and the candidates not needed are freed.  Also returns the same
    planes paired within a region (what an allocator that knows nothing of the regions usually produces: the layout
    to compare against), a description, and, when stage_bytes is given and spare candidates allow it, one staging
    buffer per layer cut from a spare candidate of the region that holds neither of the layer's planes (else None:
    the caller allocates them wherever the allocator puts them); with stage_rotation = n, at most n buffers per region,
    taken in turn.  Contents are left as allocated."""
    from paper_2605_03375_amd import placement
    free, _ = torch.cuda.mem_get_info()
    fit = int((free - reserve_bytes) // plane_bytes)
    if not place or fit < 2 * n_layers + 2:
        n = min(n_layers, fit // 2)
        cands = [torch.empty(plane_bytes, dtype=torch.uint8, device=dev) for _ in range(2 * n)]
        planes = [(cands[2 * l], cands[2 * l + 1]) for l in range(n)]
        return planes, [], {"placed": False, "why": "switched off" if not place else "no room for spare candidates"}, None
    n_cand = min(fit, max(3 * n_layers, int((200 << 30) // plane_bytes)))
    cands = []
    try:
        cands = [torch.empty(plane_bytes, dtype=torch.uint8, device=dev) for _ in range(n_cand)]
        classes, report = placement.classify_planes(cands, dev)
    except (RuntimeError, ValueError) as e:       # out of memory, or a probe that reported a status: go on unplaced
        del cands
        torch.cuda.empty_cache()
        log(f"[bench] placement failed ({type(e).__name__}: {str(e)[:200]}); taking the planes as allocated")
        return placed_planes(torch, n_layers, plane_bytes, dev, reserve_bytes, place=False)
    info = {"candidates": n_cand, "candidate_GiB": round(n_cand * plane_bytes / 2 ** 30, 1),
            "regions_in_allocation_order": "".join("ABC?"[c] for c in classes), "rounds": report["rounds"]}
    pairs = placement.choose_pairs(classes, n_layers, strict=False)
    info["placed"] = True
    used = sorted(i for p in pairs for i in p)
    same = placement.same_region_pairs([classes[i] for i in used], n_layers)
    planes = [(cands[i], cands[j]) for i, j in pairs]
    planes_same = [(cands[used[i]], cands[used[j]]) for i, j in same]
    info["layers_with_K_and_V_in_different_regions"] = sum(1 for i, j in pairs if classes[i] != classes[j] and
                                                            classes[i] >= 0 and classes[j] >= 0)
    stages = None
    if stage_bytes and plane_bytes >= stage_bytes:
        # spare candidates cut into staging buffers, by region; a layer takes one from the region of neither plane
        spare = {}
        taken = set(used)
        for i, c in enumerate(classes):
            if i not in taken and c >= 0:
                spare.setdefault(c, []).append(i)
        per_cand = plane_bytes // stage_bytes
        cut = {c: [] for c in spare}                     # views not handed out yet
        nxt = {c: 0 for c in spare}                      # spare candidates of the class not yet cut
        handed = {c: [] for c in spare}                  # views handed out (they are taken in turn once
        turn = {c: 0 for c in spare}                     # stage_rotation of them exist)
        def take(c):
            if stage_rotation and len(handed[c]) >= stage_rotation:
                turn[c] += 1
                return handed[c][turn[c] % len(handed[c])]
            if not cut[c] and nxt[c] < len(spare[c]):
                t = cands[spare[c][nxt[c]]]
                nxt[c] += 1
                cut[c] = [t[k * stage_bytes:(k + 1) * stage_bytes] for k in range(per_cand)]
            if not cut[c]:
                if handed[c]:
                    turn[c] += 1
                    return handed[c][turn[c] % len(handed[c])]
                return None
            handed[c].append(cut[c].pop(0))
            return handed[c][-1]
        stages, third, loose = [], 0, []
        for i, j in pairs:
            want = [c for c in sorted(spare) if c not in (classes[i], classes[j])]
            st = None
            for c in want:
                st = take(c)
                if st is not None:
                    third += 1
                    break
            if st is None:
                if stage_rotation and len(loose) >= stage_rotation:
                    st = loose[len(stages) % len(loose)]
                else:
                    st = torch.empty(stage_bytes, dtype=torch.uint8, device=dev)
                    loose.append(st)
            stages.append(st)
        info["staging_buffers_in_a_third_region"] = third
    del cands
    torch.cuda.empty_cache()
    return planes, planes_same, info, stages


def region_map(torch, dev, mib):
    """The HBM regions in the order the allocator hands memory out: candidates of `mib` MiB covering the free memory
    (at most 1,000 of them), classified by tutti_place_classify; the classes as runs in allocation order."""
    from paper_2605_03375_amd import placement
    size = max(128, mib) << 20
    free, _ = torch.cuda.mem_get_info()
    n = int(min(1000, (free - (10 << 30)) // size))
    cands = [torch.empty(size, dtype=torch.uint8, device=dev) for _ in range(n)]
    classes, report = placement.classify_planes(cands, dev, max_regions=4)
    runs = []
    for c in classes:
        ch = "ABCD?"[c]
        if runs and runs[-1][0] == ch:
            runs[-1][1] += 1
        else:
            runs.append([ch, 1])
    return {"candidate_MiB": size >> 20, "candidates": n, "GiB": round(n * size / 2 ** 30, 2), "rounds": report["rounds"],
            "runs_in_allocation_order": [[ch, k, round(k * size / 2 ** 30, 2)] for ch, k in runs],
            "GiB_per_class": {ch: round(sum(k for c2, k in runs if c2 == ch) * size / 2 ** 30, 2)
                              for ch in sorted({r[0] for r in runs})}}


def region_matrix(torch, B, w, dev, layers=16, reps=6):
    """Config 2's fused restore and save, microseconds per layer, for every combination of the HBM region of the K
    plane, the V plane and the staging buffer that the candidates of this process allow (about 220 GiB of 2 GiB
    candidates, classified by tutti_place_classify; `layers` layers rotate so that every launch is cold; staging
    buffers are 128 MiB pieces of two spare candidates of the wanted region)."""
    from paper_2605_03375_amd import placement
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    plane = s.num_blocks * bb
    n_tab = int(w.block_table.size)
    payload = 2 * n_tab * bb
    n_sqe = 2 * ((n_tab * bb + w.chunk_bytes - 1) // w.chunk_bytes)
    free, _ = torch.cuda.mem_get_info()
    n_cand = int(min(112, (free - (12 << 30)) // plane))
    cands = [torch.empty(plane, dtype=torch.uint8, device=dev) for _ in range(n_cand)]
    classes, report = placement.classify_planes(cands, dev)
    by = {c: [i for i in range(n_cand) if classes[i] == c] for c in range(3)}
    L = layers
    geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                head_dim=s.head_dim, elt_bytes=s.elt_bytes)
    cfg = B.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
    d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
    d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
    ext = torch.zeros(L, 32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(L, 2, dtype=torch.int64, device=dev)
    sqe = torch.zeros(L, n_sqe * 64, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    def us_per_layer(pools, stages, fn):
        def train():
            for l in range(L):
                fn(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload, stages[l].data_ptr(), 1, ext[l],
                   tot[l], sqe[l], n_sqe, 0, status)
        train()
        train()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            train()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / L)
        return round(median(ts), 2)

    rows = []
    for ka, kb in ((0, 1), (1, 0), (0, 2), (1, 2), (0, 0), (1, 1), (2, 2)):
        # planes from the front of a class, staging pieces from its last two candidates
        need_a = 2 * L + 2 if ka == kb else L + 2
        if len(by[ka]) < need_a or len(by[kb]) < L + 2:
            continue
        ia = by[ka][:2 * L]
        ib = by[kb][:2 * L]
        pools = [B.make_pool(cands[ia[2 * l if ka == kb else l]], cands[ib[2 * l + 1 if ka == kb else l]], **geom)
                 for l in range(L)]
        for kc in range(3):
            if len(by[kc]) < 2:
                continue
            stages = [cands[c][k * payload:(k + 1) * payload] for c in by[kc][-2:] for k in range(plane // payload)][:L]
            rows.append({"K": "ABC"[ka], "V": "ABC"[kb], "staging": "ABC"[kc],
                         "restore_us": us_per_layer(pools, stages, B.tutti_layer_restore),
                         "save_us": us_per_layer(pools, stages, B.tutti_layer_save)})
            log(f"[bench] region matrix: {rows[-1]}")
    assert int(status.item()) == 0
    return {"workload": "config 2 layer (2048 blocks of 32 KiB, 128 MiB of payload), fused restore / save, us per layer",
            "regions_in_allocation_order": "".join("ABC?"[c] for c in classes), "rounds": report["rounds"],
            "layers_rotating": L, "rows": rows}


def carved_planes(torch, n_layers, plane_bytes, dev, reserve_bytes, place, stage_bytes):
    """placed_planes for planes much smaller than the pieces the driver hands memory out in: 2 GiB buffers are placed
    (K buffer and V buffer of a group in different regions, the group's staging buffer in the third) and every group
    of layers cuts its planes and staging buffers out of them."""
    big = 2 << 30
    plane_al = (plane_bytes + 4095) // 4096 * 4096
    stage_al = (stage_bytes + 4095) // 4096 * 4096
    per = max(1, min(big // plane_al, big // stage_al))
    groups = (n_layers + per - 1) // per
    bplanes, bsame, info, bstages = placed_planes(torch, groups, big, dev, reserve_bytes, place=place,
                                                  stage_bytes=per * stage_al, stage_rotation=3)
    def cut(buf, k, step, size):
        return buf[k * step: k * step + size]
    planes, stages = [], []
    for l in range(min(n_layers, len(bplanes) * per)):
        g, k = divmod(l, per)
        planes.append((cut(bplanes[g][0], k, plane_al, plane_bytes), cut(bplanes[g][1], k, plane_al, plane_bytes)))
        if bstages is not None:
            stages.append(cut(bstages[g], k, stage_al, stage_bytes))
    same = []
    for g, (a, b) in enumerate(bsame):
        for k in range(per):
            same.append((cut(a, k, plane_al, plane_bytes), cut(b, k, plane_al, plane_bytes)))
    info = dict(info, planes_cut_from_buffers_of_GiB=2, layers_per_buffer_pair=per)
    for key in ("layers_with_K_and_V_in_different_regions", "staging_buffers_in_a_third_region"):
        if key in info:                                     # counted in buffer pairs so far
            info[key] = min(len(planes), info[key] * per)
    return planes, same[:len(planes)], info, (stages if bstages is not None else None)


def host_us_per_call(torch, fn, n_calls, reps=7):
    """Host microseconds one call costs: wall time of the enqueueing loop alone, started on an idle stream and not
    waiting for the device (through the Python binding, so ctypes marshalling is in it).  The paper's point is that
    this is constant per layer whatever the number of blocks (sec. 3.2: the CPU launches one I/O kernel per layer)."""
    ts = []
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        ts.append((time.perf_counter() - t0) * 1e6 / n_calls)
    torch.cuda.synchronize()
    return round(median(ts), 2)


def ordered_restore(torch, B, num_blocks, pools, cfg, d_n, d_tab, n_tab, d_fid, stages, payload, n_sqe, dev, reps=5):
    """Config 2's restore again, once in table order (tutti_layer_restore) and once with the blocks visited by
    ascending pool address (tutti_table_order once, then tutti_layer_restore_ordered per layer), back to back on
    the same buffers."""
    L = len(pools)
    ext = torch.zeros(32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    sqe = torch.zeros(max(n_sqe, 1) * 64, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    d_visit = torch.zeros(n_tab, dtype=torch.int32, device=dev)
    work = torch.empty(B.tutti_table_order_work_bytes(num_blocks), dtype=torch.uint8, device=dev)

    def order():
        B.tutti_table_order(num_blocks, d_tab, n_tab, d_visit, work, work.numel(), status)

    def train(ordered):
        for l in range(L):
            if ordered:
                B.tutti_layer_restore_ordered(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload,
                                              stages[l].data_ptr(), 1, ext, tot, sqe, n_sqe, d_visit, 0, status)
            else:
                B.tutti_layer_restore(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload,
                                      stages[l].data_ptr(), 1, ext, tot, sqe, n_sqe, 0, status)

    def timed(fn, per):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / per)
        return median(ts)

    order_us = timed(order, 1)
    plain = timed(lambda: train(False), L)
    ordered = timed(lambda: train(True), L)
    plain2 = timed(lambda: train(False), L)
    assert int(status.item()) == 0
    res = {"table_order_us_per_layer": round(min(plain, plain2), 2), "address_order_us_per_layer": round(ordered, 2),
           "gain_pct": round(100 * (1 - ordered / min(plain, plain2)), 2), "table_order_call_us_once": round(order_us, 2)}
    log(f"[bench] restore, blocks visited by address: {res}")
    return res


def restore_leg(torch, B, w, dev, max_layers, reps=5, place=True):
    """Per-layer tutti_layer_restore of another workload at its real pool size: as many layers resident
    as fit (each with its own planes and staging buffer, so launches stay cold), contents left as
    allocated (timing only; parity for these shapes is in the tests)."""
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    plane_bytes = s.num_blocks * bb
    n_tab = int(w.block_table.size)
    payload = 2 * n_tab * bb
    n_sqe = int(2 * np.sum((w.n_blocks.astype(np.int64) * bb + w.chunk_bytes - 1) // w.chunk_bytes))
    torch.cuda.empty_cache()            # what an earlier leg's allocator cache still holds
    free, _ = torch.cuda.mem_get_info()
    n_stage = 8  # staging buffers rotate (8 x payload is well beyond the 256 MB Infinity Cache)
    L = max(1, min(max_layers, s.num_layers, int((free - (8 << 30) - n_stage * payload) // (2 * plane_bytes))))
    geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                head_dim=s.head_dim, elt_bytes=s.elt_bytes)
    cfg = B.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    if plane_bytes < (1 << 30):
        planes, planes_same, placement_info, layer_stage = carved_planes(
            torch, L, plane_bytes, dev, reserve_bytes=n_stage * payload + (10 << 30), place=place, stage_bytes=payload)
    else:
        planes, planes_same, placement_info, layer_stage = placed_planes(
            torch, L, plane_bytes, dev, reserve_bytes=n_stage * payload + (10 << 30), place=place,
            stage_bytes=payload, stage_rotation=3)
    L = len(planes)
    pools = [B.make_pool(k, v, **geom) for k, v in planes]
    pools_same = [B.make_pool(k, v, **geom) for k, v in planes_same]
    if layer_stage is not None:
        stages = layer_stage[:L]            # per layer: a buffer in the region of neither plane, three per region in turn
    else:
        few = [torch.empty(payload, dtype=torch.uint8, device=dev) for _ in range(min(L, n_stage))]
        stages = [few[l % len(few)] for l in range(L)]
    d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
    d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
    d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
    ext = torch.zeros(w.n_req * 32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    # the table's address order, computed once on the device and used by every layer of the ordered variant
    d_visit = torch.zeros(max(n_tab, 1), dtype=torch.int32, device=dev)
    work = torch.empty(B.tutti_table_order_work_bytes(s.num_blocks), dtype=torch.uint8, device=dev)

    def order():
        B.tutti_table_order(s.num_blocks, d_tab, n_tab, d_visit, work, work.numel(), status)

    def train(ordered=False):
        for l in range(L):
            st = stages[l % len(stages)]
            if ordered:
                B.tutti_layer_restore_ordered(pools[l], cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, st, payload,
                                              st.data_ptr(), 1, ext, tot, sqe, n_sqe, d_visit, 0, status)
            else:
                B.tutti_layer_restore(pools[l], cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, st, payload,
                                      st.data_ptr(), 1, ext, tot, sqe, n_sqe, 0, status)

    def timed(fn, per):
        fn()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / per)
        return median(times)

    def save_train():
        for l in range(L):
            st = stages[l % len(stages)]
            B.tutti_layer_save(pools[l], cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, st, payload, st.data_ptr(), 1, ext,
                               tot, sqe, n_sqe, 0, status)

    def same_train():
        for l, p in enumerate(pools_same):
            st = stages[l % len(stages)]
            B.tutti_layer_restore(p, cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, st, payload, st.data_ptr(), 1, ext,
                                  tot, sqe, n_sqe, 0, status)

    us = timed(train, L)
    us_same = timed(same_train, len(pools_same)) if pools_same else None
    order_us = timed(order, 1)
    us_ordered = timed(lambda: train(True), L)
    us_save = timed(save_train, L)
    host_us = host_us_per_call(torch, train, L, reps=3)
    assert int(status.item()) == 0 and int(tot[1].item()) == n_sqe
    res = {"layers_resident": L, "layers_model": s.num_layers, "pool_blocks": s.num_blocks, "requests": w.n_req,
           "blocks_per_layer": n_tab, "payload_bytes_per_layer": payload, "entries_per_layer": n_sqe,
           "us_per_layer": round(us, 2), "payload_GBps": round(payload / (us * 1e-6) / 1e9, 1),
           "traffic_GBps": round(2 * payload / (us * 1e-6) / 1e9, 1),
           "pct_hbm_peak": round(100 * 2 * payload / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
           "host_us_per_call": host_us,
           "placement": {k: v for k, v in placement_info.items() if k != "rounds"},
           "restore_K_and_V_in_one_region": None if us_same is None else {
               "layers": len(pools_same), "us_per_layer": round(us_same, 2),
               "pct_hbm_peak": round(100 * 2 * payload / (us_same * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)},
           "save": {"us_per_layer": round(us_save, 2),
                    "pct_hbm_peak": round(100 * 2 * payload / (us_save * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)},
           "address_order": {"us_per_layer": round(us_ordered, 2), "gain_pct": round(100 * (1 - us_ordered / us), 2),
                             "table_order_us_once": round(order_us, 2),
                             "pct_hbm_peak": round(100 * 2 * payload / (us_ordered * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)}}
    log(f"[bench] {w.name}: {res}")
    return res


def ring_leg(torch, B, w, pools, planes, cfg, d_n, d_tab, n_tab, d_fid, payload, dev, reps=5):
    """The paper's data path on config 2: per layer, the GPU fills two IOCBs (4096 contexts, one per hit block
    and plane) and tutti_issue_io moves each block between the request's GPU file (an HBM buffer standing in
    for the SSD) and the pool block its SGL descriptor names.  No staging copy."""
    s = w.shape
    L = len(pools)
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    obj = n_tab * bb
    file_stride = 2 * s.num_layers * obj                      # one request, all layers: 4 GiB
    store = torch.empty(file_stride, dtype=torch.uint8, device=dev)
    fs = B.make_filestore(store, file_stride, int(w.file_id[0]), 1)
    nd = 2 * s.num_blocks
    sgls = []
    for l in range(L):
        t = torch.empty(nd * 16, dtype=torch.uint8, device=dev)
        B.tutti_sgl_table_build(pools[l], planes[l][0].data_ptr(), planes[l][1].data_ptr(), 1, t, nd)
        sgls.append(t)
    n_slots = (2 * n_tab + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS
    depth = n_slots * L
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.empty(sq_bytes, dtype=torch.uint8, device=dev)
    cq = torch.empty(cq_bytes, dtype=torch.uint8, device=dev)
    ring = B.make_ring(sq, cq, depth)
    ext = torch.zeros(32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    B.tutti_obj_layout(pools[0], cfg, d_n, 1, ext, tot)

    def train(op, fill=True, issue=True):
        if fill:
            B.tutti_ring_init(ring)
        for l in range(L):
            if fill:
                B.tutti_iocb_fill_direct(ring, l * n_slots, n_slots, pools[l], cfg, ext, 1, d_tab, n_tab, d_fid, l, op,
                                         sgls[l].data_ptr(), 1, status)
            if issue:
                B.tutti_issue_io(ring, l * n_slots, n_slots, sgls[l], nd, sgls[l].data_ptr(), fs, bb, 0, status)

    res = {"contexts_per_layer": 2 * n_tab, "iocbs_per_layer": n_slots, "file_store_bytes": file_stride}
    for label, op in (("save_WRITE", B.OP_WRITE), ("restore_READ", B.OP_READ)):
        train(op)
        torch.cuda.synchronize()
        both, only_io = [], []
        for _ in range(reps):
            a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            a.record()
            train(op)
            b.record()
            torch.cuda.synchronize()
            both.append(a.elapsed_time(b) * 1e3 / L)
            train(op, issue=False)                 # IOCBs are FILLED again
            torch.cuda.synchronize()
            a.record()
            train(op, fill=False)
            c.record()
            torch.cuda.synchronize()
            only_io.append(a.elapsed_time(c) * 1e3 / L)
        one_call = B.tutti_store_layer if op == B.OP_WRITE else B.tutti_retrieve_layer
        fused = []
        for _ in range(reps):
            B.tutti_ring_init(ring)
            torch.cuda.synchronize()
            a, b = (torch.cuda.Event(enable_timing=True) for _ in range(2))
            a.record()
            for l in range(L):
                one_call(ring, l * n_slots, n_slots, pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l,
                         sgls[l].data_ptr(), 1, fs, ext, tot, 0, status)
            b.record()
            torch.cuda.synchronize()
            fused.append(a.elapsed_time(b) * 1e3 / L)
        # the same one-call train (ring initialisation included) as one HIP-graph replay: launch gaps at their smallest
        def one_call_train():
            B.tutti_ring_init(ring)
            for l in range(L):
                one_call(ring, l * n_slots, n_slots, pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l,
                         sgls[l].data_ptr(), 1, fs, ext, tot, 0, status)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                one_call_train()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replay = []
        for _ in range(reps):
            a, b = (torch.cuda.Event(enable_timing=True) for _ in range(2))
            a.record()
            graph.replay()
            b.record()
            torch.cuda.synchronize()
            replay.append(a.elapsed_time(b) * 1e3 / L)
        del graph
        # the two halves: data launches on this stream, every completion on a second stream behind an event, so that
        # the next layer's data kernel does not wait for the completion kernel of the layer before it
        issue = B.tutti_store_layer_issue if op == B.OP_WRITE else B.tutti_retrieve_layer_issue
        comp = torch.cuda.Stream()
        main = torch.cuda.current_stream()
        halves = []
        for _ in range(reps):
            B.tutti_ring_init(ring)
            torch.cuda.synchronize()
            a, b = (torch.cuda.Event(enable_timing=True) for _ in range(2))
            a.record()
            for l in range(L):
                issue(ring, l * n_slots, n_slots, pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l,
                      sgls[l].data_ptr(), 1, fs, ext, tot, 0, status)
                ev = torch.cuda.Event()
                ev.record(main)
                comp.wait_event(ev)
                B.tutti_complete_io(ring, l * n_slots, n_slots, comp)
            main.wait_stream(comp)             # the train has ended when its last completion has
            b.record()
            torch.cuda.synchronize()
            halves.append(a.elapsed_time(b) * 1e3 / L)
        # a train whose launches each complete the layer before them (no completion kernel but the last one)
        chained_call = B.tutti_store_layer_chained if op == B.OP_WRITE else B.tutti_retrieve_layer_chained
        chained = []
        for _ in range(reps):
            B.tutti_ring_init(ring)
            torch.cuda.synchronize()
            a, b = (torch.cuda.Event(enable_timing=True) for _ in range(2))
            a.record()
            for l in range(L):
                chained_call(ring, l * n_slots, n_slots, (l - 1) * n_slots if l else 0, n_slots if l else 0, pools[l],
                             cfg, d_n, 1, d_tab, n_tab, d_fid, l, sgls[l].data_ptr(), 1, fs, ext, tot, 0, status)
            B.tutti_complete_io(ring, (L - 1) * n_slots, n_slots)
            b.record()
            torch.cuda.synchronize()
            chained.append(a.elapsed_time(b) * 1e3 / L)
        done_now = int(cq[:4].view(torch.int32)[0].item())
        assert done_now == L * n_slots, (done_now, L * n_slots)
        # the entry-driven issue in the same way: IOCBs already FILLED, every issue completes the one before it
        io_chained = []
        for _ in range(reps):
            train(op, issue=False)
            torch.cuda.synchronize()
            a, b = (torch.cuda.Event(enable_timing=True) for _ in range(2))
            a.record()
            for l in range(L):
                B.tutti_issue_io_chained(ring, l * n_slots, n_slots, (l - 1) * n_slots if l else 0, n_slots if l else 0,
                                         sgls[l], nd, sgls[l].data_ptr(), fs, bb, 0, status)
            B.tutti_complete_io(ring, (L - 1) * n_slots, n_slots)
            b.record()
            torch.cuda.synchronize()
            io_chained.append(a.elapsed_time(b) * 1e3 / L)
        us, us_io, us_one, us_ch = median(both), median(only_io), median(fused), median(chained)
        res[label] = {"us_per_layer_chained_completions": round(us_ch, 2),
                      "pct_hbm_peak_chained": round(100 * 2 * payload / (us_ch * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
                      "us_per_layer_completions_on_second_stream": round(median(halves), 2),
"us_per_layer_fill_plus_io": round(us, 2), "us_per_layer_issue_io": round(us_io, 2),
                      "us_per_layer_issue_io_chained": round(median(io_chained), 2),
                      "us_per_layer_one_call": round(us_one, 2),
                      "us_per_layer_one_call_graph_replay": round(median(replay), 2),
                      "pct_hbm_peak_one_call": round(100 * 2 * payload / (us_one * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
                      "payload_GBps": round(payload / (us * 1e-6) / 1e9, 1),
                      "traffic_GBps_issue_io": round(2 * payload / (us_io * 1e-6) / 1e9, 1),
                      "pct_hbm_peak_issue_io": round(100 * 2 * payload / (us_io * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)}
    done = int(cq[:4].view(torch.int32)[0].item())
    assert int(status.item()) == 0 and done == depth, (int(status.item()), done, depth)
    log(f"[bench] rings: {res}")
    return res


def hnd_rows(torch, B, w, planes, stages, dev, layers=8, reps=5):
    """Head-major pools ([h][T][d] blocks) of config 2's block size (32 KiB, 16 tokens) with (token, head) rows of
    256, 128, 64 and 32 bytes: tutti_obj_unpack / tutti_obj_pack alone, once moved 16 bytes per lane straight
    between the two orders and once through token tiles in LDS (the choice forced with the measurement library's
    switch; the product library takes LDS for rows shorter than 128 bytes).  Random table of 2048 blocks."""
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    n_tab = int(w.block_table.size)
    payload = 2 * n_tab * bb
    L = min(layers, len(stages), len(planes))
    planes = planes[:L]                 # the bench's own planes (their contents are not needed any more)
    d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
    d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
    ext = torch.zeros(32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    cfg = B.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    res = {}
    B.use_bench_library(True)
    try:
        for heads, dim in ((8, 128), (16, 64), (32, 32), (64, 16)):
            row = dim * s.elt_bytes
            geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=heads, head_dim=dim,
                        elt_bytes=s.elt_bytes, pool_layout=1)
            pools = [B.make_pool(k, v, **geom) for k, v in planes]
            B.tutti_obj_layout(pools[0], cfg, d_n, 1, ext, tot)
            r = {}
            for mode, label in ((1, "direct"), (2, "lds")):
                B.tutti_set_hnd_mode(mode)
                for fn, name in ((B.tutti_obj_unpack, "unpack"), (B.tutti_obj_pack, "pack")):
                    def train():
                        for l in range(L):
                            fn(pools[l], cfg, ext, 1, d_tab, n_tab, stages[l], payload, 0, status)
                    train()
                    torch.cuda.synchronize()
                    ts = []
                    for _ in range(reps):
                        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        a.record()
                        train()
                        b.record()
                        torch.cuda.synchronize()
                        ts.append(a.elapsed_time(b) * 1e3 / L)
                    r[f"{label}_{name}_us"] = round(median(ts), 2)
            r["product_choice"] = "lds" if row < 128 else "direct"
            res[f"row_{row}B ({heads} heads x {dim})"] = r
            log(f"[bench] head-major rows of {row} B: {r}")
    finally:
        B.tutti_set_hnd_mode(0)
        B.use_bench_library(False)
    assert int(status.item()) == 0
    return res


def pinned_leg(torch, B, pools, cfg, d_n, d_tab, n_tab, d_fid, payload, n_sqe, dev, layers=4, reps=3):
    """Config 2's per-layer restore and pack with the staging buffer in pinned host memory: the copy
    crosses the host link, so this is NOT an HBM figure and never the headline value."""
    L = min(layers, len(pools))
    stages = [torch.empty(payload, dtype=torch.uint8, pin_memory=True) for _ in range(L)]
    ext = torch.zeros(32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    B.tutti_obj_layout(pools[0], cfg, d_n, 1, ext, tot)

    def pack():
        for l in range(L):
            B.tutti_obj_pack(pools[l], cfg, ext, 1, d_tab, n_tab, stages[l], payload, 0, status)

    def restore():
        for l in range(L):
            B.tutti_layer_restore(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, stages[l], payload,
                                  stages[l].data_ptr(), 1, ext, tot, sqe, n_sqe, 0, status)

    res = {"layers": L, "note": "staging buffer in pinned host memory: host-link bound, not an HBM figure"}
    for label, fn in (("pack", pack), ("restore", restore)):
        fn()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / L)
        us = median(times)
        res[label] = {"us_per_layer": round(us, 1), "payload_GBps": round(payload / (us * 1e-6) / 1e9, 2)}
    assert int(status.item()) == 0
    log(f"[bench] pinned-host staging: {res}")
    return res


def scatter_floor(torch, B, w, stages, nbytes, dev, n_buf=6, reps=5):
    """What the memory system gives for config 2's access pattern with nothing else in the kernel: a
    128 MiB contiguous buffer against 4096 pieces of 32 KiB placed by the same block table inside a 4 GiB
    span (K plane then V plane), written (the unpack's pattern) or read (the pack's)."""
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    span = 2 * s.num_blocks * bb
    perm = np.concatenate([w.block_table, w.block_table + s.num_blocks]).astype(np.uint32)
    d_perm = torch.from_numpy(perm.view(np.int32)).to(dev)
    bufs = [torch.empty(span, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    res = {"pieces": int(perm.size), "piece_bytes": bb, "span_bytes": span}
    for label, wr in (("scattered_writes", 1), ("scattered_reads", 0)):
        def run():
            for i in range(len(stages)):
                B.tutti_scatter_baseline(bufs[i % n_buf], span, stages[i], nbytes, d_perm, bb, wr)
        if not wr:   # do not clobber the staging buffers the parity check reads later: reads go to a scratch copy
            scratch = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]

            def run():  # noqa: F811
                for i in range(len(stages)):
                    B.tutti_scatter_baseline(bufs[i % n_buf], span, scratch[i % 4], nbytes, d_perm, bb, wr)
        run()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            run()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / len(stages))
        us = median(times)
        res[label] = {"us": round(us, 2), "traffic_GBps": round(2 * nbytes / (us * 1e-6) / 1e9, 1),
                      "pct_hbm_peak": round(100 * 2 * nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)}
    return res


def scatter_sweep(torch, B, stages, nbytes, dev, span=2 << 30, n_buf=6, reps=3):
    """tutti_scatter_baseline at every granularity from 4 KiB to 4 MiB: 128 MiB contiguous against pieces
    placed inside a 2 GiB span at random, in sorted order, or contiguously; microseconds per 128 MiB."""
    rng = np.random.default_rng(1)
    bufs = [torch.empty(span, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    scratch = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]
    res = {}
    gran = 4096
    while gran <= (4 << 20):
        n = nbytes // gran
        perms = {"random": rng.permutation(span // gran)[:n]}
        perms["sorted"] = np.sort(perms["random"])
        perms["contiguous"] = np.arange(n)
        row = {}
        for order, p in perms.items():
            d_perm = torch.from_numpy(p.astype(np.uint32).view(np.int32)).to(dev)
            for label, wr in (("writes", 1), ("reads", 0)):
                def run():
                    for i in range(len(stages)):
                        B.tutti_scatter_baseline(bufs[i % n_buf], span, scratch[i % 4] if not wr else stages[i], nbytes,
                                                 d_perm, gran, wr)
                run()
                torch.cuda.synchronize()
                ts = []
                for _ in range(reps):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    run()
                    b.record()
                    torch.cuda.synchronize()
                    ts.append(a.elapsed_time(b) * 1e3 / len(stages))
                row[f"{order}_{label}_us"] = round(median(ts), 2)
        res[str(gran)] = row
        log(f"[bench] scatter sweep gran {gran}: {row}")
        gran *= 2
    return res


def scatter_orders(torch, B, stages, nbytes, dev, gran=32768, span=4 << 30, n_buf=4, reps=5):
    """Does the ORDER in which scattered 32 KiB pieces are visited matter?  The same random set of pieces visited
    at random, ascending, or dealt round-robin over the residues of the piece index mod M (so that pieces in flight
    together differ in the address bits just above the piece size), and regular strides for comparison."""
    rng = np.random.default_rng(1)
    n = nbytes // gran
    slots = span // gran
    ids = rng.permutation(slots)[:n]

    def dealt(M):
        buckets = [list(ids[ids % M == r]) for r in range(M)]
        out = []
        while any(buckets):
            for b in buckets:
                if b:
                    out.append(b.pop())
        return np.array(out)

    orders = {"random": ids, "ascending": np.sort(ids), "contiguous": np.arange(n)}
    for S in (2, 32, 1024):
        orders[f"stride_{S}_pieces"] = (np.arange(n) * S) % slots + (np.arange(n) * S) // slots
    for M in (8, 32, 256):
        orders[f"dealt_mod_{M}"] = dealt(M)
    # whole aligned regions taken at random, their pieces visited in random order: the placement keeps every
    # neighbour, the order keeps none
    for region in (1 << 20, 4 << 20, 32 << 20):
        per = region // gran
        starts = rng.permutation(slots // per)[: n // per]
        orders[f"random_order_inside_{region >> 20}MiB_regions"] = rng.permutation(
            (starts[:, None] * per + np.arange(per)[None, :]).reshape(-1))
    bufs = [torch.empty(span, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    scratch = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]
    res = {}
    for name, p in orders.items():
        assert len(set(p.tolist())) == n and int(p.max()) < slots
        d_perm = torch.from_numpy(p.astype(np.uint32).view(np.int32)).to(dev)
        row = {}
        for label, wr in (("writes_us", 1), ("reads_us", 0)):
            def run():
                for i in range(len(stages)):
                    B.tutti_scatter_baseline(bufs[i % n_buf], span, scratch[i % 4] if not wr else stages[i], nbytes,
                                             d_perm, gran, wr)
            run()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) * 1e3 / len(stages))
            row[label] = round(median(ts), 2)
        res[name] = row
        log(f"[bench] scatter order {name}: {row}")
    return res


def copy_ceiling(torch, B, stages, nbytes, dev, reps=5):
    """Same-size contiguous copy with the same access shape, rotating over cold sources."""
    dsts = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]
    for i, s in enumerate(stages):
        B.tutti_copy_baseline(dsts[i % 4], s, nbytes)
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i, s in enumerate(stages):
            B.tutti_copy_baseline(dsts[i % 4], s, nbytes)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) * 1e3 / len(stages))
    us = median(times)
    # the runtime's own device-to-device copy of the same buffers, for reference (torch's copy_ of a
    # contiguous same-device tensor is a hipMemcpyAsync)
    rt = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i, s in enumerate(stages):
            dsts[i % 4].copy_(s, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        rt.append(a.elapsed_time(b) * 1e3 / len(stages))
    return {"bytes": nbytes, "us_per_copy": round(us, 2), "traffic_GBps": round(2 * nbytes / (us * 1e-6) / 1e9, 1),
            "pct_hbm_peak": round(100 * 2 * nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
            "runtime_d2d_copy_us": round(median(rt), 2)}


def sqe_rate(torch, B, W, dev, reps=50):
    """Entries built per second on config 3's batch of 64 requests, per-chunk and per-block."""
    res = {}
    for label, chunk in (("chunk_2MiB", 2 << 20), ("per_block_32KiB", 32768)):
        w = W.batch64_zipf(chunk_bytes=chunk)
        s = w.shape
        geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                    head_dim=s.head_dim, elt_bytes=s.elt_bytes)
        pool = B.make_pool(4096, 4096, **geom)  # entries are arithmetic only: the planes are never touched
        cfg = B.make_cfg(w.align, chunk, s.num_layers)
        d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
        d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
        ext = torch.zeros(w.n_req * 32, dtype=torch.uint8, device=dev)
        tot = torch.zeros(2, dtype=torch.int64, device=dev)
        B.tutti_obj_layout(pool, cfg, d_n, w.n_req, ext, tot)
        torch.cuda.synchronize()
        n_sqe = int(tot[1].item())
        sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=dev)
        for _ in range(3):
            B.tutti_sqe_build(pool, cfg, ext, w.n_req, d_fid, 3, B.OP_READ, 1 << 40, 1, sqe, n_sqe)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            B.tutti_sqe_build(pool, cfg, ext, w.n_req, d_fid, i % s.num_layers, B.OP_READ, 1 << 40, 1, sqe, n_sqe)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        res[label] = {"entries_per_layer": n_sqe, "us_per_launch": round(us, 2),
                      "sqes_per_s": round(n_sqe / (us * 1e-6), 0),
                      "regime": "launch-latency bound" if us < 20 else "kernel bound"}
    return res


def direct_rate(torch, B, W, dev, reps=50):
    """Direct-to-block mode (no staging copy): mapping table build for config 2's pool and per-block
    entries per second for config 3's batch (one entry per hit block and plane)."""
    w = W.batch64_zipf(chunk_bytes=32768)
    s = w.shape
    geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                head_dim=s.head_dim, elt_bytes=s.elt_bytes)
    pool = B.make_pool(4096, 4096, **geom)  # arithmetic only
    cfg = B.make_cfg(w.align, 32768, s.num_layers)
    d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
    d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
    d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
    ext = torch.zeros(w.n_req * 32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    B.tutti_obj_layout(pool, cfg, d_n, w.n_req, ext, tot)
    n_desc = 2 * s.num_blocks
    sgl = torch.zeros(n_desc * 16, dtype=torch.uint8, device=dev)
    n_sqe = 2 * int(w.block_table.size)
    sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=dev)
    E = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    res = {}
    for label, fn, n in (
            ("sgl_table", lambda i: B.tutti_sgl_table_build(pool, 1 << 40, 1 << 41, 1, sgl, n_desc), n_desc),
            ("entries", lambda i: B.tutti_sqe_build_direct(pool, cfg, ext, w.n_req, d_tab, d_tab.numel(), d_fid,
                                                           i % s.num_layers, B.OP_READ, sgl.data_ptr(), 1, sqe, n_sqe),
             n_sqe)):
        for i in range(3):
            fn(i)
        a, b = E(), E()
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        res[label] = {"count": n, "us_per_launch": round(us, 2), "per_s": round(n / (us * 1e-6), 0)}
    return res


def big_entry_rate(torch, B, dev, n_req=2048, blocks_per_req=512, reps=20):
    """Entries per second once the count is large enough to leave the launch-latency regime: 2048 requests
    x 512 blocks = 2,097,152 per-block entries (128 MiB of entries) in one tutti_sqe_build_direct launch."""
    rng = np.random.default_rng(7)
    n_tab = n_req * blocks_per_req
    num_blocks = 2 * n_tab
    geom = dict(num_blocks=num_blocks, block_tokens=16, num_kv_heads=8, head_dim=128, elt_bytes=2)
    pool = B.make_pool(4096, 4096, **geom)  # arithmetic only
    cfg = B.make_cfg(4096, 32768, 32)
    d_n = torch.full((n_req,), blocks_per_req, dtype=torch.int32, device=dev)
    d_tab = torch.from_numpy(rng.permutation(num_blocks)[:n_tab].astype(np.uint32).view(np.int32)).to(dev)
    d_fid = torch.arange(n_req, dtype=torch.int32, device=dev)
    ext = torch.zeros(n_req * 32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    B.tutti_obj_layout(pool, cfg, d_n, n_req, ext, tot)
    n_sqe = 2 * n_tab
    sqes = [torch.empty(n_sqe * 64, dtype=torch.uint8, device=dev) for _ in range(3)]  # 3 x 128 MiB: cold writes
    for i in range(3):
        B.tutti_sqe_build_direct(pool, cfg, ext, n_req, d_tab, n_tab, d_fid, i, B.OP_READ, 1 << 40, 1, sqes[i], n_sqe)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(reps):
        B.tutti_sqe_build_direct(pool, cfg, ext, n_req, d_tab, n_tab, d_fid, i % 32, B.OP_READ, 1 << 40, 1, sqes[i % 3],
                                 n_sqe)
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / reps
    return {"requests": n_req, "entries": n_sqe, "us_per_launch": round(us, 2),
            "sqes_per_s": round(n_sqe / (us * 1e-6), 0), "entry_write_GBps": round(64 * n_sqe / (us * 1e-6) / 1e9, 1),
            "regime": "per-entry dependent chain (owner walk in LDS, table word, file id) hidden by occupancy and "
                      "one-entry pipelining; compare entry_write_GBps with chip_stream_ceilings.write"}


def per_cu_limits(torch, B, dev, nbytes=256 << 20, budgets=(8, 32, 128, 0), reps=3, n_buf=4):
    """What B compute units (0 = the chip) move when they only read, only write, or copy: GB/s of memory traffic,
    in total and per budgeted CU.  The budgeted restore is compared with the copy line."""
    src = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 256) for _ in range(n_buf)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    acc = torch.zeros(4 * B.STREAM_SLOTS, dtype=torch.int32, device=dev)
    cus = B.tutti_cu_count()
    res = {}
    for budget in budgets:
        row = {}
        for label, traffic, fn in (("read", nbytes, lambda i: B.tutti_stream_baseline(src[i], nbytes, False, acc, budget)),
                                   ("write", nbytes, lambda i: B.tutti_stream_baseline(dst[i], nbytes, True, None, budget)),
                                   ("copy", 2 * nbytes, lambda i: B.tutti_copy_baseline(dst[i], src[i], nbytes, budget))):
            for i in range(n_buf):
                fn(i)
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for i in range(n_buf):
                    fn(i)
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) * 1e-3 / n_buf)
            gbps = traffic / median(ts) / 1e9
            row[label] = {"traffic_GBps": round(gbps, 1), "per_cu_GBps": round(gbps / (budget or cus), 1)}
        res[str(budget)] = row
        log(f"[bench] per-CU limits, budget {budget}: {row}")
    return res


def corun_sweep(torch, B, restore_layers, L, payload_layer, dev, gemm_iters=60, reps=3, gemm_n=(4096, 4096, 4096),
                budgets=(8, 16, 32, 64, 0), domains=(8, 16, 32, 64)):
    """Config 5: restore under a CU budget (or on a CU-masked stream) while a bf16 GEMM loops on another stream.

    gemm_n = (M, N, K).  Each figure is taken under FULL overlap: to time the GEMM, a restore loop long enough
    to outlast it is queued first on the other stream (and the other way round), and the events are checked
    afterwards to confirm the background work was still running when the measured loop ended.
    Rows "budget B": cu_budget = B on an ordinary stream (B workgroups of 1024 threads: bounds occupancy, not
    placement).  Rows "domain B": cu_budget = 0 on a stream from tutti_io_domain_create(B) (the hardware
    dispatches the launch to the first B compute units only).
    """
    M, N, K = gemm_n
    a = torch.randn(M, K, dtype=torch.bfloat16, device=dev)
    b = torch.randn(K, N, dtype=torch.bfloat16, device=dev)
    side = torch.cuda.Stream()
    E = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731

    def gemm_loop(n):
        e0, e1 = E(), E()
        with torch.cuda.stream(side):
            e0.record(side)
            for _ in range(n):
                torch.matmul(a, b)
            e1.record(side)
        return e0, e1

    def restore_loop(stream, budget, trains):
        e0, e1 = E(), E()
        with torch.cuda.stream(stream):
            e0.record(stream)
            for _ in range(trains):
                restore_layers(budget, stream)
            e1.record(stream)
        return e0, e1

    gemm_loop(10)
    torch.cuda.synchronize()
    out = {}
    rows_spec = [(f"budget {x}", x, None) for x in budgets] + [(f"domain {x}", 0, x) for x in domains]
    for label, budget, domain in rows_spec:
        handle = None
        if domain is None:
            main = torch.cuda.Stream()
        else:
            try:
                handle = B.tutti_io_domain_create(domain)
            except B.TuttiError as e:
                out[label] = {"skipped": f"the runtime refuses the compute-unit mask: {e}"}
                continue
            main = torch.cuda.ExternalStream(handle)
        rows = []
        for _ in range(reps):
            g0, g1 = gemm_loop(gemm_iters)
            torch.cuda.synchronize()
            gemm_solo = g0.elapsed_time(g1) / gemm_iters                      # ms per GEMM
            r0, r1 = restore_loop(main, budget, 1)
            torch.cuda.synchronize()
            train_solo = r0.elapsed_time(r1)                                  # ms per layer train
            # (a) GEMM timed while restores run in the background for ~4x as long (12x on a second try, should the
            # background have ended first)
            for factor in (4, 12):
                bg_trains = max(2, int(factor * gemm_solo * gemm_iters / train_solo) + 1)
                r0, r1 = restore_loop(main, budget, bg_trains)
                g0, g1 = gemm_loop(gemm_iters)
                torch.cuda.synchronize()
                gemm_co = g0.elapsed_time(g1) / gemm_iters
                ok_a = g1.elapsed_time(r1) > 0                                # restores ended after the GEMMs
                if ok_a:
                    break
            # (b) restore timed while GEMMs run in the background for ~4x (12x) as long
            trains = max(1, int(gemm_solo * gemm_iters / train_solo))
            for factor in (4, 12):
                bg_gemms = int(factor * trains * train_solo / gemm_solo) + 1
                g0, g1 = gemm_loop(bg_gemms)
                r0, r1 = restore_loop(main, budget, trains)
                torch.cuda.synchronize()
                train_co = r0.elapsed_time(r1) / trains
                ok_b = r1.elapsed_time(g1) > 0
                if ok_b:
                    break
            # (c) both loops, sized to last equally long alone, started together: time until both have ended, against
            # the sum of their solo times (a figure that needs no overlap check: 1.0 = no better than taking turns)
            e0, e1 = E(), E()
            e0.record(main)
            side.wait_event(e0)
            restore_loop(main, budget, trains)
            gemm_loop(gemm_iters)
            main.wait_stream(side)
            e1.record(main)
            torch.cuda.synchronize()
            pair = e0.elapsed_time(e1) / (gemm_solo * gemm_iters + trains * train_solo)
            rows.append((gemm_solo, gemm_co, train_solo / L, train_co / L, ok_a, ok_b, pair))
        gs, gc, rs, rc = (median([r[i] for r in rows]) for i in range(4))
        out[label] = {"gemm_ms_solo": round(gs, 4), "gemm_ms_corun": round(gc, 4),
                      "gemm_slowdown": round(gc / gs, 3),
                      "restore_us_per_layer_solo": round(rs * 1e3, 1),
                      "restore_us_per_layer_corun": round(rc * 1e3, 1),
                      "restore_payload_GBps_solo": round(payload_layer / (rs * 1e-3) / 1e9, 1),
                      "restore_payload_GBps_corun": round(payload_layer / (rc * 1e-3) / 1e9, 1),
                      "restore_slowdown": round(rc / rs, 3),
                      "both_together_vs_taking_turns": round(median([r[6] for r in rows]), 3),
                      # a figure taken while the other side had already finished is not a co-run figure
                      "gemm_figure_under_overlap": all(r[4] for r in rows),
                      "restore_figure_under_overlap": all(r[5] for r in rows)}
        log(f"[bench] corun gemm {M}x{N}x{K} {label}: {out[label]}")
        if handle is not None:
            torch.cuda.synchronize()
            B.tutti_io_domain_destroy(handle)
    return out


def slack_lut(torch, B, w, pools, planes, cfg, d_tab, d_fid, dev, budgets=(8, 16, 32, 64, 0), iocbs=(1, 2, 4), reps=3):
    """The offline profile of the I/O kernels that the slack-aware scheduler looks launch sizes up in (sec. 3.3):
    duration of tutti_retrieve_layer / tutti_store_layer for 1, 2 and 4 IOCBs (2048 contexts = 1024 blocks of K
    and V each) under every CU budget, config 2's pool and block shape, alone on the GPU.  The rows are what
    tutti_iocbs_for_slack / tutti_budget_for_slack take (tutti_io_profile)."""
    s = w.shape
    L = min(len(pools), 8)
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    rng = np.random.default_rng(w.seed + 9)
    max_blocks = max(iocbs) * B.IOCB_SLOTS // 2
    table = rng.permutation(s.num_blocks)[:max_blocks].astype(np.uint32)
    d_table = torch.from_numpy(table.view(np.int32)).to(dev)
    file_stride = 2 * L * max_blocks * bb
    store = torch.empty(file_stride, dtype=torch.uint8, device=dev)
    fs = B.make_filestore(store, file_stride, int(w.file_id[0]), 1)
    depth = max(iocbs) * L
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.empty(sq_bytes, dtype=torch.uint8, device=dev)
    cq = torch.empty(cq_bytes, dtype=torch.uint8, device=dev)
    ring = B.make_ring(sq, cq, depth)
    ext = torch.zeros(32, dtype=torch.uint8, device=dev)
    tot = torch.zeros(2, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    cfg_l = B.make_cfg(cfg.align, cfg.chunk_bytes, L)
    rows = []
    for n_io in iocbs:
        n_blk = n_io * B.IOCB_SLOTS // 2
        d_n = torch.tensor([n_blk], dtype=torch.int32, device=dev)
        for budget in budgets:
            us = {}
            for label, fn in (("write", B.tutti_store_layer), ("read", B.tutti_retrieve_layer)):
                ts = []
                for rep in range(reps + 1):
                    B.tutti_ring_init(ring)
                    torch.cuda.synchronize()
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    for l in range(L):
                        fn(ring, l * n_io, n_io, pools[l], cfg_l, d_n, 1, d_table, n_blk, d_fid, l, 0, 1, fs, ext, tot,
                           budget, status)
                    b.record()
                    torch.cuda.synchronize()
                    if rep:
                        ts.append(a.elapsed_time(b) * 1e3 / L)
                us[label] = median(ts)
            rows.append({"cu_budget": budget, "n_iocbs": n_io, "read_us": round(us["read"], 2),
                         "write_us": round(us["write"], 2)})
    assert int(status.item()) == 0
    # what the lookups answer for a few slack windows (the runtime's question before each layer)
    prof, n = B.make_io_profile([(r["cu_budget"], r["n_iocbs"], r["read_us"], r["write_us"]) for r in rows])
    examples = []
    for slack_us, budget in ((100.0, 64), (300.0, 32), (300.0, 8), (1000.0, 16)):
        examples.append({"slack_us": slack_us, "cu_budget": budget,
                         "read_iocbs_that_fit": B.tutti_iocbs_for_slack(prof, n, budget, B.OP_READ, slack_us),
                         "smallest_budget_for_2_read_iocbs": B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, slack_us, 64)})
    res = {"made_by": "python bench.py --write-lut <this file>   (on one MI355X; the same table is in the bench line as slack_lut)",
           "workload": "config 2 pool and block shape (32 KiB blocks; one IOCB = 1024 blocks of K and of V = 64 MiB)",
           "what": "tutti_retrieve_layer (read_us) / tutti_store_layer (write_us), completion kernel included, "
                   "microseconds per call, alone on the GPU; cu_budget 0 = whole GPU",
           "rows": rows, "lookups": examples}
    log(f"[bench] slack table: {res}")
    return res


def length_sweep(torch, B, W, pools, cfg, dev, lengths=(1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072), reps=5):
    """Config 2's shape at prefix lengths from 1K to 128K tokens (the range of the paper's raw-bandwidth ablation,
    sec. 4): per-layer restore and save over all resident layers, as eager launches and as one HIP-graph replay
    of the whole layer train (which removes the host's launch cost but not the kernels' own start-up)."""
    L = len(pools)
    n_stage = 8
    out = {}
    for T in lengths:
        w = W.llama8b_32k(tokens=T)
        s = w.shape
        bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
        n_tab = int(w.block_table.size)
        payload = 2 * n_tab * bb
        n_sqe = 2 * ((n_tab * bb + w.chunk_bytes - 1) // w.chunk_bytes)
        stages = [torch.empty(payload, dtype=torch.uint8, device=dev) for _ in range(n_stage)]
        d_n = torch.from_numpy(w.n_blocks.view(np.int32)).to(dev)
        d_tab = torch.from_numpy(w.block_table.view(np.int32)).to(dev)
        d_fid = torch.from_numpy(w.file_id.view(np.int32)).to(dev)
        ext = torch.zeros(32, dtype=torch.uint8, device=dev)
        tot = torch.zeros(2, dtype=torch.int64, device=dev)
        sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=dev)
        status = torch.zeros(1, dtype=torch.int32, device=dev)

        def train(fn):
            for l in range(L):
                st = stages[l % n_stage]
                fn(pools[l], cfg, d_n, 1, d_tab, n_tab, d_fid, l, st, payload, st.data_ptr(), 1, ext, tot, sqe, n_sqe, 0,
                   status)

        row = {"blocks": n_tab, "payload_bytes_per_layer": payload}
        for label, fn in (("restore", B.tutti_layer_restore), ("save", B.tutti_layer_save)):
            train(fn)
            torch.cuda.synchronize()
            eager = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                train(fn)
                b.record()
                torch.cuda.synchronize()
                eager.append(a.elapsed_time(b) * 1e3 / L)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    train(fn)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            replay = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                graph.replay()
                b.record()
                torch.cuda.synchronize()
                replay.append(a.elapsed_time(b) * 1e3 / L)
            del graph
            us_e, us_g = median(eager), median(replay)
            best = min(us_e, us_g)
            pct = 100 * 2 * payload / (best * 1e-6) / 1e9 / HBM_PEAK_GBPS
            # against the time the bytes alone would take at the rate of the largest size
            row[label] = {"us_per_layer_eager": round(us_e, 2), "us_per_layer_graph": round(us_g, 2),
                          "payload_GBps": round(payload / (best * 1e-6) / 1e9, 1), "pct_hbm_peak": round(pct, 2)}
        assert int(status.item()) == 0
        out[str(T)] = row
        log(f"[bench] prefix {T} tokens: {row}")
        del stages
    # regime of each point: how much of the time is the bytes moving at the rate the longest prefix reaches
    for label in ("restore", "save"):
        top = max(out[str(T)][label]["payload_GBps"] for T in lengths)
        for T in lengths:
            r = out[str(T)][label]
            share = r["payload_GBps"] / top
            r["regime"] = ("bandwidth bound" if share >= 0.9 else
                           "transition (launch start-up and tail still visible)" if share >= 0.5 else
                           "launch-latency bound")
    out["context"] = ("the paper's retrieve bandwidth over the same lengths is bound by its SSDs (at most 25.9 GB/s on "
                      "its 4-SSD H100 box, sec. 4); quoted as context only")
    return out


def visit_order(torch, B, W, dev, reps=5):
    """Would it pay to visit the blocks of a restore in the order of their pool addresses instead of token order?
    (A one-off argsort of the block table, reused by every layer, would make that free per layer.)  The tables of
    configs 2, 3 and 4 as scattered writes of 32 KiB pieces (K plane then V plane of one layer), in table order
    and sorted by address, with the kernel that has the product's access shape and nothing else in it."""
    res = {}
    for name, w in (("config2", W.llama8b_32k()), ("config3", W.batch64_zipf()), ("config4", W.llama70b_128k())):
        s = w.shape
        bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
        span = 2 * s.num_blocks * bb
        perm = np.concatenate([w.block_table, w.block_table + s.num_blocks]).astype(np.uint32)
        nbytes = int(perm.size) * bb
        bufs = [torch.empty(span, dtype=torch.uint8, device=dev) for _ in range(3)]
        src = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(2)]
        row = {"pieces": int(perm.size), "pool_blocks": s.num_blocks,
               "fill": round(w.block_table.size / s.num_blocks, 3)}
        for order, p in (("table_order", perm), ("address_order", np.sort(perm))):
            d_perm = torch.from_numpy(p.view(np.int32)).to(dev)

            def run():
                for i in range(6):
                    B.tutti_scatter_baseline(bufs[i % 3], span, src[i % 2], nbytes, d_perm, bb, 1)
            run()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) * 1e3 / 6)
            row[f"{order}_us"] = round(median(ts), 2)
        row["gain_pct"] = round(100 * (1 - row["address_order_us"] / row["table_order_us"]), 2)
        res[name] = row
        log(f"[bench] visit order {name}: {row}")
        del bufs, src
    return res


def scatter_shapes(torch, B, w, stages, nbytes, dev, n_buf=6, reps=5):
    """Config 2's own table (4096 pieces of 32 KiB inside the 4 GiB of a layer's K and V planes) moved by every
    shape of tutti_scatter_baseline: would dealing the same bytes to the wavefronts differently, or another
    cache policy, suit the memory system better than the product's wavefront-per-4-KiB with nt accesses?"""
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    span = 2 * s.num_blocks * bb
    perm = np.concatenate([w.block_table, w.block_table + s.num_blocks]).astype(np.uint32)
    d_perm = torch.from_numpy(perm.view(np.int32)).to(dev)
    bufs = [torch.empty(span, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    scratch = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]
    res = {}
    for shape in B.SCATTER_SHAPES:
        row = {}
        for label, wr in (("scattered_writes_us", 1), ("scattered_reads_us", 0)):
            def run():
                for i in range(len(stages)):
                    B.tutti_scatter_baseline(bufs[i % n_buf], span, scratch[i % 4], nbytes, d_perm, bb, wr, shape)
            run()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) * 1e3 / len(stages))
            row[label] = round(median(ts), 2)
        res[shape] = row
        log(f"[bench] scatter shape {shape}: {row}")
    return res


def cpu_baseline(torch, W, w, plane0, pristine, stage0, geom, payload_layer, budget_s=8.0):
    """The CPU oracle on layer 0 of the same workload: pack + restore of its 2048 blocks, on the host copy
    of the planes taken before any kernel ran; single thread, then all cores of the affinity mask.
    Also a free full-size parity check: after all the timed save + restore steps the pool must still hold
    those bytes, and the GPU's staging buffer of layer 0 must equal what the oracle packs from them."""
    from oracle import tutti_oracle as orc
    k_host, v_host = pristine
    unchanged = bool(np.array_equal(plane0[0].cpu().numpy(), k_host) and np.array_equal(plane0[1].cpu().numpy(), v_host))
    assert unchanged, "layer 0 of the pool changed under save + restore"
    gpu_stage = stage0.cpu().numpy()
    pool = orc.make_pool(k_host, v_host, **geom)
    cfg = orc.make_cfg(w.align, w.chunk_bytes, w.shape.num_layers)
    ext, tot = orc.obj_layout(pool, cfg, w.n_blocks)
    stage = np.zeros(int(tot[0]), np.uint8)
    cores = len(os.sched_getaffinity(0))     # every core the process may run on; the count goes into the line

    def one_pass(nt):
        t = time.perf_counter()
        orc.obj_pack(pool, cfg, ext, w.block_table, stage, n_threads=nt)
        if nt:
            orc.obj_unpack(pool, cfg, ext, w.block_table, stage, n_threads=nt)
        else:
            orc.layer_restore(pool, cfg, w.n_blocks, w.block_table, w.file_id, 0, stage, 0, 1, int(tot[1]))
        return time.perf_counter() - t

    res = {}
    for label, nt in (("1thread", 0), ("allcores", cores)):
        one_pass(nt)
        times, t_start = [], time.perf_counter()
        while len(times) < 5 or (time.perf_counter() - t_start < budget_s and len(times) < 200):
            times.append(one_pass(nt))
        res[label] = (2 * payload_layer / median(times) / 1e9, len(times))
    # entries per second of the oracle on config 3's batch, one entry per block (81,438 entries per layer)
    w3 = W.batch64_zipf(chunk_bytes=32768)
    s3 = w3.shape
    p3 = orc.make_pool(None, None, num_blocks=s3.num_blocks, block_tokens=s3.block_tokens, num_kv_heads=s3.num_kv_heads,
                       head_dim=s3.head_dim, elt_bytes=s3.elt_bytes)
    c3 = orc.make_cfg(w3.align, 32768, s3.num_layers)
    e3, t3 = orc.obj_layout(p3, c3, w3.n_blocks)
    ts = []
    for i in range(7):
        t = time.perf_counter()
        orc.sqe_build(p3, c3, e3, w3.file_id, i, orc.OP_READ, 1 << 40, 1)
        ts.append(time.perf_counter() - t)
    oracle_sqes = int(t3[1]) / median(ts[1:])
    parity = bool(np.array_equal(stage, gpu_stage))
    log(f"[bench] oracle: 1 thread {res['1thread'][0]:.2f} GB/s, {cores} threads {res['allcores'][0]:.2f} GB/s; "
        f"GPU staging buffer of layer 0 equals the oracle's: {parity}")
    assert parity, "GPU-packed layer 0 differs from the CPU oracle"
    return {"value": round(res["allcores"][0], 3), "unit": "GB/s (bytes packed + bytes restored per second)", "cores": cores,
            "kind": "oracle", "value_1thread": round(res["1thread"][0], 3),
            "sqes_per_s_1thread": round(oracle_sqes, 0),
            "sample": f"layer 0 of config 2 (2048 blocks, {payload_layer >> 20} MiB packed + {payload_layer >> 20} MiB "
                      f"restored per pass), median of {res['allcores'][1]} passes with {cores} threads "
                      f"({res['1thread'][1]} passes single-threaded)"}


def cpu_baseline_others(W, budget_s=3.0):
    """The oracle on one layer of configs 1, 3 and 4 (config 2 is the headline sample): pack + restore, one thread
    and every core of the affinity mask.  Pool contents are a constant fill (the oracle's time does not depend on
    the values); tables, extents and shapes are the workloads' own."""
    from oracle import tutti_oracle as orc
    cores = len(os.sched_getaffinity(0))
    out = {}
    for name, w in (("config1_tiny", W.tiny()), ("config3_batch64_zipf", W.batch64_zipf()),
                    ("config4_llama70b_128k", W.llama70b_128k())):
        s = w.shape
        bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
        k = np.full(s.num_blocks * bb, 0x5A, np.uint8)
        v = np.full(s.num_blocks * bb, 0xA5, np.uint8)
        pool = orc.make_pool(k, v, num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads,
                             head_dim=s.head_dim, elt_bytes=s.elt_bytes)
        cfg = orc.make_cfg(w.align, w.chunk_bytes, s.num_layers)
        ext, tot = orc.obj_layout(pool, cfg, w.n_blocks)
        stage = np.zeros(int(tot[0]), np.uint8)
        payload = 2 * int(w.block_table.size) * bb
        row = {"payload_bytes_per_layer": payload}
        for label, nt in (("1thread", 0), ("allcores", cores)):
            def one_pass():
                t = time.perf_counter()
                orc.obj_pack(pool, cfg, ext, w.block_table, stage, n_threads=nt)
                orc.obj_unpack(pool, cfg, ext, w.block_table, stage, n_threads=nt)
                return time.perf_counter() - t
            one_pass()
            times, t0 = [], time.perf_counter()
            while len(times) < 2 or (time.perf_counter() - t0 < budget_s and len(times) < 500):
                times.append(one_pass())
            row[f"GBps_{label}"] = round(2 * payload / median(times) / 1e9, 3)
            row[f"passes_{label}"] = len(times)
        out[name] = row
        log(f"[bench] oracle on {name}: {row}")
        del k, v, stage
    out["cores"] = cores
    out["sample"] = "one layer of each config, pack + restore per pass, median over the passes that fit about 3 s"
    return out


if __name__ == "__main__":
    main()
