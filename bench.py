#!/usr/bin/env python3
"""Benchmark driver: random-line read GB/s vs region size (1..256 GiB) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" is one pass of the hot path over the region-size sweep: for each region size
(1, 2, 4, ..., 128, 192, 256 GiB prefixes of one filled allocation) one read launch (all of a
step's launches go out in one rr_rand_read_batch call, which waits once at the end) in
which every wave slot of the device is occupied and every 32-lane logical wave reads 4096
uniformly random, aligned 128-byte lines (paper Sec. 2.1).  The fill is done once before the
timed region (the region is resident in HBM when timing starts).  Prints ONE JSON line.

`value` is whole-job throughput: bytes read in the K timed steps / wall time between two device
synchronisations, i.e. it includes launch, the 8-byte result read-back and host overhead.
`roofline` is for the read kernels alone: algorithmic bytes per launch / average launch duration
measured by the library with HIP events on the launch stream, against the 8 TB/s HBM3E peak; its
top-level figures are those of the dominant kernel (the plain-order read) over regions of 4 GiB and
more, `kernels` lists every kernel of the timed steps with its own figures, `all_timed_launches`
is all of them together.
`cpu_baseline` times the CPU oracle (recompute mode) on one whole step on the host's cores and
checks that its checksums equal the GPU's for the same arguments.
`beyond_the_sweep` is context measured after the timed steps: if the card has the memory, the
allocation is 280 GiB rather than 256, and the same launch is timed over 264, 272 and 280 GiB
in plain order, zone by zone and with one window per XCD (paper Sec. 2.4).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def read_traffic_file(path):
    """Bytes per launch that the L2 fetched from the fabric plus those it wrote back, from the committed rocprofv3
    --pmc summary (FETCH_SIZE and WRITE_SIZE, each scaled by a copy of known size), or None."""
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("fabric_traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-region-gib", type=int, default=256)
    ap.add_argument("--allocation-gib", type=int, default=280,
                    help="allocate up to this much (a multiple of 8 GiB) if the card has it: what lies beyond "
                         "--max-region-gib is measured after the timed steps, as context (beyond_the_sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--one-by-one", action="store_true",
                    help="one rr_rand_read call (and one wait) per region size instead of one rr_rand_read_batch per step")
    ap.add_argument("--plain-order", action="store_true",
                    help="read every region in plain order (no zone probe, no zone-by-zone launches)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark is a single-GPU measurement; --gpus must be 1 "
              "(no multi-GPU path is built; each GPU would run its own range of logical waves and the checksums add).",
              file=sys.stderr)
        return 2

    from paper_2405_11425_amd import envinfo
    env = envinfo.environment()          # before this process touches the GPU
    import torch
    import paper_2405_11425_amd as rl
    from paper_2405_11425_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        return 3
    env.update(envinfo.device_facts())
    if not os.path.exists(rl.library_path()):
        print("bench.py: librandline.so is not built (run __graft_entry__.build()).", file=sys.stderr)
        return 3

    GiB = wl.GiB
    free, total = torch.cuda.mem_get_info()
    max_gib = min(args.max_region_gib, int((free - 4 * GiB) // GiB))
    cu_table = rl.enumerate_cus()
    n_cus = len(cu_table)
    # the sweep's regions are prefixes of one allocation; if the card has more than the sweep needs, the allocation
    # is larger still, for the context measurements beyond the sweep's largest region
    alloc_gib = max(max_gib, min(args.allocation_gib, int((free - 6 * GiB) // (8 * GiB)) * 8))
    try:
        region = torch.empty(alloc_gib * GiB, dtype=torch.uint8, device="cuda")
    except RuntimeError:
        if alloc_gib == max_gib:
            raise
        alloc_gib = max_gib
        region = torch.empty(alloc_gib * GiB, dtype=torch.uint8, device="cuda")
    t0 = time.perf_counter()
    rl.fill(region, wl.FILL_SEED)
    torch.cuda.synchronize()
    fill_s = time.perf_counter() - t0
    configs = wl.region_sweep(max_gib * GiB, n_cus)

    def read(cfg, seed, zm=None):
        kw = {"zone_of_window": zm} if zm is not None else {}
        return rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, seed,
                            lanes_per_line=cfg.lanes_per_line, region_bytes=cfg.region_bytes, **kw)

    # Before the timed region (like the fill): regions that span several memory zones may be read zone by zone
    # (opts.zone_of_window: same lines, same checksum, ordered so that the device works on one zone at a time).
    # The zone map of this allocation is probed, both orders are timed on every such region, and the faster
    # one is used for it from here on, warm-up included.
    order = {cfg.name: None for cfg in configs}
    zone_info = None
    if not args.plain_order and max_gib >= 32:
        try:
            t0 = time.perf_counter()
            whole = (max_gib // 32) * 32 * GiB
            win = whole // 32
            probe = {}
            zone_of_window = rl.detect_zones(region, 32, region_bytes=whole, details=probe)
            probe = {k: (round(v, 1) if isinstance(v, float) and k != "seconds" else v) for k, v in probe.items()}
            probe["row"] = [round(x, 1) for x in probe["row"]]
            tried = []
            for cfg in configs:
                if cfg.region_bytes > whole or cfg.region_bytes % win != 0:
                    continue
                zm = zone_of_window[:cfg.region_bytes // win]
                ids = {z: i for i, z in enumerate(dict.fromkeys(zm))}
                if len(ids) < 2:
                    continue
                zm = [ids[z] for z in zm]
                rate = {}
                for name, m in (("plain", None), ("zone-by-zone", zm)):
                    read(cfg, 1000, m)
                    ms = sorted(read(cfg, 2000 + i, m).kernel_ms_event for i in range(4))[1]   # second fastest: what
                    # disturbs a launch only ever makes it slower
                    rate[name] = round(cfg.bytes_read / ms / 1e6, 1)
                if rate["zone-by-zone"] > rate["plain"]:
                    order[cfg.name] = zm
                tried.append({"region_gib": cfg.region_bytes // GiB, "zones": len(ids), "gbps_plain": rate["plain"],
                              "gbps_zone_by_zone": rate["zone-by-zone"],
                              "chosen": "zone-by-zone" if order[cfg.name] is not None else "plain"})
            zone_info = {"zone_of_window_8gib": zone_of_window, "probe": probe, "regions_spanning_zones": tried,
                         "seconds_before_timing": round(time.perf_counter() - t0, 2)}
        except Exception as e:   # the sweep itself does not depend on this: go on in plain order, and say so
            order = {cfg.name: None for cfg in configs}
            zone_info = {"error": f"{type(e).__name__}: {e}"}

    # What the timed launches are, from one untimed launch of each kind: the kernel's name as a trace shows it, and
    # how its working wavefronts spread over the XCDs.  And, as context, the same reads as one wavefront per pair of
    # logical waves with every wave slot of the device occupied (RR_MODE_FLAT), three launches per region.
    xcd_of_cu = cu_table[:, 0]
    kinds = {}
    for cfg in configs:
        kind = "plain" if order[cfg.name] is None else "zone-by-zone"
        if kind in kinds:
            continue
        kw = {"zone_of_window": order[cfg.name]} if order[cfg.name] is not None else {}
        r = rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, 999, lanes_per_line=cfg.lanes_per_line,
                         region_bytes=cfg.region_bytes, want_cu_waves=True, **kw)
        per_xcd = [int(r.cu_waves[:n_cus][xcd_of_cu == x].sum()) for x in sorted(set(xcd_of_cu.tolist()))]
        per_cu = r.cu_waves[:n_cus]
        kinds[kind] = {"kernel": rl.last_kernel(), "wavefronts": int(r.waves_run), "wavefronts_per_xcd": per_xcd,
                       "wavefronts_per_cu_min_max": [int(per_cu.min()), int(per_cu.max())]}
    full_occupancy = []
    for cfg in configs:
        ms = sorted(rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, 3000 + i,
                                 lanes_per_line=cfg.lanes_per_line, region_bytes=cfg.region_bytes,
                                 mode=rl.MODE_FLAT).kernel_ms_event for i in range(3))[1]
        full_occupancy.append({"region_gib": cfg.region_bytes // GiB, "gbps": round(cfg.bytes_read / ms / 1e6, 1)})
    flat_kernel = rl.last_kernel()

    c0 = configs[0]   # the points differ in region size (and read order) only

    # the same calls as one by one, queued back to back with one wait at the end of the step; the arguments are
    # marshalled once, a step only sets its seed
    batch = rl.ReadBatch(region, [(cfg.region_bytes, 0, {"zone_of_window": order[cfg.name]} if order[cfg.name] is not None
                                   else None) for cfg in configs],
                         c0.line_bytes, c0.n_reads, c0.iters_per_wave, lanes_per_line=c0.lanes_per_line)

    def step(seed, record=None):
        if args.one_by_one:
            results = [read(cfg, seed, order[cfg.name]) for cfg in configs]
        else:
            results = batch.run(read_seed=seed)
        if record is not None:
            for cfg, r in zip(configs, results):
                record.setdefault(cfg.name, []).append(r)

    for i in range(args.warmup):
        step(1000 + i)
    records = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(wl.READ_SEED + k, records)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0

    # Context, after the timed steps: regions beyond the sweep, up to the whole allocation.  Above 256 GiB a region
    # holds more translations than the second-level translation cache of an XCD; what that costs uniform reads in
    # plain order, and what the library's division of the region between the halves of the XCDs, zone order (direction
    # alternating from launch to launch) and one window per XCD (paper Sec. 2.4) make of it.
    beyond = []
    for gib in sorted({g for g in (264, 272, alloc_gib) if max_gib < g <= alloc_gib and g % 8 == 0}):
        R = gib * GiB
        row = {"region_gib": gib}
        try:
            rd = lambda seed, wm=None, **kw: rl.rand_read(region, c0.line_bytes, c0.n_reads, c0.iters_per_wave, seed, wm,
                                                          lanes_per_line=c0.lanes_per_line, region_bytes=R, **kw)
            rate = lambda rs: round(c0.bytes_read / sorted(r.kernel_ms_event for r in rs)[len(rs) // 2] / 1e6, 1)
            rd(999)
            plain = [rd(wl.READ_SEED + i) for i in range(4)]
            row["gbps_plain"] = rate(plain)           # the library divides such a region between the halves of the XCDs
            row["kernel_plain"] = rl.last_kernel()
            rd(999, xcd_split=rl.SPLIT_OFF)
            row["gbps_plain_not_divided_between_the_xcd_halves"] = rate([rd(wl.READ_SEED + i, xcd_split=rl.SPLIT_OFF) for i in range(4)])
            zm = rl.detect_zones(region, gib // 8, region_bytes=R)
            rd(999, zone_of_window=zm, zone_descending=True)
            zoned = [rd(wl.READ_SEED + i, zone_of_window=zm, zone_descending=bool(i % 2)) for i in range(6)]
            row["gbps_zone_by_zone_direction_alternating"] = rate(zoned)
            g_of_cu, w_of_g = wl.window_map_by_xcd(cu_table, 8)
            wm = rl.WindowMap(8, g_of_cu, w_of_g)
            rd(999, wm)
            row["gbps_one_window_of_8_per_xcd"] = rate([rd(wl.READ_SEED + i, wm) for i in range(4)])
            row["zone_of_window_8gib"] = zm
            row["zone_order_checksums_equal_plain"] = all(a.checksum == b.checksum for a, b in zip(plain, zoned))
            row["checksum_plain_first_seed"] = f"{plain[0].checksum:#018x}"
        except Exception as e:   # context only: say what went wrong and go on
            row["error"] = f"{type(e).__name__}: {e}"
        beyond.append(row)

    bytes_per_step = sum(c.bytes_read for c in configs)
    value = bytes_per_step * args.steps / wall_s / 1e9
    curve = []
    groups = {}     # launches of the timed steps by kernel and region class
    for cfg in configs:
        ms = [r.kernel_ms_event for r in records[cfg.name]]
        ms_dev = [r.kernel_ms_device for r in records[cfg.name]]
        kind = "plain" if order[cfg.name] is None else "zone-by-zone"
        gib = cfg.region_bytes // GiB
        # The device has a 256 MB memory-side cache that no counter on this machine shows: a region of 1-2 GiB may be
        # served from it to 12-25 %, so those launches are not counted as HBM rates (4 GiB: at most 6 %).
        cls = kind if gib >= 4 else kind + ", regions below 4 GiB"
        groups.setdefault(cls, {"kind": kind, "regions_gib": [], "ms": []})
        groups[cls]["regions_gib"].append(gib)
        groups[cls]["ms"] += ms
        med = statistics.median(ms)
        curve.append({"region_gib": gib, "order": kind,
                      "gbps": round(cfg.bytes_read / med / 1e6, 1),
                      "gbps_min": round(cfg.bytes_read / max(ms) / 1e6, 1),
                      "gbps_max": round(cfg.bytes_read / min(ms) / 1e6, 1),
                      "pct_of_hbm_peak": round(cfg.bytes_read / med / 1e6 / HBM_PEAK_GBPS * 100, 1),
                      "kernel_ms": round(med, 4), "kernel_ms_in_kernel_clock": round(statistics.median(ms_dev), 4),
                      "n_reads": cfg.n_reads, "line_bytes": cfg.line_bytes, "lanes_per_line": cfg.lanes_per_line,
                      "checksum_first_step": f"{records[cfg.name][0].checksum:#018x}"})
    bytes_per_launch = configs[0].bytes_read
    per_kernel = []
    for cls, g in groups.items():
        avg = sum(g["ms"]) / len(g["ms"])
        per_kernel.append({"launches_of": cls, "kernel": kinds[g["kind"]]["kernel"], "regions_gib": g["regions_gib"],
                           "launches_timed": len(g["ms"]), "avg_launch_ms": round(avg, 4),
                           "achieved": round(bytes_per_launch / avg / 1e6, 1),
                           "frac": round(bytes_per_launch / avg / 1e6 / HBM_PEAK_GBPS, 4),
                           "wavefronts": kinds[g["kind"]]["wavefronts"],
                           "wavefronts_per_xcd": kinds[g["kind"]]["wavefronts_per_xcd"],
                           "wavefronts_per_cu_min_max": kinds[g["kind"]]["wavefronts_per_cu_min_max"]})
    dominant = max((k for k in per_kernel if "below" not in k["launches_of"]), key=lambda k: k["launches_timed"])
    all_ms = [m for g in groups.values() for m in g["ms"]]
    avg_all = sum(all_ms) / len(all_ms)
    roofline = {"bound": "hbm", "kernel": dominant["kernel"], "achieved": dominant["achieved"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": dominant["frac"],
                "traffic": read_traffic_file(os.path.join(ROOT, "profiles", "rand_read_region_sweep_pmc.txt")),
                "traffic_is": "bytes per launch between the L2 and the fabric (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled "
                              "by a copy of known size), from the committed profile of this command, not of this run; "
                              "reads served by the 256 MB memory-side cache are included in it",
                "bytes_per_launch": bytes_per_launch, "avg_launch_ms": dominant["avg_launch_ms"],
                "launches_timed": dominant["launches_timed"], "regions_gib": dominant["regions_gib"],
                "kernels": per_kernel,
                "all_timed_launches": {"launches": len(all_ms), "avg_launch_ms": round(avg_all, 4),
                                       "achieved": round(bytes_per_launch / avg_all / 1e6, 1),
                                       "frac": round(bytes_per_launch / avg_all / 1e6 / HBM_PEAK_GBPS, 4)}}

    # the knee of the paper's Fig. 1: the first region from which the curve stays more than 10 % below the median of the
    # smaller regions (None: flat)
    from paper_2405_11425_amd.report import find_knee
    knee_at, plateau = find_knee([c["region_gib"] for c in curve], [c["gbps"] for c in curve], 0.10)
    knee = {"rule": "first region from which the curve stays more than 10 % below the median of the smaller regions",
            "region_gib": knee_at, "median_gbps": round(plateau, 1),
            "lowest_point_pct_below_median": round((1 - min(c["gbps"] for c in curve) / plateau) * 100, 2)}

    out = {
        "metric": "random-line read GB/s vs region size (1-256 GiB); % of 8 TB/s HBM peak",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_s / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "region-size sweep (configs[1]): per region size one launch with all "
                               f"{configs[0].logical_waves} 32-lane logical waves (two for each of the device's "
                               f"{n_cus * wl.WAVES_PER_CU} wave slots), each reading "
                               "4096 uniformly random 128-B lines, executed by 8 wavefronts per compute unit that take "
                               "the logical waves' iterations in chunks and never let their loads run dry (measured "
                               "faster than one wavefront per pair with every slot occupied: see full_occupancy_flat); "
                               "regions are prefixes of one filled allocation; "
                               "regions that span several memory zones are read in whichever order was faster "
                               "before the timed steps, plain or zone by zone (same lines, same checksums); "
                               + ("one call and one wait per launch" if args.one_by_one else
                                  "a step's launches are queued back to back by one batched call that waits once"),
                   "regions_gib": [c.region_bytes // GiB for c in configs], "line_bytes": 128,
                   "lanes_per_line": 32, "logical_waves": configs[0].logical_waves,
                   "iters_per_wave": configs[0].iters_per_wave, "reads_per_launch": configs[0].n_reads,
                   "allocation_gib": alloc_gib, "fill_seed": wl.FILL_SEED, "first_read_seed": wl.READ_SEED,
                   "n_cus": n_cus},
        "pct_of_hbm_peak": round(value / HBM_PEAK_GBPS * 100, 1),
        "curve": curve,
        "environment": env,
        "gbps_at_largest_region": curve[-1]["gbps"],
        "knee_of_curve": knee,
        "fill_gbps": round(alloc_gib * GiB / fill_s / 1e9, 1),
        "roofline": roofline,
        # context: the same launches as one wavefront per pair of logical waves, every wave slot occupied
        "full_occupancy_flat": {"kernel": flat_kernel, "launches_per_region": 3, "curve": full_occupancy},
        # the paper's own figures (A100 SXM4-80GB, Sec. 2.1): context, not a target, hence vs_baseline is null
        "paper_context_a100": {"theoretical_hbm_gbps": 1900, "random_256B_lines_gbps": 1400,
                               "random_512B_lines_gbps": 1600, "throughput_collapses_above_gb": 64},
    }

    if beyond:
        out["beyond_the_sweep"] = {
            "what": "context, measured after the timed steps and not part of value: the same launch over regions larger "
                    "than the sweep's largest, up to the whole allocation; median of 4 launches (zone order: of 6, "
                    "ascending and descending in turn)",
            "curve": beyond}
    if zone_info is not None:
        out["zone_order"] = zone_info

    if not args.no_cpu_baseline:
        # CPU-baseline leg: the oracle as it stands, on one whole step (every sweep point), first timed seed.
        from oracle import randline as orc
        cores = len(os.sched_getaffinity(0))
        picks = list(configs)
        t_all, reads_all, used, match = 0.0, 0, 0, True
        oracle_first = {}
        for cfg in picks:
            t0 = time.perf_counter()
            c_all, used = orc.checksum_ex(cfg.region_bytes, cfg.line_bytes, cfg.logical_waves, cfg.iters_per_wave,
                                          cfg.fill_seed, wl.READ_SEED, n_threads=cores)
            t_all += time.perf_counter() - t0
            reads_all += cfg.n_reads
            oracle_first[cfg.name] = c_all
            match = match and c_all == records[cfg.name][0].checksum
        # the last timed step too (not timed: the rate above is from the first pass only)
        last_seed = wl.READ_SEED + args.steps - 1
        match_last = all(orc.checksum(c.region_bytes, c.line_bytes, c.logical_waves, c.iters_per_wave, c.fill_seed,
                                      last_seed, n_threads=cores) == records[c.name][-1].checksum for c in picks)
        cfg = configs[-1]
        sample_waves = cfg.logical_waves // 4           # single thread: a quarter of one point's waves
        t0 = time.perf_counter()
        orc.checksum(cfg.region_bytes, cfg.line_bytes, sample_waves, cfg.iters_per_wave, cfg.fill_seed,
                     wl.READ_SEED, n_threads=1)
        t_one = time.perf_counter() - t0
        # materialised mode: real random reads from a 2 GiB host buffer (host-DRAM analogue)
        mat_bytes = 2 * GiB
        host = orc.fill_buffer(mat_bytes, cfg.fill_seed)
        mat_waves = 16384
        t0 = time.perf_counter()
        orc.checksum_materialised(host, cfg.line_bytes, mat_waves, 1024, wl.READ_SEED, n_threads=cores)
        t_mat = time.perf_counter() - t0
        del host
        for c, cfg in zip(curve, configs):
            c["oracle_checksum_first_step"] = f"{oracle_first[cfg.name]:#018x}"
        for row in beyond:      # not timed
            if "checksum_plain_first_seed" in row:
                want = orc.checksum(row["region_gib"] * GiB, c0.line_bytes, c0.logical_waves, c0.iters_per_wave,
                                    c0.fill_seed, wl.READ_SEED, n_threads=cores)
                row["oracle_checksum_plain_first_seed"] = f"{want:#018x}"
        out["cpu_baseline"] = {
            "value": round(reads_all * cfg.line_bytes / t_all / 1e9, 3), "unit": "GB/s", "cores": used,
            "kind": "oracle",
            "sample": f"recompute mode, one whole step = all {len(picks)} sweep points: {cfg.logical_waves} logical "
                      f"waves x {cfg.iters_per_wave} reads of 128 B each per point (same arguments as the GPU launches "
                      f"of the first timed step, all checksums compared), {used} threads, {t_all:.2f} s wall",
            "reads_per_s": round(reads_all / t_all),
            "single_thread_gbps": round(sample_waves * cfg.iters_per_wave * cfg.line_bytes / t_one / 1e9, 3),
            "single_thread_sample": f"{sample_waves} logical waves of {cfg.name}, {t_one:.2f} s",
            "materialised_gbps": round(mat_waves * 1024 * cfg.line_bytes / t_mat / 1e9, 3),
            "materialised_sample": f"{mat_waves} logical waves x 1024 reads from a {mat_bytes // GiB} GiB host buffer, "
                                   f"{cores} threads, {t_mat:.2f} s",
            "checksum_matches_gpu": bool(match and match_last),
            "checksums_compared": f"all {len(picks)} region sizes, first timed step (seed {wl.READ_SEED}) and last "
                                  f"(seed {last_seed})",
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
