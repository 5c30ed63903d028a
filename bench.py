#!/usr/bin/env python3
"""Benchmark of the layout-conversion / gather hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--only-main] [--strategy N]

A step is one pass of the headline workload (benchmark configuration 4, the largest and slowest
of the five: 4096 tiles of 65536 int32 converted between two random invertible XOR layouts, 2 GiB
of algorithmic bytes) with inputs already resident in HBM.  The
JSON line printed at the end carries the whole-job GB/s (read + write algorithmic
bytes), a roofline object for the dominant kernel, the CPU oracle timed on a
bounded sample, and per-config figures for all five configurations next to a
plain 16-byte copy at the same footprint.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E peak


MAIN_SETS = 4          # buffer sets the main line rotates through
TABLE_SETS = 3         # ... and each per-config table entry
TABLE_WARMUP = 10      # untimed launches before each table entry, at least; extended to TABLE_WARMUP_MS of device time
TABLE_WARMUP_MS = 25.0 # (the first launches after an idle spell or on fresh buffers run up to 10 % slower: clocks ramp up)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--only-main", action="store_true", help="skip the per-config table")
    ap.add_argument("--workload", type=int, default=4, help="config id timed as the main line (default 4: the largest)")
    ap.add_argument("--table-steps", type=int, default=100, help="launches per config in the per-config table")
    ap.add_argument("--strategy", type=int, default=None,
                    help="force a conversion strategy for every plan (3: element-wide LDS, 4: 128-bit LDS "
                         "where it applies); default: the planner's choice")
    ap.add_argument("--mark", action="store_true",
                    help="for profiler runs: before every timed section launch a tiny copy whose grid size is unique "
                         "(256 * (k + 1) threads for the k-th section) and list the sections in the JSON field 'sections', "
                         "so that a kernel trace can be cut into sections")
    ap.add_argument("--opt", action="append", default=[], metavar="FIELD=VALUE",
                    help="set a field of ll_options for the main workload and the per-config table (repeatable), "
                         "e.g. --opt elem_threads_log2=8 --opt xcd_chunk=0")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; tiles are independent, so more GPUs would each "
              "take a tile range with no communication, but no multi-GPU path is built or measured. "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2505_23819_amd as ll
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = "cuda"

    fields = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.opt}
    if args.strategy is not None:
        fields["strategy"] = args.strategy
    forced = ll.ll_options_init(**fields) if fields else None

    def make_case(cfg, nsets, opts=forced):
        """Device buffers (nsets rotating copies) and a launcher for one configuration."""
        a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
        sets = []
        for s in range(nsets):
            x = cfg.gen_data(0, cfg.ntiles, dev) if s == 0 else sets[0][0].clone()
            if cfg.kind == "gather":
                idx = cfg.gen_idx(0, cfg.ntiles, dev) if s == 0 else sets[0][1].clone()
                sets.append((x, idx, torch.empty_like(x)))
            else:
                sets.append((x, None, torch.empty_like(x)))
        if cfg.kind == "gather":
            info = {"strategy_name": ll.ll_gather_info(a, cfg.axis, cfg.elem_bytes, opts)["kernel_name"], "kind_name": "gather"}

            def launch(k):
                x, idx, out = sets[k % nsets]
                ll.ll_gather(a, cfg.axis, cfg.elem_bytes, x, idx, out, cfg.ntiles, opts=opts)
        else:
            b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
            plan = ll.ll_plan_convert(a, b, cfg.elem_bytes, opts)
            info = plan.info()

            def launch(k, plan=plan):
                x, _, out = sets[k % nsets]
                ll.ll_convert(plan, x, out, cfg.ntiles)
        return launch, info, sets

    # what rocprofv3 measured for each timed section in an earlier profiled run (profiles/per_section_summary.txt):
    # HBM traffic, LDS bank conflict cycles per wave, kernel-only duration
    profiled = {}
    ppath = os.path.join(ROOT, "profiles", "per_section_summary.txt")
    if os.path.exists(ppath):
        for line in open(ppath):
            f = line.rstrip("\n").split("\t")
            if len(f) == 6 and not line.startswith(("#", "section\t")):
                profiled[f[0]] = {"kernel": f[1], "hbm_read_MiB": float(f[2]), "hbm_written_MiB": float(f[3]),
                                  "lds_conflict_cycles_per_wave": float(f[4]), "kernel_us": float(f[5])}

    def annotate(entry, label, alg_bytes):
        """Adds the profiled figures of section `label` to a table entry."""
        p = profiled.get(label)
        if not p:
            return
        traffic = (p["hbm_read_MiB"] + p["hbm_written_MiB"]) * (1 << 20)
        entry["profiled"] = {"kernel": p["kernel"], "kernel_us": p["kernel_us"],
                             "GBps_kernel_time": round(alg_bytes / p["kernel_us"] / 1e3, 1),
                             "hbm_traffic_bytes": int(traffic), "hbm_traffic_over_algorithmic": round(traffic / alg_bytes, 4),
                             "GBps_of_hbm_traffic": round(traffic / p["kernel_us"] / 1e3, 1),
                             "lds_conflict_cycles_per_wave": p["lds_conflict_cycles_per_wave"]}

    sections = []
    mark_buf = torch.zeros(2, 1 << 20, dtype=torch.uint8, device=dev) if args.mark else None

    def time_launches(launch, steps, warmup, warm_ms=TABLE_WARMUP_MS, label=""):
        """Returns (wall ms per step, mean ms per launch, median, min).

        The timed region is exactly `steps` back-to-back launches between two HIP events on the stream
        the kernels run on (torch's current stream is the stream handed to the library) and between two
        host clock readings around synchronize(): mean = event time / steps, wall = host time / steps.
        Median and minimum come from a second, untimed pass with an event after every launch (each
        such event costs about 3 us of stream time, which is why it is not done in the timed region)."""
        if args.mark:
            ll.ll_copy(mark_buf[0], mark_buf[1], 4096 * (len(sections) + 1))
            sections.append(label)
        t_w = time.perf_counter()
        for k in range(warmup):
            launch(k)
        torch.cuda.synchronize()
        if warm_ms and warmup:
            spent = (time.perf_counter() - t_w) * 1e3
            extra = min(5000, int((warm_ms - spent) / max(spent / warmup, 1e-3))) if spent < warm_ms else 0
            for k in range(extra):
                launch(k)
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for k in range(steps):
            launch(k)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        mean_ms = e0.elapsed_time(e1) / steps
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        evs[0].record()
        for k in range(steps):
            launch(k)
            evs[k + 1].record()
        torch.cuda.synchronize()
        per = [evs[k].elapsed_time(evs[k + 1]) for k in range(steps)]
        return wall_ms, mean_ms, statistics.median(per), min(per)

    def copy_ceiling(nbytes_each, steps=None, label="copy yardstick"):
        steps = steps or max(20, args.table_steps)
        """Plain 16-byte vector copy moving the same read + write footprint."""
        n = max(16, (nbytes_each // 16) * 16)
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dsts = [torch.empty_like(src) for _ in range(2)]
        _, mean_ms, _, _ = time_launches(lambda k: ll.ll_copy(src, dsts[k % 2], n), steps, TABLE_WARMUP, label="%s, %d MiB each way" % (label, n >> 20))
        return 2.0 * n / mean_ms / 1e6

    main_cfg = wl.config(args.workload)
    # four buffer sets in rotation: nothing is re-read from a cache, and the rate is the mean over four placements of the
    # buffers (where a buffer lands in HBM moves the same kernel on the same data by up to 5 %)
    launch, info, sets = make_case(main_cfg, nsets=MAIN_SETS)
    wall_ms, mean_ms, med_ms, min_ms = time_launches(launch, args.steps, args.warmup, warm_ms=0,      # exactly W warm-up steps
                                                     label="main: config %d" % main_cfg.cid)
    alg_bytes = main_cfg.algorithmic_bytes()
    value = alg_bytes / wall_ms / 1e6                      # GB/s over the timed region (wall clock)
    achieved = alg_bytes / mean_ms / 1e6                   # GB/s of the kernel itself (HIP events)
    ceiling = copy_ceiling(alg_bytes // 2, label="copy yardstick for the main line")

    traffic, kernel_us = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_config%d.txt" % main_cfg.cid)
    if os.path.exists(tpath) and not fields:               # measured separately with rocprofv3 --pmc (default options only)
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split()[1])
    spath = os.path.join(ROOT, "profiles", "config%d_kernel_stats.txt" % main_cfg.cid)
    if os.path.exists(spath) and not fields:               # rocprofv3 --kernel-trace --stats of the same command
        for line in open(spath):
            if line.startswith("ll::") and "k_copy" not in line:
                kernel_us = float(line.split(", ")[-4]) / 1e3

    result = {
        "metric": "layout-conversion GB/s (read+write) vs HBM peak",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {1: "u8", 2: "u16", 4: "u32", 8: "u64"}[main_cfg.elem_bytes],      # raw bits are moved, no arithmetic
        "element_type": str(main_cfg.dtype).replace("torch.", ""),
        "data": "synthetic",
        "config": {"workload": "config %d: %s, %d tiles of 2^%d elements x %d B" %
                               (main_cfg.cid, main_cfg.name, main_cfg.ntiles, main_cfg.d, main_cfg.elem_bytes),
                   "kernel": info["strategy_name"], "class": info["kind_name"],
                   "threads_per_workgroup": info.get("threads"), "vectors_per_thread": info.get("vectors_per_thread"),
                   "options": fields or None, "buffer_sets_rotated": MAIN_SETS},
        "fraction_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "copy_kernel_ceiling_GBps": round(ceiling, 1),
        "fraction_of_copy_ceiling": round(achieved / ceiling, 4),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": info["strategy_name"], "launch_ms_mean": round(mean_ms, 5),
                     "launch_ms_median": round(med_ms, 5), "launch_ms_min": round(min_ms, 5),
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "profiled_kernel_us": kernel_us,
                     "profiled_frac": round(alg_bytes / kernel_us / 1e3 / HBM_PEAK_GBPS, 4) if kernel_us else None,
                     "how": "achieved = algorithmic bytes / mean launch duration, HIP events around the timed region on the launch stream; "
                            "profiled_* = the same kernel's average under rocprofv3 --kernel-trace (profiles/), traffic = FETCH_SIZE + WRITE_SIZE"},
    }
    # Buffers go back to torch's caching allocator, not to the driver: memory that is freed and allocated again
    # during the run lands less well (configs 2-5 read 0.5-1.3 % lower with a release after every section)
    del sets, launch

    if not args.only_main:
        table = []
        for cfg in wl.configs():
            nsets = TABLE_SETS
            l, inf, s = make_case(cfg, nsets)
            steps = args.table_steps if cfg.cid != 1 else max(args.table_steps, 200 if args.table_steps >= 30 else 0)
            w_ms, m_ms, md_ms, mn_ms = time_launches(l, steps, TABLE_WARMUP, label="config %d" % cfg.cid)
            ab = cfg.algorithmic_bytes()
            entry = {"config": cfg.cid, "name": cfg.name, "kernel": inf["strategy_name"], "class": inf["kind_name"],
                     "algorithmic_bytes": ab, "us_mean": round(m_ms * 1e3, 2), "us_median_with_events": round(md_ms * 1e3, 2),
                     "us_min": round(mn_ms * 1e3, 2),
                     "GBps": round(ab / m_ms / 1e6, 1), "frac_hbm_peak": round(ab / m_ms / 1e6 / HBM_PEAK_GBPS, 4)}
            if inf.get("lds_write_bytes"):
                entry.update({"lds_access_bytes": inf["lds_write_bytes"], "lds_bytes": inf["lds_bytes"],
                              "predicted_wavefronts": [inf["predicted_wavefronts_write"], inf["predicted_wavefronts_read"]]})
            del s, l
            if cfg.cid != 1:
                entry["copy_GBps_same_footprint"] = round(copy_ceiling(ab // 2, label="copy yardstick for config %d" % cfg.cid), 1)
            if cfg.kind == "convert" and args.strategy is None and inf["strategy_name"] in ("reg_permute", "wave_shuffle"):
                # the same conversion staged through LDS (128-bit accesses), for comparison
                l2, inf2, s2 = make_case(cfg, nsets, ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_VEC))
                _, md2, _, _ = time_launches(l2, steps, TABLE_WARMUP, label="config %d through 128-bit LDS" % cfg.cid)
                entry["through_lds"] = {"kernel": inf2["strategy_name"], "lds_access_bytes": inf2["lds_write_bytes"],
                                        "GBps": round(ab / md2 / 1e6, 1),
                                        "predicted_wavefronts": [inf2["predicted_wavefronts_write"], inf2["predicted_wavefronts_read"]]}
                del s2, l2
            annotate(entry, "config %d" % cfg.cid, ab)
            table.append(entry)
        result["per_config"] = table

        # config 1 is launch bound: the same launch recorded 100 times into a HIP graph and replayed
        c1 = wl.config(1)
        l1, inf1, s1 = make_case(c1, 2)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            l1(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for k in range(100):
                l1(k)
        _, g_ms, _, _ = time_launches(lambda k: graph.replay(), 20, 2, label="config 1, graph of 100 launches")
        result["config1_graph_replay"] = {"launches_per_graph": 100, "us_per_launch": round(g_ms * 1e3 / 100, 3),
                                          "kernel": inf1["strategy_name"]}
        del graph, l1, s1

        # config 1's layouts on many tiles: the lane <-> register butterfly kernel (Sec. 5.4 "Intra-warp Data
        # Exchange") at a size where bandwidth, not the launch, is what is measured; and the same through LDS
        nt1 = 32768
        a1 = ll.distributed_layout(c1.nreg, c1.nlane, c1.nwave, c1.out_dim_bits, c1.src_bases)
        b1 = ll.distributed_layout(c1.nreg, c1.nlane, c1.nwave, c1.out_dim_bits, c1.dst_bases)
        x1 = wl.gen_int32(11, 0, nt1 * c1.tile_elems, dev)
        o1 = [torch.empty_like(x1) for _ in range(2)]
        ab1 = 2 * nt1 * c1.tile_elems * c1.elem_bytes
        many = []
        for force in (None, ll.LL_STRATEGY_LDS_VEC, ll.LL_STRATEGY_LDS_ELEM):
            p1 = ll.ll_plan_convert(a1, b1, c1.elem_bytes, None if force is None else ll.ll_options_init(strategy=force))
            i1 = p1.info()
            _, m_ms, _, _ = time_launches(lambda k: ll.ll_convert(p1, x1, o1[k % 2], nt1), args.table_steps, TABLE_WARMUP,
                                          label="config 1's layouts on 32768 tiles, %s" % i1["strategy_name"])
            many.append({"kernel": i1["strategy_name"], "shuffle_stages": i1["shuffle_rounds"], "lds_bytes": i1["lds_bytes"],
                         "us_mean": round(m_ms * 1e3, 2), "GBps": round(ab1 / m_ms / 1e6, 1),
                         "frac_hbm_peak": round(ab1 / m_ms / 1e6 / HBM_PEAK_GBPS, 4)})
        result["config1_layouts_32768_tiles"] = {"algorithmic_bytes": ab1, "kernels": many}
        del x1, o1

        # conversions between layouts that replicate data (zero columns): one copy of every logical
        # element read, every destination slot written
        btable = []
        for case in wl.broadcast_cases():
            a = ll.distributed_layout(*case.src_in, case.out_dim_bits, case.src_bases)
            b = ll.distributed_layout(*case.dst_in, case.out_dim_bits, case.dst_bases)
            plan = ll.ll_plan_convert(a, b, case.elem_bytes)
            inf = plan.info()
            x = case.gen_data(0, case.ntiles, dev)
            outs = [torch.empty(case.ntiles << case.d_dst, dtype=x.dtype, device=dev) for _ in range(2)]
            _, md_ms, _, mn_ms = time_launches(lambda k: ll.ll_convert(plan, x, outs[k % 2], case.ntiles),
                                               args.table_steps, TABLE_WARMUP, label="broadcast: " + case.name)
            ab = case.algorithmic_bytes()
            btable.append({"name": case.name, "kernel": inf["strategy_name"], "src_tile_bits": case.d_src,
                           "dst_tile_bits": case.d_dst, "logical_bits": case.d_out, "algorithmic_bytes": ab,
                           "us_mean": round(md_ms * 1e3, 2), "GBps": round(ab / md_ms / 1e6, 1),
                           "frac_hbm_peak": round(ab / md_ms / 1e6 / HBM_PEAK_GBPS, 4),
                           "predicted_wavefronts": [inf["predicted_wavefronts_write"], inf["predicted_wavefronts_read"]]})
            annotate(btable[-1], "broadcast: " + case.name, ab)
            del x, outs
        result["broadcast_conversions"] = btable

        # the 128 x 128 transpose of config 2 with 1-byte (float8-sized) and 2-byte elements: the planner's
        # choice, and the same conversion through the transposing LDS loads of gfx950 / 128-bit LDS
        ttable = []
        c2 = wl.config(2)
        for w_, dt_, force_ in ((1, torch.uint8, None), (1, torch.uint8, ll.LL_STRATEGY_LDS_TR), (2, torch.int16, ll.LL_STRATEGY_LDS_TR),
                                (2, torch.int16, ll.LL_STRATEGY_LDS_VEC)):
            a = ll.distributed_layout(c2.nreg, c2.nlane, c2.nwave, c2.out_dim_bits, c2.src_bases)
            b = ll.distributed_layout(c2.nreg, c2.nlane, c2.nwave, c2.out_dim_bits, c2.dst_bases)
            plan = ll.ll_plan_convert(a, b, w_, None if force_ is None else ll.ll_options_init(strategy=force_))
            inf = plan.info()
            nt = (256 << 20) // (c2.tile_elems * w_)            # 256 MiB per side
            x = wl.raw_bits(21, 0, nt * c2.tile_elems * w_ // 8, dev).view(dt_)
            outs = [torch.empty_like(x) for _ in range(2)]
            _, md_ms, _, _ = time_launches(lambda k: ll.ll_convert(plan, x, outs[k % 2], nt), args.table_steps, TABLE_WARMUP,
                                           label="transpose 128x128, %d-byte elements, %s" % (w_, inf["strategy_name"]))
            ab = 2 * nt * c2.tile_elems * w_
            ttable.append({"name": "transpose 128x128, %d-byte elements, %d tiles" % (w_, nt), "kernel": inf["strategy_name"],
                           "lds_access_bytes": [inf["lds_write_bytes"], inf["lds_read_bytes"]], "block_bytes": (1 << inf["block_bits"]) * w_,
                           "algorithmic_bytes": ab, "us_mean": round(md_ms * 1e3, 2), "GBps": round(ab / md_ms / 1e6, 1),
                           "frac_hbm_peak": round(ab / md_ms / 1e6 / HBM_PEAK_GBPS, 4),
                           "predicted_wavefronts": [inf["predicted_wavefronts_write"], inf["predicted_wavefronts_read"]]})
            del x, outs
        result["narrow_element_transposes"] = ttable

        # gather variants on config 5's layout: rows (lane axis) with each of the three kernels, and
        # columns (an axis on register and wave bits: 16 shuffle rounds in the paper's scheme)
        gtable = []
        c5 = wl.config(5)
        lay5 = ll.distributed_layout(c5.nreg, c5.nlane, c5.nwave, c5.out_dim_bits, c5.src_bases)
        x5 = c5.gen_data(0, c5.ntiles, dev)
        out5 = torch.empty_like(x5)
        for axis_, kern_ in ((0, None), (0, ll.LL_GATHER_SHUFFLE_ROWS), (0, ll.LL_GATHER_SHUFFLE), (0, ll.LL_GATHER_BLOCK_STAGED), (1, None)):
            gopts = None if kern_ is None else ll.ll_options_init(gather_kernel=kern_)
            ginfo = ll.ll_gather_info(lay5, axis_, c5.elem_bytes, gopts)
            idx5 = wl.gen_index(51 + axis_, 0, c5.ntiles * c5.tile_elems, 1 << c5.out_dim_bits[axis_], dev)
            _, md_ms, _, _ = time_launches(lambda k: ll.ll_gather(lay5, axis_, c5.elem_bytes, x5, idx5, out5, c5.ntiles, opts=gopts),
                                           args.table_steps, TABLE_WARMUP,
                                           label="gather: config 5 layout, dim %d, %s" % (axis_, ginfo["kernel_name"]))
            ab = c5.algorithmic_bytes()
            gtable.append({"name": "config 5 layout, gather along dim %d" % axis_, "kernel": ginfo["kernel_name"],
                           "axis_bits_reg_lane_wave": [ginfo["axis_reg_bits"], ginfo["axis_lane_bits"], ginfo["axis_wave_bits"]],
                           "paper_rounds": ginfo["paper_rounds"], "staged_bytes": ginfo["block_bytes"],
                           "algorithmic_bytes": ab, "us_mean": round(md_ms * 1e3, 2), "GBps": round(ab / md_ms / 1e6, 1),
                           "frac_hbm_peak": round(ab / md_ms / 1e6 / HBM_PEAK_GBPS, 4)})
            annotate(gtable[-1], "gather: config 5 layout, dim %d, %s" % (axis_, ginfo["kernel_name"]), ab)
            del idx5
        del x5, out5
        # axes whose aligned block exceeds LDS, row-major two-byte tiles of 2^18 elements (512 KiB), gather along
        # the rows: 512 x 512 is staged as 512 rows x 128-byte runs; 8192 x 32 has no closed block with runs of
        # 64 bytes that fits LDS, its 512 KiB range is walked through LDS in chunks; 32768 x 32 (2 MiB) is read
        # straight from memory
        xb = wl.raw_bits(23, 0, (512 << 18) * 2 // 8, dev).view(torch.int16)
        ob = torch.empty_like(xb)
        for rows_b, cols_b in ((9, 9), (13, 5), (15, 5)):
            db = rows_b + cols_b
            ntb = (512 << 18) >> db
            big = ll.distributed_layout(4, 6, db - 10, [rows_b, cols_b], [1 << k for k in range(db)])
            ib = wl.gen_index(53, 0, ntb << db, 1 << rows_b, dev)
            ginfo = ll.ll_gather_info(big, 0, 2)
            _, md_ms, _, _ = time_launches(lambda k: ll.ll_gather(big, 0, 2, xb, ib, ob, ntb), args.table_steps, TABLE_WARMUP,
                                           label="gather: row-major %dx%d two-byte tile, rows, %s" % (1 << rows_b, 1 << cols_b, ginfo["kernel_name"]))
            ab = (ntb << db) * (2 + 2 + 4)
            gtable.append({"name": "row-major %dx%d tile, 2-byte elements, gather along dim 0" % (1 << rows_b, 1 << cols_b),
                           "kernel": ginfo["kernel_name"],
                           "axis_bits_reg_lane_wave": [ginfo["axis_reg_bits"], ginfo["axis_lane_bits"], ginfo["axis_wave_bits"]],
                           "paper_rounds": ginfo["paper_rounds"], "staged_bytes": ginfo["block_bytes"],
                           "algorithmic_bytes": ab, "us_mean": round(md_ms * 1e3, 2), "GBps": round(ab / md_ms / 1e6, 1),
                           "frac_hbm_peak": round(ab / md_ms / 1e6 / HBM_PEAK_GBPS, 4)})
            annotate(gtable[-1], "gather: row-major %dx%d two-byte tile, rows, %s" % (1 << rows_b, 1 << cols_b, ginfo["kernel_name"]), ab)
            del ib
        del xb, ob
        result["gather_variants"] = gtable

        # affine layouts (y = A x xor b): config 2 with the destination flipped along both dims (element
        # positions inside every 16-byte vector reverse as well) and config 4 with an arbitrary constant
        atable = []
        for cid_, off_ in ((2, (1 << 14) - 1), (4, 0xB46B)):
            cfg = wl.config(cid_)
            a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
            b = ll.ll_layout_with_offset(ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases), off_)
            plan = ll.ll_plan_convert(a, b, cfg.elem_bytes)
            inf = plan.info()
            x = cfg.gen_data(0, cfg.ntiles, dev)
            outs = [torch.empty_like(x) for _ in range(2 if cid_ == 2 else 1)]
            _, md_ms, _, _ = time_launches(lambda k: ll.ll_convert(plan, x, outs[k % len(outs)], cfg.ntiles), args.table_steps, TABLE_WARMUP,
                                           label="affine: config %d, destination offset 0x%x" % (cid_, off_))
            ab = cfg.algorithmic_bytes()
            atable.append({"name": "config %d, destination offset 0x%x" % (cid_, off_), "kernel": inf["strategy_name"],
                           "conv_offset": inf["conv_offset"], "algorithmic_bytes": ab, "us_mean": round(md_ms * 1e3, 2),
                           "GBps": round(ab / md_ms / 1e6, 1), "frac_hbm_peak": round(ab / md_ms / 1e6 / HBM_PEAK_GBPS, 4)})
            del x, outs
        result["affine_conversions"] = atable

    if args.mark:
        result["sections"] = sections
    if not args.only_main:
        result["c_abi_eager_calls"] = c_abi_call_cost()

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(main_cfg)

    print(json.dumps(result))
    return 0


def c_abi_call_cost():
    """Host cost of an eager ll_convert / ll_gather call through the C ABI, measured by the plain C
    client (tests/c/gpu_client.c --time: 20000 calls back to back on one stream, one tile each,
    configuration 1's layouts), which is compiled here with gcc and run as a child process."""
    import subprocess
    import tempfile
    import paper_2505_23819_amd as ll
    import oracle
    libdir, odir = os.path.dirname(ll.LIBRARY_PATH), os.path.dirname(oracle.build())
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "gpu_client")
        cmd = ["gcc", "-std=c99", "-O1", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
               os.path.join(ROOT, "tests", "c", "gpu_client.c"), "-o", exe,
               "-L", libdir, "-lll355", "-L", odir, "-lll_oracle", "-L", "/opt/rocm/lib", "-lamdhip64",
               "-Wl,-rpath," + libdir, "-Wl,-rpath," + odir, "-Wl,-rpath,/opt/rocm/lib"]
        try:
            subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=120)
            res = subprocess.run([exe, "--time"], capture_output=True, text=True, timeout=120)
        except (OSError, subprocess.SubprocessError) as e:
            return {"error": str(e)[:200]}
    if res.returncode != 0:
        return {"error": res.stderr[-200:]}
    f = res.stdout.split()
    return {"us_per_ll_convert_config1": float(f[1]), "us_per_ll_gather_one_tile": float(f[3]), "calls": int(f[5]),
            "how": "plain C client, back-to-back eager calls on one stream, host clock around the loop and one synchronize"}


def cpu_baseline(cfg):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    import workloads as wl
    if cfg.kind == "gather":
        nt = 256
        x, idx = wl.to_numpy_bits(cfg.gen_data(0, nt)), cfg.gen_idx(0, nt).numpy()
        t0 = time.perf_counter()
        oracle.gather(cfg.src_bases, cfg.out_dim_bits, cfg.axis, x, idx)
        dt = time.perf_counter() - t0
        return {"value": round(cfg.algorithmic_bytes(nt) / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": "oracle_gather on the first %d of %d tiles, single thread" % (nt, cfg.ntiles)}
    nt_table = min(cfg.ntiles, max(1, (512 << 20) // (cfg.tile_elems * cfg.elem_bytes)))   # at most 512 MiB of input
    nt_plain = min(cfg.ntiles, max(1, (256 << 20) // (cfg.tile_elems * cfg.elem_bytes)))   # about 256 MiB of input: 5 s or so
    src = wl.to_numpy_bits(cfg.gen_data(0, nt_table))
    oracle.convert(cfg.src_bases, cfg.dst_bases, src[: cfg.tile_elems])                    # builds / loads the C library
    best, threads = None, 1
    for _ in range(3):
        t0 = time.perf_counter()
        _, threads = oracle.convert(cfg.src_bases, cfg.dst_bases, src, table=True)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    t0 = time.perf_counter()
    oracle.convert(cfg.src_bases, cfg.dst_bases, src[: nt_plain * cfg.tile_elems])
    dt_plain = time.perf_counter() - t0
    return {"value": round(cfg.algorithmic_bytes(nt_table) / best / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": "oracle_convert_table (tabulated map, OpenMP over tiles) on the first %d of %d tiles, best of 3"
                      % (nt_table, cfg.ntiles),
            "plain_single_thread_GBps": round(cfg.algorithmic_bytes(nt_plain) / dt_plain / 1e9, 4),
            "plain_sample": "oracle_convert (bit-by-bit definition) on the first %d tiles, 1 thread" % nt_plain}


if __name__ == "__main__":
    sys.exit(main())
