#!/usr/bin/env python3
"""Benchmark of the per-partition einsum hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--headline-only] [--only NAME] [--calibrate-copy] [--probe-power]

A step is one pass of the hot path over the Transformer feed-forward share
(BSM,MH->BSH, B=8 S=2048 M=8192 H_local=8192, bf16 operands, fp32 accumulate, bf16 out):
shard bounds + dot classification + problem planning on the host and the fused
pad/mask + MFMA contraction + epilogue on the GPU, through the C ABI's grouped entry
point, inputs resident in HBM.  Prints ONE JSON line.  The other benchmark configs
(contracting split with on-GPU reduce, MoE experts, 4x8 nested mesh), the second einsum of each layer
and the backward contractions of the feed-forward layer are timed the same way and reported under "others".  The CPU oracle is timed on a bounded row sample of the
same workload and its result is compared with the GPU output of those rows.  Before the W warm-up steps the step is run
untimed for 80 ms, so that the clock has recovered from the idle staging period whatever W is.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 4096 flop/clk/CU x 2.4 GHz (dense bf16 MFMA)
PEAK_HBM_GBS = 8000.0
# L2 <-> fabric bytes of one dot_mfma_kernel launch on the FFN share, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled
# by a copy kernel of known size (profiles/dot_mfma_kernel_ffn_share.md): 3.224e9 fetched + 0.268e9 written
FFN_TRAFFIC_BYTES = 3.224e9 + 0.268e9
FFN_TRAFFIC_SOURCE = ("profiles/dot_mfma_kernel_ffn_share.md: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE per dispatch, scaled by "
                      "bench.py --calibrate-copy; a profiler figure quoted here, not measured by this run")
METRIC = "per-shard einsum bf16 TFLOP/s and % of MI355X MFMA peak (1 GPU)"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=40,
                    help="untimed warm-up steps (after an idle period the GPU needs about 30 launches = 50 ms to reach its steady clock)")
    ap.add_argument("--headline-only", action="store_true", help="skip the other configs and the CPU baseline")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="rows of the FFN output the CPU oracle is timed on")
    ap.add_argument("--only", default=None,
                    help="time just one of the other workloads (by name, e.g. moe_ecm_emh) and print its entry; for profiling")
    ap.add_argument("--moe-fill", type=int, default=None,
                    help="with --only moe_ecm_emh (or another workload with fill counts): every expert filled to this many "
                         "rows instead of the seed-drawn counts (a diagnostic variant, not the benchmark's configuration)")
    ap.add_argument("--tile-timeline", default=None, metavar="NAME",
                    help="per-workgroup timeline of dot_mfma_kernel on one workload (its name, or ffn_bsm_mh for the headline): "
                         "where a tile's time goes and how fast each XCD works; prints one JSON line")
    ap.add_argument("--probe-power", action="store_true",
                    help="run only the power probe: the headline kernel looped for 4 s on the benchmark's data and on all-zero "
                         "operands, with the shader clock and package power sampled from rocm-smi (the kernel is power-limited: "
                         "same cycles per launch, different clock)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain copy of known size (shard_extract of a [16384,8192] bf16 tensor on a 1-partition "
                         "mesh: 268435456 bytes read, 268435456 written per launch) for scaling HBM byte counters")
    return ap.parse_args()


def sample_clock_under_load(step, torch, seconds=1.5):
    """Shader clock and package power as rocm-smi reports them while the headline step runs back to back (outside the
    timed region): the kernel is power-limited, so the clock the data allows is part of the result.  None if rocm-smi
    is missing or prints something else."""
    import re
    import shutil
    import subprocess
    import threading
    # Not under a profiler: its preloaded library would initialise the GPU in every child process, and rocm-smi is a
    # script that re-executes an interpreter.  The script is run with this interpreter directly for the same reason.
    if any("rocprof" in os.environ.get(k, "").lower() for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "ROCPROFILER_LIBRARY_CTOR")):
        return None
    smi = shutil.which("rocm-smi")
    if smi is None:
        return None
    samples, done = [], threading.Event()

    def sampler():
        time.sleep(0.4)
        while not done.is_set():
            try:
                out = subprocess.run([sys.executable, smi, "--showclocks", "--showpower", "--json"], capture_output=True,
                                     text=True, timeout=10).stdout
                card = json.loads(out)
                card = card[sorted(card)[0]]
                entry = {}
                for key, val in card.items():
                    lk = key.lower()
                    m = re.search(r"(\d+(?:\.\d+)?)", str(val))
                    if not m:
                        continue
                    if "sclk" in lk and "speed" in lk:
                        entry["sclk_mhz"] = float(m.group(1))
                    elif "power" in lk and "max" not in lk:
                        entry["power_w"] = float(m.group(1))
                if entry:
                    samples.append(entry)
            except Exception:
                return
            time.sleep(0.1)
    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    done.set()
    th.join(timeout=15)
    if not samples:
        return None
    out = {"samples": len(samples), "source": "rocm-smi --showclocks --showpower, sampled while the headline step loops"}
    for k in ("sclk_mhz", "power_w"):
        vals = [e[k] for e in samples if k in e]
        if vals:
            out[k] = round(sum(vals) / len(vals), 1)
    return out


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs all mesh partitions as virtual partitions on ONE GPU; "
                         "--gpus must be 1 (no multi-GPU path exists)\n")
        sys.exit(2)
    import torch
    import paper_2105_04663_amd as g
    import workloads as wl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(2)
    g.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream

    if args.calibrate_copy:
        src = torch.randn(16384, 8192, device=dev).to(torch.bfloat16)
        dst = torch.empty_like(src)
        mesh, sh = g.Mesh((1,), (0,)), g.Sharding((16384, 8192), (-1, -1))
        for _ in range(5):
            g.shard_extract(mesh, sh, 0, src.data_ptr(), g.ShardBuf.of(dst, 0), 0, stream)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"calibrate_copy": "shard_copy_kernel", "launches": 5, "bytes_read_per_launch": src.numel() * 2,
                          "bytes_written_per_launch": src.numel() * 2}), flush=True)
        return

    def dev_tensor(arr, dtype):
        if dtype == "bf16":
            return torch.from_numpy(arr.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(arr).to(dev)

    class Staged:
        """Per-partition shard buffers of one workload (rows padded to 8 elements)."""

        def __init__(self, w, lhs_np=None, rhs_np=None):
            self.w = w
            self.mesh = g.Mesh(tuple(w.mesh_shape), tuple(w.device_ids))
            self.dims = g.DotDims(tuple(w.lhs_batch), tuple(w.rhs_batch), tuple(w.lhs_contract), tuple(w.rhs_contract))
            self.lhs_sh = g.Sharding(tuple(w.lhs_shape), tuple(w.lhs_map))
            self.rhs_sh = g.Sharding(tuple(w.rhs_shape), tuple(w.rhs_map))
            self.out_sh = g.Sharding(tuple(w.out_shape), tuple(w.out_map))
            if w.fill_range is not None and args.moe_fill is not None:
                # the override replaces the drawn counts before the lhs is drawn, so that exactly the rows beyond it are zero
                n_experts = w.lhs_shape[0]
                w.draw_fill = lambda: np.full(n_experts, args.moe_fill, dtype=np.int64)
            self.fill = w.draw_fill()
            lhs_np = w.draw_lhs() if lhs_np is None else lhs_np
            rhs_np = w.draw_rhs() if rhs_np is None else rhs_np
            gl, gr = dev_tensor(lhs_np, w.dtype), dev_tensor(rhs_np, w.dtype)
            self.keep, cache = [], {}
            self.lhs, self.rhs, self.out = [], [], []
            tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
            odt = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
            P = w.n_partitions
            for pid in range(P):
                for tag, sh, glob, store, dt in (("l", self.lhs_sh, gl, self.lhs, tdt), ("r", self.rhs_sh, gr, self.rhs, tdt),
                                                 ("o", self.out_sh, None, self.out, odt)):
                    off, valid, shard = g.shard_bounds(self.mesh, sh, pid)
                    key = (tag, off)
                    if key not in cache:
                        if P == 1 and glob is not None:
                            t, ld = glob, 0           # one partition: the global tensor is the shard
                        else:
                            ld = -(-shard[-1] // 8) * 8
                            rows = int(np.prod(shard[:-1], dtype=np.int64))
                            t = torch.zeros(rows * ld, dtype=dt, device=dev)
                            if glob is not None:
                                g.shard_extract(self.mesh, sh, pid, glob.data_ptr(), g.ShardBuf.of(t, ld), 0, stream)
                        cache[key] = (g.ShardBuf.of(t, ld), t, ld, shard)
                    store.append(cache[key])
            nbytes = g.dot_workspace_bytes(self.mesh, self.dims, self.lhs_sh, self.rhs_sh, self.out_sh, -1, self.fill is not None)
            self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
            self.ws_base = (self.ws.data_ptr() + 255) // 256 * 256
            self.ws_bytes = nbytes
            torch.cuda.synchronize()
            if P > 1:
                del gl, gr

        def step(self):
            g.grouped_dot(self.mesh, self.dims, [x[0] for x in self.lhs], self.lhs_sh, [x[0] for x in self.rhs], self.rhs_sh,
                          [x[0] for x in self.out], self.out_sh, self.fill, self.ws_base, self.ws_bytes, stream)

    def timed(st, steps, warmup):
        for _ in range(warmup):
            st.step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            st.step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        ev_ms = e0.elapsed_time(e1) / steps
        return wall_ms, ev_ms

    other_makers = (wl.ksplit, wl.moe, wl.mesh2d, wl.ffn_second, lambda: wl.ffn_second(scatter=True), wl.moe_second, wl.ffn_wgrad,
                    wl.ffn_dgrad, wl.moe_wgrad)

    def run_other(ww):
        s2 = Staged(ww)
        # staging leaves the GPU idle for seconds: warm up for at least 80 ms (and 5 steps) before timing
        t_w, n_w = time.perf_counter(), 0
        while n_w < 5 or time.perf_counter() - t_w < 0.08:
            s2.step()
            n_w += 1
            if n_w % 5 == 0:
                torch.cuda.synchronize()
        wall, ev = timed(s2, max(10, args.steps // 2), 2)
        fl = ww.useful_flops(s2.fill)
        entry = {"ms_per_step": round(wall, 4), "tflops": round(fl / (wall * 1e-3) / 1e12, 2),
                 "pct_of_peak": round(100.0 * fl / (wall * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2), "useful_flops": fl,
                 # the other convention: static shard shapes and all capacity slots counted as work
                 "padded_flops": ww.padded_flops(),
                 "einsum": ww.einsum, "partitions": ww.n_partitions,
                 # the step's device time between two events on the launch stream: the contraction kernel plus, where the
                 # workload has them, the zero fill and the sum of partials
                 "roofline": {"bound": "mfma", "achieved": round(fl / (ev * 1e-3) / 1e12, 2), "peak": PEAK_BF16_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(fl / (ev * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "flops": fl,
                              "kernel": "dot_mfma_kernel", "device_ms": round(ev, 4)}}
        if s2.fill is not None:
            entry["fill"] = [int(x) for x in s2.fill]
        del s2
        torch.cuda.empty_cache()
        return entry

    if args.probe_power:
        w = wl.ffn()
        st = Staged(w)
        flops = w.useful_flops()
        out = {"probe": "power", "workload": w.einsum, "seconds_per_case": 4.0}
        for tag in ("benchmark_data", "all_zero_operands"):
            if tag == "all_zero_operands":
                for x in st.lhs + st.rhs:
                    x[1].zero_()
            for _ in range(40):
                st.step()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n_steps = [0]

            def counted():
                n_steps[0] += 1
                st.step()
            e0.record()
            load = sample_clock_under_load(counted, torch, seconds=4.0)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / max(n_steps[0], 1)
            out[tag] = {"ms_per_launch": round(ms, 4), "tflops": round(flops / ms / 1e9, 1), "launches": n_steps[0], "rocm_smi": load}
        print(json.dumps(out), flush=True)
        return

    if args.tile_timeline:
        ww = None
        for make in (wl.ffn,) + other_makers:
            cand = make()
            if cand.name == args.tile_timeline:
                ww = cand
        if ww is None:
            sys.stderr.write("bench.py: no workload named %r\n" % args.tile_timeline)
            sys.exit(2)
        st = Staged(ww)
        for _ in range(40):
            st.step()
        torch.cuda.synchronize()
        cap = 1 << 17
        rec = torch.zeros(cap * g.TILE_TIMELINE_WORDS, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        # several launches back to back, each overwriting the records of the one before: what is read back is the
        # last one, which started on a busy GPU like the launches the benchmark times
        g.set_tile_timeline(rec.data_ptr(), cap)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(5):
            st.step()
        e0.record()
        st.step()
        e1.record()
        torch.cuda.synchronize()
        g.set_tile_timeline(0, 0)
        d = rec.cpu().numpy().view(np.uint64).reshape(cap, g.TILE_TIMELINE_WORDS)
        d = d[d[:, 0] != 0]
        where = (d[:, 0] >> np.uint64(52)).astype(np.int64)
        ts = d.copy()
        ts[:, 0] &= np.uint64((1 << 52) - 1)
        ts = ts.astype(np.float64) * 0.01                      # microseconds (100 MHz counter)
        done = ts[:, 7] > 0                                    # workgroups that stored an output tile
        t0 = ts[:, 0].min()

        def seg(i, j, rows):
            x = ts[rows, j] - ts[rows, i]
            return {"mean": round(float(x.mean()), 2), "median": round(float(np.median(x)), 2),
                    "p10": round(float(np.percentile(x, 10)), 2), "p90": round(float(np.percentile(x, 90)), 2)}
        every = np.ones(len(ts), dtype=bool)
        out = {"tile_timeline": ww.name, "unit": "us", "workgroups": int(len(ts)), "call_ms": round(e0.elapsed_time(e1), 4),
               "first_entry_to_last_store_ms": round(float(ts[done, 7].max() - t0) / 1e3, 4),
               "entry_to_tile_decoded": seg(0, 1, every), "decoded_to_first_loads_issued": seg(1, 2, every),
               "loads_issued_to_k_loop_entered": seg(2, 3, every), "k_loop": seg(3, 4, every),
               "k_loop_left_to_epilogue": seg(4, 5, done), "epilogue_stores_issued": seg(5, 6, done),
               "stores_complete": seg(6, 7, done), "whole_workgroup": seg(0, 7, done)}
        xcd = where >> 8
        cu = where                                             # XCD id and compute-unit bits together name a compute unit
        gaps, last_end = [], []
        for c in np.unique(cu):
            idx = np.where((cu == c) & done)[0]
            if len(idx) == 0:
                continue
            o = idx[np.argsort(ts[idx, 0])]
            gaps.extend((ts[o[1:], 0] - ts[o[:-1], 7]).tolist())
            last_end.append(ts[o[-1], 7] - t0)
        if gaps:
            out["stores_complete_to_next_entry_same_cu"] = {"mean": round(float(np.mean(gaps)), 2), "median": round(float(np.median(gaps)), 2),
                                                            "p90": round(float(np.percentile(gaps, 90)), 2)}
        # every workgroup, also those that leave after handing in a joined contribution: from entry to the end of its K loop
        busy = []
        for c in np.unique(cu):
            idx = np.where(cu == c)[0]
            o = idx[np.argsort(ts[idx, 0])]
            end = np.where(done[o], ts[o, 7], ts[o, 4])
            busy.append(float((end - ts[o, 0]).sum()))
        out["busy_per_cu_entry_to_last_stamp"] = {"min": round(min(busy), 1), "mean": round(float(np.mean(busy)), 1), "max": round(max(busy), 1)}
        out["compute_units"] = int(len(np.unique(cu)))
        out["last_store_per_cu"] = {"min": round(float(np.min(last_end)), 1), "mean": round(float(np.mean(last_end)), 1),
                                    "max": round(float(np.max(last_end)), 1)}
        out["per_xcd"] = {str(int(x)): {"workgroups": int((xcd == x).sum()),
                                        "mean_workgroup": round(float((ts[(xcd == x) & done, 7] - ts[(xcd == x) & done, 0]).mean()), 2),
                                        "mean_k_loop": round(float((ts[xcd == x, 4] - ts[xcd == x, 3]).mean()), 2)}
                          for x in np.unique(xcd)}
        order = np.argsort(ts[:, 0])
        kl = (ts[:, 4] - ts[:, 3])[order]
        n8 = max(len(kl) // 8, 1)
        out["mean_k_loop_by_start_order_eighths"] = [round(float(kl[i * n8:(i + 1) * n8].mean()), 2) for i in range(8) if i * n8 < len(kl)]
        print(json.dumps(out), flush=True)
        return

    if args.only:
        for make in other_makers:
            ww = make()
            if ww.name == args.only:
                print(json.dumps({ww.name: run_other(ww)}), flush=True)
                return
        sys.stderr.write("bench.py: no workload named %r\n" % args.only)
        sys.exit(2)

    # ------------------------------------------------------------------ headline: FFN share
    w = wl.ffn()
    lhs_np, rhs_np = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs_np, rhs_np)
    # staging left the GPU idle for seconds and its clock low: run the step for at least 80 ms before the W warm-up steps,
    # so that a small --warmup still times the steady state (none of this is timed)
    t_w, n_w = time.perf_counter(), 0
    while time.perf_counter() - t_w < 0.08:
        st.step()
        n_w += 1
        if n_w % 5 == 0:
            torch.cuda.synchronize()
    wall_ms, ev_ms = timed(st, args.steps, args.warmup)
    # per-launch durations of a second pass (one event pair per step): median and minimum beside the mean
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    evs[0].record()
    for i in range(args.steps):
        st.step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    prop = torch.cuda.get_device_properties(0)
    flops = w.useful_flops()
    under_load = None if args.headline_only else sample_clock_under_load(st.step, torch)
    tflops = flops / (wall_ms * 1e-3) / 1e12
    kern_tflops = flops / (ev_ms * 1e-3) / 1e12
    result = {
        "metric": METRIC, "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ffn_bsm_mh: BSM,MH->BSH B=8 S=2048 M=8192 H_local=8192 (one device's share of a 2D mesh)",
                   "einsum": w.einsum, "useful_flops": flops, "padded_flops": w.padded_flops(), "entry_point": "gspmd_grouped_dot"},
        "pct_of_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {"bound": "mfma", "achieved": round(kern_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(kern_tflops / PEAK_BF16_TFLOPS, 4), "traffic": FFN_TRAFFIC_BYTES,
                     "traffic_source": FFN_TRAFFIC_SOURCE,
                     "algorithmic_bytes": 16384 * 8192 * 2 + 8192 * 8192 * 2 + 16384 * 8192 * 2,
                     "kernel": "dot_mfma_kernel", "kernel_ms": round(ev_ms, 4),
                     "kernel_ms_median": round(per[len(per) // 2], 4), "kernel_ms_min": round(per[0], 4)},
        "device": {"name": prop.name, "compute_units": prop.multi_processor_count, "hbm_gib": round(prop.total_memory / 2 ** 30, 1),
                   "max_clock_mhz": getattr(prop, "clock_rate", 0) // 1000 or None,
                   "peak_used": "256 CU x 4096 flop/clk x 2.4 GHz = 2516.6 TFLOP/s dense bf16; HBM 8 TB/s",
                   "under_load": under_load},
    }

    if under_load and under_load.get("sclk_mhz"):
        # Clock-normalised view, so that a kernel change can be told from a faster or slower box: shader cycles a
        # compute unit spends per 64-wide K step of one 256 x 256 tile (2048 of them would be back-to-back MFMAs), and the
        # fraction of the peak AT THE SAMPLED CLOCK.  The clock is sampled outside the timed region, under the same load.
        tiles_per_cu = (16384 // 256) * (8192 // 256) / prop.multi_processor_count
        k_steps = 8192 // 64
        clk = under_load["sclk_mhz"] * 1e6
        result["roofline"]["sclk_mhz_under_load"] = under_load["sclk_mhz"]
        result["roofline"]["shader_cycles_per_k_step"] = round(ev_ms * 1e-3 * clk / (tiles_per_cu * k_steps), 1)
        result["roofline"]["frac_at_sampled_clock"] = round(kern_tflops * 1e12 / (prop.multi_processor_count * 4096 * clk), 4)

    # ------------------------------------------------------------------ CPU oracle on a row sample
    if not args.headline_only:
        from oracle import dot as od
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        rows = min(args.cpu_rows, w.lhs_shape[1] * w.lhs_shape[0])
        b_take = max(1, rows // w.lhs_shape[1])
        s_take = rows // b_take
        t0 = time.perf_counter()
        a64 = wl.bf16_bits_to_f64(lhs_np[:b_take, :s_take])
        b64 = wl.bf16_bits_to_f64(rhs_np)
        ref = od.dot_general(a64, b64, w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
        cpu_s = time.perf_counter() - t0
        cpu_flops = 2.0 * b_take * s_take * w.lhs_shape[2] * w.rhs_shape[1]
        got = st.out[0][1].view(w.out_shape)[:b_take, :s_take].float().cpu().numpy().astype(np.float64)
        scaled, fro = od.error_metrics(got, ref)
        result["cpu_baseline"] = {"value": round(cpu_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores),
                                  "kind": "oracle", "seconds": round(cpu_s, 2),
                                  "sample": f"fp64 oracle on output rows [0:{b_take},0:{s_take}] of the FFN share "
                                            f"({b_take * s_take} of 16384 rows, all 8192 columns), incl. bf16->fp64 widening"}
        result["parity_vs_oracle"] = {"rows": b_take * s_take, "max_scaled_err": float(f"{scaled:.3e}"),
                                      "rel_frobenius": float(f"{fro:.3e}"), "ok": bool(scaled <= 1e-2 and fro <= 5e-3)}
        del a64, b64, ref, got
    del st, lhs_np, rhs_np
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ the other configs
    if not args.headline_only:
        others = {}
        for make in other_makers:
            ww = make()
            others[ww.name] = run_other(ww)
        # the HBM-bound helpers: sum of the four fp32 K-partials of config 3 (public reduce call on buffers of that size),
        # and the AllGather of BSM's M over a 4-partition mesh dimension that precedes the feed-forward einsum (Table 1)
        def timed_call(fn, steps, warmup):
            t_w = time.perf_counter()
            while warmup > 0 or time.perf_counter() - t_w < 0.08:
                fn()
                warmup -= 1
                if warmup % 5 == 0:
                    torch.cuda.synchronize()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps

        n_el = 4096 * 8192
        parts = [torch.randn(n_el, device=dev) for _ in range(4)]
        red = torch.empty(n_el, device=dev)
        ms = timed_call(lambda: g.reduce_partials([t.data_ptr() for t in parts], n_el, red.data_ptr(), g.F32, stream), 20, 3)
        rbytes = 5 * n_el * 4
        others["ksplit_matmul"]["reduce_alone"] = {"kernel": "reduce_partials_kernel", "ms": round(ms, 4), "algorithmic_bytes": rbytes,
                                                   "gbs": round(rbytes / ms / 1e6, 1), "frac_of_hbm_peak": round(rbytes / ms / 1e6 / PEAK_HBM_GBS, 3),
                                                   "roofline": {"bound": "hbm", "achieved": round(rbytes / ms / 1e6, 1), "peak": PEAK_HBM_GBS,
                                                                "unit": "GB/s", "frac": round(rbytes / ms / 1e6 / PEAK_HBM_GBS, 4),
                                                                "algorithmic_bytes": rbytes, "kernel": "reduce_partials_kernel"}}
        del parts, red
        # the contraction part of config 3 alone: the four partitions' partial products as one launch of four problems
        # (the partition index as a batch dimension), fp32 partials written, no sum
        mesh1 = g.Mesh((1,), (0,))
        pd = g.DotDims((0,), (0,), (2,), (1,))
        pa = torch.randn(4, 4096, 4096, device=dev).to(torch.bfloat16)
        pb = (torch.randn(4, 4096, 8192, device=dev) * 0.02).to(torch.bfloat16)
        pc = torch.empty(4, 4096, 8192, device=dev)
        psh = [g.Sharding(tuple(t.shape), (-1, -1, -1)) for t in (pa, pb, pc)]
        pn = g.dot_workspace_bytes(mesh1, pd, psh[0], psh[1], psh[2], -1, False)
        pws = torch.empty(pn + 256, dtype=torch.uint8, device=dev)
        pbase = (pws.data_ptr() + 255) // 256 * 256
        ms = timed_call(lambda: g.grouped_dot(mesh1, pd, [g.ShardBuf.of(pa, 0)], psh[0], [g.ShardBuf.of(pb, 0)], psh[1],
                                              [g.ShardBuf.of(pc, 0)], psh[2], None, pbase, pn, stream), 20, 3)
        pfl = 2.0 * 4 * 4096 * 4096 * 8192
        others["ksplit_matmul"]["gemm_alone"] = {"kernel": "dot_mfma_kernel (fp32 partials)", "ms": round(ms, 4),
                                                 "tflops": round(pfl / ms / 1e9, 2),
                                                 "pct_of_peak": round(100.0 * pfl / ms / 1e9 / PEAK_BF16_TFLOPS, 2),
                                                 "roofline": {"bound": "mfma", "achieved": round(pfl / ms / 1e9, 2), "peak": PEAK_BF16_TFLOPS,
                                                              "unit": "TFLOP/s", "frac": round(pfl / ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                                                              "flops": pfl, "kernel": "dot_mfma_kernel"}}
        del pa, pb, pc, pws
        mesh4 = g.Mesh((4,), (0, 1, 2, 3))
        shp = (8, 2048, 8192)
        src_sh, dst_sh = g.Sharding(shp, (-1, -1, 0)), g.Sharding(shp, (-1, -1, -1))
        srcs = [torch.randn(8 * 2048 * 2048, device=dev).to(torch.bfloat16) for _ in range(4)]
        dst = torch.empty(8 * 2048 * 8192, dtype=torch.bfloat16, device=dev)
        nws = g.reshard_workspace_bytes(mesh4)
        wsr = torch.empty(nws + 256, dtype=torch.uint8, device=dev)
        wbase = (wsr.data_ptr() + 255) // 256 * 256
        sb, db = [g.ShardBuf.of(t, 0) for t in srcs], [g.ShardBuf.of(dst, 0)] * 4
        ms = timed_call(lambda: g.reshard(mesh4, src_sh, sb, dst_sh, db, wbase, nws, stream), 20, 3)
        gbytes = 2 * dst.numel() * 2
        others["reshard_allgather_bsm"] = {"kernel": "reshard_kernel", "what": "BSM [8,2048,8192] bf16, M split 4 ways -> whole (one shared dst buffer)",
                                           "ms": round(ms, 4), "algorithmic_bytes": gbytes, "gbs": round(gbytes / ms / 1e6, 1),
                                           "frac_of_hbm_peak": round(gbytes / ms / 1e6 / PEAK_HBM_GBS, 3),
                                           "roofline": {"bound": "hbm", "achieved": round(gbytes / ms / 1e6, 1), "peak": PEAK_HBM_GBS,
                                                        "unit": "GB/s", "frac": round(gbytes / ms / 1e6 / PEAK_HBM_GBS, 4),
                                                        "algorithmic_bytes": gbytes, "kernel": "reshard_kernel"}}
        del srcs, dst
        result["others"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
