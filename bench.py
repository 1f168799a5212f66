#!/usr/bin/env python3
"""Benchmark of the fused Hydragen decode-attention call on one MI355X.

A "step" is one hg_hydragen_attn call (batched shared-prefix kernel + per-sequence suffix kernel + LSE merge)
over one synthetic batch that is already resident in HBM.  The default workload is the long-shared-context
configuration the headline metric is quoted on: B=1024 decode queries, MHA 40 heads x 128, shared prefix
P=16384, ragged suffix lengths uniform in [32,128], bf16, N(0,1) values (seed 3).

Prints ONE JSON line: queries/s per layer (mean over the timed region, plus median and minimum of per-step events),
per-kernel rooflines from a second, serialised pass (stage durations measured with HIP events on the streams the
kernels run on), the same for the other configurations (`configs`), the chip's own ceilings measured in the same
run (`ceilings`: a register-only matrix-instruction loop on constant and on random operands, a streaming read), the
speed-up over the non-decomposed per-sequence kernel, and the fp64 CPU oracle timed on a bounded sample of the same
workload (which doubles as a parity spot check of the timed configuration).

`--power-table` is a separate mode: three-second loops of the kernels with the board's power sensor sampled
meanwhile, printed as a text table.
"""
import argparse
import glob
import hashlib
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
CSRC = os.path.join(ROOT, "paper_2402_05099_amd", "csrc")
# the source files each kernel's counters depend on (a stored counter reading is only quoted while they are unchanged)
KERNEL_SOURCES = {
    "prefix_level": ["prefix_wide_impl.h", "prefix_wide.hip", "prefix_wide_step.inc", "prefix.hip", "prefix_common.h", "hg_internal.h"],
    "suffix": ["decode.hip", "decode_mfma.hip", "hg_internal.h"],
}


def sources_sha16(kind: str) -> str:
    h = hashlib.sha256()
    for f in KERNEL_SOURCES[kind]:
        h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()[:16]


def stored_counters(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload` from the tracked rocprofv3 --pmc summaries under profiles/ (lines
    `# machine: {...}`), or None if there is none or the kernel's sources have changed since it was taken."""
    kind = "prefix_level" if kernel.startswith("prefix_level") else kernel
    if kind not in KERNEL_SOURCES:
        return None
    sha = sources_sha16(kind)
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path, errors="replace"):
            m = re.match(r"#\s*machine:\s*(\{.*\})\s*$", line)
            if not m:
                continue
            try:
                rec = json.loads(m.group(1))
            except ValueError:
                continue
            if rec.get("kernel") == kernel and rec.get("workload") == workload and rec.get("sources_sha16") == sha:
                rec["file"] = os.path.relpath(path, ROOT)
                return rec
    return None


def stats(xs):
    import numpy as np
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min())}


def algorithmic_work(w, fp8_kv=False):
    """bytes / flops the method itself has to move per launch of each kernel (what the rooflines are priced on)"""
    import numpy as np
    B, Hq, Hkv, D, nq = w.B, w.Hq, w.Hkv, w.D, w.nq
    rows = B * nq * Hq
    T = int(np.minimum(w.lengths, w.max_len).sum())
    kv_elem = 1 if fp8_kv else 2
    suffix_bytes = 2 * kv_elem * T * Hkv * D + rows * D * 2 + rows * (D + 1) * 4          # K+V rows, Q, partial (O, LSE)
    level_flops, level_bytes = [], []
    for lv in w.levels:
        f = by = 0
        for g in range(lv.Gn):
            nk = int(lv.kv_off[g + 1] - lv.kv_off[g])
            ns = int(lv.seq_off[g + 1] - lv.seq_off[g])
            f += 4 * ns * nq * Hq * nk * D
            by += 4 * nk * Hkv * D + ns * nq * Hq * D * 2 + ns * nq * Hq * (D + 1) * 4
        level_flops.append(f)
        level_bytes.append(by)
    return suffix_bytes, level_flops, level_bytes


def kernel_table(w, stage_stats, nlev, fp8_kv=False):
    """per-kernel rooflines from per-stage duration statistics [suffix, levels.., merge] (ms)"""
    suffix_bytes, level_flops, level_bytes = algorithmic_work(w, fp8_kv)
    kernels = {}
    s = stage_stats[0]
    if s["mean"] > 0:
        kernels["suffix"] = {"bound": "hbm", "ms": s["mean"], "ms_median": s["median"], "ms_min": s["min"],
                             "achieved": suffix_bytes / (s["mean"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "algorithmic": suffix_bytes}
    for i in range(nlev):
        s = stage_stats[1 + i]
        if s["mean"] <= 0:
            continue
        ms = s["mean"]
        tf = level_flops[i] / (ms * 1e-3) / 1e12
        gb = level_bytes[i] / (ms * 1e-3) / 1e9
        # a level is priced against the roofline that binds it: flops/byte above ~312 -> matrix cores, else HBM
        mfma_bound = level_flops[i] / max(level_bytes[i], 1) >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
        base = {"ms": ms, "ms_median": s["median"], "ms_min": s["min"]}
        kernels[f"prefix_level{i}"] = dict(base, **(
            {"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "algorithmic": level_flops[i], "hbm_GBs": gb}
            if mfma_bound else
            {"bound": "hbm", "achieved": gb, "peak": PEAK_HBM_GBS, "unit": "GB/s", "algorithmic": level_bytes[i], "TFLOPs": tf}))
    s = stage_stats[1 + nlev]
    kernels["merge"] = {"bound": "hbm", "ms": s["mean"], "ms_median": s["median"], "ms_min": s["min"], "unit": "GB/s", "peak": PEAK_HBM_GBS}
    for k in kernels.values():
        if "achieved" in k:
            k["frac"] = k["achieved"] / k["peak"]
    return kernels


class Runner:
    """One workload on the device and the ways of timing the fused call on it."""

    def __init__(self, w, args, hb, dev, torch, variant_step=None):
        self.w, self.args, self.hb, self.torch = w, args, hb, torch
        self.dw = dev.to_device(w)
        torch.cuda.synchronize()
        self.ctx = dev.make_context(self.dw, parts=args.parts)
        self.O = torch.empty(self.dw.lead + (self.dw.D,), dtype=torch.bfloat16, device="cuda:0")
        self.L = torch.empty(self.dw.lead, dtype=torch.float32, device="cuda:0")
        self._step = variant_step

    def step(self):
        if self._step is not None:
            return self._step(self)
        dw = self.dw
        self.hb.hg_hydragen_attn(self.ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, self.O, self.L, dw.scale)

    def timed_region(self, n):
        """n calls between two synchronisations, nothing else enqueued: milliseconds per step (the headline)"""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def per_step_events(self, n, flush=None):
        """n calls, each bracketed by its own pair of events on the stream (optionally a cache-flushing write between
        them, outside the brackets): statistics of the device-side duration of a call"""
        torch = self.torch
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        torch.cuda.synchronize()
        for e0, e1 in ev:
            if flush is not None:
                flush.add_(1)
            e0.record()
            self.step()
            e1.record()
        torch.cuda.synchronize()
        return stats([e0.elapsed_time(e1) for e0, e1 in ev])

    def staged(self, n):
        """n calls with the library's per-kernel timing events: (ms per step by the host clock, per-stage statistics)"""
        hb, torch = self.hb, self.torch
        import numpy as np
        self.ctx.set_option(hb.HG_OPT_STAGE_TIMING, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            self.step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st = np.array(self.ctx.read_stage_timings(min(n, hb.HG_TIMING_RING)), dtype=np.float64)
        self.ctx.set_option(hb.HG_OPT_STAGE_TIMING, 0)
        return (t1 - t0) * 1e3 / n, [stats(st[:, i]) for i in range(st.shape[1])]

    def close(self):
        self.ctx.close()


def measure_config(w, args, hb, dev, torch, steps, warmup):
    """the default and the serialised pass of one plain configuration (an entry of `configs`)"""
    r = Runner(w, args, hb, dev, torch)
    for _ in range(warmup):
        r.step()
    ms = r.timed_region(steps)
    ev = r.per_step_events(steps)
    r.ctx.set_option(hb.HG_OPT_OVERLAP, 1)
    for _ in range(3):
        r.step()
    serial_ms, st = r.staged(steps)
    nlev = len(r.dw.levels)
    out = {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
           "shared_levels": [{"blocks": lv.Gn, "rows_per_block": lv.max_rows, "seqs_per_block": lv.max_seqs} for lv in w.levels],
           "suffix_len": [int(w.lengths.min()), int(w.lengths.max())],
           "ms_per_step": ms, "ms_per_step_events": ev, "queries_per_s": w.B * w.nq / (ms * 1e-3),
           "ms_per_step_serialised": serial_ms, "kernels": kernel_table(w, st, nlev)}
    r.close()
    del r
    torch.cuda.empty_cache()
    return out


def device_info(torch):
    """the GPU the figures were taken on: name, CU count, maximum clock, memory, and the board's power cap if the
    sensor is readable"""
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "max_clock_MHz": getattr(p, "clock_rate", 0) / 1e3,
            "memory_GiB": round(p.total_memory / 2 ** 30, 1), "power_cap_W": None}
    try:
        caps = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
        if caps:
            info["power_cap_W"] = int(open(caps[0]).read()) / 1e6
        if not info["max_clock_MHz"]:      # the driver's table of shader clock levels: the highest one
            for f in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
                mhz = [int(m) for m in re.findall(r"(\d+)\s*[Mm][Hh]z", open(f).read())]
                if mhz:
                    info["max_clock_MHz"] = float(max(mhz))
                    break
    except (OSError, ValueError):
        pass
    return info


def measure_ceilings(hb, torch, ctx):
    """what this chip sustains: the matrix instruction alone (constant / random operands) and a streaming read"""
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    iters = 4000
    flops = 256 * 8 * iters * 16 * 32768.0
    out = {}
    for name, rnd in (("mfma_constant_operands", False), ("mfma_random_operands", True)):
        hb.hg_debug_mfma_loop(ctx, rnd, 200, clocks, sink)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            hb.hg_debug_mfma_loop(ctx, rnd, iters, clocks, sink)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            c = clocks.cpu().numpy()
            rec = {"TFLOPs": flops / (ms * 1e-3) / 1e12, "clock_GHz": float(c[0]) / max(float(c[1]), 1.0) * 0.1, "ms": ms}
            if best is None or rec["TFLOPs"] > best["TFLOPs"]:
                best = rec
        best["frac_of_peak"] = best["TFLOPs"] / PEAK_BF16_TFLOPS
        out[name] = best
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    hb.hg_debug_stream_read(ctx, buf, sink)
    torch.cuda.synchronize()
    best = 0.0
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        hb.hg_debug_stream_read(ctx, buf, sink)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["stream_read"] = {"GBs": best, "frac_of_peak": best / PEAK_HBM_GBS, "bytes": buf.numel()}
    del buf
    torch.cuda.empty_cache()
    return out


def power_table(args, hb, dev, wl, torch):
    """three-second loops of the kernels of config 3 and of the two ceiling kernels, board power sampled every 20 ms"""
    files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
    cap = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
    def power():
        for f in files:
            try:
                return int(open(f).read().strip()) / 1e6
            except (OSError, ValueError):
                pass
        return float("nan")
    w = wl.config(args.config, P=args.prefix or None)
    r = Runner(w, args, hb, dev, torch)
    dw, ctx = r.dw, r.ctx
    lv = dw.levels[0]
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    Of = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    print(f"# board power while one call is repeated for 3 s ({w.name}); sensor {files[:1]}, cap {[open(c).read().strip() for c in cap[:1]]} uW, idle {power():.0f} W")
    print("# loop | ms per call | mean W | max W | clock GHz (matrix loops: shader cycles / 100 MHz ticks inside the kernel)")
    def run(name, fn, clock=False):
        samples, stop = [], [False]
        def poll():
            while not stop[0]:
                samples.append((time.time(), power()))
                time.sleep(0.02)
        th = threading.Thread(target=poll)
        th.start()
        t0, n = time.time(), 0
        while time.time() - t0 < 3.0:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
            n += 20
        dt = time.time() - t0
        stop[0] = True
        th.join()
        ps = [p for (t, p) in samples if t - t0 > 1.0]
        ghz = ""
        if clock:
            c = clocks.cpu().numpy()
            ghz = f"{float(c[0]) / max(float(c[1]), 1.0) * 0.1:.2f}"
        print(f"{name} | {dt / n * 1e3:.4f} | {sum(ps) / max(len(ps), 1):.0f} | {max(ps) if ps else float('nan'):.0f} | {ghz}", flush=True)
        time.sleep(1.0)
    run("matrix instruction loop, constant operands (4000 x 16 per wavefront)", lambda: hb.hg_debug_mfma_loop(ctx, False, 4000, clocks, sink), True)
    run("matrix instruction loop, random operands", lambda: hb.hg_debug_mfma_loop(ctx, True, 4000, clocks, sink), True)
    run("streaming read, 2 GiB", lambda: hb.hg_debug_stream_read(ctx, buf, sink))
    run("suffix kernel", lambda: hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, Of, r.L, dw.scale))
    run("shared-block kernel (+ its merge)", lambda: hb.hg_prefix_attn(ctx, dw.Q, lv.K, lv.V, Of, r.L, dw.scale))
    run("fused call, default", r.step)
    ctx.set_option(hb.HG_OPT_OVERLAP, 1)
    run("fused call, serialised", r.step)
    r.close()
    return 0


def wide_timeline(args, hb, dev, wl, torch):
    """Phase time stamps of the persistent shared-block kernel on every shared level of the workload, from a library
    built with -DHG_TRACE (python -m paper_2402_05099_amd.build --out <lib> -DHG_TRACE; HYDRAGEN_LIB=<lib>)."""
    import ctypes
    import numpy as np
    L = hb.lib()
    if not hasattr(L, "hg_debug_read_wide_trace"):
        print("bench.py --wide-timeline needs a -DHG_TRACE build of the library (see HYDRAGEN_LIB)", file=sys.stderr)
        return 2
    L.hg_debug_read_wide_trace.argtypes = [ctypes.c_void_p]
    w = wl.config(args.config, P=args.prefix or None)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=args.parts)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, 2)
    O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    LS = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
    print(f"# prefix_kernel_wide, phase time stamps per workgroup (100 MHz counter; us from the first workgroup's entry), {w.name}")
    for li, lv in enumerate(dw.levels):
        plan = hb.hg_debug_wide_plan(lv.n_blocks, lv.max_rows, lv.max_seqs if lv.kv_off is not None else dw.B, dw.Hkv,
                                     dw.nq * (dw.Hq // dw.Hkv), args.parts, 32)
        for _ in range(3):
            hb.hg_prefix_attn_grouped(ctx, dw.Q, lv, O, LS, dw.scale)
        torch.cuda.synchronize()
        hb.hg_prefix_attn_grouped(ctx, dw.Q, lv, O, LS, dw.scale)
        buf = np.zeros(256 * 32, dtype=np.uint64)
        assert L.hg_debug_read_wide_trace(buf.ctypes.data_as(ctypes.c_void_p)) == 0
        t = buf.reshape(256, 32).astype(np.float64)[:8 * plan["slots"]]
        t0 = t[:, 0].min()
        print(f"level {li}: plan { {k: v for k, v in plan.items() if k not in ('starts', 'first_part')} }")
        print(f"  kernel span {(t[:, 15].max() - t0) / 100:.1f} us; workgroups start between 0 and {(t[:, 0].max() - t0) / 100:.1f} us (mean {(t[:, 0] - t0).mean() / 100:.2f}) "
              f"and leave between {(t[:, 15].min() - t0) / 100:.1f} and {(t[:, 15].max() - t0) / 100:.1f} us; from a workgroup's start to its first piece's entry "
              f"{(t[:, 1] - t[:, 0]).mean() / 100:.2f} (max {(t[:, 1] - t[:, 0]).max() / 100:.2f}): first piece looked up {(t[:, 24] - t[:, 0]).mean() / 100:.2f}, "
              f"copy cursor set {(t[:, 25] - t[:, 24]).mean() / 100:.2f}, two stages' copies issued {(t[:, 26] - t[:, 25]).mean() / 100:.2f}, Q requested "
              f"{(t[:, 27] - t[:, 26]).mean() / 100:.2f}, five more stages {(t[:, 1] - t[:, 27]).mean() / 100:.2f}")
        for p in range(3):
            b = 1 + 4 * p
            ok = t[:, b + 3] > t[:, b]
            if not ok.any():
                continue
            a_, b_, c_, d_ = (t[ok, b + k] for k in range(4))
            cyc = t[ok, 16 + p]
            nst = t[ok, 23 if p == 2 else 13 + p]
            print(f"  piece {p}: {int(ok.sum())} workgroups; entry at {(a_ - t0).mean() / 100:.1f}; wait + first scores {(b_ - a_).mean() / 100:.2f} "
                  f"(max {(b_ - a_).max() / 100:.2f}); steps {(c_ - b_).mean() / 100:.2f} (max {(c_ - b_).max() / 100:.2f}) = {cyc.mean():.0f} cycles "
                  f"at {cyc.mean() / ((c_ - b_).mean() * 10):.2f} GHz, {nst.mean():.1f} stages, {cyc.sum() / nst.sum():.0f} cycles per stage; next Q request + result stores {(d_ - c_).mean() / 100:.2f} (max {(d_ - c_).max() / 100:.2f})")
        # the XCDs one by one (workgroup id % 8; which physical XCD that is varies by launch): the shader clock each ran
        # piece 0 at, its cycles per stage, and when its workgroups left
        ok0 = t[:, 3] > t[:, 2]
        if ok0.all():
            xcd = np.arange(t.shape[0]) & 7
            clk = t[:, 16] / ((t[:, 3] - t[:, 2]) * 10.0)
            cps = t[:, 16] / np.maximum(t[:, 13], 1)
            print("  by XCD (workgroup id % 8): clock GHz " + " ".join(f"{clk[xcd == x].mean():.3f}" for x in range(8))
                  + "; cycles per stage " + " ".join(f"{cps[xcd == x].mean():.0f}" for x in range(8))
                  + "; workgroups leave at " + " ".join(f"{(t[xcd == x, 15] - t0).mean() / 100:.1f}" for x in range(8)))
        ok = t[:, 22] > t[:, 19]
        if ok.any():
            x = t[ok]
            print(f"  boundary between pieces 0 and 1 ({int(ok.sum())} workgroups): next piece looked up {(x[:, 19] - x[:, 3]).mean() / 100:.2f}; "
                  f"Q requested {(x[:, 20] - x[:, 19]).mean() / 100:.2f}; results stored {(x[:, 4] - x[:, 20]).mean() / 100:.2f}; "
                  f"wait for Q {(x[:, 21] - x[:, 5]).mean() / 100:.2f}; barrier {(x[:, 22] - x[:, 21]).mean() / 100:.2f}; "
                  f"first scores {(x[:, 6] - x[:, 22]).mean() / 100:.2f}")
    ctx.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload index 1..6 (default: the headline config 3; 6 = the paper's microbenchmark shape)")
    ap.add_argument("--batch", type=int, default=0, help="config 6: batch size")
    ap.add_argument("--suffix-len", type=int, default=0, help="config 6: suffix length of every sequence")
    ap.add_argument("--prefix", type=int, default=0, help="override the level-0 prefix length")
    ap.add_argument("--head-dim", type=int, default=0, help="head dimension of configs 2..6 (128; 64 is a variant, never the headline)")
    ap.add_argument("--naive-steps", type=int, default=3)
    ap.add_argument("--cpu-sample", type=int, default=256, help="sequences the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--overlap", type=int, default=0, help="HG_OPT_OVERLAP: 0 library default (two streams), 1 one stream, 2 two streams, shared blocks first")
    ap.add_argument("--suffix-chunk", type=int, default=0)
    ap.add_argument("--parts", type=int, default=24)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--prefix-kernel", type=int, default=0, help="0 auto, 1 128-row workgroups, 2 256-row workgroups")
    ap.add_argument("--paged", type=int, default=0, help="rows per page: the suffix cache is a page pool read through a page table (0 = packed rows, the default)")
    ap.add_argument("--fp8-kv", action="store_true", help="the suffix cache holds 8-bit E4M3 codes with one scale per tensor (hg_hydragen_attn_fp8); a variant, not the headline")
    ap.add_argument("--append-steps", type=int, default=0, help="also time this many KV-cache updates (hg_kv_append / _paged), reported as kv_append_ms")
    ap.add_argument("--nq", type=int, default=1, help="queries per sequence (App. B's num_queries: the last nq suffix tokens are queried at once); a variant, value then counts B * nq queries")
    ap.add_argument("--suffix-kernel", type=int, default=0, help="HG_OPT_SUFFIX_KERNEL: 0 automatic, 1 vector-ALU, 2 matrix-core")
    ap.add_argument("--fused-kernel", type=int, default=0, help="HG_OPT_FUSED_KERNEL: 0 automatic, 1 separate kernels, 2 single launch whenever it applies")
    ap.add_argument("--graph", action="store_true", help="also time the fused call replayed from a captured HIP graph (reported as graph_ms_per_step; the headline stays the eager call)")
    ap.add_argument("--wide-slots", type=int, default=0, help="HG_OPT_WIDE_SLOTS: CUs per XCD for the persistent shared-block kernel (0 = library default)")
    ap.add_argument("--flush-mib", type=int, default=0, help="per-step events pass: write a buffer of this many MiB between steps (more than the 256 MiB last-level cache), reported as ms_per_step_events_flushed")
    ap.add_argument("--extra-configs", type=int, default=-1, help="1: also measure configs 2, 3 at P=1024/4096, 4 and 5 (`configs`); default: only in the plain headline run")
    ap.add_argument("--ceilings", type=int, default=-1, help="1: also measure the matrix-instruction and streaming-read ceilings (`ceilings`); default: only in the plain headline run")
    ap.add_argument("--wide-timeline", action="store_true", help="separate mode: per-workgroup phase time stamps of the persistent shared-block kernel (needs a -DHG_TRACE build of the library selected with HYDRAGEN_LIB); prints a text table")
    ap.add_argument("--power-table", action="store_true", help="separate mode: board power while each kernel of the workload is repeated for three seconds; prints a text table")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (attention shards by KV head with no collective inside it); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2402_05099_amd import binding as hb
    from paper_2402_05099_amd import device as dev
    from paper_2402_05099_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    hb.lib()  # fail loudly if the HIP library is missing
    if args.power_table:
        return power_table(args, hb, dev, wl, torch)
    if args.wide_timeline:
        return wide_timeline(args, hb, dev, wl, torch)

    plain = (args.config == 3 and not (args.head_dim or args.prefix or args.batch or args.suffix_len or args.paged or args.fp8_kv or args.nq > 1
                                       or args.splits or args.overlap or args.suffix_chunk or args.prefix_kernel
                                       or args.suffix_kernel or args.fused_kernel or args.wide_slots))
    want_configs = plain if args.extra_configs < 0 else bool(args.extra_configs)
    want_ceilings = plain if args.ceilings < 0 else bool(args.ceilings)

    t0 = time.time()
    variant = {"nq": args.nq} if args.nq > 1 else {}
    w = wl.config(args.config, P=args.prefix or None, B=args.batch or None, L=args.suffix_len or None, D=args.head_dim or None, **variant)

    kv = None
    f8 = None          # packed 8-bit cache
    f8_paged = None    # (PagedSuffix of codes, k_scale, v_scale)

    def variant_step(r):
        dw = r.dw
        if f8 is not None:
            hb.hg_hydragen_attn_fp8(r.ctx, dw.Q, dw.levels, dK8, dV8, f8.k_scale, f8.v_scale, doff8, dw.lengths, dw.max_len, r.O, r.L, dw.scale)
        elif kv is not None:
            hb.hg_hydragen_attn_paged(r.ctx, dw.Q, dw.levels, kv, dw.lengths, dw.max_len, r.O, r.L, dw.scale)
        else:
            hb.hg_hydragen_attn(r.ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, r.O, r.L, dw.scale)

    r = Runner(w, args, hb, dev, torch, variant_step)
    dw, ctx, O, L = r.dw, r.ctx, r.O, r.L
    print(f"[bench] workload {w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} levels={[int(l.K.shape[0]) for l in w.levels]} "
          f"T={w.T} (generated + uploaded in {time.time() - t0:.1f}s)", file=sys.stderr, flush=True)
    if args.splits:
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, args.splits)
    if args.suffix_chunk:
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, args.suffix_chunk)
    ctx.set_option(hb.HG_OPT_OVERLAP, args.overlap)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, args.prefix_kernel)
    if args.wide_slots:
        ctx.set_option(hb.HG_OPT_WIDE_SLOTS, args.wide_slots)
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, args.suffix_kernel)
    ctx.set_option(hb.HG_OPT_FUSED_KERNEL, args.fused_kernel)

    if args.paged and args.fp8_kv:
        f8_paged = wl.make_paged_fp8(w, args.paged, reserve=args.append_steps)
        pg8 = f8_paged[0]
        kv = hb.PagedKV(K=torch.from_numpy(pg8.K).cuda(), V=torch.from_numpy(pg8.V).cuda(),
                        page_table=torch.from_numpy(pg8.table).cuda(), page_size=pg8.page_size, kv_format=hb.HG_KV_E4M3,
                        k_scale=f8_paged[1], v_scale=f8_paged[2])
        torch.cuda.synchronize()
    elif args.paged:
        kv = dev.paged_to_device(wl.make_paged(w, args.paged, reserve=args.append_steps))
        torch.cuda.synchronize()
    elif args.fp8_kv:
        f8 = wl.make_fp8(w, reserve=args.append_steps, junk_code=None)
        dK8, dV8 = torch.from_numpy(f8.Ks8).cuda(), torch.from_numpy(f8.Vs8).cuda()
        doff8 = torch.from_numpy(f8.offsets).cuda()
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        r.step()
    torch.cuda.synchronize()
    if args.calibration_copy_mib > 0:   # a copy kernel of known size: reads and writes exactly this many bytes
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: the library's default configuration, nothing but the calls between two synchronisations ----
    ms_per_step = r.timed_region(args.steps)
    # device-side duration of a call, step by step (median and minimum next to the mean)
    ev_stats = r.per_step_events(args.steps)
    ev_flushed = None
    if args.flush_mib > 0:
        fb = torch.zeros(args.flush_mib << 20, dtype=torch.uint8, device="cuda:0")
        ev_flushed = r.per_step_events(args.steps, flush=fb)
        del fb
    graph_ms = None
    if args.graph:
        # the same call captured once in a HIP graph on a side stream and replayed: no per-launch host work
        gs = torch.cuda.Stream()
        ctx.set_stream(gs)
        with torch.cuda.stream(gs):
            r.step()
        gs.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=gs):
            r.step()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ctx.set_stream(None)
    # per-kernel durations for the rooflines: a second pass of K steps with the kernels serialised on one stream (when
    # they overlap, each one's events also span the other's work) and the library's per-kernel events switched on
    # (which also keeps the call on the separate kernels)
    _, st_overlapped = r.staged(min(args.steps, 20)) if args.overlap != 1 else (None, None)
    ctx.set_option(hb.HG_OPT_OVERLAP, 1)
    for _ in range(3):
        r.step()
    serial_ms_per_step, st = r.staged(args.steps)
    ctx.set_option(hb.HG_OPT_OVERLAP, args.overlap)
    nlev = len(dw.levels)
    kernels = kernel_table(w, st, nlev, args.fp8_kv)

    dom_name = max((k for k in kernels if k != "merge"), key=lambda k: kernels[k]["ms"])
    dom = kernels[dom_name]
    counters = stored_counters(dom_name, w.name)
    roofline = {"kernel": dom_name, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
                "frac": dom["frac"], "traffic": None if counters is None else counters.get("traffic_bytes"),
                "traffic_source": None if counters is None else counters.get("file"),
                "avg_launch_ms": dom["ms"], "median_launch_ms": dom["ms_median"], "min_launch_ms": dom["ms_min"],
                "measured": "HIP events around the kernel on its stream, over the serialised pass of the same K steps"}

    # ---- non-decomposed comparison ----------------------------------------------------------------------------
    naive_ms = None
    if args.naive_steps > 0:
        On = torch.empty_like(O)
        Ln = torch.empty_like(L)
        hb.hg_naive_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, On, Ln, dw.scale)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.naive_steps):
            hb.hg_naive_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, On, Ln, dw.scale)
        e1.record()
        torch.cuda.synchronize()
        naive_ms = e0.elapsed_time(e1) / args.naive_steps

    # ---- KV-cache update of a decode step (optional): the new token's K/V rows appended on the device --------------
    append_ms = None
    if args.append_steps > 0:
        Kn, Vn = wl.new_rows(w)
        dKn, dVn = dev.bf16_tensor(Kn, "cuda:0"), dev.bf16_tensor(Vn, "cuda:0")
        dlen = dw.lengths.clone()
        cap = w.max_len + args.append_steps
        if f8 is not None:
            dK, dV, doff, cap = dK8, dV8, doff8, f8.capacity
        elif kv is None:
            hK, hV, hoff, cap = wl.with_room(w, args.append_steps)
            dK, dV, doff = dev.bf16_tensor(hK, "cuda:0"), dev.bf16_tensor(hV, "cuda:0"), torch.from_numpy(hoff).cuda()
            del hK, hV
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.append_steps):
            if f8 is not None:
                hb.hg_kv_append_fp8(ctx, dKn, dVn, dK, dV, f8.k_scale, f8.v_scale, doff, dlen, cap)
            elif kv is not None:
                hb.hg_kv_append_paged(ctx, dKn, dVn, kv, dlen, cap)
            else:
                hb.hg_kv_append(ctx, dKn, dVn, dK, dV, doff, dlen, cap)
        e1.record()
        torch.cuda.synchronize()
        append_ms = e0.elapsed_time(e1) / args.append_steps
        assert bool((dlen == dw.lengths + args.append_steps).all())

    # ---- CPU oracle on a bounded sample: baseline figure + parity spot check of the timed configuration --------
    cpu = None
    parity = None
    B, Hq, Hkv, nq = w.B, w.Hq, w.Hkv, w.nq
    if args.cpu_sample > 0:
        import oracle
        r.step()                 # the outputs of the default configuration (the serialised pass ran last)
        torch.cuda.synchronize()
        n = min(args.cpu_sample, B)
        seqs = np.unique(np.concatenate([np.linspace(0, B - 1, n).astype(np.int64),
                                         [int(np.argmin(w.lengths)), int(np.argmax(w.lengths))]])).astype(np.int32)
        oracle.attention(w, seqs=seqs[:2])  # warm (library load, page-in)
        c0 = time.perf_counter()
        Oref, Lref = oracle.attention(w, seqs=seqs)
        c1 = time.perf_counter()
        if args.fp8_kv:
            # the timed call read the 8-bit cache: its reference is the merge of the exact attention over the shared
            # levels and the exact attention over the decoded codes (the bf16 run above only times the oracle)
            from oracle import fp8 as ofp8
            Op, Lp = oracle.attention(w, suffix=False, seqs=seqs)
            if f8 is not None:
                K8, V8, off8, ks8, vs8 = f8.Ks8, f8.Vs8, f8.offsets[seqs], f8.k_scale, f8.v_scale
            else:
                pg8, ks8, vs8 = f8_paged
                K8, V8, off8 = oracle.paged_to_packed(pg8.K, pg8.V, pg8.table[seqs], pg8.page_size, w.lengths[seqs])
            Os, Ls = ofp8.suffix_attention_fp8(w.Q[seqs], Hkv, K8, V8, ks8, vs8, off8, w.lengths[seqs], w.scale)
            Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
        cpu = {"value": len(seqs) * nq / (c1 - c0), "unit": "queries/s per layer", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{len(seqs)} of {B} sequences (evenly spaced + shortest and longest suffix), all {Hq} heads, full key lists; "
                         f"{c1 - c0:.1f}s wall"}
        idx = torch.from_numpy(seqs.astype(np.int64)).cuda()
        Og = O[idx].float().cpu().numpy().astype(np.float64)
        Lg = L[idx].cpu().numpy().astype(np.float64)
        dO = float(np.abs(Og - Oref).max())
        dL = float((np.abs(Lg - Lref) / np.abs(Lref)).max())
        rel = float(np.linalg.norm(Og - Oref) / np.linalg.norm(Oref))
        parity = {"max_abs_dO": dO, "max_rel_dLSE": dL, "rel_l2_O": rel, "max_abs_O": float(np.abs(Oref).max()), "sequences": len(seqs)}
        if naive_ms is not None and not args.fp8_kv:    # the comparison call read the bf16 cache
            Ogn = On[idx].float().cpu().numpy().astype(np.float64)
            parity["naive_max_abs_dO"] = float(np.abs(Ogn - Oref).max())
        ok = dO <= 1e-2 and dL <= 1e-3 and rel <= 1e-2
        parity["ok"] = bool(ok)

    ceilings = measure_ceilings(hb, torch, ctx) if want_ceilings else None
    shared_levels = [{"blocks": lv.Gn, "rows_per_block": lv.max_rows, "seqs_per_block": lv.max_seqs} for lv in w.levels]
    r.close()
    del r, dw, O, L
    torch.cuda.empty_cache()

    # ---- the other configurations (their own default and serialised passes) ------------------------------------------
    configs = None
    if want_configs:
        configs = []
        csteps, cwarm = min(args.steps, 30), 5
        for idx, P in ((2, None), (3, 1024), (3, 4096), (4, None), (5, None)):
            t1 = time.time()
            wc = wl.config(idx, P=P)
            configs.append(measure_config(wc, args, hb, dev, torch, csteps, cwarm))
            print(f"[bench] config {idx}{'' if P is None else f' P={P}'}: {configs[-1]['ms_per_step']:.4f} ms per call "
                  f"({time.time() - t1:.1f}s)", file=sys.stderr, flush=True)
            del wc

    st_ms = [s["mean"] for s in st]
    out = {
        "metric": "decode-attn queries/s per layer (B=1024, 16K prefix); MFMA util + HBM GB/s",
        "value": B * nq / (ms_per_step * 1e-3),
        "unit": "queries/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "Hq": Hq, "Hkv": Hkv, "D": w.D, "queries_per_sequence": nq,
                   "shared_levels": shared_levels,
                   "suffix_len": [int(w.lengths.min()), int(w.lengths.max())], "suffix_tokens": int(w.T), "seed": w.seed,
                   "overlap_streams": args.overlap, "suffix_cache": (f"paged, {args.paged} rows per page" if args.paged else "packed rows") + (", 8-bit E4M3 codes" if args.fp8_kv else "")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "ms_per_step_events": ev_stats,
        "ms_per_step_events_flushed": ev_flushed,
        "kernels": kernels,
        "stage_ms": {"suffix": st_ms[0], "prefix_levels": st_ms[1:1 + nlev], "merge": st_ms[1 + nlev], "sum": float(sum(st_ms)),
                     "ms_per_step_serialised": serial_ms_per_step},
        "stage_ms_overlapped": None if st_overlapped is None else {
            "suffix": st_overlapped[0]["mean"], "prefix_levels": [s["mean"] for s in st_overlapped[1:1 + nlev]],
            "merge": st_overlapped[1 + nlev]["mean"], "note": "kernels side by side: each span includes the other's work"},
        "naive": None if naive_ms is None else {"ms_per_step": naive_ms, "queries_per_s": B * nq / (naive_ms * 1e-3),
                                                 "speedup_hydragen_over_naive": naive_ms / ms_per_step},
        "kv_append_ms": append_ms,
        "graph_ms_per_step": graph_ms,
        "parity": parity,
        "ceilings": ceilings,
        "configs": configs,
        "device": device_info(torch),
    }
    print(json.dumps(out))
    if parity is not None and not parity["ok"]:
        print("bench.py: parity spot check FAILED", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
