#!/usr/bin/env python3
"""Benchmark of the fused Hydragen decode-attention call on one MI355X.

A "step" is one hg_hydragen_attn call (batched shared-prefix kernel + per-sequence suffix kernel + LSE merge)
over one synthetic batch that is already resident in HBM.  The default workload is the long-shared-context
configuration the headline metric is quoted on: B=1024 decode queries, MHA 40 heads x 128, shared prefix
P=16384, ragged suffix lengths uniform in [32,128], bf16, N(0,1) values (seed 3).

Prints ONE JSON line: queries/s per layer, per-kernel rooflines (stage durations measured with HIP events on
the streams the kernels run on, inside the timed region), the speed-up over the non-decomposed per-sequence
kernel, and the fp64 CPU oracle timed on a bounded sample of the same workload (which doubles as a parity
spot check of the timed configuration).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/fused_c3_P16384_hbm_traffic.txt),
# each counter scaled by its reading for a 1 GiB device copy (FETCH_SIZE reads 0.50002 of the true KiB on this
# chip, WRITE_SIZE 1.0), keyed by (kernel, workload); None for pairs not measured.
MEASURED_TRAFFIC = {
    ("prefix_level0", "c3_long_P16384"): int((173540.0 / 0.50002 + 51880.4) * 1024),
    ("suffix", "c3_long_P16384"): int((834136.4 / 0.50002 + 20804.8) * 1024),
    ("prefix_level0", "c4_gqa"): int((12480.9 / 0.50003 + 35728.4) * 1024),
    ("suffix", "c4_gqa"): int((276987.8 / 0.50003 + 16513.9) * 1024),
}
# Matrix-core busy fraction of the shared-block kernel from a rocprofv3 --pmc run of its own
# (profiles/fused_c3_P16384_mfma_util.txt): SQ_VALU_MFMA_BUSY_CYCLES / (active cycles x 1024 SIMDs), and the clock
# the kernel ran at (active cycles / duration); keyed like MEASURED_TRAFFIC.
MEASURED_MFMA_UTIL = {
    ("prefix_level0", "c3_long_P16384"): {"mfma_busy_frac_of_cycles": 0.596, "clock_ghz": 1.81},
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload index 1..6 (default: the headline config 3; 6 = the paper's microbenchmark shape)")
    ap.add_argument("--batch", type=int, default=0, help="config 6: batch size")
    ap.add_argument("--suffix-len", type=int, default=0, help="config 6: suffix length of every sequence")
    ap.add_argument("--prefix", type=int, default=0, help="override the level-0 prefix length")
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
    ap.add_argument("--graph", action="store_true", help="also time the fused call replayed from a captured HIP graph (reported as graph_ms_per_step; the headline stays the eager call)")
    ap.add_argument("--wide-slots", type=int, default=0, help="HG_OPT_WIDE_SLOTS: CUs per XCD for the persistent shared-block kernel (0 = library default)")
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

    t0 = time.time()
    variant = {"nq": args.nq} if args.nq > 1 else {}
    w = wl.config(args.config, P=args.prefix or None, B=args.batch or None, L=args.suffix_len or None, **variant)
    dw = dev.to_device(w)
    torch.cuda.synchronize()
    print(f"[bench] workload {w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} levels={[int(l.K.shape[0]) for l in w.levels]} "
          f"T={w.T} (generated + uploaded in {time.time() - t0:.1f}s)", file=sys.stderr, flush=True)

    ctx = dev.make_context(dw, parts=args.parts)
    if args.splits:
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, args.splits)
    if args.suffix_chunk:
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, args.suffix_chunk)
    ctx.set_option(hb.HG_OPT_OVERLAP, args.overlap)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, args.prefix_kernel)
    if args.wide_slots:
        ctx.set_option(hb.HG_OPT_WIDE_SLOTS, args.wide_slots)
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, args.suffix_kernel)

    O = torch.empty(dw.lead + (dw.D,), dtype=torch.bfloat16, device="cuda:0")
    L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")

    kv = None
    f8 = None          # packed 8-bit cache
    f8_paged = None    # (PagedSuffix of codes, k_scale, v_scale)
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

    def step():
        if f8 is not None:
            hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, dK8, dV8, f8.k_scale, f8.v_scale, doff8, dw.lengths, dw.max_len, O, L, dw.scale)
        elif kv is not None:
            hb.hg_hydragen_attn_paged(ctx, dw.Q, dw.levels, kv, dw.lengths, dw.max_len, O, L, dw.scale)
        else:
            hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibration_copy_mib > 0:   # a copy kernel of known size: reads and writes exactly this many bytes
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def timed(n):
        """n fused calls bracketed by synchronisation; returns (ms per step, mean stage ms [suffix, levels.., merge])"""
        ctx.set_option(hb.HG_OPT_STAGE_TIMING, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        stages = np.array(ctx.read_stage_timings(min(n, hb.HG_TIMING_RING)), dtype=np.float64)
        ctx.set_option(hb.HG_OPT_STAGE_TIMING, 0)
        return (t1 - t0) * 1e3 / n, stages.mean(axis=0)

    # the timed region: the library's default configuration (suffix and shared-block kernels overlap on two streams)
    ms_per_step, st_timed = timed(args.steps)
    graph_ms = None
    if args.graph:
        # the same call captured once in a HIP graph on a side stream and replayed: no per-launch host work
        gs = torch.cuda.Stream()
        ctx.set_stream(gs)
        with torch.cuda.stream(gs):
            step()
        gs.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=gs):
            step()
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
    # per-kernel durations for the rooflines: the same K steps again with the kernels serialised on one stream, so
    # that each duration is that kernel alone (when they overlap, each one's events also span the other's work)
    serial_ms_per_step = None
    st = st_timed
    if args.overlap != 1:
        ctx.set_option(hb.HG_OPT_OVERLAP, 1)
        for _ in range(3):
            step()
        serial_ms_per_step, st = timed(args.steps)
        ctx.set_option(hb.HG_OPT_OVERLAP, args.overlap)
    nlev = len(dw.levels)
    suffix_ms, level_ms, merge_ms = float(st[0]), [float(x) for x in st[1:1 + nlev]], float(st[1 + nlev])

    # ---- algorithmic work per launch --------------------------------------------------------------------------
    B, Hq, Hkv, D, G = w.B, w.Hq, w.Hkv, w.D, w.G
    nq = w.nq
    rows = B * nq * Hq
    T = int(np.minimum(w.lengths, w.max_len).sum())
    kv_elem = 1 if args.fp8_kv else 2
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
    kernels = {"suffix": {"bound": "hbm", "ms": suffix_ms, "achieved": suffix_bytes / (suffix_ms * 1e-3) / 1e9 if suffix_ms else 0.0,
                          "peak": PEAK_HBM_GBS, "unit": "GB/s", "algorithmic": suffix_bytes}}
    for i in range(nlev):
        ms = level_ms[i]
        tf = level_flops[i] / (ms * 1e-3) / 1e12 if ms else 0.0
        gb = level_bytes[i] / (ms * 1e-3) / 1e9 if ms else 0.0
        # a level is priced against the roofline that binds it: flops/byte above ~312 -> matrix cores, else HBM
        mfma_bound = level_flops[i] / max(level_bytes[i], 1) >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
        kernels[f"prefix_level{i}"] = (
            {"bound": "mfma", "ms": ms, "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "algorithmic": level_flops[i], "hbm_GBs": gb}
            if mfma_bound else
            {"bound": "hbm", "ms": ms, "achieved": gb, "peak": PEAK_HBM_GBS, "unit": "GB/s", "algorithmic": level_bytes[i], "TFLOPs": tf})
    nparts_bytes = None  # merge: reads every partial once, writes bf16 O + LSE
    kernels["merge"] = {"bound": "hbm", "ms": merge_ms, "unit": "GB/s", "peak": PEAK_HBM_GBS}
    for k in kernels.values():
        if "achieved" in k:
            k["frac"] = k["achieved"] / k["peak"]
    dom_name = max((k for k in kernels if k != "merge"), key=lambda k: kernels[k]["ms"])
    dom = kernels[dom_name]
    roofline = {"kernel": dom_name, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
                "frac": dom["frac"], "traffic": MEASURED_TRAFFIC.get((dom_name, w.name)), "avg_launch_ms": dom["ms"],
                "mfma_util": MEASURED_MFMA_UTIL.get((dom_name, w.name)),
                "measured": "HIP events around the kernel on its stream, mean over the serialised pass of the same K steps"
                            if serial_ms_per_step is not None else "HIP events around the kernel on its stream, mean over the timed region"}

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
    if args.cpu_sample > 0:
        import oracle
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

    out = {
        "metric": "decode-attn queries/s per layer (B=1024, 16K prefix); MFMA util + HBM GB/s",
        "value": B * nq / (ms_per_step * 1e-3),
        "unit": "queries/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "Hq": Hq, "Hkv": Hkv, "D": D, "queries_per_sequence": nq,
                   "shared_levels": [{"blocks": lv.Gn, "rows_per_block": lv.max_rows, "seqs_per_block": lv.max_seqs} for lv in w.levels],
                   "suffix_len": [int(w.lengths.min()), int(w.lengths.max())], "suffix_tokens": int(w.T), "seed": w.seed,
                   "overlap_streams": args.overlap, "suffix_cache": (f"paged, {args.paged} rows per page" if args.paged else "packed rows") + (", 8-bit E4M3 codes" if args.fp8_kv else "")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "stage_ms": {"suffix": suffix_ms, "prefix_levels": level_ms, "merge": merge_ms, "sum": float(st.sum()),
                     "ms_per_step_serialised": serial_ms_per_step},
        "stage_ms_timed_region": {"suffix": float(st_timed[0]), "prefix_levels": [float(x) for x in st_timed[1:1 + nlev]],
                                  "merge": float(st_timed[1 + nlev]), "note": "kernels overlap: each span includes the other's work"},
        "naive": None if naive_ms is None else {"ms_per_step": naive_ms, "queries_per_s": B * nq / (naive_ms * 1e-3),
                                                 "speedup_hydragen_over_naive": naive_ms / ms_per_step},
        "kv_append_ms": append_ms,
        "graph_ms_per_step": graph_ms,
        "parity": parity,
    }
    print(json.dumps(out))
    ctx.close()
    if parity is not None and not parity["ok"]:
        print("bench.py: parity spot check FAILED", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
