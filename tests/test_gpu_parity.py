"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle on identical seeded inputs."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2402_05099_amd import binding as hb
from paper_2402_05099_amd import device as dev
from paper_2402_05099_amd import workloads as wl
from parity import check, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def outputs(dw, dtype=torch.float32, canary=True):
    """O/LSE buffers surrounded by NaN canaries so that out-of-range writes are seen."""
    n = dw.rows * dw.D
    pad = 256
    fo = torch.full((n + 2 * pad,), float("nan"), dtype=dtype, device="cuda:0")
    fl = torch.full((dw.rows + 2 * pad,), float("nan"), dtype=torch.float32, device="cuda:0")
    O = fo[pad:pad + n].view(dw.lead + (dw.D,))
    L = fl[pad:pad + dw.rows].view(dw.lead)

    def intact():
        torch.cuda.synchronize()
        return bool(torch.isnan(fo[:pad]).all() and torch.isnan(fo[pad + n:]).all()
                    and torch.isnan(fl[:pad]).all() and torch.isnan(fl[pad + dw.rows:]).all())
    return O, L, intact


WORKLOADS = {}


def workload(key, **variant):
    k = (key, tuple(sorted(variant.items())))
    if k not in WORKLOADS:
        w = wl.scaled_down(key, **variant) if isinstance(key, int) else key()
        WORKLOADS[k] = (w, dev.to_device(w))
    return WORKLOADS[k]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("in_bf16,out_bf16", [(False, False), (False, True), (True, True), (True, False)])
def test_merge(D, in_bf16, out_bf16):
    say(f"merge D={D} in_bf16={in_bf16} out_bf16={out_bf16}")
    rng = np.random.default_rng(11)
    rows = 1000 + 37
    ctx = hb.Context(0, 0)
    for n in (1, 2, 3, 7):
        Os = [wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(rng.standard_normal((rows, D)).astype(np.float32))) for _ in range(n)]
        Ls = [(rng.standard_normal(rows) * 4).astype(np.float32) for _ in range(n)]
        for i in range(n):  # sprinkle empty parts, and make row 5 empty everywhere
            Ls[i][rng.integers(0, rows, 50)] = -np.inf
            Ls[i][5] = -np.inf
        Oref, Lref = oracle.merge(Os, Ls)
        tin = torch.bfloat16 if in_bf16 else torch.float32
        tO = [torch.from_numpy(o).cuda().to(tin) for o in Os]
        tL = [torch.from_numpy(l).cuda() for l in Ls]
        # uninitialised O of an empty part must never leak into the result
        for i in range(n):
            tO[i][torch.isneginf(tL[i])] = float("nan")
        Oout = torch.full((rows, D), float("nan"), dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda:0")
        Lout = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda:0")
        hb.hg_merge(ctx, tO, tL, Oout, Lout)
        torch.cuda.synchronize()
        check(to_np(Oout), to_np(Lout), Oref, Lref, f"merge n={n}", out_bf16=out_bf16)
        assert float(Oout[5].abs().max()) == 0.0
    ctx.close()


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("chunk", [0, 32])
def test_suffix_attn(idx, chunk):
    say(f"suffix idx={idx} chunk={chunk}")
    w, dw = workload(idx)
    ctx = dev.make_context(dw, parts=8)
    if chunk:
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
    Oref, Lref = oracle.attention(w, levels=[], suffix=True)
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"suffix idx={idx} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


@pytest.mark.parametrize("kernel", [1, 2, 3, 4, 5], ids=["valu", "mfma", "mfma_ipw3", "mfma_ipw1000", "mfma_tile32"])
@pytest.mark.parametrize("chunk", [0, 32, 96])
@pytest.mark.parametrize("case", ["mha", "gqa8", "gqa4_nq3", "mha_nq5", "gqa8_nq7_two_row_tiles", "long", "d64_gqa8", "d64_mha_nq3", "d64_long"])
def test_suffix_kernels(case, chunk, kernel):
    """Both suffix kernels (vector-ALU, matrix-core) on every shape class: one row per KV head, grouped heads, several
    queries per sequence (causal tail, suffixes shorter than the query block), more than 32 rows per KV head, and
    suffixes of several hundred rows cut into chunks that start and end inside 32-key stages."""
    say(f"suffix kernels {case} chunk={chunk} kernel={kernel}")
    rng = np.random.default_rng(len(case))
    def lens(B, hi, nq):
        ln = rng.integers(0, hi + 1, size=B).astype(np.int32)
        ln[:6] = [0, 1, max(nq - 1, 0), nq, 31, 33]
        return ln
    if case == "mha":
        w = wl.make_workload(case, 81, 29, 4, 4, 128, [], 0, 0, lengths=lens(29, 150, 1))
    elif case == "gqa8":
        w = wl.make_workload(case, 82, 23, 16, 2, 128, [], 0, 0, lengths=lens(23, 200, 1))
    elif case == "gqa4_nq3":
        w = wl.make_workload(case, 83, 19, 8, 2, 128, [], 0, 0, lengths=lens(19, 120, 3), nq=3)
    elif case == "mha_nq5":
        w = wl.make_workload(case, 84, 17, 4, 4, 128, [], 0, 0, lengths=lens(17, 100, 5), nq=5)
    elif case == "gqa8_nq7_two_row_tiles":   # 56 rows per KV head: two 32-row tiles, the second half empty
        w = wl.make_workload(case, 85, 11, 8, 1, 128, [], 0, 0, lengths=lens(11, 90, 7), nq=7)
    elif case == "d64_gqa8":                 # head dimension 64: 128-byte rows, other swizzles, half as many k-steps
        w = wl.make_workload(case, 87, 23, 16, 2, 64, [], 0, 0, lengths=lens(23, 200, 1))
    elif case == "d64_mha_nq3":
        w = wl.make_workload(case, 88, 19, 3, 3, 64, [], 0, 0, lengths=lens(19, 130, 3), nq=3)
    elif case == "d64_long":
        w = wl.make_workload(case, 89, 9, 8, 2, 64, [], 0, 0, lengths=lens(9, 700, 1))
    else:
        w = wl.make_workload(case, 86, 9, 8, 2, 128, [], 0, 0, lengths=lens(9, 700, 1))
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=24)
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, min(kernel, 2))
    if kernel in (3, 4):   # several work items per wavefront: copies of the next item are in flight while one finishes
        ctx.set_option(hb.HG_OPT_SUFFIX_ITEMS_PER_WAVE, 3 if kernel == 3 else 1000)
    if kernel == 5:        # 32-row tiles also where 16-row tiles would be chosen (at most 16 rows per KV head)
        ctx.set_option(hb.HG_OPT_SUFFIX_TILE_ROWS, 32)
    if chunk:
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"suffix {case} kernel={kernel} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
@pytest.mark.parametrize("splits", [0, 1, 3])
@pytest.mark.parametrize("kernel", [1, 2], ids=["rows128", "rows256"])
def test_prefix_attn(idx, splits, kernel):
    say(f"prefix idx={idx} splits={splits} kernel={kernel}")
    w, dw = workload(idx)
    ctx = dev.make_context(dw, parts=8)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
    if splits:
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, splits)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    lv = dw.levels[0]
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_prefix_attn(ctx, dw.Q, lv.K, lv.V, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"prefix idx={idx} splits={splits} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


@pytest.mark.parametrize("case", ["ragged_1000", "exactly_64", "one_past_64", "short_20", "gqa_tiles", "two_queries", "long_3333"])
@pytest.mark.parametrize("parts", [8, 1])
def test_prefix_attn_persistent_kernel_d64(case, parts):
    """The 256-row kernel at head dimension 64 walks stages of 64 keys (two score tiles per stage): ranges that end
    inside a stage, inside its first tile, exactly at a stage, a single partial stage, several row tiles, several
    queries per sequence, and with one part only (whole columns per team)."""
    say(f"persistent D=64 {case} parts={parts}")
    B, Hq, Hkv, P, nq = {"ragged_1000": (300, 8, 2, 1000, 1), "exactly_64": (150, 4, 4, 64, 1), "one_past_64": (150, 4, 4, 65, 1),
                         "short_20": (260, 2, 1, 20, 1), "gqa_tiles": (90, 16, 2, 700, 1), "two_queries": (70, 4, 2, 333, 2),
                         "long_3333": (40, 8, 8, 3333, 1)}[case]
    w = wl.make_workload(case, 71, B, Hq, Hkv, 64, [(1, P, B)], 0, 0, lengths=np.zeros(B, np.int32) + nq, nq=nq)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=parts)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, 2)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    lv = dw.levels[0]
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_prefix_attn(ctx, dw.Q, lv.K, lv.V, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"persistent D=64 {case} parts={parts} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


def test_persistent_kernel_d64_grouped_and_fused():
    """Unequal blocks with uncovered sequences at D = 64 on the 256-row kernel, alone and inside the fused call (which
    picks that kernel by itself for blocks of more than 128 query rows)."""
    say("persistent D=64 grouped + fused")
    w = wl.make_workload("gaps64", 23, 400, 8, 4, 64, [(3, 150, 120)], 5, 90)
    lv = w.levels[0]
    lv.kv_off = np.array([0, 150, 215, 450], np.int32)    # unequal rows: 150, 65, 235
    lv.seq_off = np.array([0, 180, 330, 360], np.int32)   # unequal sequences: 180, 150, 30; 360..399 uncovered
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=8)
    Op, Lp = oracle.attention(w, levels=[0], suffix=False)
    Of, Lf = oracle.attention(w)
    assert np.isneginf(Lp[380]).all()
    for kernel in (2, 0):
        ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
        O, L, intact = outputs(dw)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[0], O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Op, Lp, f"D=64 grouped kernel={kernel}")
        O2, L2 = dev.hydragen(ctx, dw, torch.float32)
        torch.cuda.synchronize()
        check(to_np(O2), to_np(L2), Of, Lf, f"D=64 fused kernel={kernel}")
    plan = hb.hg_debug_wide_plan(3, 235, 180, 4, 2, 8, 32, 64)
    assert plan is not None and plan["n_c"] == 4       # 235 keys: four stages of 64
    ctx.close()


@pytest.mark.parametrize("splits", [0, 2])
@pytest.mark.parametrize("kernel", [1, 2], ids=["rows128", "rows256"])
def test_prefix_attn_grouped_tree_levels(splits, kernel):
    say(f"grouped splits={splits} kernel={kernel}")
    w, dw = workload(5)
    ctx = dev.make_context(dw, parts=8)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
    if splits:
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, splits)
    for li in (0, 1):
        Oref, Lref = oracle.attention(w, levels=[li], suffix=False)
        O, L, intact = outputs(dw)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[li], O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"grouped level {li}")
    ctx.close()


def test_grouped_level_with_uncovered_sequences_and_unequal_blocks():
    say("grouped uncovered")
    w = wl.make_workload("gaps", 21, 50, 8, 4, 128, [(3, 90, 11)], 5, 9)  # blocks cover sequences 0..32 only
    lv = w.levels[0]
    lv.kv_off = np.array([0, 90, 150, 270], np.int32)     # unequal rows: 90, 60, 120
    lv.seq_off = np.array([0, 11, 30, 33], np.int32)      # unequal sequences: 11, 19, 3
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=8)
    for splits, kernel in ((1, 0), (2, 0), (0, 2)):   # kernel 2: the persistent 256-row kernel on the same ragged blocks
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, splits)
        ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
        Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
        assert np.isneginf(Lref[40]).all()
        O, L, intact = outputs(dw)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[0], O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"uncovered splits={splits}")
        Of, Lf = oracle.attention(w)
        O2, L2 = dev.hydragen(ctx, dw, torch.float32)
        torch.cuda.synchronize()
        check(to_np(O2), to_np(L2), Of, Lf, "uncovered fused")
        O3, L3 = dev.naive(ctx, dw, torch.float32)
        torch.cuda.synchronize()
        check(to_np(O3), to_np(L3), Of, Lf, "uncovered naive")
    ctx.close()


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("kernel", [1, 2], ids=["rows128", "rows256"])
def test_shared_blocks_ignore_rows_that_are_nobodys_keys(kernel, D):
    """Blocks truncated by max_rows leave rows in the level's tensors that are no block's keys; here they hold NaN,
    as do the rows around the blocks.  The kernels re-read a window of 32 rows around a short block (the rows just
    below it, the rows past a range that ends before row 32 of the tensor): none of that may reach a result."""
    say(f"nobody's keys kernel={kernel} D={D}")
    B, Hq, Hkv = 300, 4, 2
    max_rows = 20
    first = 7                               # rows before the first block
    stored = [50, 5, 45]                    # rows each block owns in the tensors
    used = [min(n, max_rows) for n in stored]      # ... of which these count: 20, 5, 20
    w = wl.make_workload("truncated", 61, B, Hq, Hkv, D, [(1, sum(used), B)], 0, 33)
    lv = w.levels[0]
    seq_off = np.array([0, 140, 150, 300], np.int32)
    lv.kv_off = np.concatenate([[0], np.cumsum(used)]).astype(np.int32)     # the oracle's view: the used rows, back to back
    lv.seq_off = seq_off
    Oref, Lref = oracle.attention(w)
    Op, Lp = oracle.attention(w, levels=[0], suffix=False)
    # the device's view: NaN rows before the first block, and every block followed by its unused rows, all NaN
    Kd = np.full((first + sum(stored), Hkv, D), 0x7FC0, np.uint16)
    Vd = np.full((first + sum(stored), Hkv, D), 0x7FC0, np.uint16)
    kv_off_d = (first + np.concatenate([[0], np.cumsum(stored)])).astype(np.int32)
    for g in range(3):
        Kd[kv_off_d[g]: kv_off_d[g] + used[g]] = lv.K[lv.kv_off[g]: lv.kv_off[g + 1]]
        Vd[kv_off_d[g]: kv_off_d[g] + used[g]] = lv.V[lv.kv_off[g]: lv.kv_off[g + 1]]
    dw = dev.to_device(w)
    level = hb.Level(K=dev.bf16_tensor(Kd, "cuda:0"), V=dev.bf16_tensor(Vd, "cuda:0"), n_blocks=3,
                     kv_off=torch.from_numpy(kv_off_d).cuda(), seq_off=torch.from_numpy(seq_off).cuda(), max_rows=max_rows, max_seqs=150)
    ctx = dev.make_context(dw, parts=8)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
    for splits in (0, 2):
        ctx.set_option(hb.HG_OPT_PREFIX_SPLITS, splits)
        O, L, intact = outputs(dw)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, level, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Op, Lp, f"truncated blocks kernel={kernel} splits={splits}")
        O, L, intact = outputs(dw)
        hb.hg_hydragen_attn(ctx, dw.Q, [level], dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"truncated blocks, fused kernel={kernel} splits={splits}")
    O, L, intact = outputs(dw)
    hb.hg_naive_attn(ctx, dw.Q, [level], dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    assert intact()
    check(to_np(O), to_np(L), Oref, Lref, f"truncated blocks, comparison call kernel={kernel}")
    ctx.set_option(hb.HG_OPT_FUSED_KERNEL, 2)
    O, L, intact = outputs(dw)
    hb.hg_hydragen_attn(ctx, dw.Q, [level], dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    assert intact()
    check(to_np(O), to_np(L), Oref, Lref, f"truncated blocks, single launch")
    ctx.close()


@pytest.mark.parametrize("name,B,Hq,Hkv,P,parts", [
    ("three_tiles", 75, 8, 1, 1000, 8),      # 600 query rows per KV head: teams of 3 workgroups, ragged last tile and stage
    ("three_tiles_two_parts", 75, 8, 1, 1000, 2),   # workspace for two partial results only: longer ranges per team
    ("one_part", 40, 8, 2, 700, 1),          # no workspace for partials: one team per column, direct output
    ("row_groups", 1030, 8, 1, 100, 8),      # 8240 rows = 33 tiles of 256: two row groups of 17 tiles
    ("tiny_block", 40, 8, 2, 5, 8),          # fewer keys than one 32-key stage, at the very start of the tensor
    ("one_stage_plus_one", 33, 8, 1, 33, 8),
])
def test_persistent_kernel_partitions(name, B, Hq, Hkv, P, parts):
    """Work partitions of the persistent 256-row shared-block kernel that the five configs do not reach."""
    say(f"persistent partitions {name}")
    w = wl.make_workload(name, 77, B, Hq, Hkv, 128, [(1, P, B)], 0, 0)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=parts)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, 2)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    lv = dw.levels[0]
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_prefix_attn(ctx, dw.Q, lv.K, lv.V, O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"persistent {name} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


@pytest.mark.parametrize("name,n_blocks,P,B,Hq,Hkv,D,slots,nparts", [
    ("five_columns_eight_teams", 1, 2500, 300, 5, 5, 128, 2, 3),     # ranges of 54 stages without a column boundary, 45 with one
    ("five_columns_eight_teams_d64", 1, 2500, 300, 5, 5, 64, 2, 2),
    ("two_blocks_three_tiles", 2, 1300, 145, 6, 3, 128, 3, 2),       # 290 rows per block and KV head: teams of three workgroups
])
def test_persistent_kernel_ranges_of_equal_cost(name, n_blocks, P, B, Hq, Hkv, D, slots, nparts):
    """Where equal ranges would give some teams a column boundary and others none, the planner hands out ranges of equal
    cost from a table (a boundary counts as nine stages): every key is still multiplied exactly once."""
    say(f"equal-cost ranges {name}")
    G = Hq // Hkv
    plan = hb.hg_debug_wide_plan(n_blocks, P, B, Hkv, G, 8, slots, D)
    assert plan["mode"] == 2 and plan["nparts"] == nparts, plan
    w = wl.make_workload(name, 79, B * n_blocks, Hq, Hkv, D, [(n_blocks, P, B)], 0, 0)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=8)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, 2)
    ctx.set_option(hb.HG_OPT_WIDE_SLOTS, slots)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    for dtype in (torch.float32, torch.bfloat16):
        O, L, intact = outputs(dw, dtype)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[0], O, L, dw.scale)
        assert intact()
        check(to_np(O), to_np(L), Oref, Lref, f"equal-cost ranges {name} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


VARIANTS = [dict(), dict(q_gain=4.0), dict(plant="suffix"), dict(plant="prefix")]


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("variant", VARIANTS, ids=["normal", "peaked", "plant_suffix", "plant_prefix"])
@pytest.mark.parametrize("kernel", [0, 2], ids=["auto", "rows256"])
def test_fused_hydragen_and_naive(idx, variant, kernel):
    say(f"fused idx={idx} {variant} kernel={kernel}")
    w, dw = workload(idx, **variant)
    ctx = dev.make_context(dw, parts=24)
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.bfloat16, torch.float32):
        O, L, intact = outputs(dw, dtype)
        hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
        assert intact()
        st = check(to_np(O), to_np(L), Oref, Lref, f"hydragen idx={idx} {variant} {dtype}", out_bf16=dtype == torch.bfloat16)
        say(f"   hydragen {dtype}: {st}")
    O, L, intact = outputs(dw, torch.float32)
    hb.hg_naive_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    assert intact()
    check(to_np(O), to_np(L), Oref, Lref, f"naive idx={idx} {variant}")
    # every stream arrangement of the fused call meets the same bar (the key ranges of the partial results may
    # differ between them, so the bits may), and each is deterministic
    for mode in (2, 1, 0):
        ctx.set_option(hb.HG_OPT_OVERLAP, mode)
        Oa, La = dev.hydragen(ctx, dw, torch.float32)
        Ob, Lb = dev.hydragen(ctx, dw, torch.float32)
        torch.cuda.synchronize()
        check(to_np(Oa), to_np(La), Oref, Lref, f"hydragen idx={idx} {variant} overlap={mode}")
        assert torch.equal(Oa, Ob) and torch.equal(La, Lb)
    ctx.close()


def test_config1_exact_sizes_and_determinism():
    say("config1")
    w = wl.config(1)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw)
    Oref, Lref = oracle.attention(w)
    O, L = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, "config1")
    O2, L2 = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(L, L2)
    ctx.close()


def test_edge_cases_empty_parts():
    say("edge cases")
    # P = 0 (standard attention), all-empty suffixes, some empty suffixes, B = 1, no suffix tensors at all
    w = wl.make_workload("p0", 31, 9, 8, 4, 128, [(1, 0, 9)], 0, 40)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw)
    Oref, Lref = oracle.attention(w)
    O, L = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, "P=0")
    Op, Lp, intact = outputs(dw)
    hb.hg_prefix_attn(ctx, dw.Q, dw.levels[0].K, dw.levels[0].V, Op, Lp, dw.scale)
    assert intact() and float(Op.abs().max()) == 0.0 and bool(torch.isneginf(Lp).all())
    ctx.close()

    w = wl.make_workload("l0", 32, 5, 4, 4, 64, [(1, 70, 5)], 0, 0)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw)
    Oref, Lref = oracle.attention(w)
    O, L = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, "L=0 everywhere")
    Os, Ls, intact = outputs(dw)
    hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, 0, Os, Ls, dw.scale)
    assert intact() and bool(torch.isneginf(Ls).all())
    # lengths given but Ks absent: treated as no suffix
    O2 = torch.empty_like(O)
    L2 = torch.empty_like(L)
    hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, None, None, None, None, 0, O2, L2, dw.scale)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)
    ctx.close()

    w = wl.make_workload("b1", 33, 1, 2, 1, 128, [(1, 65, 1)], 1, 1)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw)
    Oref, Lref = oracle.attention(w)
    O, L = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, "B=1")
    ctx.close()


def test_lengths_change_on_device_without_host_work():
    """Suffix lengths live on the device: shrinking them between calls changes the result accordingly."""
    say("device lengths")
    w, dw = workload(2)
    ctx = dev.make_context(dw)
    new_len = np.maximum(w.lengths // 2, 0).astype(np.int32)
    dw.lengths.copy_(torch.from_numpy(new_len))
    w2 = wl.scaled_down(2)
    w2.lengths = new_len
    Oref, Lref = oracle.attention(w2)
    O, L = dev.hydragen(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    dw.lengths.copy_(torch.from_numpy(w.lengths))
    check(to_np(O), to_np(L), Oref, Lref, "halved lengths")
    ctx.close()


def test_error_paths_launch_nothing():
    say("errors")
    w, dw = workload(1)
    ctx = dev.make_context(dw, parts=1)
    O = torch.full((dw.B, dw.Hq, dw.D), 7.0, device="cuda:0")
    L = torch.full((dw.B, dw.Hq), 7.0, device="cuda:0")
    lib = hb.lib()
    lv = dw.levels[0]
    p = lambda t: t.data_ptr()
    # unsupported head dim
    assert lib.hg_prefix_attn(ctx.h, p(dw.Q), p(lv.K), p(lv.V), 4, 4, 4, 96, 128, 0.0, p(O), hb.HG_F32, p(L)) == hb.HG_ERR_UNSUPPORTED
    # Hq not a multiple of Hkv
    assert lib.hg_prefix_attn(ctx.h, p(dw.Q), p(lv.K), p(lv.V), 4, 4, 3, 64, 128, 0.0, p(O), hb.HG_F32, p(L)) == hb.HG_ERR_UNSUPPORTED
    # null output, negative length, bad dtype
    assert lib.hg_prefix_attn(ctx.h, p(dw.Q), p(lv.K), p(lv.V), 4, 4, 4, 64, 128, 0.0, None, hb.HG_F32, p(L)) == hb.HG_ERR_INVALID_ARG
    assert lib.hg_prefix_attn(ctx.h, p(dw.Q), p(lv.K), p(lv.V), 4, 4, 4, 64, -1, 0.0, p(O), hb.HG_F32, p(L)) == hb.HG_ERR_INVALID_ARG
    assert lib.hg_prefix_attn(ctx.h, p(dw.Q), p(lv.K), p(lv.V), 4, 4, 4, 64, 128, 0.0, p(O), 9, p(L)) == hb.HG_ERR_INVALID_ARG
    assert lib.hg_suffix_attn(ctx.h, p(dw.Q), p(dw.Ks), p(dw.Vs), p(dw.offsets), p(dw.lengths), -5, 4, 4, 4, 64, 0.0, p(O), hb.HG_F32, p(L)) == hb.HG_ERR_INVALID_ARG
    # a suffix so long that 32-bit byte offsets inside one sequence's rows would overflow
    assert lib.hg_suffix_attn(ctx.h, p(dw.Q), p(dw.Ks), p(dw.Vs), p(dw.offsets), p(dw.lengths), 1 << 23, 4, 4, 4, 64, 0.0, p(O), hb.HG_F32, p(L)) == hb.HG_ERR_UNSUPPORTED
    # options out of range
    for opt, bad in ((hb.HG_OPT_SUFFIX_TILE_ROWS, 7), (hb.HG_OPT_SUFFIX_KERNEL, 3), (hb.HG_OPT_SUFFIX_ITEMS_PER_WAVE, 5000)):
        with pytest.raises(hb.HydragenError) as e:
            ctx.set_option(opt, bad)
        assert e.value.code == hb.HG_ERR_INVALID_ARG
    # fused call needs room for levels+1 partials: one part is not enough
    with pytest.raises(hb.HydragenError) as e:
        dev.hydragen(ctx, dw, torch.float32)
    assert e.value.code == hb.HG_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(O.min()) == 7.0 and float(L.min()) == 7.0  # nothing was written
    assert hb.strerror(hb.HG_ERR_WORKSPACE) == "workspace too small"
    ctx.close()


@pytest.mark.parametrize("nq", [2, 5])
@pytest.mark.parametrize("shape", ["mha", "gqa_tree", "d64"])
def test_several_queries_per_sequence(nq, shape):
    """App. B's num_queries > 1: Q [B, nq, Hq, D]; query t sees the suffix up to its own token (suffixes shorter than nq included)."""
    say(f"several queries nq={nq} {shape}")
    def lengths(B, hi, seed):
        ln = np.random.default_rng(seed).integers(0, hi + 1, size=B).astype(np.int32)
        ln[:4] = [0, 1, nq - 1, nq]          # suffixes shorter than, and exactly as long as, the query block
        return ln
    if shape == "mha":       # 120 (nq=2) or 300 (nq=5) query rows per KV head: 128-row and persistent 256-row kernels
        w = wl.make_workload("nq_mha", 51, 60, 4, 4, 128, [(1, 700, 60)], 0, 0, lengths=lengths(60, 90, 1), nq=nq)
    elif shape == "gqa_tree":
        w = wl.make_workload("nq_tree", 52, 48, 8, 2, 128, [(1, 150, 48), (4, 77, 12)], 0, 0, lengths=lengths(48, 40, 2), nq=nq)
    else:
        w = wl.make_workload("nq_d64", 53, 21, 4, 2, 64, [(1, 100, 21)], 0, 0, lengths=lengths(21, 70, 3), nq=nq)
    assert w.lengths.min() < nq
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=24)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.float32, torch.bfloat16):
        O, L = dev.hydragen(ctx, dw, dtype)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Oref, Lref, f"hydragen nq={nq} {shape} {dtype}", out_bf16=dtype == torch.bfloat16)
    O, L = dev.naive(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"naive nq={nq} {shape}")
    # the parts on their own
    Os, Ls, intact = outputs(dw)
    hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, Os, Ls, dw.scale)
    assert intact()
    Or, Lr = oracle.attention(w, levels=[], suffix=True)
    check(to_np(Os), to_np(Ls), Or, Lr, f"suffix nq={nq} {shape}")
    for li in range(len(dw.levels)):
        Op, Lp, intact = outputs(dw)
        hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[li], Op, Lp, dw.scale)
        assert intact()
        Or, Lr = oracle.attention(w, levels=[li], suffix=False)
        check(to_np(Op), to_np(Lp), Or, Lr, f"level {li} nq={nq} {shape}")
    ctx.close()


@pytest.mark.parametrize("shape", ["mha", "gqa8", "gqa4_nq3"])
def test_suffix_ignores_unwritten_cache_rows(shape):
    """A padded cache: every sequence owns a slot longer than its suffix, and the rows behind the suffix (and the slots
    of empty sequences) hold NaN, as memory that was never written may.  No such row may reach a result: the kernels
    read rows outside a sequence's range when they re-read a window or fill a batch, and must neutralise them."""
    say(f"unwritten cache rows {shape}")
    rng = np.random.default_rng(7)
    B = 33
    ln = rng.integers(0, 60, size=B).astype(np.int32)
    ln[:8] = [0, 1, 2, 5, 31, 32, 33, 0]
    if shape == "mha":
        w = wl.make_workload(shape, 91, B, 4, 4, 128, [(1, 70, B)], 0, 0, lengths=ln)
    elif shape == "gqa8":
        w = wl.make_workload(shape, 92, B, 16, 2, 128, [(1, 70, B)], 0, 0, lengths=ln)
    else:
        w = wl.make_workload(shape, 93, B, 8, 2, 128, [(1, 70, B)], 0, 0, lengths=ln, nq=3)
    Ks, Vs, off, cap = wl.with_room(w, 9)
    owned = np.zeros(Ks.shape[0], dtype=bool)
    for b in range(B):
        owned[off[b]: off[b] + ln[b]] = True
    Ks[~owned] = 0x7FC0     # bf16 NaN
    Vs[~owned] = 0x7FC0
    dw = dev.to_device(w)
    dK, dV, doff = dev.bf16_tensor(Ks, "cuda:0"), dev.bf16_tensor(Vs, "cuda:0"), torch.from_numpy(off).cuda()
    Oref, Lref = oracle.attention(w)
    Osuf, Lsuf = oracle.attention(w, levels=[])
    for kernel in (1, 2):
        ctx = dev.make_context(dw, parts=16)
        ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, kernel)
        for chunk in (0, 32):
            ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
            O, L, intact = outputs(dw, torch.float32)
            hb.hg_suffix_attn(ctx, dw.Q, dK, dV, doff, dw.lengths, dw.max_len, O, L, dw.scale)
            assert intact()
            check(to_np(O), to_np(L), Osuf, Lsuf, f"suffix over a padded cache {shape} kernel={kernel} chunk={chunk}")
            O, L, intact = outputs(dw, torch.float32)
            hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dK, dV, doff, dw.lengths, dw.max_len, O, L, dw.scale)
            assert intact()
            check(to_np(O), to_np(L), Oref, Lref, f"fused over a padded cache {shape} kernel={kernel} chunk={chunk}")
            O, L, intact = outputs(dw, torch.float32)
            hb.hg_naive_attn(ctx, dw.Q, dw.levels, dK, dV, doff, dw.lengths, dw.max_len, O, L, dw.scale)
            assert intact()
            check(to_np(O), to_np(L), Oref, Lref, f"naive over a padded cache {shape} kernel={kernel} chunk={chunk}")
        ctx.close()


def test_persistent_kernel_more_columns_than_teams_and_one_part():
    """320 (block, KV head) columns against 256 teams with room for a single partial result: every team must take
    whole columns, and all of them (a plan that gave each team one column dropped the rest)."""
    say("many columns, one part")
    w = wl.make_workload("many_columns", 97, 1600, 32, 8, 128, [(40, 45, 40)], 0, 0, lengths=np.zeros(1600, np.int32))
    dw = dev.to_device(w)
    plan = hb.hg_debug_wide_plan(40, 45, 40, 8, 4, 1, 32)
    assert plan["ncols"] == 320 > 8 * plan["tpx"] and plan["nparts"] == 1 and plan["quota"] == 2 * plan["n_c"]
    ctx = hb.Context(0, 0)                       # no workspace: the level must run with one part, written directly
    ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, 2)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    O, L, intact = outputs(dw, torch.float32)
    hb.hg_prefix_attn_grouped(ctx, dw.Q, dw.levels[0], O, L, dw.scale)
    assert intact()
    check(to_np(O), to_np(L), Oref, Lref, "many columns, one part")
    ctx.close()


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_fused_call_at_every_workspace_size(idx):
    """The planner trades partial results for parallelism: from the smallest workspace the call accepts (one part per
    level and one for the suffix) upwards, every size must give the same attention."""
    say(f"workspace sweep idx={idx}")
    w, dw = workload(idx)
    Oref, Lref = oracle.attention(w)
    need = len(w.levels) + 1
    for parts in list(range(need, need + 6)) + [12, 64]:
        for kernel in (1, 2):
            ctx = dev.make_context(dw, parts=parts)
            ctx.set_option(hb.HG_OPT_PREFIX_KERNEL, kernel)
            ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, 32)     # many suffix chunks wanted: the planner has to give way
            O, L, intact = outputs(dw, torch.float32)
            hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
            assert intact()
            check(to_np(O), to_np(L), Oref, Lref, f"fused idx={idx} parts={parts} kernel={kernel}")
            ctx.close()
    small = dev.make_context(dw, parts=need - 1)
    with pytest.raises(hb.HydragenError) as e:
        dev.hydragen(small, dw, torch.float32)
    assert e.value.code == hb.HG_ERR_WORKSPACE
    small.close()


def test_workgroups_go_round_robin_over_the_xcds():
    """The shared-block kernels place the workgroups that share K/V rows on one XCD by giving them ids that are equal
    modulo 8.  The hardware's own id register agrees, for launches shaped like the persistent kernel's: XCD = (id + c) % 8
    with one c per launch (the round-robin goes on where the launch before stopped)."""
    say("xcd map")
    ctx = hb.Context(0, 0)
    for n in (256, 160, 2048):
        out = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
        hb.hg_debug_xcd_of_workgroups(ctx, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert got.min() >= 0 and got.max() <= 7, (n, got[:32])
        assert np.array_equal(got, (np.arange(n) + got[0]) % 8), (n, got[:32])
    ctx.close()
