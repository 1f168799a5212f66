"""Seeded random shapes and option settings through the fused call, the comparison kernel, the paged variant and the
8-bit suffix cache (packed and paged), each against the fp64 oracle: tree depth 0..3 with unequal blocks and uncovered sequences, MHA and grouped heads,
1..6 queries per sequence, D in {64, 128}, ragged suffixes with empty ones, every kernel choice and split setting."""
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


def random_workload(seed: int) -> wl.Workload:
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128, 128, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 4, 8]))
    nq = int(rng.choice([1, 1, 1, 2, 3, 6]))
    B = int(rng.integers(1, 70))
    Hq = Hkv * G
    hi = int(rng.choice([0, 5, 40, 130, 300]))
    lengths = rng.integers(0, hi + 1, size=B).astype(np.int32)
    w = wl.make_workload(f"rand{seed}", 2000 + seed, B, Hq, Hkv, D, [], 0, 0, lengths=lengths, nq=nq)
    # levels: random contiguous blocks with unequal rows; some sequences stay uncovered
    nlev = int(rng.integers(0, 4))
    for li in range(nlev):
        nb = int(rng.integers(1, 5))
        cuts = np.sort(rng.choice(np.arange(0, B + 1), size=min(nb + 1, B + 1), replace=False))
        if cuts.size < 2:
            continue
        seq_off = cuts.astype(np.int32)
        rows = rng.integers(0, int(rng.choice([3, 70, 400])) + 1, size=seq_off.size - 1)
        kv_off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
        tot = int(kv_off[-1])
        w.levels.append(wl.Level(K=wl.normal_bf16(w.seed, 10 + 2 * li, (tot, Hkv, D)), V=wl.normal_bf16(w.seed, 11 + 2 * li, (tot, Hkv, D)),
                                 kv_off=kv_off, seq_off=seq_off))
    return w


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(seed):
    w = random_workload(seed)
    rng = np.random.default_rng(5000 + seed)
    opts = {
        hb.HG_OPT_PREFIX_KERNEL: int(rng.integers(0, 3)), hb.HG_OPT_SUFFIX_KERNEL: int(rng.integers(0, 3)),
        hb.HG_OPT_PREFIX_SPLITS: int(rng.choice([0, 0, 1, 2, 5])), hb.HG_OPT_SUFFIX_CHUNK: int(rng.choice([0, 0, 32, 64, 160])),
        hb.HG_OPT_OVERLAP: int(rng.integers(0, 3)), hb.HG_OPT_SUFFIX_ITEMS_PER_WAVE: int(rng.choice([0, 0, 1, 3, 50])),
    }
    print(f"random shape {seed}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} nq={w.nq} levels={[(l.Gn, l.max_rows) for l in w.levels]} "
          f"max_len={w.max_len} options={opts}", file=sys.stderr, flush=True)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=32)
    for k, v in opts.items():
        ctx.set_option(k, v)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.float32, torch.bfloat16):
        O, L = dev.hydragen(ctx, dw, dtype)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Oref, Lref, f"hydragen seed={seed} {dtype}", out_bf16=dtype == torch.bfloat16)
    O, L = dev.naive(ctx, dw, torch.float32)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"naive seed={seed}")
    if w.max_len > 0:
        kv = dev.paged_to_device(wl.make_paged(w, int(rng.choice([16, 32, 128]))))
        O, L = dev.hydragen_paged(ctx, dw, kv, out_dtype=torch.float32)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Oref, Lref, f"paged seed={seed}")
        # the same suffix as an 8-bit cache, packed and through pages: reference = merge of the exact attention over
        # the levels and over the decoded codes
        from oracle import fp8
        f8 = wl.make_fp8(w, reserve=int(rng.integers(0, 4)))
        Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, f8.Ks8, f8.Vs8, f8.k_scale, f8.v_scale, f8.offsets, w.lengths, w.scale)
        if w.levels:
            Op, Lp = oracle.attention(w, suffix=False)
            O8ref, L8ref = oracle.merge([Op, Os], [Lp, Ls])
        else:
            O8ref, L8ref = Os, Ls
        O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.float32, device="cuda:0")
        L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
        hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, torch.from_numpy(f8.Ks8).cuda(), torch.from_numpy(f8.Vs8).cuda(), f8.k_scale,
                                f8.v_scale, torch.from_numpy(f8.offsets).cuda(), dw.lengths, dw.max_len, O, L, dw.scale)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), O8ref, L8ref, f"fp8 seed={seed}")
        pg8, ks8, vs8 = wl.make_paged_fp8(w, int(rng.choice([16, 64])))
        kv8 = hb.PagedKV(K=torch.from_numpy(pg8.K).cuda(), V=torch.from_numpy(pg8.V).cuda(), page_table=torch.from_numpy(pg8.table).cuda(),
                         page_size=pg8.page_size, kv_format=hb.HG_KV_E4M3, k_scale=ks8, v_scale=vs8)
        O, L = dev.hydragen_paged(ctx, dw, kv8, out_dtype=torch.float32)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), O8ref, L8ref, f"paged fp8 seed={seed}")
    ctx.close()
