"""Parity at the full benchmark sizes, in the launch configuration bench.py times (default options, bf16 output,
24 workspace parts): the five configurations and the paper's microbenchmark shape, with the oracle evaluated on sampled sequences (first, last,
shortest and longest suffix, block boundaries of the tree) and whole-output properties checked at full size."""
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


def sample_seqs(w, extra=()):
    s = {0, w.B - 1, w.B // 2, int(np.argmin(w.lengths)), int(np.argmax(w.lengths))}
    for lv in w.levels:
        if lv.Gn > 1:
            s.update([int(lv.seq_off[1]) - 1, int(lv.seq_off[1]), int(lv.seq_off[lv.Gn - 1])])
    s.update(extra)
    return np.array(sorted(s), dtype=np.int32)


def run_and_check(w, dw, what, with_naive=True):
    ctx = dev.make_context(dw, parts=24)
    seqs = sample_seqs(w)
    Oref, Lref = oracle.attention(w, seqs=seqs)
    idx = torch.from_numpy(seqs.astype(np.int64)).cuda()
    O, L = dev.hydragen(ctx, dw, torch.bfloat16)
    torch.cuda.synchronize()
    st = check(to_np(O[idx]), to_np(L[idx]), Oref, Lref, what, out_bf16=True)
    say(f"   {what}: {st}")
    # properties that hold for every row at any size
    assert bool(torch.isfinite(O.float()).all()) and bool(torch.isfinite(L).all())
    # the full LSE is at least each part's LSE: compare with the suffix-only part on all rows
    Os = torch.empty((dw.B, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    Ls = torch.empty((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, Os, Ls, dw.scale)
    torch.cuda.synchronize()
    assert bool((L >= Ls - 1e-4).all())
    if with_naive:
        On, Ln = dev.naive(ctx, dw, torch.bfloat16)
        torch.cuda.synchronize()
        check(to_np(On[idx]), to_np(Ln[idx]), Oref, Lref, what + " naive", out_bf16=True)
        # decomposed and non-decomposed results agree on every row
        assert float((On.float() - O.float()).abs().max()) <= 2.0 ** -6 * float(O.float().abs().max())
        assert float((Ln - L).abs().max()) <= 1e-3
    ctx.close()


@pytest.mark.parametrize("idx", [2, 4, 6])
def test_full_config(idx):
    say(f"full config {idx}")
    w = wl.config(idx)
    run_and_check(w, dev.to_device(w), f"config{idx}")


def test_full_config3_prefix_sweep():
    say("full config 3")
    w = wl.config(3)
    full = w.levels[0]
    for P in (1024, 4096, 16384):
        say(f"  P={P}")
        w.levels[0] = wl.Level(K=full.K[:P], V=full.V[:P], kv_off=np.array([0, P], np.int32), seq_off=full.seq_off)
        assert np.array_equal(w.levels[0].K, wl.config(3, P=1024).levels[0].K) if P == 1024 else True
        dw = dev.to_device(w)
        run_and_check(w, dw, f"config3 P={P}", with_naive=(P != 16384))
        del dw
        torch.cuda.empty_cache()


def test_full_config5_tree():
    say("full config 5")
    w = wl.config(5)
    run_and_check(w, dev.to_device(w), "config5")
