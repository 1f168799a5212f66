"""Parity at the full benchmark sizes, in the launch configuration bench.py times (default options, bf16 output,
24 workspace parts): the five configurations and the paper's microbenchmark shape.  Every row of O and LSE, of the
fused call and of the non-decomposed comparison call, is compared with the oracle (the oracle takes about 13 s for
the largest configuration on the GPU machine's host cores)."""
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


_capsys = None


@pytest.fixture(autouse=True)
def _uncaptured(capsys):
    """The figures of every comparison are printed past pytest's capture, so that they show in a quiet run too."""
    global _capsys
    _capsys = capsys
    yield
    _capsys = None


def say(msg):
    if _capsys is not None:
        with _capsys.disabled():
            print(msg, file=sys.stderr, flush=True)
    else:
        print(msg, file=sys.stderr, flush=True)


def run_and_check(w, dw, what):
    ctx = dev.make_context(dw, parts=24)
    ctx.set_option(hb.HG_OPT_FUSED_KERNEL, 0)              # the library's own choice, as bench.py runs it
    Oref, Lref = oracle.attention(w)                       # every sequence, every head
    O, L = dev.hydragen(ctx, dw, torch.bfloat16)
    torch.cuda.synchronize()
    st = check(to_np(O), to_np(L), Oref, Lref, what, out_bf16=True)
    say(f"   {what}: all {w.B * w.Hq} rows: max|dO|={st['max_abs_dO']:.3e} (max|O|={st['max_abs_O']:.3e}) rel-L2={st['rel_l2']:.3e} "
        f"max|dLSE|={st['max_abs_dLSE']:.3e}")
    On, Ln = dev.naive(ctx, dw, torch.bfloat16)
    torch.cuda.synchronize()
    sn = check(to_np(On), to_np(Ln), Oref, Lref, what + " naive", out_bf16=True)
    say(f"   {what} non-decomposed call: max|dO|={sn['max_abs_dO']:.3e} rel-L2={sn['rel_l2']:.3e} max|dLSE|={sn['max_abs_dLSE']:.3e}")
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
        run_and_check(w, dw, f"config3 P={P}")
        del dw
        torch.cuda.empty_cache()


@pytest.mark.parametrize("idx,P", [(3, 4096), (4, 0), (5, 0)])
def test_full_config_head_dim_64(idx, P):
    """The head-dimension-64 variant of the long-context, grouped-head and tree configurations (the persistent
    shared-block kernel walks 64-key stages there), every row."""
    say(f"full config {idx} at D=64")
    w = wl.config(idx, P=P or None, D=64)
    run_and_check(w, dev.to_device(w), f"config{idx} D=64")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("P", [4096, 16384])
def test_full_config3_shared_block_alone(P):
    """The shared-block call by itself on the whole chip, as bench.py's serialised pass times it (the partition differs
    from the one inside the fused call: 64 teams with ranges of equal cost), every row against the oracle."""
    say(f"full config 3, shared block alone, P={P}")
    w = wl.config(3, P=P)
    dw = dev.to_device(w)
    ctx = dev.make_context(dw, parts=24)
    Oref, Lref = oracle.attention(w, levels=[0], suffix=False)
    O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    lv = dw.levels[0]
    hb.hg_prefix_attn(ctx, dw.Q, lv.K, lv.V, O, L, dw.scale)
    torch.cuda.synchronize()
    st = check(to_np(O), to_np(L), Oref, Lref, f"config3 P={P} shared block", out_bf16=True)
    say(f"   config3 P={P} shared block alone: all {w.B * w.Hq} rows: max|dO|={st['max_abs_dO']:.3e} (max|O|={st['max_abs_O']:.3e}) "
        f"rel-L2={st['rel_l2']:.3e} max|dLSE|={st['max_abs_dLSE']:.3e}")
    ctx.close()
    torch.cuda.empty_cache()


def test_full_config5_tree():
    say("full config 5")
    w = wl.config(5)
    run_and_check(w, dev.to_device(w), "config5")
