"""The single-launch form of the fused call (HG_OPT_FUSED_KERNEL = 2: every shared level, the suffixes and the merge in
one kernel, no workspace) against the fp64 oracle: the scaled-down configurations with their sharper variants, seeded
random trees (unequal blocks, uncovered sequences, block boundaries inside a 32-row tile, grouped heads, several
queries per sequence, both head dimensions), empty parts, a padded cache whose unowned rows hold NaN, and the
automatic choice on a tiny call."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2402_05099_amd import binding as hb
from paper_2402_05099_amd import device as dev
from paper_2402_05099_amd import workloads as wl
from parity import check, to_np
from test_gpu_random_shapes import random_workload

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def single_launch(w, what, Ks=None, Vs=None, off=None):
    """The call with the single launch forced, on a context WITHOUT a workspace, both output types, canaries around."""
    dw = dev.to_device(w)
    ctx = hb.Context(0, 0)
    ctx.set_option(hb.HG_OPT_FUSED_KERNEL, 2)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.float32, torch.bfloat16):
        n, pad = dw.rows * dw.D, 256
        fo = torch.full((n + 2 * pad,), float("nan"), dtype=dtype, device="cuda:0")
        fl = torch.full((dw.rows + 2 * pad,), float("nan"), dtype=torch.float32, device="cuda:0")
        O, L = fo[pad:pad + n].view(dw.lead + (dw.D,)), fl[pad:pad + dw.rows].view(dw.lead)
        hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks if Ks is None else Ks, dw.Vs if Vs is None else Vs,
                            dw.offsets if off is None else off, dw.lengths, dw.max_len, O, L, dw.scale)
        torch.cuda.synchronize()
        assert bool(torch.isnan(fo[:pad]).all() and torch.isnan(fo[pad + n:]).all() and torch.isnan(fl[:pad]).all()
                    and torch.isnan(fl[pad + dw.rows:]).all()), f"{what}: wrote outside its outputs"
        st = check(to_np(O), to_np(L), Oref, Lref, f"{what} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()
    return st


VARIANTS = [dict(), dict(q_gain=4.0), dict(plant="suffix"), dict(plant="prefix")]


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("variant", VARIANTS, ids=["normal", "peaked", "plant_suffix", "plant_prefix"])
def test_single_launch_scaled_down_configs(idx, variant):
    say(f"single launch: scaled-down config {idx} {variant}")
    single_launch(wl.scaled_down(idx, **variant), f"config {idx} {variant}")


@pytest.mark.parametrize("seed", range(40))
def test_single_launch_random_trees(seed):
    w = random_workload(seed)
    say(f"single launch: random shape {seed}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} nq={w.nq} "
        f"levels={[(l.Gn, l.max_rows) for l in w.levels]} max_len={w.max_len}")
    if w.max_len == 0 and not any(l.max_rows for l in w.levels):
        pytest.skip("no key anywhere: the call fills the outputs without any attention kernel")
    single_launch(w, f"random {seed}")


def test_single_launch_empty_parts_and_tiny_batches():
    say("single launch: empty parts")
    single_launch(wl.make_workload("p0", 31, 9, 8, 4, 128, [(1, 0, 9)], 0, 40), "P=0")
    single_launch(wl.make_workload("l0", 32, 5, 4, 4, 64, [(1, 70, 5)], 0, 0), "L=0 everywhere")
    single_launch(wl.make_workload("b1", 33, 1, 2, 1, 128, [(1, 65, 1)], 1, 1), "B=1")
    single_launch(wl.make_workload("nolevel", 34, 37, 6, 2, 128, [], 0, 90), "no shared level")
    ln = np.zeros(70, np.int32)
    ln[::3] = 17
    single_launch(wl.make_workload("gaps", 35, 70, 4, 4, 128, [(1, 33, 70)], 0, 0, lengths=ln), "two sequences in three without a suffix")


@pytest.mark.parametrize("shape", ["mha", "gqa8", "gqa4_nq3"])
def test_single_launch_ignores_unwritten_cache_rows(shape):
    """A padded cache whose rows behind every suffix hold NaN, and a shared block shorter than a stage: no row that is
    nobody's key may reach a result."""
    say(f"single launch: unwritten cache rows {shape}")
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
    single_launch(w, f"padded cache {shape}", dev.bf16_tensor(Ks, "cuda:0"), dev.bf16_tensor(Vs, "cuda:0"), torch.from_numpy(off).cuda())


def test_tiny_call_takes_the_single_launch_by_itself():
    """Config 1 (4 sequences) with the library's defaults: the result is bit for bit the forced single launch's, on a
    context that has no workspace at all (the separate kernels would refuse it)."""
    say("single launch: automatic choice")
    w = wl.config(1)
    dw = dev.to_device(w)
    outs = []
    for opt in (0, 2):
        ctx = hb.Context(0, 0)
        ctx.set_option(hb.HG_OPT_FUSED_KERNEL, opt)
        outs.append(dev.hydragen(ctx, dw, torch.float32))
        torch.cuda.synchronize()
        ctx.close()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    Oref, Lref = oracle.attention(w)
    check(to_np(outs[0][0]), to_np(outs[0][1]), Oref, Lref, "config 1, defaults")
    ctx = hb.Context(0, 0)
    ctx.set_option(hb.HG_OPT_FUSED_KERNEL, 1)
    with pytest.raises(hb.HydragenError) as e:
        dev.hydragen(ctx, dw, torch.float32)
    assert e.value.code == hb.HG_ERR_WORKSPACE
    ctx.close()
