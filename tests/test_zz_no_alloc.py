"""hg_hydragen_attn_static, the fused call that keeps its partial results in a fixed array inside the library instead
of a caller-provided workspace: same results as hg_hydragen_attn on two calls in a row (the second on a smaller
input, so that whatever the first call left in the array is in the way), sizes beyond the array are refused."""
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


def both_calls(w, what):
    """(static call, workspace call, oracle) on one workload; the static call runs on a context without a workspace."""
    dw = dev.to_device(w)
    ctx_ws = dev.make_context(dw, parts=24)
    ctx_static = hb.Context(0, 0)
    O0, L0 = dev.hydragen(ctx_ws, dw, torch.float32)
    O1 = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.float32, device="cuda:0")
    L1 = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    hb.hg_hydragen_attn_static(ctx_static, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O1, L1, dw.scale)
    torch.cuda.synchronize()
    st = check(to_np(O1), to_np(L1), to_np(O0), to_np(L0), what + " static vs workspace call")
    Oref, Lref = oracle.attention(w)
    st2 = check(to_np(O1), to_np(L1), Oref, Lref, what + " static vs oracle")
    say(f"   {what}: vs workspace call {st}; vs oracle {st2}")
    ctx_ws.close()
    ctx_static.close()


def test_static_call_twice_second_input_smaller():
    say("static scratch: scaled-down config 3 (one long shared block, 150 sequences)")
    both_calls(wl.scaled_down(3), "config 3 scaled down")
    say("static scratch: scaled-down config 5 (two-level tree, 96 sequences, fewer rows than the call before)")
    both_calls(wl.scaled_down(5), "config 5 scaled down")
    say("static scratch: config 1 (4 sequences)")
    both_calls(wl.config(1), "config 1")


def test_static_call_refuses_what_does_not_fit():
    # scaled-down config 3 stacked to more rows than two partial results of 64 MiB / 2 can hold: the call must
    # return its own error before anything is enqueued (tensors are real and large enough, outputs stay untouched)
    w = wl.scaled_down(3)
    dw = dev.to_device(w)
    reps = hb.HG_STATIC_SCRATCH_BYTES // (2 * dw.B * dw.Hq * (dw.D + 1) * 4) + 1
    B = dw.B * reps
    Q = dw.Q.repeat(reps, 1, 1).contiguous()
    off = dw.offsets.repeat(reps).contiguous()
    ln = dw.lengths.repeat(reps).contiguous()
    O = torch.full((B, dw.Hq, dw.D), 7.0, dtype=torch.float32, device="cuda:0")
    L = torch.full((B, dw.Hq), 7.0, dtype=torch.float32, device="cuda:0")
    ctx = hb.Context(0, 0)
    say(f"static scratch: B={B} rows={B * dw.Hq} must be refused")
    with pytest.raises(hb.HydragenError) as e:
        hb.hg_hydragen_attn_static(ctx, Q, dw.levels, dw.Ks, dw.Vs, off, ln, dw.max_len, O, L, dw.scale)
    assert e.value.code == hb.HG_ERR_STATIC_LIMIT
    torch.cuda.synchronize()
    assert bool((O == 7.0).all()) and bool((L == 7.0).all())
    # one row fewer than the limit still runs, and agrees with the workspace call
    B2 = dw.B * (reps - 1)
    ctx_ws = hb.Context(0, hb.hg_workspace_bytes(B2, dw.Hq, dw.D, 4))
    O0 = torch.empty((B2, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    L0 = torch.empty((B2, dw.Hq), dtype=torch.float32, device="cuda:0")
    hb.hg_hydragen_attn(ctx_ws, Q[:B2], dw.levels, dw.Ks, dw.Vs, off[:B2], ln[:B2], dw.max_len, O0, L0, dw.scale)
    hb.hg_hydragen_attn_static(ctx, Q[:B2], dw.levels, dw.Ks, dw.Vs, off[:B2], ln[:B2], dw.max_len, O[:B2], L[:B2], dw.scale)
    torch.cuda.synchronize()
    check(to_np(O[:B2]), to_np(L[:B2]), to_np(O0), to_np(L0), "largest size that fits")
    ctx.close()
    ctx_ws.close()
