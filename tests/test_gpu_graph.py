"""The fused call under HIP graph capture: it enqueues only kernels and event edges, reads lengths on the device,
and allocates nothing, so a captured call can be replayed on new device-side lengths."""
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


@pytest.mark.parametrize("idx", [3, 4, 5])
def test_fused_call_captured_in_a_graph_and_replayed(idx):
    print(f"graph capture idx={idx}", file=sys.stderr, flush=True)
    w = wl.scaled_down(idx)
    dw = dev.to_device(w)
    s = torch.cuda.Stream()
    ctx = hb.Context(0, hb.hg_workspace_bytes(dw.B, dw.Hq, dw.D, 24), stream=s)
    O = torch.zeros((dw.B, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    L = torch.zeros((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")
    with torch.cuda.stream(s):   # first call outside capture (one-time kernel attribute set-up)
        hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    full = w.lengths.copy()
    for trial, new_len in enumerate([full, np.maximum(full // 2, 0).astype(np.int32), np.zeros_like(full), full]):
        # the program's own eager work and synchronisations sit between the replays
        dw.lengths.copy_(torch.from_numpy(new_len))
        torch.cuda.synchronize()
        O.fill_(float("nan"))
        L.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        Og, Lg = O.clone(), L.clone()
        with torch.cuda.stream(s):
            Oe, Le = dev.hydragen(ctx, dw, torch.float32)
        s.synchronize()
        assert torch.equal(Og, Oe) and torch.equal(Lg, Le), f"replay {trial} differs from the eager call"
        w2 = wl.scaled_down(idx)
        w2.lengths = new_len
        Oref, Lref = oracle.attention(w2)
        check(to_np(Og), to_np(Lg), Oref, Lref, f"graph replay {trial} idx={idx}")
    dw.lengths.copy_(torch.from_numpy(full))
    ctx.close()
