"""Moves a host workload (bf16 bit patterns in numpy) into device tensors and calls the library on it.

Plumbing only: PyTorch holds the device memory; all attention arithmetic happens inside libhydragen.so.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from . import binding as hb


def bf16_tensor(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bit patterns -> bf16 device tensor with the same bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


@dataclass
class DeviceWorkload:
    B: int
    Hq: int
    Hkv: int
    D: int
    scale: float
    Q: torch.Tensor
    levels: List[hb.Level]
    Ks: Optional[torch.Tensor]
    Vs: Optional[torch.Tensor]
    offsets: torch.Tensor
    lengths: torch.Tensor
    max_len: int

    @property
    def nq(self) -> int:
        return int(self.Q.shape[1]) if self.Q.dim() == 4 else 1

    @property
    def rows(self) -> int:
        return self.B * self.nq * self.Hq

    @property
    def lead(self):
        """Leading shape of O and LSE: (B, Hq), or (B, nq, Hq) with several queries per sequence."""
        return tuple(self.Q.shape[:-1])


def to_device(w, device="cuda:0") -> DeviceWorkload:
    levels = []
    for lv in w.levels:
        single = lv.Gn == 1 and int(lv.seq_off[0]) == 0 and int(lv.seq_off[1]) == w.B and int(lv.kv_off[0]) == 0
        levels.append(hb.Level(
            K=bf16_tensor(lv.K, device), V=bf16_tensor(lv.V, device), n_blocks=lv.Gn,
            kv_off=None if single else torch.from_numpy(lv.kv_off).to(device),
            seq_off=None if single else torch.from_numpy(lv.seq_off).to(device),
            max_rows=lv.max_rows, max_seqs=lv.max_seqs,
        ))
    return DeviceWorkload(
        B=w.B, Hq=w.Hq, Hkv=w.Hkv, D=w.D, scale=float(w.scale), Q=bf16_tensor(w.Q, device), levels=levels,
        Ks=bf16_tensor(w.Ks, device), Vs=bf16_tensor(w.Vs, device),
        offsets=torch.from_numpy(w.offsets).to(device), lengths=torch.from_numpy(w.lengths).to(device),
        max_len=w.max_len,
    )


def make_context(dw: DeviceWorkload, parts: int = 24, device: int = 0) -> hb.Context:
    return hb.Context(device, hb.hg_workspace_bytes(dw.B * dw.nq, dw.Hq, dw.D, parts))


def hydragen(ctx: hb.Context, dw: DeviceWorkload, out_dtype=torch.bfloat16, want_lse: bool = True):
    O = torch.empty(dw.lead + (dw.D,), dtype=out_dtype, device=dw.Q.device)
    L = torch.empty(dw.lead, dtype=torch.float32, device=dw.Q.device) if want_lse else None
    hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    return O, L


def naive(ctx: hb.Context, dw: DeviceWorkload, out_dtype=torch.bfloat16, want_lse: bool = True):
    O = torch.empty(dw.lead + (dw.D,), dtype=out_dtype, device=dw.Q.device)
    L = torch.empty(dw.lead, dtype=torch.float32, device=dw.Q.device) if want_lse else None
    hb.hg_naive_attn(ctx, dw.Q, dw.levels, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O, L, dw.scale)
    return O, L


def paged_to_device(pg, device="cuda:0") -> hb.PagedKV:
    """A workloads.PagedSuffix as device tensors."""
    return hb.PagedKV(K=bf16_tensor(pg.K, device), V=bf16_tensor(pg.V, device),
                      page_table=torch.from_numpy(pg.table).to(device), page_size=pg.page_size)


def hydragen_paged(ctx: hb.Context, dw: DeviceWorkload, kv: hb.PagedKV, lengths=None, max_len=None, out_dtype=torch.bfloat16):
    O = torch.empty(dw.lead + (dw.D,), dtype=out_dtype, device=dw.Q.device)
    L = torch.empty(dw.lead, dtype=torch.float32, device=dw.Q.device)
    hb.hg_hydragen_attn_paged(ctx, dw.Q, dw.levels, kv, dw.lengths if lengths is None else lengths,
                              dw.max_len if max_len is None else max_len, O, L, dw.scale)
    return O, L
