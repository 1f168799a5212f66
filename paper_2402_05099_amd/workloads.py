"""Seeded synthetic decode-attention workloads (inputs only; no attention arithmetic here).

This module is the single source of inputs for both the HIP path and the CPU
oracle.  It draws N(0,1) values from numpy's PCG64 streams, rounds them to
bf16 (round-to-nearest-even) and returns the raw 16-bit patterns, so that both
sides consume identical bits.  It knows nothing about softmax, LSE or merging.

Shapes follow the paper's problem statement (App. B docstring of the
Hydragen attention routine): queries [B, Hq, D] (one decode token per
sequence), a shared KV block stored once as [P, Hkv, D], and per-sequence
suffix KV.  The suffix cache is kept packed and ragged: [T, Hkv, D] with
offsets[B] and lengths[B]; the paper's padded [B, Lmax, Hkv, D] cache is the
special case offsets[b] = b * Lmax.  Tree-shaped sharing (Sec. 3.3) is a list
of levels; level l holds Gn_l shared blocks, block g owning KV rows
[kv_off[g], kv_off[g+1]) and the contiguous sequences [seq_off[g], seq_off[g+1]).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_CHUNK = 1 << 22  # elements per independent child stream


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, tensor_id: int, shape, gain: float = 1.0, threads: int = 8) -> np.ndarray:
    """N(0,1)*gain as bf16 bits, shape `shape`.

    Element i lives in chunk i // _CHUNK, and each chunk is drawn from
    default_rng(SeedSequence([seed, tensor_id, chunk])) as float32, so the
    result does not depend on the thread count.
    """
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c: int) -> None:
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        rng = np.random.default_rng(np.random.SeedSequence([seed, tensor_id, c]))
        x = rng.standard_normal(hi - lo, dtype=np.float32)
        if gain != 1.0:
            x *= np.float32(gain)
        out[lo:hi] = f32_to_bf16_bits(x)

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nchunks)))
    return out.reshape(shape)


@dataclass
class Level:
    """One level of shared KV blocks (Sec. 3.3: a tree vertex's KV is shared by its descendants)."""
    K: np.ndarray        # uint16 [Ptot, Hkv, D]
    V: np.ndarray        # uint16 [Ptot, Hkv, D]
    kv_off: np.ndarray   # int32 [Gn+1], rows of K/V owned by each block
    seq_off: np.ndarray  # int32 [Gn+1], sequences covered by each block

    @property
    def Gn(self) -> int:
        return int(self.kv_off.shape[0] - 1)

    @property
    def max_rows(self) -> int:
        return int(np.max(np.diff(self.kv_off))) if self.Gn else 0

    @property
    def max_seqs(self) -> int:
        return int(np.max(np.diff(self.seq_off))) if self.Gn else 0


@dataclass
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    scale: float
    Q: np.ndarray                      # uint16 [B, Hq, D], or [B, nq, Hq, D] with nq > 1 queries per sequence
    levels: List[Level]
    Ks: np.ndarray                     # uint16 [T, Hkv, D]
    Vs: np.ndarray                     # uint16 [T, Hkv, D]
    offsets: np.ndarray                # int32 [B]
    lengths: np.ndarray                # int32 [B]
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def nq(self) -> int:
        """Queries per sequence (App. B's num_queries): the last nq tokens of every suffix are queried at once."""
        return int(self.Q.shape[1]) if self.Q.ndim == 4 else 1

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def T(self) -> int:
        return int(self.Ks.shape[0])

    @property
    def max_len(self) -> int:
        return int(self.lengths.max()) if self.B else 0

    def kv_rows_of(self, b: int):
        """(level_index, row_begin, row_end) of every shared block covering sequence b, root first."""
        out = []
        for li, lv in enumerate(self.levels):
            g = int(np.searchsorted(lv.seq_off, b, side="right") - 1)
            if 0 <= g < lv.Gn and lv.seq_off[g] <= b < lv.seq_off[g + 1]:
                out.append((li, int(lv.kv_off[g]), int(lv.kv_off[g + 1])))
        return out


def _single_block_level(seed: int, tid: int, P: int, B: int, Hkv: int, D: int) -> Level:
    return Level(
        K=normal_bf16(seed, tid, (P, Hkv, D)),
        V=normal_bf16(seed, tid + 1, (P, Hkv, D)),
        kv_off=np.array([0, P], dtype=np.int32),
        seq_off=np.array([0, B], dtype=np.int32),
    )


def make_workload(
    name: str,
    seed: int,
    B: int,
    Hq: int,
    Hkv: int,
    D: int,
    level_specs,                 # list of (Gn, rows_per_block, seqs_per_block)
    len_lo: int,
    len_hi: int,
    q_gain: float = 1.0,
    plant: Optional[str] = None,  # None | "suffix" | "prefix"
    lengths: Optional[np.ndarray] = None,
    nq: int = 1,
) -> Workload:
    """Build a workload.  Tensor ids (fixed): Q=0, level l K=10+2l, V=11+2l, lengths=90, Ks=100, Vs=101.

    Suffix lengths are integers uniform on [len_lo, len_hi] inclusive.
    `q_gain` scales Q before the bf16 cast (q_gain=4 gives a peaked softmax).
    `nq` > 1 draws Q as [B, nq, Hq, D]: nq queries per sequence (the last nq suffix tokens).
    `plant` overwrites a few K rows with 2*q so that one key dominates a
    query's softmax: in the suffix (every sequence, its middle row, first
    query head of each KV group) or in each shared block of level 0 (rows
    first/middle/last for the first/middle/last sequence of that block).
    """
    assert Hq % Hkv == 0
    G = Hq // Hkv
    assert nq >= 1 and (nq == 1 or plant is None), "planted keys are defined for one query per sequence"
    Q = normal_bf16(seed, 0, (B, Hq, D) if nq == 1 else (B, nq, Hq, D), gain=q_gain)
    levels = []
    for li, (Gn, rows, seqs) in enumerate(level_specs):
        assert Gn * seqs <= B
        levels.append(
            Level(
                K=normal_bf16(seed, 10 + 2 * li, (Gn * rows, Hkv, D)),
                V=normal_bf16(seed, 11 + 2 * li, (Gn * rows, Hkv, D)),
                kv_off=(np.arange(Gn + 1, dtype=np.int64) * rows).astype(np.int32),
                seq_off=(np.arange(Gn + 1, dtype=np.int64) * seqs).astype(np.int32),
            )
        )
    if lengths is None:
        rng = np.random.default_rng(np.random.SeedSequence([seed, 90]))
        lengths = rng.integers(len_lo, len_hi + 1, size=B, dtype=np.int64).astype(np.int32)
    else:
        lengths = np.asarray(lengths, dtype=np.int32)
        assert lengths.shape == (B,)
    offsets = np.zeros(B, dtype=np.int32)
    if B > 1:
        offsets[1:] = np.cumsum(lengths[:-1], dtype=np.int64).astype(np.int32)
    T = int(lengths.sum(dtype=np.int64))
    Ks = normal_bf16(seed, 100, (T, Hkv, D))
    Vs = normal_bf16(seed, 101, (T, Hkv, D))

    def dominant_row(b: int, kvh: int) -> np.ndarray:
        q = bf16_bits_to_f32(Q[b, kvh * G])
        return f32_to_bf16_bits(2.0 * q)  # exact doubling of a bf16 value

    notes = {}
    if plant == "suffix":
        for b in range(B):
            if lengths[b] > 0:
                row = int(offsets[b]) + int(lengths[b]) // 2
                for kvh in range(Hkv):
                    Ks[row, kvh] = dominant_row(b, kvh)
    elif plant == "prefix":
        lv = levels[0]
        planted = []
        for g in range(lv.Gn):
            r0, r1 = int(lv.kv_off[g]), int(lv.kv_off[g + 1])
            s0, s1 = int(lv.seq_off[g]), int(lv.seq_off[g + 1])
            if r1 <= r0 or s1 <= s0:
                continue
            for row, b in ((r0, s0), ((r0 + r1) // 2, (s0 + s1) // 2), (r1 - 1, s1 - 1)):
                for kvh in range(Hkv):
                    lv.K[row, kvh] = dominant_row(b, kvh)
                planted.append((row, b))
        notes["planted"] = planted
    elif plant is not None:
        raise ValueError(plant)

    return Workload(
        name=name, B=B, Hq=Hq, Hkv=Hkv, D=D, scale=1.0 / math.sqrt(D), Q=Q, levels=levels,
        Ks=Ks, Vs=Vs, offsets=offsets, lengths=lengths, seed=seed, notes=notes,
    )


# The five benchmark configurations (index 1..5), each with its fixed seed.
def config(idx: int, P: Optional[int] = None, B: Optional[int] = None, L: Optional[int] = None, D: Optional[int] = None,
           **variant) -> Workload:
    """idx in 1..6.  `P` overrides the level-0 prefix length (config 3 sweeps 1024/4096/16384), `D` the head dimension
    of configs 2..6 (128 in the paper's models; 64 is the variant the kernels also cover).

    6 is the shape of the paper's attention microbenchmark (Sec. 4.2: eight query heads, one KV head, head
    dimension 128), swept over batch size `B`, prefix length `P` and suffix length `L` (every sequence has L rows).
    """
    if idx == 1:
        return make_workload("c1_tiny", 1, 4, 4, 4, 64, [(1, P or 128, 4)], 16, 16, **variant)
    d = D or 128
    tag = "" if d == 128 else f"_D{d}"
    if idx == 2:
        return make_workload("c2_codellama13b" + tag, 2, 256, 40, 40, d, [(1, P or 2048, 256)], 1, 256, **variant)
    if idx == 3:
        p = P or 16384
        return make_workload(f"c3_long_P{p}" + tag, 3, 1024, 40, 40, d, [(1, p, 1024)], 32, 128, **variant)
    if idx == 4:
        return make_workload("c4_gqa" + tag, 4, 512, 64, 8, d, [(1, P or 4096, 512)], 1, 512, **variant)
    if idx == 5:
        return make_workload("c5_tree" + tag, 5, 2048, 40, 40, d, [(1, P or 1024, 2048), (16, 512, 128)], 64, 64, **variant)
    if idx == 6:
        b, p, l = B or 1024, P or 16384, L or 128
        return make_workload(f"c6_micro_B{b}_P{p}_L{l}" + tag, 6, b, 8, 1, d, [(1, p, b)], l, l, **variant)
    raise ValueError(f"no config {idx}")


def scaled_down(idx: int, **variant) -> Workload:
    """Same structure as config idx at sizes the CPU oracle finishes in seconds.

    Sizes are chosen to span several key tiles and query tiles of the GPU
    kernels and to leave ragged tails (prefix lengths and batch sizes that are
    not multiples of 32/64/128).
    """
    if idx == 2:
        return make_workload("c2_small", 12, 37, 8, 8, 128, [(1, 333, 37)], 1, 70, **variant)
    if idx == 3:
        return make_workload("c3_small", 13, 150, 4, 4, 128, [(1, 1100, 150)], 32, 128, **variant)
    if idx == 4:
        return make_workload("c4_small", 14, 45, 16, 2, 128, [(1, 515, 45)], 1, 150, **variant)
    if idx == 5:
        return make_workload("c5_small", 15, 96, 4, 4, 128, [(1, 200, 96), (4, 77, 24)], 20, 20, **variant)
    if idx == 6:
        return make_workload("c6_small", 16, 75, 8, 1, 128, [(1, 700, 75)], 50, 50, **variant)
    return config(1, **variant)


# ---- suffix-cache layouts for the decode-step neighbours of the path (inputs only: scatter, no arithmetic) ---------

@dataclass
class PagedSuffix:
    """The suffix rows of a workload stored in fixed-size pages of one pool (the layout Sec. 3.5 contrasts with)."""
    K: np.ndarray          # uint16 [n_pages * page_size, Hkv, D]
    V: np.ndarray
    table: np.ndarray      # int32 [B, stride]: physical page of each logical page, -1 where none is assigned
    page_size: int
    capacity: int          # rows every sequence may hold: max_len + reserve (its pages cover at least that many)

    @property
    def n_pages(self) -> int:
        return int(self.K.shape[0]) // self.page_size


def make_paged(w: Workload, page_size: int, reserve: int = 0, spare_pages: int = 3, junk_gain: float = 8.0) -> PagedSuffix:
    """Scatter w's packed suffix rows into pages handed out in a seeded random physical order.

    Every sequence gets pages for max_len + reserve rows (room to append).  Rows no sequence owns (page tails,
    reserved rows, spare pages) hold N(0,1)*junk_gain values (tensor ids 110, 111) so that a kernel that reads a
    row it should not shows up in the result.  Table entries past a sequence's pages are -1.
    """
    ps = int(page_size)
    cap = w.max_len + reserve
    per_seq = (cap + ps - 1) // ps
    stride = per_seq + 1
    n_pages = w.B * per_seq + spare_pages
    rng = np.random.default_rng(np.random.SeedSequence([w.seed, 112, ps]))
    phys = rng.permutation(n_pages).astype(np.int32)[: w.B * per_seq].reshape(w.B, per_seq) if w.B else np.zeros((0, per_seq), np.int32)
    table = np.full((w.B, stride), -1, dtype=np.int32)
    table[:, :per_seq] = phys
    K = normal_bf16(w.seed, 110, (n_pages * ps, w.Hkv, w.D), gain=junk_gain)
    V = normal_bf16(w.seed, 111, (n_pages * ps, w.Hkv, w.D), gain=junk_gain)
    for b in range(w.B):
        n = int(w.lengths[b])
        j = np.arange(n)
        rows = phys[b, j // ps].astype(np.int64) * ps + j % ps
        K[rows] = w.Ks[w.offsets[b]: w.offsets[b] + n]
        V[rows] = w.Vs[w.offsets[b]: w.offsets[b] + n]
    return PagedSuffix(K=K, V=V, table=table, page_size=ps, capacity=cap)


def with_room(w: Workload, reserve: int, junk_gain: float = 8.0):
    """(Ks, Vs, offsets, capacity): w's suffix re-packed so that every sequence owns max_len + reserve rows.

    The rows behind a sequence's last one hold N(0,1)*junk_gain values (tensor ids 113, 114).
    """
    cap = w.max_len + reserve
    Ks = normal_bf16(w.seed, 113, (w.B * cap, w.Hkv, w.D), gain=junk_gain)
    Vs = normal_bf16(w.seed, 114, (w.B * cap, w.Hkv, w.D), gain=junk_gain)
    offsets = (np.arange(w.B, dtype=np.int64) * cap).astype(np.int32)
    for b in range(w.B):
        n = int(w.lengths[b])
        Ks[offsets[b]: offsets[b] + n] = w.Ks[w.offsets[b]: w.offsets[b] + n]
        Vs[offsets[b]: offsets[b] + n] = w.Vs[w.offsets[b]: w.offsets[b] + n]
    return Ks, Vs, offsets, cap


def new_rows(w: Workload, step: int = 0):
    """(Knew, Vnew) uint16 [B, Hkv, D] (or [B, nq, Hkv, D]): the K/V rows of the tokens a decode step adds (tensor ids 120+2*step, 121+2*step)."""
    shape = (w.B, w.Hkv, w.D) if w.nq == 1 else (w.B, w.nq, w.Hkv, w.D)
    return normal_bf16(w.seed, 120 + 2 * step, shape), normal_bf16(w.seed, 121 + 2 * step, shape)


@dataclass
class Fp8Suffix:
    """An 8-bit suffix cache for a workload: E4M3 codes, one scale per tensor (value = code * scale)."""
    Ks8: np.ndarray        # uint8 [T, Hkv, D]
    Vs8: np.ndarray
    k_scale: float
    v_scale: float
    offsets: np.ndarray    # int32 [B]
    capacity: int          # rows every sequence may hold


def make_fp8(w: Workload, reserve: int = 0, headroom: float = 1.0, junk_code: Optional[int] = 0x7F) -> Fp8Suffix:
    """w's suffix rows as an 8-bit cache with room for `reserve` more rows per sequence.

    Scales are per-tensor calibration values: largest magnitude * headroom / 448 (headroom < 1 makes the largest values
    saturate).  The codes come from torch's float8_e4m3fn conversion of value / scale (a library routine: this module
    holds no arithmetic of the method).  Rows no sequence owns hold `junk_code` (0x7f is a NaN code; None: zero).
    """
    import torch

    cap = w.max_len + reserve
    offsets = (np.arange(w.B, dtype=np.int64) * cap).astype(np.int32)
    out = []
    scales = []
    for bits in (w.Ks, w.Vs):
        x = bf16_bits_to_f32(bits)
        amax = float(np.abs(x).max()) if x.size else 1.0
        scale = float(np.float32(max(amax, 1e-6) * headroom / 448.0))
        q = torch.from_numpy(x / np.float32(scale)).clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        full = np.full((w.B * cap, w.Hkv, w.D), 0 if junk_code is None else junk_code, dtype=np.uint8)
        for b in range(w.B):
            n = int(w.lengths[b])
            full[offsets[b]: offsets[b] + n] = q[w.offsets[b]: w.offsets[b] + n]
        out.append(full)
        scales.append(scale)
    return Fp8Suffix(Ks8=out[0], Vs8=out[1], k_scale=scales[0], v_scale=scales[1], offsets=offsets, capacity=cap)


def make_paged_fp8(w: Workload, page_size: int, reserve: int = 0, spare_pages: int = 3, headroom: float = 1.0):
    """(PagedSuffix with uint8 pools, k_scale, v_scale): make_fp8's codes scattered into pages as make_paged does.

    Rows no sequence owns (page tails, reserved rows, spare pages) hold the NaN code 0x7f.
    """
    f8 = make_fp8(w, headroom=headroom, junk_code=None)
    ps = int(page_size)
    cap = w.max_len + reserve
    per_seq = (cap + ps - 1) // ps
    n_pages = w.B * per_seq + spare_pages
    rng = np.random.default_rng(np.random.SeedSequence([w.seed, 115, ps]))
    phys = rng.permutation(n_pages).astype(np.int32)[: w.B * per_seq].reshape(w.B, per_seq) if w.B else np.zeros((0, per_seq), np.int32)
    table = np.full((w.B, per_seq + 1), -1, dtype=np.int32)
    table[:, :per_seq] = phys
    K = np.full((n_pages * ps, w.Hkv, w.D), 0x7F, dtype=np.uint8)
    V = np.full((n_pages * ps, w.Hkv, w.D), 0x7F, dtype=np.uint8)
    for b in range(w.B):
        n = int(w.lengths[b])
        j = np.arange(n)
        rows = phys[b, j // ps].astype(np.int64) * ps + j % ps
        K[rows] = f8.Ks8[f8.offsets[b]: f8.offsets[b] + n]
        V[rows] = f8.Vs8[f8.offsets[b]: f8.offsets[b] + n]
    return PagedSuffix(K=K, V=V, table=table, page_size=ps, capacity=cap), f8.k_scale, f8.v_scale
