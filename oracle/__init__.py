"""ctypes front end of the fp64 CPU oracle (oracle/hydragen_oracle.c).  TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package: it exists for tests/,
the smoke check and the benchmark's cpu_baseline leg.  It shares no code with
the HIP library; it only accepts the same seeded input arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

from .kvcache import kv_append, kv_append_paged, paged_to_packed  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hydragen_oracle.c")
_LIB = os.path.join(_HERE, "libhydragen_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 -fopenmp (no fast-math: fp64 sums stay in index order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.hgo_attention.restype = ctypes.c_int
        lib.hgo_merge.restype = ctypes.c_int
        lib.hgo_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().hgo_num_threads())


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def attention_arrays(
    Q, Hkv: int, levels: Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]],
    Ks=None, Vs=None, offsets=None, lengths=None, scale: Optional[float] = None, seqs=None,
):
    """Exact attention over (shared blocks covering b) || (suffix of b) for each sequence.

    Q: uint16 [B,Hq,D], or [B,nq,Hq,D] for nq queries per sequence (query t sees suffix rows
    [0, length - (nq-1-t))); levels: list of (K, V, kv_off, seq_off); suffix arrays optional.
    Returns (O float64 [n,Hq,D], LSE float64 [n,Hq]) for the n selected sequences ([n,nq,Hq,D] and [n,nq,Hq] for 4-d Q).
    """
    lib = _load()
    Q = _u16(Q)
    four = Q.ndim == 4
    if four:
        B, nq, Hq, D = Q.shape
    else:
        B, Hq, D = Q.shape
        nq = 1
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    nl = len(levels)
    keep = []
    Kp = (ctypes.c_void_p * max(nl, 1))()
    Vp = (ctypes.c_void_p * max(nl, 1))()
    kop = (ctypes.c_void_p * max(nl, 1))()
    sop = (ctypes.c_void_p * max(nl, 1))()
    Gn = np.zeros(max(nl, 1), dtype=np.int32)
    for i, (K, V, kv_off, seq_off) in enumerate(levels):
        K, V, kv_off, seq_off = _u16(K), _u16(V), _i32(kv_off), _i32(seq_off)
        assert K.shape == V.shape and K.shape[1:] == (Hkv, D), (K.shape, V.shape)
        assert kv_off.shape == seq_off.shape and kv_off.ndim == 1 and kv_off.shape[0] >= 1
        assert kv_off[-1] <= K.shape[0] and seq_off[-1] <= B
        keep += [K, V, kv_off, seq_off]
        Kp[i], Vp[i], kop[i], sop[i] = K.ctypes.data, V.ctypes.data, kv_off.ctypes.data, seq_off.ctypes.data
        Gn[i] = kv_off.shape[0] - 1
    if lengths is not None:
        Ks, Vs, offsets, lengths = _u16(Ks), _u16(Vs), _i32(offsets), _i32(lengths)
        assert Ks.shape == Vs.shape and Ks.shape[1:] == (Hkv, D)
        assert offsets.shape == (B,) and lengths.shape == (B,)
        if B:
            assert int((offsets.astype(np.int64) + lengths).max()) <= Ks.shape[0]
    else:
        Ks = Vs = offsets = None
    if seqs is not None:
        seqs = _i32(seqs)
        n = int(seqs.shape[0])
    else:
        n = B
    O = np.empty((n, nq, Hq, D) if four else (n, Hq, D), dtype=np.float64)
    LSE = np.empty((n, nq, Hq) if four else (n, Hq), dtype=np.float64)
    rc = lib.hgo_attention(
        _ptr(Q), B, nq, Hq, Hkv, D, nl, Kp, Vp, _ptr(Gn), kop, sop,
        _ptr(Ks), _ptr(Vs), _ptr(offsets), _ptr(lengths), ctypes.c_double(float(scale)),
        _ptr(seqs), n, _ptr(O), _ptr(LSE),
    )
    if rc != 0:
        raise ValueError("hgo_attention rejected its arguments")
    return O, LSE


def attention(w, levels: Optional[Sequence[int]] = None, suffix: bool = True, seqs=None):
    """Oracle attention for a workload object (see paper_2402_05099_amd.workloads.Workload).

    levels=None uses every level; levels=[i] restricts to some; suffix=False drops the suffix.
    The full result is levels=None, suffix=True.
    """
    idx = range(len(w.levels)) if levels is None else levels
    lv = [(w.levels[i].K, w.levels[i].V, w.levels[i].kv_off, w.levels[i].seq_off) for i in idx]
    if suffix:
        return attention_arrays(w.Q, w.Hkv, lv, w.Ks, w.Vs, w.offsets, w.lengths, w.scale, seqs)
    return attention_arrays(w.Q, w.Hkv, lv, scale=w.scale, seqs=seqs)


def merge(parts: Sequence[np.ndarray], lses: Sequence[np.ndarray]):
    """fp64 n-way LSE merge.  parts[i]: [..., D]; lses[i]: [...].  Returns (O, LSE) with those shapes."""
    lib = _load()
    n = len(parts)
    assert n == len(lses) and n > 0
    shape = parts[0].shape
    D = shape[-1]
    P = [np.ascontiguousarray(p, dtype=np.float64).reshape(-1, D) for p in parts]
    L = [np.ascontiguousarray(l, dtype=np.float64).reshape(-1) for l in lses]
    rows = P[0].shape[0]
    for p, l in zip(P, L):
        assert p.shape == (rows, D) and l.shape == (rows,)
    pp = (ctypes.c_void_p * n)(*[p.ctypes.data for p in P])
    lp = (ctypes.c_void_p * n)(*[l.ctypes.data for l in L])
    O = np.empty((rows, D), dtype=np.float64)
    LSE = np.empty(rows, dtype=np.float64)
    rc = lib.hgo_merge(n, pp, lp, ctypes.c_int64(rows), D, _ptr(O), _ptr(LSE))
    if rc != 0:
        raise ValueError("hgo_merge rejected its arguments")
    return O.reshape(shape), LSE.reshape(shape[:-1])
