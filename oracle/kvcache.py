"""Plain definitions of the suffix-cache layouts and of the decode-step cache update.  TEST INFRASTRUCTURE ONLY.

Byte and index work only (no arithmetic on values), written as loops over sequences and rows so that each line can
be checked by eye against the definition it states:

  * paged cache: suffix row j of sequence b lives in pool row table[b, j // page_size] * page_size + j % page_size
    (the block-table indirection of the paged caches that Sec. 3.5 and Sec. 6 refer to);
  * cache update of a decode step (Sec. 2.2: the cache keeps the keys and values of all earlier tokens and each
    step adds the newest token's): the nq new rows of sequence b become suffix rows length_b .. length_b + nq - 1,
    rows at or above the capacity are dropped, and the length grows by the number of rows kept.

Pinned in tests/test_kvcache_pins.py by hand-typed tiny cases and by round trips through the scatter of the input
generator (which is independent code).
"""
from __future__ import annotations

import numpy as np


def paged_to_packed(Kpool, Vpool, table, page_size: int, lengths):
    """Gather the rows the page table designates.  Returns (Ks, Vs, offsets): packed rows [T, Hkv, D], offsets int32 [B]."""
    table = np.asarray(table)
    lengths = np.asarray(lengths)
    B = lengths.shape[0]
    offsets = np.zeros(B, dtype=np.int32)
    rows = []
    total = 0
    for b in range(B):
        offsets[b] = total
        for j in range(int(lengths[b])):
            page = int(table[b, j // page_size])
            assert 0 <= page and (page + 1) * page_size <= Kpool.shape[0], (b, j, page)
            rows.append(page * page_size + j % page_size)
        total += int(lengths[b])
    idx = np.asarray(rows, dtype=np.int64)
    return Kpool[idx].copy(), Vpool[idx].copy(), offsets


def kv_append(Ks, Vs, offsets, lengths, capacity: int, Knew, Vnew):
    """Cache update on packed rows (sequence b owns rows offsets[b] .. offsets[b] + capacity - 1).

    Knew, Vnew: [B, Hkv, D] or [B, nq, Hkv, D].  Returns new (Ks, Vs, lengths); the inputs are not modified.
    """
    Ks, Vs, lengths = Ks.copy(), Vs.copy(), np.asarray(lengths).copy()
    if Knew.ndim == 3:
        Knew, Vnew = Knew[:, None], Vnew[:, None]
    B, nq = Knew.shape[:2]
    for b in range(B):
        n = int(lengths[b])
        for t in range(nq):
            if 0 <= n < capacity:
                Ks[int(offsets[b]) + n] = Knew[b, t]
                Vs[int(offsets[b]) + n] = Vnew[b, t]
                n += 1
        lengths[b] = n
    return Ks, Vs, lengths


def kv_append_paged(Kpool, Vpool, table, page_size: int, lengths, capacity: int, Knew, Vnew):
    """Cache update through a page table.  Returns new (Kpool, Vpool, lengths); the inputs are not modified."""
    Kpool, Vpool, lengths = Kpool.copy(), Vpool.copy(), np.asarray(lengths).copy()
    if Knew.ndim == 3:
        Knew, Vnew = Knew[:, None], Vnew[:, None]
    B, nq = Knew.shape[:2]
    for b in range(B):
        n = int(lengths[b])
        for t in range(nq):
            if 0 <= n < capacity:
                page = int(table[b, n // page_size])
                assert 0 <= page and (page + 1) * page_size <= Kpool.shape[0], (b, n, page)
                Kpool[page * page_size + n % page_size] = Knew[b, t]
                Vpool[page * page_size + n % page_size] = Vnew[b, t]
                n += 1
        lengths[b] = n
    return Kpool, Vpool, lengths
