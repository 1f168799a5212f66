"""GPU parity of the decode-step neighbours of the path: suffix attention through a page table, and the KV-cache
update (append) on packed and paged caches.  Attention results are compared with the fp64 oracle on the rows the
table designates; cache contents and lengths are byte and index work and must be equal bit for bit."""
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


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 device tensor -> uint16 bit patterns on the host"""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("page_size", [16, 64, 256])
@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_paged_suffix_attn(idx, page_size):
    say(f"paged suffix idx={idx} page_size={page_size}")
    w = wl.scaled_down(idx)
    dw = dev.to_device(w)
    pg = wl.make_paged(w, page_size)
    kv = dev.paged_to_device(pg)
    ctx = dev.make_context(dw, parts=24)
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, 1)
    Oref, Lref = oracle.attention(w, levels=[])
    O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.float32, device="cuda:0")
    L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_paged(ctx, dw.Q, kv, dw.lengths, dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"paged suffix idx={idx} ps={page_size}")
    # the packed cache holds the same rows and the same (vector-ALU) kernel walks them in the same order: identical bits
    O2, L2 = torch.empty_like(O), torch.empty_like(L)
    hb.hg_suffix_attn(ctx, dw.Q, dw.Ks, dw.Vs, dw.offsets, dw.lengths, dw.max_len, O2, L2, dw.scale)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(L, L2)
    ctx.close()


@pytest.mark.parametrize("kernel", [1, 2], ids=["valu", "mfma"])
@pytest.mark.parametrize("page_size", [16, 32, 128])
@pytest.mark.parametrize("shape", ["mha", "gqa8", "gqa4_nq3"])
def test_paged_suffix_both_kernels_and_unwritten_rows(shape, page_size, kernel):
    """Both suffix kernels through the page table; the pool rows that no sequence owns (page tails, free pages) hold
    NaN, as memory that was never written may, and must not reach a result."""
    say(f"paged {shape} page_size={page_size} kernel={kernel}")
    rng = np.random.default_rng(11)
    B = 27
    ln = rng.integers(0, 330, size=B).astype(np.int32)
    ln[:8] = [0, 1, 15, 16, 17, 31, 32, 33]
    if shape == "mha":
        w = wl.make_workload(shape, 94, B, 4, 4, 128, [(1, 60, B)], 0, 0, lengths=ln)
    elif shape == "gqa8":
        w = wl.make_workload(shape, 95, B, 16, 2, 128, [(1, 60, B)], 0, 0, lengths=ln)
    else:
        w = wl.make_workload(shape, 96, B, 8, 2, 128, [(1, 60, B)], 0, 0, lengths=ln, nq=3)
    pg = wl.make_paged(w, page_size)
    owned = np.zeros(pg.K.shape[0], dtype=bool)
    for b in range(B):
        j = np.arange(int(ln[b]))
        owned[pg.table[b, j // page_size].astype(np.int64) * page_size + j % page_size] = True
    pg.K[~owned] = 0x7FC0     # bf16 NaN
    pg.V[~owned] = 0x7FC0
    dw = dev.to_device(w)
    kv = dev.paged_to_device(pg)
    ctx = dev.make_context(dw, parts=24)
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, kernel)
    Osuf, Lsuf = oracle.attention(w, levels=[])
    Oref, Lref = oracle.attention(w)
    for chunk in (0, 64):
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
        O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.float32, device="cuda:0")
        L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
        hb.hg_suffix_attn_paged(ctx, dw.Q, kv, dw.lengths, dw.max_len, O, L, dw.scale)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Osuf, Lsuf, f"paged suffix {shape} ps={page_size} kernel={kernel} chunk={chunk}")
        O, L = dev.hydragen_paged(ctx, dw, kv, out_dtype=torch.float32)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Oref, Lref, f"paged fused {shape} ps={page_size} kernel={kernel} chunk={chunk}")
    ctx.close()


@pytest.mark.parametrize("chunk", [32, 96, 512])
def test_paged_suffix_long_ragged_chunks(chunk):
    """Suffixes of several hundred rows over 16-row pages: work items cover many pages, start mid-table, end mid-page."""
    say(f"paged suffix long chunk={chunk}")
    rng = np.random.default_rng(5)
    ln = rng.integers(0, 700, size=23).astype(np.int32)
    ln[:5] = [0, 1, 15, 16, 17]
    w = wl.make_workload("paged_long", 61, 23, 8, 2, 128, [], 0, 0, lengths=ln)
    dw = dev.to_device(w)
    kv = dev.paged_to_device(wl.make_paged(w, 16))
    ctx = dev.make_context(dw, parts=32)
    ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
    Oref, Lref = oracle.attention(w)
    O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_paged(ctx, dw.Q, kv, dw.lengths, dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"paged long chunk={chunk}")
    ctx.close()


@pytest.mark.parametrize("idx,nq", [(3, 1), (5, 1), (6, 1), (4, 3)])
def test_paged_fused_hydragen(idx, nq):
    say(f"paged fused idx={idx} nq={nq}")
    w = wl.scaled_down(idx, nq=nq) if nq > 1 else wl.scaled_down(idx)
    dw = dev.to_device(w)
    kv = dev.paged_to_device(wl.make_paged(w, 32))
    ctx = dev.make_context(dw, parts=24)
    Oref, Lref = oracle.attention(w)
    for dtype in (torch.float32, torch.bfloat16):
        O, L = dev.hydragen_paged(ctx, dw, kv, out_dtype=dtype)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Oref, Lref, f"paged fused idx={idx} nq={nq} {dtype}", out_bf16=dtype == torch.bfloat16)
    ctx.close()


@pytest.mark.parametrize("nq", [1, 3])
def test_kv_append_packed_and_paged(nq):
    """New rows land behind each sequence's last row, lengths advance on the device, full sequences drop rows."""
    say(f"append nq={nq}")
    rng = np.random.default_rng(6)
    B = 37
    ln = rng.integers(0, 60, size=B).astype(np.int32)
    w = wl.make_workload("append", 62, B, 8, 2, 128, [], 0, 0, lengths=ln, nq=nq)
    reserve = 2                       # the longest sequences run out of room when nq = 3
    Kn, Vn = wl.new_rows(w)
    dKn, dVn = dev.bf16_tensor(Kn, "cuda:0"), dev.bf16_tensor(Vn, "cuda:0")
    ctx = hb.Context(0, hb.hg_workspace_bytes(B * nq, 8, 128, 8))
    # packed rows with room behind each sequence
    Kr, Vr, offr, cap = wl.with_room(w, reserve)
    K2, V2, L2 = oracle.kv_append(Kr, Vr, offr, w.lengths, cap, Kn, Vn)
    dK, dV = dev.bf16_tensor(Kr, "cuda:0"), dev.bf16_tensor(Vr, "cuda:0")
    doff, dlen = torch.from_numpy(offr).cuda(), torch.from_numpy(w.lengths.copy()).cuda()
    hb.hg_kv_append(ctx, dKn, dVn, dK, dV, doff, dlen, cap)
    torch.cuda.synchronize()
    assert np.array_equal(dlen.cpu().numpy(), L2)
    assert np.array_equal(bits(dK), K2) and np.array_equal(bits(dV), V2)
    if nq == 3:
        assert (L2 - w.lengths < nq).any(), "the case must contain a sequence that runs out of room"
    # paged
    pg = wl.make_paged(w, 16, reserve=reserve)
    Kp, Vp, Lp = oracle.kv_append_paged(pg.K, pg.V, pg.table, 16, w.lengths, pg.capacity, Kn, Vn)
    kv = dev.paged_to_device(pg)
    dlen = torch.from_numpy(w.lengths.copy()).cuda()
    hb.hg_kv_append_paged(ctx, dKn, dVn, kv, dlen, pg.capacity)
    torch.cuda.synchronize()
    assert np.array_equal(dlen.cpu().numpy(), Lp) and np.array_equal(Lp, L2)
    assert np.array_equal(bits(kv.K), Kp) and np.array_equal(bits(kv.V), Vp)
    ctx.close()


@pytest.mark.parametrize("idx", [5, 4], ids=["tree_mha", "gqa"])
@pytest.mark.parametrize("paged", [False, True])
def test_decode_steps_append_then_attend_in_a_graph(paged, idx):
    """One decode step = cache update + fused attention, captured once and replayed: lengths advance on the device,
    the launch sequence never changes (Sec. 3.5), and every step matches the oracle on the grown cache."""
    say(f"decode steps paged={paged} idx={idx}")
    steps = 4
    w = wl.scaled_down(idx)
    dw = dev.to_device(w)
    s = torch.cuda.Stream()
    ctx = hb.Context(0, hb.hg_workspace_bytes(dw.B, dw.Hq, dw.D, 24), stream=s)
    max_len = w.max_len + steps
    # host-side mirror of the cache, advanced by the oracle's definition of the update
    if paged:
        pg = wl.make_paged(w, 16, reserve=steps)
        kv = dev.paged_to_device(pg)
        hK, hV, cap = pg.K, pg.V, pg.capacity
    else:
        hK, hV, hoff, cap = wl.with_room(w, steps)
        dK, dV, doff = dev.bf16_tensor(hK, "cuda:0"), dev.bf16_tensor(hV, "cuda:0"), torch.from_numpy(hoff).cuda()
    hlen = w.lengths.copy()
    dlen = torch.from_numpy(hlen.copy()).cuda()
    dKn = torch.zeros((w.B, w.Hkv, w.D), dtype=torch.bfloat16, device="cuda:0")
    dVn = torch.zeros_like(dKn)
    O = torch.zeros((dw.B, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    L = torch.zeros((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")

    def step():
        if paged:
            hb.hg_kv_append_paged(ctx, dKn, dVn, kv, dlen, cap)
            hb.hg_hydragen_attn_paged(ctx, dw.Q, dw.levels, kv, dlen, max_len, O, L, dw.scale)
        else:
            hb.hg_kv_append(ctx, dKn, dVn, dK, dV, doff, dlen, cap)
            hb.hg_hydragen_attn(ctx, dw.Q, dw.levels, dK, dV, doff, dlen, max_len, O, L, dw.scale)

    g = None
    lv = [(l.K, l.V, l.kv_off, l.seq_off) for l in w.levels]
    for k in range(steps):
        Kn, Vn = wl.new_rows(w, step=k)
        dKn.copy_(dev.bf16_tensor(Kn, "cuda:0"))
        dVn.copy_(dev.bf16_tensor(Vn, "cuda:0"))
        torch.cuda.synchronize()
        if k == 0:
            with torch.cuda.stream(s):   # first step eagerly (one-time kernel attribute set-up happens outside capture)
                step()
            s.synchronize()
            g = torch.cuda.CUDAGraph()
        elif k == 1:
            with torch.cuda.graph(g, stream=s):
                step()
            torch.cuda.synchronize()
            g.replay()                   # capture does not execute: this replay is step 1
        else:
            g.replay()
        torch.cuda.synchronize()
        if paged:
            hK, hV, hlen = oracle.kv_append_paged(hK, hV, pg.table, 16, hlen, cap, Kn, Vn)
            Ks, Vs, off = oracle.paged_to_packed(hK, hV, pg.table, 16, hlen)
        else:
            hK, hV, hlen = oracle.kv_append(hK, hV, hoff, hlen, cap, Kn, Vn)
            Ks, Vs, off = hK, hV, hoff
        assert np.array_equal(dlen.cpu().numpy(), hlen), f"lengths after step {k}"
        Oref, Lref = oracle.attention_arrays(w.Q, w.Hkv, lv, Ks, Vs, off, hlen, w.scale)
        check(to_np(O), to_np(L), Oref, Lref, f"decode step {k} paged={paged}")
    assert np.array_equal(hlen, w.lengths + steps)
    ctx.close()


def test_paged_error_paths_launch_nothing():
    say("paged errors")
    w = wl.scaled_down(2)
    dw = dev.to_device(w)
    pg = wl.make_paged(w, 16)
    kv = dev.paged_to_device(pg)
    ctx = dev.make_context(dw, parts=24)
    O = torch.full(dw.lead + (dw.D,), 7.0, dtype=torch.float32, device="cuda:0")
    L = torch.full(dw.lead, 7.0, dtype=torch.float32, device="cuda:0")
    lib = hb.lib()
    import ctypes

    def call(st, max_len=dw.max_len, c=ctx):
        return lib.hg_suffix_attn_paged(c.h, dw.Q.data_ptr(), ctypes.byref(st), dw.lengths.data_ptr(), max_len, dw.B, dw.Hq,
                                        dw.Hkv, dw.D, 0.0, O.data_ptr(), hb.HG_F32, L.data_ptr())
    st = kv.c_struct(); st.page_size = 24          # not a power of two
    assert call(st) == hb.HG_ERR_INVALID_ARG
    st = kv.c_struct(); st.page_size = 8           # below the smallest page
    assert call(st) == hb.HG_ERR_INVALID_ARG
    st = kv.c_struct(); st.table_stride = 1        # the table cannot address max_len rows
    assert call(st) == hb.HG_ERR_INVALID_ARG
    st = kv.c_struct(); st.page_table = None
    assert call(st) == hb.HG_ERR_INVALID_ARG
    st = kv.c_struct(); st.n_pages = 0
    assert call(st) == hb.HG_ERR_INVALID_ARG
    assert lib.hg_suffix_attn_paged(ctx.h, dw.Q.data_ptr(), None, dw.lengths.data_ptr(), dw.max_len, dw.B, dw.Hq, dw.Hkv, dw.D,
                                    0.0, O.data_ptr(), hb.HG_F32, L.data_ptr()) == hb.HG_ERR_INVALID_ARG
    # one partial result cannot cover more than 32 pages: max_len 4096 over 16-row pages needs 8
    # (a limit of the vector-ALU kernel, which such long suffixes get only on request)
    small = hb.Context(0, hb.hg_workspace_bytes(dw.B, dw.Hq, dw.D, 2))
    small.set_option(hb.HG_OPT_SUFFIX_KERNEL, 1)
    st = kv.c_struct(); st.table_stride = 256
    assert call(st, max_len=4096, c=small) == hb.HG_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(O.min()) == 7.0 and float(L.min()) == 7.0
    small.close()
    ctx.close()
