"""GPU parity of the 8-bit (E4M3) suffix cache: suffix attention and the fused call over such a cache against the fp64
oracle on the decoded values, and the quantising cache update against the oracle's codes, bit for bit."""
import sys

import numpy as np
import pytest
import torch

import oracle
from oracle import fp8
from paper_2402_05099_amd import binding as hb
from paper_2402_05099_amd import device as dev
from paper_2402_05099_amd import workloads as wl
from parity import check, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def u8(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def i32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


def finite_codes(n_rows: int) -> np.ndarray:
    """[n_rows, 2, 128]: every row holds all 256 codes in order (heads 0 and 1), the two NaN codes replaced by 0x3a."""
    row = np.arange(256, dtype=np.uint8)
    row[(row & 0x7F) == 0x7F] = 0x3A
    return np.broadcast_to(row.reshape(1, 2, 128), (n_rows, 2, 128)).copy()


KERNELS = pytest.mark.parametrize("kernel", [1, 2, 3], ids=["valu", "mfma", "mfma_tile32"])


def choose_kernel(ctx, kernel):
    """1: vector-ALU; 2: matrix cores (16-row tiles where a KV head serves at most 16 rows); 3: matrix cores, 32-row tiles."""
    ctx.set_option(hb.HG_OPT_SUFFIX_KERNEL, min(kernel, 2))
    if kernel == 3:
        ctx.set_option(hb.HG_OPT_SUFFIX_TILE_ROWS, 32)


@KERNELS
def test_every_value_code_is_decoded_exactly(kernel):
    """One key per sequence, so the softmax weight is exactly 1 and O = decode(V code) * v_scale, one fp32 product."""
    say(f"fp8 decode of every V code, kernel {kernel}")
    B, H, D = 3, 2, 128
    Vs8 = finite_codes(B)
    Ks8 = np.full((B, H, D), 0x38, dtype=np.uint8)
    Q = dev.bf16_tensor(wl.normal_bf16(1, 0, (B, H, D)), "cuda:0")
    offsets, lengths = i32(np.arange(B)), i32(np.ones(B))
    ctx = hb.Context(0, hb.hg_workspace_bytes(B, H, D, 4))
    choose_kernel(ctx, kernel)
    O = torch.full((B, H, D), float("nan"), dtype=torch.float32, device="cuda:0")
    L = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda:0")
    v_scale = 0.37
    hb.hg_suffix_attn_fp8(ctx, Q, u8(Ks8), u8(Vs8), 0.5, v_scale, offsets, lengths, 1, O, L)
    torch.cuda.synchronize()
    want = fp8.e4m3_decode(Vs8).astype(np.float32) * np.float32(v_scale)
    if kernel == 1:
        assert np.array_equal(O.cpu().numpy(), want)
    else:
        # the matrix-core kernel takes exp2(s c - round(m c)): the single weight is 1 up to a few ulps, and cancels
        # only up to that in O = p v / p.  Neighbouring codes differ by 6 % or more.
        assert np.allclose(O.cpu().numpy(), want, rtol=1e-5, atol=0.0)
    ctx.close()


@KERNELS
def test_every_key_code_is_decoded_exactly(kernel):
    """One key per sequence and a one-hot query: LSE is the single score q_d * decode(K code) * k_scale * scale."""
    say(f"fp8 decode of every K code, kernel {kernel}")
    B, H, D = 128, 2, 128
    Ks8 = finite_codes(B)
    Vs8 = np.full((B, H, D), 0x38, dtype=np.uint8)
    q = np.zeros((B, H, D), dtype=np.float32)
    for b in range(B):
        q[b, :, b] = 2.0
    Q = dev.bf16_tensor(wl.f32_to_bf16_bits(q), "cuda:0")
    offsets, lengths = i32(np.arange(B)), i32(np.ones(B))
    ctx = hb.Context(0, hb.hg_workspace_bytes(B, H, D, 4))
    choose_kernel(ctx, kernel)
    O = torch.empty((B, H, D), dtype=torch.float32, device="cuda:0")
    L = torch.empty((B, H), dtype=torch.float32, device="cuda:0")
    k_scale, scale = 0.75, 0.25
    hb.hg_suffix_attn_fp8(ctx, Q, u8(Ks8), u8(Vs8), k_scale, 1.0, offsets, lengths, 1, O, L, scale)
    torch.cuda.synchronize()
    vals = fp8.e4m3_decode(Ks8[0])                                  # [2, 128]
    want = 2.0 * vals.T * k_scale * scale                           # [B = d, H]
    got = L.cpu().numpy().astype(np.float64)
    assert np.allclose(got, want, rtol=2e-6, atol=1e-9), float(np.abs(got - want).max())
    assert np.allclose(O.cpu().numpy(), np.ones((B, H, D), dtype=np.float32), rtol=1e-5 if kernel >= 2 else 0.0, atol=0.0)
    ctx.close()


CASES = {
    "tiny_d64": dict(idx=1),
    "mha": dict(idx=2),
    "ragged": dict(idx=3),
    "gqa8": dict(idx=4),
    "tree": dict(idx=5),
    "one_kv_head": dict(idx=6),
    "ragged_nq3": dict(idx=3, nq=3),
}


@KERNELS
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("chunk", [0, 64], ids=["auto", "chunk64"])
@pytest.mark.parametrize("case", sorted(CASES))
def test_suffix_attn_fp8(case, chunk, out_dtype, kernel):
    say(f"fp8 suffix {case} chunk={chunk} {out_dtype} kernel={kernel}")
    kw = dict(CASES[case])
    w = wl.scaled_down(kw.pop("idx"), **kw)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w, reserve=5)                  # unowned rows hold a NaN code
    ctx = dev.make_context(dw, parts=24)
    choose_kernel(ctx, kernel)   # an 8-bit cache at D = 64 stays on the vector ALU
    if chunk:
        ctx.set_option(hb.HG_OPT_SUFFIX_CHUNK, chunk)
    Oref, Lref = fp8.suffix_attention_fp8(w.Q, w.Hkv, f8.Ks8, f8.Vs8, f8.k_scale, f8.v_scale, f8.offsets, w.lengths, w.scale)
    O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=out_dtype, device="cuda:0")
    L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_fp8(ctx, dw.Q, u8(f8.Ks8), u8(f8.Vs8), f8.k_scale, f8.v_scale, i32(f8.offsets), dw.lengths, dw.max_len,
                          O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"fp8 suffix {case}", out_bf16=out_dtype == torch.bfloat16)
    ctx.close()


def test_suffix_attn_fp8_saturated_cache_and_small_workspace():
    """Scales so small that the largest values saturate at 448, and a workspace with room for two partial results."""
    say("fp8 suffix saturated")
    w = wl.scaled_down(3)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w, headroom=0.5, junk_code=None)
    assert (f8.Ks8 & 0x7F).max() == 0x7E and ((f8.Ks8 & 0x7F) == 0x7E).sum() > 10
    ctx = dev.make_context(dw, parts=2)
    Oref, Lref = fp8.suffix_attention_fp8(w.Q, w.Hkv, f8.Ks8, f8.Vs8, f8.k_scale, f8.v_scale, f8.offsets, w.lengths, w.scale)
    O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_fp8(ctx, dw.Q, u8(f8.Ks8), u8(f8.Vs8), f8.k_scale, f8.v_scale, i32(f8.offsets), dw.lengths, dw.max_len,
                          O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, "fp8 suffix saturated")
    ctx.close()


@pytest.mark.parametrize("case", ["mha", "ragged", "gqa8", "tree", "ragged_nq3"])
def test_hydragen_attn_fp8(case):
    """Fused call: bf16 shared levels, 8-bit suffix.  Oracle: the merge (Eq. 5) of the exact attention over the levels
    and the exact attention over the decoded suffix."""
    say(f"fp8 fused {case}")
    kw = dict(CASES[case])
    w = wl.scaled_down(kw.pop("idx"), **kw)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w, reserve=3)
    ctx = dev.make_context(dw, parts=24)
    Op, Lp = oracle.attention(w, suffix=False)
    Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, f8.Ks8, f8.Vs8, f8.k_scale, f8.v_scale, f8.offsets, w.lengths, w.scale)
    Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
    O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, u8(f8.Ks8), u8(f8.Vs8), f8.k_scale, f8.v_scale, i32(f8.offsets), dw.lengths,
                            dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Oref, Lref, f"fp8 fused {case}", out_bf16=True)
    ctx.close()


def special_rows(shape, scale: float, seed: int) -> np.ndarray:
    """bf16 bit patterns: N(0, 1) * 40 * scale values with, sprinkled in, every tie between neighbouring codes (times the
    scale, which is a power of two so that the quotient is the tie again), values beyond the largest code, values that
    round to zero and to the smallest subnormal, both zeros and a NaN."""
    rng = np.random.default_rng(seed)
    x = (rng.normal(0, 40.0, shape) * scale).astype(np.float32)
    grid = fp8.e4m3_decode(np.arange(127, dtype=np.uint8))
    ties = (grid[:-1] + grid[1:]) / 2
    extra = np.concatenate([ties, -ties, [449.0, 464.0, 480.0, 1e6, -1e6, 2.0 ** -10, 2.0 ** -11, 1.5 * 2.0 ** -10,
                                          0.0, -0.0, np.nan, 448.0, -448.0, 2.0 ** -9]]) * scale
    flat = x.reshape(-1)
    pos = rng.choice(flat.shape[0], size=extra.shape[0], replace=False)
    flat[pos] = extra.astype(np.float32)
    bits = wl.f32_to_bf16_bits(flat.reshape(shape))
    return bits


@pytest.mark.parametrize("nq", [1, 3])
def test_kv_append_fp8_codes_bit_for_bit(nq):
    say(f"fp8 append nq={nq}")
    w = wl.scaled_down(3, nq=nq)
    f8 = wl.make_fp8(w, reserve=4, junk_code=None)
    cap = f8.capacity
    k_scale, v_scale = 0.125, 2.0            # powers of two: ties stay ties, and every tie is a bf16 value
    lengths = w.lengths.copy()
    lengths[0] = cap                          # full: nothing fits
    lengths[1] = cap - 1                      # room for one row only
    shape = (w.B, w.Hkv, w.D) if nq == 1 else (w.B, nq, w.Hkv, w.D)
    Knew, Vnew = special_rows(shape, k_scale, 21), special_rows(shape, v_scale, 22)
    Kd, Vd, Ld = u8(f8.Ks8), u8(f8.Vs8), i32(lengths)
    ctx = hb.Context(0, hb.hg_workspace_bytes(w.B * nq, w.Hq, w.D, 4))
    ctx.set_option(hb.HG_OPT_NUM_QUERIES, nq)
    hb.hg_kv_append_fp8(ctx, dev.bf16_tensor(Knew, "cuda:0"), dev.bf16_tensor(Vnew, "cuda:0"), Kd, Vd, k_scale, v_scale,
                        i32(f8.offsets), Ld, cap)
    torch.cuda.synchronize()
    Kref, Vref, Lref = fp8.kv_append_fp8(f8.Ks8, f8.Vs8, f8.offsets, lengths, cap, wl.bf16_bits_to_f32(Knew),
                                         wl.bf16_bits_to_f32(Vnew), k_scale, v_scale)
    assert np.array_equal(Ld.cpu().numpy(), Lref)
    for got, ref in ((Kd.cpu().numpy(), Kref), (Vd.cpu().numpy(), Vref)):
        nan = (ref & 0x7F) == 0x7F
        assert nan.sum() >= 1
        assert np.array_equal(got[~nan], ref[~nan])
        assert ((got[nan] & 0x7F) == 0x7F).all()
    ctx.close()


def test_decode_steps_on_an_8bit_cache():
    """Append, then attend, three times: the cache the device maintains gives the oracle's attention over the oracle's cache."""
    say("fp8 decode steps")
    w = wl.scaled_down(5)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w, reserve=3, junk_code=None)
    cap = f8.capacity
    Kd, Vd, Ld, offs = u8(f8.Ks8), u8(f8.Vs8), i32(w.lengths), i32(f8.offsets)
    Kh, Vh, Lh = f8.Ks8, f8.Vs8, w.lengths.copy()
    ctx = dev.make_context(dw, parts=24)
    Op, Lp = oracle.attention(w, suffix=False)
    for step in range(3):
        Knew, Vnew = wl.new_rows(w, step)
        hb.hg_kv_append_fp8(ctx, dev.bf16_tensor(Knew, "cuda:0"), dev.bf16_tensor(Vnew, "cuda:0"), Kd, Vd, f8.k_scale,
                            f8.v_scale, offs, Ld, cap)
        O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
        L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
        hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, Kd, Vd, f8.k_scale, f8.v_scale, offs, Ld, cap, O, L, dw.scale)
        torch.cuda.synchronize()
        Kh, Vh, Lh = fp8.kv_append_fp8(Kh, Vh, f8.offsets, Lh, cap, wl.bf16_bits_to_f32(Knew), wl.bf16_bits_to_f32(Vnew),
                                       f8.k_scale, f8.v_scale)
        assert np.array_equal(Ld.cpu().numpy(), Lh)
        assert np.array_equal(Kd.cpu().numpy(), Kh) and np.array_equal(Vd.cpu().numpy(), Vh)
        Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, Kh, Vh, f8.k_scale, f8.v_scale, f8.offsets, Lh, w.scale)
        Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
        check(to_np(O), to_np(L), Oref, Lref, f"fp8 decode step {step}")
    ctx.close()


def test_fp8_error_paths():
    say("fp8 errors")
    w = wl.scaled_down(1)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w)
    ctx = dev.make_context(dw, parts=4)
    O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
    K8, V8, offs = u8(f8.Ks8), u8(f8.Vs8), i32(f8.offsets)
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("nan"), 1.0), (1.0, float("inf"))):
        with pytest.raises(hb.HydragenError) as e:
            hb.hg_suffix_attn_fp8(ctx, dw.Q, K8, V8, ks, vs, offs, dw.lengths, dw.max_len, O, L, dw.scale)
        assert e.value.code == hb.HG_ERR_INVALID_ARG
        with pytest.raises(hb.HydragenError):
            hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, K8, V8, ks, vs, offs, dw.lengths, dw.max_len, O, L, dw.scale)
        with pytest.raises(hb.HydragenError):
            Knew, Vnew = wl.new_rows(w, 0)
            hb.hg_kv_append_fp8(ctx, dev.bf16_tensor(Knew, "cuda:0"), dev.bf16_tensor(Vnew, "cuda:0"), K8, V8, ks, vs, offs,
                                dw.lengths.clone(), f8.capacity)
    with pytest.raises(TypeError):
        hb.hg_suffix_attn_fp8(ctx, dw.Q, dw.Ks, dw.Vs, 1.0, 1.0, offs, dw.lengths, dw.max_len, O, L, dw.scale)   # bf16 cache
    ctx.close()


def test_fp8_full_size_config3():
    """The launch configuration `bench.py --fp8-kv` times (config 3, default options, bf16 output, 24 parts): sampled
    sequences against the oracle, and properties that hold for every row."""
    say("fp8 full config 3")
    w = wl.config(3)
    dw = dev.to_device(w)
    f8 = wl.make_fp8(w, junk_code=None)
    K8, V8, offs = u8(f8.Ks8), u8(f8.Vs8), i32(f8.offsets)
    ctx = dev.make_context(dw, parts=24)
    seqs = np.array(sorted({0, w.B - 1, w.B // 2, 333, int(np.argmin(w.lengths)), int(np.argmax(w.lengths))}), dtype=np.int32)
    Op, Lp = oracle.attention(w, suffix=False, seqs=seqs)
    Os, Ls = fp8.suffix_attention_fp8(w.Q[seqs], w.Hkv, f8.Ks8, f8.Vs8, f8.k_scale, f8.v_scale, f8.offsets[seqs],
                                      w.lengths[seqs], w.scale)
    Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
    O = torch.empty((dw.B, dw.Hq, dw.D), dtype=torch.bfloat16, device="cuda:0")
    L = torch.empty((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")
    hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, K8, V8, f8.k_scale, f8.v_scale, offs, dw.lengths, dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    idx = torch.from_numpy(seqs.astype(np.int64)).cuda()
    st = check(to_np(O[idx]), to_np(L[idx]), Oref, Lref, "fp8 full config 3", out_bf16=True)
    say(f"   {st}")
    assert bool(torch.isfinite(O.float()).all()) and bool(torch.isfinite(L).all())
    # suffix part alone on every row: sampled rows against the oracle, and the full LSE dominates it everywhere
    O2 = torch.empty((dw.B, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    L2 = torch.empty((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_fp8(ctx, dw.Q, K8, V8, f8.k_scale, f8.v_scale, offs, dw.lengths, dw.max_len, O2, L2, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O2[idx]), to_np(L2[idx]), Os, Ls, "fp8 full config 3 suffix")
    assert bool((L >= L2 - 1e-4).all())
    # quantisation error against the bf16 cache stays at the format's level (3 mantissa bits: <= 2^-4 relative per
    # element, averaged down by the softmax-weighted sum): a sanity bound, not a parity claim
    Ob, _ = dev.hydragen(ctx, dw, torch.bfloat16)
    torch.cuda.synchronize()
    rel = float((Ob.float() - O.float()).norm() / Ob.float().norm())
    say(f"   relative L2 difference to the bf16 cache: {rel:.4f}")
    assert rel < 0.05
    ctx.close()


def paged_fp8_to_device(pg, k_scale, v_scale) -> hb.PagedKV:
    return hb.PagedKV(K=u8(pg.K), V=u8(pg.V), page_table=i32(pg.table), page_size=pg.page_size, kv_format=hb.HG_KV_E4M3,
                      k_scale=k_scale, v_scale=v_scale)


@KERNELS
@pytest.mark.parametrize("page_size", [16, 128])
@pytest.mark.parametrize("case", ["mha", "ragged", "gqa8", "tree", "ragged_nq3"])
def test_paged_fp8_suffix_and_fused(case, page_size, kernel):
    """The 8-bit cache through a page table: the oracle gathers the rows the table designates (byte work), then takes the
    exact attention of the decoded codes; unowned pool rows hold a NaN code."""
    say(f"fp8 paged {case} page_size={page_size} kernel={kernel}")
    kw = dict(CASES[case])
    w = wl.scaled_down(kw.pop("idx"), **kw)
    dw = dev.to_device(w)
    pg, ks, vs = wl.make_paged_fp8(w, page_size)
    kv = paged_fp8_to_device(pg, ks, vs)
    K8, V8, offs = oracle.paged_to_packed(pg.K, pg.V, pg.table, pg.page_size, w.lengths)
    Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, K8, V8, ks, vs, offs, w.lengths, w.scale)
    ctx = dev.make_context(dw, parts=24)
    choose_kernel(ctx, kernel)
    O = torch.full(dw.lead + (dw.D,), float("nan"), dtype=torch.float32, device="cuda:0")
    L = torch.full(dw.lead, float("nan"), dtype=torch.float32, device="cuda:0")
    hb.hg_suffix_attn_paged(ctx, dw.Q, kv, dw.lengths, dw.max_len, O, L, dw.scale)
    torch.cuda.synchronize()
    check(to_np(O), to_np(L), Os, Ls, f"fp8 paged suffix {case}")
    # same codes in packed rows: the vector-ALU kernel walks them in the same order, identical bits (the matrix-core
    # kernel aligns its stages to logical rows when paged and to the range's end when packed: parity only)
    f8 = wl.make_fp8(w, junk_code=None)
    O2, L2 = torch.empty_like(O), torch.empty_like(L)
    hb.hg_suffix_attn_fp8(ctx, dw.Q, u8(f8.Ks8), u8(f8.Vs8), ks, vs, i32(f8.offsets), dw.lengths, dw.max_len, O2, L2, dw.scale)
    torch.cuda.synchronize()
    if kernel == 1:
        assert torch.equal(O, O2) and torch.equal(L, L2)
    else:
        check(to_np(O2), to_np(L2), Os, Ls, f"fp8 packed suffix {case}")
    Op, Lp = oracle.attention(w, suffix=False)
    Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
    Of, Lf = dev.hydragen_paged(ctx, dw, kv, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check(to_np(Of), to_np(Lf), Oref, Lref, f"fp8 paged fused {case}")
    ctx.close()


def test_paged_fp8_append_then_attend():
    say("fp8 paged append")
    w = wl.scaled_down(3, nq=2)
    dw = dev.to_device(w)
    pg, ks, vs = wl.make_paged_fp8(w, 32, reserve=4)
    kv = paged_fp8_to_device(pg, ks, vs)
    Ld = i32(w.lengths)
    Kh, Vh, Lh = pg.K, pg.V, w.lengths.copy()
    ctx = dev.make_context(dw, parts=24)
    for step in range(2):
        Knew, Vnew = wl.new_rows(w, step)
        hb.hg_kv_append_paged(ctx, dev.bf16_tensor(Knew, "cuda:0"), dev.bf16_tensor(Vnew, "cuda:0"), kv, Ld, pg.capacity)
        torch.cuda.synchronize()
        Kh, Vh, Lh = oracle.kv_append_paged(Kh, Vh, pg.table, pg.page_size, Lh, pg.capacity,
                                            fp8.quantize(wl.bf16_bits_to_f32(Knew), ks), fp8.quantize(wl.bf16_bits_to_f32(Vnew), vs))
        assert np.array_equal(Ld.cpu().numpy(), Lh)
        assert np.array_equal(kv.K.cpu().numpy(), Kh) and np.array_equal(kv.V.cpu().numpy(), Vh)
        K8, V8, offs = oracle.paged_to_packed(Kh, Vh, pg.table, pg.page_size, Lh)
        Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, K8, V8, ks, vs, offs, Lh, w.scale)
        O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
        L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
        hb.hg_suffix_attn_paged(ctx, dw.Q, kv, Ld, pg.capacity, O, L, dw.scale)
        torch.cuda.synchronize()
        check(to_np(O), to_np(L), Os, Ls, f"fp8 paged append step {step}")
    ctx.close()


def test_paged_fp8_error_paths():
    say("fp8 paged errors")
    w = wl.scaled_down(1)
    dw = dev.to_device(w)
    pg, ks, vs = wl.make_paged_fp8(w, 16)
    ctx = dev.make_context(dw, parts=4)
    O = torch.empty(dw.lead + (dw.D,), dtype=torch.float32, device="cuda:0")
    L = torch.empty(dw.lead, dtype=torch.float32, device="cuda:0")
    for bad in (dict(k_scale=0.0), dict(v_scale=float("nan"))):
        kv = paged_fp8_to_device(pg, ks, vs)
        for k, v in bad.items():
            setattr(kv, k, v)
        with pytest.raises(hb.HydragenError) as e:
            hb.hg_suffix_attn_paged(ctx, dw.Q, kv, dw.lengths, dw.max_len, O, L, dw.scale)
        assert e.value.code == hb.HG_ERR_INVALID_ARG
    # an unknown format code, straight through the C ABI (the binding would object to the tensor type first)
    import ctypes
    kv = paged_fp8_to_device(pg, ks, vs)
    st = kv.c_struct()
    st.kv_format = 7
    rc = hb.lib().hg_suffix_attn_paged(ctx.h, dw.Q.data_ptr(), ctypes.byref(st), dw.lengths.data_ptr(), dw.max_len, dw.B, dw.Hq,
                                       dw.Hkv, dw.D, dw.scale, O.data_ptr(), hb.HG_F32, L.data_ptr())
    assert rc == hb.HG_ERR_INVALID_ARG
    ctx.close()


@pytest.mark.parametrize("idx", [5, 4], ids=["tree_mha", "gqa"])
def test_fp8_decode_steps_in_a_graph(idx):
    """Quantising cache update + fused attention over the 8-bit cache, captured once and replayed: every step matches the
    oracle's codes bit for bit and the oracle's attention over them."""
    say(f"fp8 decode steps in a graph idx={idx}")
    steps = 4
    w = wl.scaled_down(idx)
    dw = dev.to_device(w)
    s = torch.cuda.Stream()
    ctx = hb.Context(0, hb.hg_workspace_bytes(dw.B, dw.Hq, dw.D, 24), stream=s)
    f8 = wl.make_fp8(w, reserve=steps, junk_code=None)
    cap = f8.capacity
    Kd, Vd, offs = u8(f8.Ks8), u8(f8.Vs8), i32(f8.offsets)
    Kh, Vh, Lh = f8.Ks8, f8.Vs8, w.lengths.copy()
    dlen = i32(w.lengths)
    dKn = torch.zeros((w.B, w.Hkv, w.D), dtype=torch.bfloat16, device="cuda:0")
    dVn = torch.zeros_like(dKn)
    O = torch.zeros((dw.B, dw.Hq, dw.D), dtype=torch.float32, device="cuda:0")
    L = torch.zeros((dw.B, dw.Hq), dtype=torch.float32, device="cuda:0")

    def step():
        hb.hg_kv_append_fp8(ctx, dKn, dVn, Kd, Vd, f8.k_scale, f8.v_scale, offs, dlen, cap)
        hb.hg_hydragen_attn_fp8(ctx, dw.Q, dw.levels, Kd, Vd, f8.k_scale, f8.v_scale, offs, dlen, cap, O, L, dw.scale)

    Op, Lp = oracle.attention(w, suffix=False)
    g = None
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
        Kh, Vh, Lh = fp8.kv_append_fp8(Kh, Vh, f8.offsets, Lh, cap, wl.bf16_bits_to_f32(Kn), wl.bf16_bits_to_f32(Vn),
                                       f8.k_scale, f8.v_scale)
        assert np.array_equal(dlen.cpu().numpy(), Lh), f"lengths after step {k}"
        assert np.array_equal(Kd.cpu().numpy(), Kh) and np.array_equal(Vd.cpu().numpy(), Vh), f"codes after step {k}"
        Os, Ls = fp8.suffix_attention_fp8(w.Q, w.Hkv, Kh, Vh, f8.k_scale, f8.v_scale, f8.offsets, Lh, w.scale)
        Oref, Lref = oracle.merge([Op, Os], [Lp, Ls])
        check(to_np(O), to_np(L), Oref, Lref, f"fp8 graph decode step {k}")
    assert np.array_equal(Lh, w.lengths + steps)
    ctx.close()
