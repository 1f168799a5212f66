"""Thin ctypes binding of libhydragen.so: same names as include/hydragen.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the attention path runs in the HIP kernels of
the shared library.  There is no fallback: if the library is missing or fails to load, importing the symbols
works but the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

HG_OK, HG_ERR_INVALID_ARG, HG_ERR_UNSUPPORTED, HG_ERR_WORKSPACE, HG_ERR_HIP, HG_ERR_STATIC_LIMIT = 0, 1, 2, 3, 4, 5
HG_STATIC_SCRATCH_BYTES = 64 << 20
HG_F32, HG_BF16 = 0, 1
HG_MAX_LEVELS, HG_MAX_PARTS = 4, 64
HG_OPT_PREFIX_SPLITS, HG_OPT_SUFFIX_CHUNK, HG_OPT_OVERLAP, HG_OPT_NAIVE_CHUNK, HG_OPT_STAGE_TIMING, HG_OPT_PREFIX_KERNEL = 1, 2, 3, 4, 5, 6
HG_OPT_WIDE_SLOTS = 7
HG_OPT_NUM_QUERIES = 8
HG_KV_BF16, HG_KV_E4M3 = 0, 1
HG_OPT_SUFFIX_KERNEL = 9
HG_OPT_SUFFIX_ITEMS_PER_WAVE = 10
HG_OPT_SUFFIX_TILE_ROWS = 11
HG_OPT_FUSED_KERNEL = 12
HG_TIMING_RING, HG_MAX_STAGES = 128, HG_MAX_LEVELS + 2

# HYDRAGEN_LIB selects another build of the same library (e.g. one compiled with extra flags)
LIB_PATH = os.environ.get("HYDRAGEN_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhydragen.so")

# every symbol include/hydragen.h and include/hydragen_debug.h declare
EXPORTS = (
    "hg_create", "hg_destroy", "hg_set_stream", "hg_set_option", "hg_workspace_bytes", "hg_prefix_attn",
    "hg_prefix_attn_grouped", "hg_suffix_attn", "hg_merge", "hg_hydragen_attn", "hg_naive_attn", "hg_read_stage_timings",
    "hg_strerror", "hg_suffix_attn_paged", "hg_hydragen_attn_paged", "hg_kv_append", "hg_kv_append_paged",
    "hg_debug_wide_plan", "hg_debug_wide_ranges", "hg_debug_suffix_plan", "hg_suffix_attn_fp8", "hg_hydragen_attn_fp8", "hg_kv_append_fp8",
    "hg_hydragen_attn_static", "hg_debug_mfma_loop", "hg_debug_stream_read", "hg_debug_xcd_of_workgroups",
)


class HydragenError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


class hg_level(ctypes.Structure):
    _fields_ = [
        ("K", ctypes.c_void_p), ("V", ctypes.c_void_p), ("n_blocks", ctypes.c_int),
        ("kv_off", ctypes.c_void_p), ("seq_off", ctypes.c_void_p),
        ("max_rows", ctypes.c_int), ("max_seqs", ctypes.c_int),
    ]


class hg_paged_kv(ctypes.Structure):
    _fields_ = [
        ("K", ctypes.c_void_p), ("V", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int), ("table_stride", ctypes.c_int), ("n_pages", ctypes.c_int),
        ("kv_format", ctypes.c_int), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libhydragen.so (built by paper_2402_05099_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2402_05099_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, cf, cs = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.hg_create.argtypes = [ctypes.POINTER(vp), ci, vp, vp, cs]
        L.hg_create.restype = ci
        L.hg_destroy.argtypes = [vp]
        L.hg_destroy.restype = None
        L.hg_set_stream.argtypes = [vp, vp]
        L.hg_set_stream.restype = ci
        L.hg_set_option.argtypes = [vp, ci, ci]
        L.hg_set_option.restype = ci
        L.hg_workspace_bytes.argtypes = [ci, ci, ci, ci]
        L.hg_workspace_bytes.restype = cs
        L.hg_prefix_attn.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_prefix_attn.restype = ci
        L.hg_prefix_attn_grouped.argtypes = [vp, vp, ctypes.POINTER(hg_level), ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_prefix_attn_grouped.restype = ci
        L.hg_suffix_attn.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_suffix_attn.restype = ci
        L.hg_merge.argtypes = [vp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, ctypes.c_int64, ci, vp, ci, vp]
        L.hg_merge.restype = ci
        fused = [vp, vp, ci, ctypes.POINTER(hg_level), vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_hydragen_attn.argtypes = fused
        L.hg_hydragen_attn.restype = ci
        L.hg_naive_attn.argtypes = fused
        L.hg_naive_attn.restype = ci
        L.hg_hydragen_attn_static.argtypes = fused
        L.hg_hydragen_attn_static.restype = ci
        L.hg_suffix_attn_paged.argtypes = [vp, vp, ctypes.POINTER(hg_paged_kv), vp, ci, ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_suffix_attn_paged.restype = ci
        L.hg_hydragen_attn_paged.argtypes = [vp, vp, ci, ctypes.POINTER(hg_level), ctypes.POINTER(hg_paged_kv), vp, ci,
                                             ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_hydragen_attn_paged.restype = ci
        L.hg_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci]
        L.hg_kv_append.restype = ci
        L.hg_suffix_attn_fp8.argtypes = [vp, vp, vp, vp, cf, cf, vp, vp, ci, ci, ci, ci, ci, cf, vp, ci, vp]
        L.hg_suffix_attn_fp8.restype = ci
        L.hg_hydragen_attn_fp8.argtypes = [vp, vp, ci, ctypes.POINTER(hg_level), vp, vp, cf, cf, vp, vp, ci, ci, ci, ci, ci, cf,
                                           vp, ci, vp]
        L.hg_hydragen_attn_fp8.restype = ci
        L.hg_kv_append_fp8.argtypes = [vp, vp, vp, vp, vp, cf, cf, vp, vp, ci, ci, ci, ci]
        L.hg_kv_append_fp8.restype = ci
        L.hg_kv_append_paged.argtypes = [vp, vp, vp, ctypes.POINTER(hg_paged_kv), vp, ci, ci, ci, ci]
        L.hg_kv_append_paged.restype = ci
        L.hg_debug_wide_plan.argtypes = [ci] * 8 + [ctypes.POINTER(ci)]
        L.hg_debug_wide_plan.restype = ci
        L.hg_debug_wide_ranges.argtypes = [ci] * 8 + [ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.hg_debug_wide_ranges.restype = ci
        L.hg_debug_suffix_plan.argtypes = [ci] * 7 + [ctypes.POINTER(ci)]
        L.hg_debug_suffix_plan.restype = ci
        L.hg_debug_mfma_loop.argtypes = [vp, ci, ci, vp, vp]
        L.hg_debug_mfma_loop.restype = ci
        L.hg_debug_stream_read.argtypes = [vp, vp, cs, vp]
        L.hg_debug_stream_read.restype = ci
        L.hg_debug_xcd_of_workgroups.argtypes = [vp, ci, vp]
        L.hg_debug_xcd_of_workgroups.restype = ci
        L.hg_read_stage_timings.argtypes = [vp, ctypes.POINTER(cf), ci]
        L.hg_read_stage_timings.restype = ci
        L.hg_strerror.argtypes = [ci]
        L.hg_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().hg_strerror(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != HG_OK:
        raise HydragenError(code, what)


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HG_F32
    if t.dtype == torch.bfloat16:
        return HG_BF16
    raise TypeError(f"O must be float32 or bfloat16, got {t.dtype}")


def _want(t: torch.Tensor, dtype, shape=None, name="tensor"):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{name}: need a contiguous device tensor of {dtype}, got {t.dtype} on {t.device}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != {tuple(shape)}")


def hg_workspace_bytes(B: int, Hq: int, D: int, parts: int) -> int:
    return int(lib().hg_workspace_bytes(B, Hq, D, parts))


@dataclass
class Level:
    """One level of shared blocks on the device (see hg_level in include/hydragen.h)."""
    K: torch.Tensor                      # bf16 [rows, Hkv, D]
    V: torch.Tensor
    n_blocks: int = 1
    kv_off: Optional[torch.Tensor] = None   # int32 [n_blocks+1] on device, or None for one block covering all
    seq_off: Optional[torch.Tensor] = None
    max_rows: int = 0
    max_seqs: int = 0

    def c_struct(self) -> hg_level:
        return hg_level(self.K.data_ptr(), self.V.data_ptr(), self.n_blocks,
                        None if self.kv_off is None else self.kv_off.data_ptr(),
                        None if self.seq_off is None else self.seq_off.data_ptr(),
                        self.max_rows, self.max_seqs)


@dataclass
class PagedKV:
    """A paged suffix cache on the device (see hg_paged_kv in include/hydragen.h)."""
    K: torch.Tensor            # bf16 (or uint8 E4M3 codes with kv_format = HG_KV_E4M3) [n_pages * page_size, Hkv, D]
    V: torch.Tensor
    page_table: torch.Tensor   # int32 [B, table_stride] on device
    page_size: int
    kv_format: int = 0         # HG_KV_BF16 | HG_KV_E4M3
    k_scale: float = 1.0
    v_scale: float = 1.0

    @property
    def n_pages(self) -> int:
        return int(self.K.shape[0]) // self.page_size

    def c_struct(self) -> hg_paged_kv:
        return hg_paged_kv(self.K.data_ptr(), self.V.data_ptr(), self.page_table.data_ptr(), self.page_size,
                           int(self.page_table.shape[1]), self.n_pages, self.kv_format, self.k_scale, self.v_scale)


class Context:
    """Owns an hg_ctx and its workspace tensor (device memory comes from PyTorch)."""

    # {option: value} set on every new context right after hg_create (empty: the library's defaults)
    default_options: dict = {}

    def __init__(self, device: int = 0, workspace_bytes: int = 0, stream: Optional[torch.cuda.Stream] = None):
        L = lib()
        self.device = device
        self.workspace = None
        if workspace_bytes:
            self.workspace = torch.empty(workspace_bytes, dtype=torch.uint8, device=f"cuda:{device}")
        self._stream = stream
        h = ctypes.c_void_p()
        sp = ctypes.c_void_p(self._stream_handle(stream))
        _check(L.hg_create(ctypes.byref(h), device, sp, _p(self.workspace), workspace_bytes), "hg_create")
        self.h = h
        for option, value in self.default_options.items():
            self.set_option(option, value)

    def _stream_handle(self, stream) -> int:
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        return int(stream.cuda_stream)

    def set_stream(self, stream: Optional[torch.cuda.Stream]) -> None:
        self._stream = stream
        _check(lib().hg_set_stream(self.h, ctypes.c_void_p(self._stream_handle(stream))), "hg_set_stream")

    def set_option(self, option: int, value: int) -> None:
        _check(lib().hg_set_option(self.h, option, value), "hg_set_option")

    def read_stage_timings(self, n_calls: int):
        """[[ms per stage] per call], newest call first (see hg_read_stage_timings)."""
        buf = (ctypes.c_float * (n_calls * HG_MAX_STAGES))()
        n = lib().hg_read_stage_timings(self.h, buf, n_calls)
        if n < 0:
            raise HydragenError(-n, "hg_read_stage_timings")
        return [[buf[c * HG_MAX_STAGES + s] for s in range(HG_MAX_STAGES)] for c in range(n)]

    def close(self) -> None:
        if getattr(self, "h", None):
            lib().hg_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _qshape(ctx: Context, Q):
    """(B, Hq, D, output leading shape) of Q [B,Hq,D] or [B,nq,Hq,D]; tells the context how many queries a sequence has."""
    if Q.ndim == 4:
        B, nq, Hq, D = Q.shape
        lead = (B, nq, Hq)
    else:
        B, Hq, D = Q.shape
        nq = 1
        lead = (B, Hq)
    if getattr(ctx, "_nq", 1) != nq:
        ctx.set_option(HG_OPT_NUM_QUERIES, nq)
        ctx._nq = nq
    return B, Hq, D, lead


def hg_prefix_attn(ctx: Context, Q, Kp, Vp, O, LSE, scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    P, Hkv, _ = Kp.shape
    _want(Q, torch.bfloat16, name="Q"); _want(Kp, torch.bfloat16, (P, Hkv, D), "Kp"); _want(Vp, torch.bfloat16, (P, Hkv, D), "Vp")
    _want(O, O.dtype, lead + (D,), "O"); _want(LSE, torch.float32, lead, "LSE")
    _check(lib().hg_prefix_attn(ctx.h, _p(Q), _p(Kp), _p(Vp), B, Hq, Hkv, D, P, scale, _p(O), _dtype_code(O), _p(LSE)),
           "hg_prefix_attn")


def hg_prefix_attn_grouped(ctx: Context, Q, level: Level, O, LSE, scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    Hkv = level.K.shape[1]
    _want(Q, torch.bfloat16, name="Q"); _want(level.K, torch.bfloat16, name="K"); _want(level.V, torch.bfloat16, level.K.shape, "V")
    _want(O, O.dtype, lead + (D,), "O"); _want(LSE, torch.float32, lead, "LSE")
    st = level.c_struct()
    _check(lib().hg_prefix_attn_grouped(ctx.h, _p(Q), ctypes.byref(st), B, Hq, Hkv, D, scale, _p(O), _dtype_code(O), _p(LSE)),
           "hg_prefix_attn_grouped")


def hg_suffix_attn(ctx: Context, Q, Ks, Vs, offsets, lengths, max_len: int, O, LSE, scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    Hkv = Ks.shape[1]
    _want(Q, torch.bfloat16, name="Q"); _want(Ks, torch.bfloat16, name="Ks"); _want(Vs, torch.bfloat16, Ks.shape, "Vs")
    _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _want(O, O.dtype, lead + (D,), "O"); _want(LSE, torch.float32, lead, "LSE")
    _check(lib().hg_suffix_attn(ctx.h, _p(Q), _p(Ks), _p(Vs), _p(offsets), _p(lengths), max_len, B, Hq, Hkv, D, scale,
                                _p(O), _dtype_code(O), _p(LSE)), "hg_suffix_attn")


def hg_merge(ctx: Context, O_parts: Sequence[torch.Tensor], LSE_parts: Sequence[torch.Tensor], O_out, LSE_out=None) -> None:
    n = len(O_parts)
    D = O_parts[0].shape[-1]
    rows = O_parts[0].numel() // D
    for o, l in zip(O_parts, LSE_parts):
        _want(o, O_parts[0].dtype, O_parts[0].shape, "O_part"); _want(l, torch.float32, O_parts[0].shape[:-1], "LSE_part")
    _want(O_out, O_out.dtype, O_parts[0].shape, "O_out")
    if LSE_out is not None:
        _want(LSE_out, torch.float32, O_parts[0].shape[:-1], "LSE_out")
    op = (ctypes.c_void_p * n)(*[o.data_ptr() for o in O_parts])
    lp = (ctypes.c_void_p * n)(*[l.data_ptr() for l in LSE_parts])
    _check(lib().hg_merge(ctx.h, n, op, lp, _dtype_code(O_parts[0]), rows, D, _p(O_out), _dtype_code(O_out), _p(LSE_out)),
           "hg_merge")


def _fused(fn, name, ctx, Q, levels: List[Level], Ks, Vs, offsets, lengths, max_len, O_out, LSE_out, scale):
    B, Hq, D, lead = _qshape(ctx, Q)
    _want(Q, torch.bfloat16, name="Q")
    if levels:
        Hkv = levels[0].K.shape[1]
    elif Ks is not None:
        Hkv = Ks.shape[1]
    else:
        raise ValueError("no keys at all")
    for lv in levels:
        _want(lv.K, torch.bfloat16, name="level K"); _want(lv.V, torch.bfloat16, lv.K.shape, "level V")
    if Ks is not None:
        _want(Ks, torch.bfloat16, name="Ks"); _want(Vs, torch.bfloat16, Ks.shape, "Vs")
        _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _want(O_out, O_out.dtype, lead + (D,), "O_out")
    if LSE_out is not None:
        _want(LSE_out, torch.float32, lead, "LSE_out")
    n = len(levels)
    arr = (hg_level * max(n, 1))(*[lv.c_struct() for lv in levels])
    _check(fn(ctx.h, _p(Q), n, arr, _p(Ks), _p(Vs), _p(offsets), _p(lengths), max_len, B, Hq, Hkv, D, scale,
              _p(O_out), _dtype_code(O_out), _p(LSE_out)), name)


def hg_hydragen_attn(ctx: Context, Q, levels: List[Level], Ks, Vs, offsets, lengths, max_len: int, O_out, LSE_out=None,
                     scale: float = 0.0) -> None:
    _fused(lib().hg_hydragen_attn, "hg_hydragen_attn", ctx, Q, levels, Ks, Vs, offsets, lengths, max_len, O_out, LSE_out, scale)


def hg_hydragen_attn_static(ctx: Context, Q, levels: List[Level], Ks, Vs, offsets, lengths, max_len: int, O_out, LSE_out=None,
                            scale: float = 0.0) -> None:
    _fused(lib().hg_hydragen_attn_static, "hg_hydragen_attn_static", ctx, Q, levels, Ks, Vs, offsets, lengths, max_len, O_out,
           LSE_out, scale)


def hg_naive_attn(ctx: Context, Q, levels: List[Level], Ks, Vs, offsets, lengths, max_len: int, O_out, LSE_out=None,
                  scale: float = 0.0) -> None:
    _fused(lib().hg_naive_attn, "hg_naive_attn", ctx, Q, levels, Ks, Vs, offsets, lengths, max_len, O_out, LSE_out, scale)


def _want_paged(kv: PagedKV, B: int, D: int) -> int:
    dt = torch.uint8 if kv.kv_format == HG_KV_E4M3 else torch.bfloat16
    _want(kv.K, dt, name="paged K"); _want(kv.V, dt, kv.K.shape, "paged V")
    _want(kv.page_table, torch.int32, name="page_table")
    if kv.page_table.ndim != 2 or kv.page_table.shape[0] != B or kv.K.shape[2] != D or kv.K.shape[0] % kv.page_size:
        raise ValueError("paged cache: page_table must be [B, stride] and K [n_pages * page_size, Hkv, D]")
    return int(kv.K.shape[1])


def hg_suffix_attn_paged(ctx: Context, Q, kv: PagedKV, lengths, max_len: int, O, LSE, scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    Hkv = _want_paged(kv, B, D)
    _want(Q, torch.bfloat16, name="Q"); _want(lengths, torch.int32, (B,), "lengths")
    _want(O, O.dtype, lead + (D,), "O"); _want(LSE, torch.float32, lead, "LSE")
    st = kv.c_struct()
    _check(lib().hg_suffix_attn_paged(ctx.h, _p(Q), ctypes.byref(st), _p(lengths), max_len, B, Hq, Hkv, D, scale,
                                      _p(O), _dtype_code(O), _p(LSE)), "hg_suffix_attn_paged")


def hg_hydragen_attn_paged(ctx: Context, Q, levels: List[Level], kv: PagedKV, lengths, max_len: int, O_out, LSE_out=None,
                           scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    Hkv = _want_paged(kv, B, D)
    _want(Q, torch.bfloat16, name="Q"); _want(lengths, torch.int32, (B,), "lengths")
    for lv in levels:
        _want(lv.K, torch.bfloat16, name="level K"); _want(lv.V, torch.bfloat16, lv.K.shape, "level V")
    _want(O_out, O_out.dtype, lead + (D,), "O_out")
    if LSE_out is not None:
        _want(LSE_out, torch.float32, lead, "LSE_out")
    n = len(levels)
    arr = (hg_level * max(n, 1))(*[lv.c_struct() for lv in levels])
    st = kv.c_struct()
    _check(lib().hg_hydragen_attn_paged(ctx.h, _p(Q), n, arr, ctypes.byref(st), _p(lengths), max_len, B, Hq, Hkv, D, scale,
                                        _p(O_out), _dtype_code(O_out), _p(LSE_out)), "hg_hydragen_attn_paged")


def _new_rows(ctx: Context, Knew, Vnew):
    """(B, Hkv, D) of the new rows [B, Hkv, D] or [B, nq, Hkv, D]; tells the context how many rows a sequence adds."""
    _want(Knew, torch.bfloat16, name="Knew"); _want(Vnew, torch.bfloat16, Knew.shape, "Vnew")
    B, Hkv, D, _ = _qshape(ctx, Knew)
    return B, Hkv, D


def hg_kv_append(ctx: Context, Knew, Vnew, Ks, Vs, offsets, lengths, capacity: int) -> None:
    B, Hkv, D = _new_rows(ctx, Knew, Vnew)
    _want(Ks, torch.bfloat16, name="Ks"); _want(Vs, torch.bfloat16, Ks.shape, "Vs")
    if tuple(Ks.shape[1:]) != (Hkv, D):
        raise ValueError("Ks must be [T, Hkv, D]")
    _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _check(lib().hg_kv_append(ctx.h, _p(Knew), _p(Vnew), _p(Ks), _p(Vs), _p(offsets), _p(lengths), capacity, B, Hkv, D),
           "hg_kv_append")


def _want_fp8(Ks8, Vs8, Hkv=None, D=None):
    _want(Ks8, torch.uint8, name="Ks8"); _want(Vs8, torch.uint8, Ks8.shape, "Vs8")
    if Ks8.ndim != 3 or (Hkv is not None and tuple(Ks8.shape[1:]) != (Hkv, D)):
        raise ValueError("Ks8 must be uint8 [T, Hkv, D]")


def hg_suffix_attn_fp8(ctx: Context, Q, Ks8, Vs8, k_scale: float, v_scale: float, offsets, lengths, max_len: int, O, LSE,
                       scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    _want(Q, torch.bfloat16, name="Q")
    _want_fp8(Ks8, Vs8)
    Hkv = Ks8.shape[1]
    _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _want(O, O.dtype, lead + (D,), "O"); _want(LSE, torch.float32, lead, "LSE")
    _check(lib().hg_suffix_attn_fp8(ctx.h, _p(Q), _p(Ks8), _p(Vs8), k_scale, v_scale, _p(offsets), _p(lengths), max_len,
                                    B, Hq, Hkv, D, scale, _p(O), _dtype_code(O), _p(LSE)), "hg_suffix_attn_fp8")


def hg_hydragen_attn_fp8(ctx: Context, Q, levels: List[Level], Ks8, Vs8, k_scale: float, v_scale: float, offsets, lengths,
                         max_len: int, O_out, LSE_out=None, scale: float = 0.0) -> None:
    B, Hq, D, lead = _qshape(ctx, Q)
    _want(Q, torch.bfloat16, name="Q")
    _want_fp8(Ks8, Vs8)
    Hkv = Ks8.shape[1]
    for lv in levels:
        _want(lv.K, torch.bfloat16, name="level K"); _want(lv.V, torch.bfloat16, lv.K.shape, "level V")
    _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _want(O_out, O_out.dtype, lead + (D,), "O_out")
    if LSE_out is not None:
        _want(LSE_out, torch.float32, lead, "LSE_out")
    n = len(levels)
    arr = (hg_level * max(n, 1))(*[lv.c_struct() for lv in levels])
    _check(lib().hg_hydragen_attn_fp8(ctx.h, _p(Q), n, arr, _p(Ks8), _p(Vs8), k_scale, v_scale, _p(offsets), _p(lengths),
                                      max_len, B, Hq, Hkv, D, scale, _p(O_out), _dtype_code(O_out), _p(LSE_out)),
           "hg_hydragen_attn_fp8")


def hg_kv_append_fp8(ctx: Context, Knew, Vnew, Ks8, Vs8, k_scale: float, v_scale: float, offsets, lengths, capacity: int) -> None:
    B, Hkv, D = _new_rows(ctx, Knew, Vnew)
    _want_fp8(Ks8, Vs8, Hkv, D)
    _want(offsets, torch.int32, (B,), "offsets"); _want(lengths, torch.int32, (B,), "lengths")
    _check(lib().hg_kv_append_fp8(ctx.h, _p(Knew), _p(Vnew), _p(Ks8), _p(Vs8), k_scale, v_scale, _p(offsets), _p(lengths),
                                  capacity, B, Hkv, D), "hg_kv_append_fp8")


def hg_kv_append_paged(ctx: Context, Knew, Vnew, kv: PagedKV, lengths, capacity: int) -> None:
    B, Hkv, D = _new_rows(ctx, Knew, Vnew)
    if _want_paged(kv, B, D) != Hkv:
        raise ValueError("paged K must be [n_pages * page_size, Hkv, D]")
    _want(lengths, torch.int32, (B,), "lengths")
    st = kv.c_struct()
    _check(lib().hg_kv_append_paged(ctx.h, _p(Knew), _p(Vnew), ctypes.byref(st), _p(lengths), capacity, B, Hkv, D),
           "hg_kv_append_paged")


def hg_debug_wide_plan(n_blocks: int, max_rows: int, max_seqs: int, Hkv: int, rows_per_seq: int, max_parts: int, slots_per_xcd: int,
                       D: int = 128):
    """dict of the persistent shared-block kernel's work partition, or None if the level does not fit (host only)."""
    out = (ctypes.c_int * 9)()
    if not lib().hg_debug_wide_plan(n_blocks, max_rows, max_seqs, Hkv, rows_per_seq, max_parts, slots_per_xcd, D, out):
        return None
    plan = dict(zip(("n_c", "ncols", "rowgroups", "T", "slots", "tpx", "quota", "nparts", "mode"), list(out)))
    if plan["mode"] == 2:      # ranges from the planner's table
        starts, first = (ctypes.c_int * 257)(), (ctypes.c_int * 256)()
        n = lib().hg_debug_wide_ranges(n_blocks, max_rows, max_seqs, Hkv, rows_per_seq, max_parts, slots_per_xcd, D, starts, first)
        assert n == 8 * plan["tpx"]
        plan["starts"], plan["first_part"] = list(starts)[:n + 1], list(first)[:n]
    return plan


def hg_debug_suffix_plan(B: int, nq: int, Hq: int, Hkv: int, D: int, max_len: int, page_size: int = 0):
    """dict of the suffix kernel choice and chunking with default options, or None on invalid arguments (host only)."""
    out = (ctypes.c_int * 4)()
    if not lib().hg_debug_suffix_plan(B, nq, Hq, Hkv, D, max_len, page_size, out):
        return None
    return dict(zip(("chunk", "nchunks", "mfma", "gt"), list(out)))


def hg_debug_mfma_loop(ctx: Context, random_operands: bool, iters: int, clocks: torch.Tensor, sink: torch.Tensor) -> None:
    """Enqueue the register-only matrix-instruction loop (see include/hydragen_debug.h); clocks: int64[2] on the device."""
    _want(clocks, torch.int64, (2,), "clocks"); _want(sink, torch.float32, (1,), "sink")
    _check(lib().hg_debug_mfma_loop(ctx.h, int(bool(random_operands)), iters, _p(clocks), _p(sink)), "hg_debug_mfma_loop")


def hg_debug_stream_read(ctx: Context, src: torch.Tensor, sink: torch.Tensor) -> None:
    """Enqueue one streaming read of the whole of `src` (see include/hydragen_debug.h)."""
    _want(sink, torch.float32, (1,), "sink")
    if not src.is_cuda or not src.is_contiguous():
        raise TypeError("src: need a contiguous device tensor")
    _check(lib().hg_debug_stream_read(ctx.h, _p(src), src.numel() * src.element_size(), _p(sink)), "hg_debug_stream_read")


def hg_debug_xcd_of_workgroups(ctx: Context, out: torch.Tensor) -> None:
    """Enqueue out.numel() workgroups shaped like the persistent kernel's; workgroup i writes its XCD to out[i] (int32)."""
    _want(out, torch.int32, (out.numel(),), "out")
    _check(lib().hg_debug_xcd_of_workgroups(ctx.h, out.numel(), _p(out)), "hg_debug_xcd_of_workgroups")
