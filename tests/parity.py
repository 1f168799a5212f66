"""Comparison gates shared by the GPU parity tests (no attention arithmetic here).

Official gate (bf16 inputs, fp32 accumulation): max-abs error on O <= 1e-2, relative error on LSE <= 1e-3.
With N(0,1) inputs |O| itself is ~1e-2 at 16K keys, so that gate alone would pass garbage; the tests also
enforce a gate derived from the arithmetic of the kernels:
  - O:   max|dO| <= 2^-7 * max|O_ref|   and   ||dO||_2 / ||O_ref||_2 <= 1e-2
         (probabilities are rounded to bf16 before the second matrix product: <= 2^-9 relative per term, and
          a bf16 output adds 2^-9 relative; 2^-7 leaves a factor 2-4 for accumulation order)
  - LSE: |dLSE| <= 1e-4 * max(1, |LSE_ref|)   (fp32 max/sum/log; measured ~1e-6)
A bf16 OUTPUT cannot represent a value of magnitude >= 4 to within 1e-2 (half an ulp is 2^-8 relative, i.e.
0.0156 at 4): for bf16 outputs the official gate is therefore applied elementwise as
|dO| <= max(1e-2, 2^-7 |O_ref|); fp32 outputs take the plain 1e-2 gate.
"""
import numpy as np


def to_np(t):
    import torch
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy().astype(np.float64)


def check(O_gpu, L_gpu, O_ref, L_ref, what="", out_bf16=False):
    O_gpu = np.asarray(O_gpu, dtype=np.float64)
    O_ref = np.asarray(O_ref, dtype=np.float64)
    assert O_gpu.shape == O_ref.shape, (what, O_gpu.shape, O_ref.shape)
    assert np.all(np.isfinite(O_gpu)), f"{what}: non-finite O"
    dO = np.abs(O_gpu - O_ref)
    omax = float(np.abs(O_ref).max()) if O_ref.size else 0.0
    stats = {"max_abs_dO": float(dO.max()) if dO.size else 0.0, "max_abs_O": omax}
    if O_ref.size:
        nr = float(np.linalg.norm(O_ref))
        stats["rel_l2"] = float(np.linalg.norm(O_gpu - O_ref)) / nr if nr > 0 else float(np.linalg.norm(O_gpu))
        official = np.maximum(1e-2, 2.0 ** -7 * np.abs(O_ref)) if out_bf16 else 1e-2
        assert np.all(dO <= official), f"{what}: official O gate {stats}"
        assert stats["max_abs_dO"] <= 2.0 ** -7 * omax + 1e-30, f"{what}: tight O gate {stats}"
        assert stats["rel_l2"] <= 1e-2, f"{what}: rel-L2 gate {stats}"
    if L_gpu is not None:
        L_gpu = np.asarray(L_gpu, dtype=np.float64)
        L_ref = np.asarray(L_ref, dtype=np.float64)
        assert L_gpu.shape == L_ref.shape
        inf = np.isneginf(L_ref)
        assert np.array_equal(np.isneginf(L_gpu), inf), f"{what}: -inf LSE pattern differs"
        if (~inf).any():
            dL = np.abs(L_gpu[~inf] - L_ref[~inf])
            stats["max_abs_dLSE"] = float(dL.max())
            assert np.all(dL <= 1e-3 * np.abs(L_ref[~inf]) + 1e-6), f"{what}: official LSE gate {stats}"
            assert np.all(dL <= 1e-4 * np.maximum(1.0, np.abs(L_ref[~inf]))), f"{what}: tight LSE gate {stats}"
    return stats
