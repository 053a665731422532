"""Comparison of the HIP path's outputs with the oracle's, under the stated parity rule.

  * packed codes are unpacked and compared element by element; a code may differ from the
    oracle's only where the oracle's pre-round value t lies within 1e-6 of a rounding
    boundary k + 1/2, and then by exactly one step; such differences (and the exempt set
    itself, on inputs large enough for the fraction to mean something) must stay within
    1e-5 of all elements;
  * scales agree within 1e-5 relative;
  * dequantized values agree within 1e-5 of the row's max |y| away from the exempt set.
"""
from __future__ import annotations

import numpy as np

import rotq_oracle as oracle

T_TOL = 1e-6
FRAC_TOL = 1e-5
REL_TOL = 1e-5


def to_device(x_np, device="cuda"):
    """numpy float32 or uint16 (bf16 bits) -> torch tensor on the device, same bits."""
    import torch
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x_np).to(device)


def check_rotate_quantize(x_np, n, b, clip, codes_gpu, scales_gpu, what="", rotated=None):
    """x_np: the rows given to the GPU; codes_gpu uint8 [rows, n*b/8]; scales_gpu float32 [rows].
    rotated: the oracle's rotated rows when the caller has formed them another way (orders whose
    dense matrix is too large to build in one piece)."""
    if rotated is None:
        q, delta, t, y = oracle.rotate_quantize(x_np, n, b, clip)
    else:
        y = rotated
        q, delta, t = oracle.quantize(y, b, clip)
    rows = q.shape[0]
    codes_gpu = np.asarray(codes_gpu).reshape(rows, n * b // 8)
    scales_gpu = np.asarray(scales_gpu, dtype=np.float64).reshape(rows)
    q_gpu = oracle.unpack_codes(codes_gpu, b, n)
    _, qmin, qmax = oracle.quant_params(b)
    assert q_gpu.min() >= qmin and q_gpu.max() <= qmax
    mism = q_gpu != q
    exempt = oracle.boundary_exempt(t, b, T_TOL)
    bad = mism & ~exempt
    nbad = int(bad.sum())
    if nbad:
        r, j = np.argwhere(bad)[0]
        raise AssertionError(
            f"{what}: {nbad} code mismatches away from rounding boundaries; first at row {r} col {j}: "
            f"gpu {q_gpu[r, j]} oracle {q[r, j]} t {t[r, j]!r}")
    if mism.any():
        assert np.all(np.abs(q_gpu.astype(np.int32) - q.astype(np.int32))[mism] == 1)
    total = q.size
    allowed = max(1, int(np.ceil(FRAC_TOL * total)))
    assert int(mism.sum()) <= allowed, f"{what}: {int(mism.sum())} boundary mismatches > {allowed}"
    if total >= 1_000_000:
        assert exempt.sum() <= FRAC_TOL * total, f"{what}: exempt fraction {exempt.mean():.3g}"
    # scales
    zero = delta == 0
    assert np.all(scales_gpu[zero] == 0)
    rel = np.abs(scales_gpu[~zero] - delta[~zero]) / delta[~zero]
    assert rel.size == 0 or rel.max() <= REL_TOL, f"{what}: scale rel err {rel.max():.3g}"
    # dequantized values
    amax = np.abs(y).max(axis=1)
    dq_gpu = q_gpu.astype(np.float64) * scales_gpu[:, None]
    dq = oracle.dequantize(q, delta)
    err = np.abs(dq_gpu - dq)
    err[exempt] = 0
    assert np.all(err <= REL_TOL * amax[:, None] + 0.0), f"{what}: dequantized values differ"
    # byte-exact packing where no code differs
    if not mism.any():
        assert np.array_equal(codes_gpu, oracle.pack_codes(q, b)), f"{what}: packed bytes differ"
    return {"elements": int(total), "mismatches": int(mism.sum()), "exempt": int(exempt.sum()),
            "max_scale_rel": float(rel.max()) if rel.size else 0.0}


def check_rotate_quantize_asym(x_np, n, b, clip, codes_gpu, scales_gpu, mins_gpu, what="", rotate=True):
    """Asymmetric group-128 variant: codes exact away from rounding boundaries, Delta within 1e-5
    relative, lo within 1e-5 of the group's range, dequantized values within 1e-5 of the range.
    rotate=False: the rotation-free quantizer (the rows themselves are quantized, n = their width)."""
    y = oracle.rotate(x_np, n) if rotate else oracle.as_f64(x_np)
    q, delta, lo, t = oracle.quantize_asym(y, b, clip)
    rows = q.shape[0]
    groups = n // oracle.GROUP
    lvl = (1 << b) - 1
    codes_gpu = np.asarray(codes_gpu).reshape(rows, n * b // 8)
    scales_gpu = np.asarray(scales_gpu, dtype=np.float64).reshape(rows, groups)
    mins_gpu = np.asarray(mins_gpu, dtype=np.float64).reshape(rows, groups)
    q_gpu = oracle.unpack_codes(codes_gpu, b, n, signed=False)
    assert q_gpu.max() <= lvl
    mism = q_gpu != q
    exempt = oracle.boundary_exempt_asym(t, b, T_TOL)
    bad = mism & ~exempt
    if bad.any():
        r, j = np.argwhere(bad)[0]
        raise AssertionError(
            f"{what}: {int(bad.sum())} code mismatches away from rounding boundaries; first at row {r} "
            f"col {j}: gpu {q_gpu[r, j]} oracle {q[r, j]} t {t[r, j]!r}")
    if mism.any():
        assert np.all(np.abs(q_gpu.astype(np.int32) - q.astype(np.int32))[mism] == 1)
    total = q.size
    allowed = max(1, int(np.ceil(FRAC_TOL * total)))
    assert int(mism.sum()) <= allowed, f"{what}: {int(mism.sum())} boundary mismatches > {allowed}"
    if total >= 1_000_000:
        assert exempt.sum() <= FRAC_TOL * total, f"{what}: exempt fraction {exempt.mean():.3g}"
    zero = delta == 0
    assert np.all(scales_gpu[zero] == 0)
    rel = np.abs(scales_gpu[~zero] - delta[~zero]) / delta[~zero]
    assert rel.size == 0 or rel.max() <= REL_TOL, f"{what}: scale rel err {rel.max():.3g}"
    span = np.maximum(delta * lvl, np.abs(lo))
    assert np.all(np.abs(mins_gpu - lo) <= REL_TOL * span), f"{what}: group minima differ"
    dq_gpu = oracle.dequantize_asym(q_gpu, scales_gpu, mins_gpu)
    dq = oracle.dequantize_asym(q, delta, lo)
    err = np.abs(dq_gpu - dq)
    err[exempt] = 0
    assert np.all(err <= REL_TOL * np.repeat(span, oracle.GROUP, axis=1)), f"{what}: dequantized values differ"
    if not mism.any():
        assert np.array_equal(codes_gpu, oracle.pack_codes(q, b)), f"{what}: packed bytes differ"
    return {"elements": int(total), "mismatches": int(mism.sum()), "exempt": int(exempt.sum())}


def check_quantize_plain(x_np, b, clip, codes_gpu, scales_gpu, what=""):
    """Rotation-free quantizer: same rule as check_rotate_quantize with y = x."""
    q, delta, t = oracle.quantize_plain(x_np, b, clip)
    rows, d = q.shape
    codes_gpu = np.asarray(codes_gpu).reshape(rows, d * b // 8)
    scales_gpu = np.asarray(scales_gpu, dtype=np.float64).reshape(rows)
    q_gpu = oracle.unpack_codes(codes_gpu, b, d)
    mism = q_gpu != q
    exempt = oracle.boundary_exempt(t, b, T_TOL)
    bad = mism & ~exempt
    assert not bad.any(), f"{what}: {int(bad.sum())} code mismatches away from rounding boundaries"
    assert int(mism.sum()) <= max(1, int(np.ceil(FRAC_TOL * q.size)))
    zero = delta == 0
    assert np.all(scales_gpu[zero] == 0)
    rel = np.abs(scales_gpu[~zero] - delta[~zero]) / delta[~zero]
    assert rel.size == 0 or rel.max() <= REL_TOL, f"{what}: scale rel err {rel.max():.3g}"
    if not mism.any():
        assert np.array_equal(codes_gpu, oracle.pack_codes(q, b)), f"{what}: packed bytes differ"
    return {"elements": int(q.size), "mismatches": int(mism.sum())}


def check_quant_error(x_np, n, b, clips, mse_gpu, rtol=REL_TOL, what="", asym=False):
    want = (oracle.quant_error_asym if asym else oracle.quant_error)(x_np, n, b, clips)
    got = np.asarray(mse_gpu, dtype=np.float64)
    rel = np.abs(got - want) / np.maximum(want, 1e-300)
    assert np.all(rel <= rtol), f"{what}: mse rel err {rel.max():.3g} (got {got}, want {want})"
    return float(rel.max())


def check_float_rows(got, want, rtol=REL_TOL, what="", bf16=False):
    """Floating-point rows against the oracle's fp64 rows: every element within rtol of the row's
    largest magnitude (fp32 results), plus one bf16 rounding step of the element for bf16 results."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    amax = np.abs(want).max(axis=1, keepdims=True)
    tol = rtol * amax + (np.abs(want) * 2.0 ** -8 if bf16 else 0.0)
    err = np.abs(got - want)
    assert np.all(err <= tol), f"{what}: max err {err.max():.3g} (row max {amax.max():.3g})"
    return float((err / np.maximum(amax, 1e-300)).max())
