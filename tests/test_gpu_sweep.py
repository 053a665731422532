"""GPU parity on seeded random shapes: orders that exercise every kernel and the borders between
them, widths with and without padding, leading dimensions beyond the width, ragged row counts,
all three input formats, both bit widths."""
import sys

import numpy as np
import pytest

import parity
from paper_2504_13989_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

ORDERS = [128, 256, 384, 512, 640, 768, 896, 1024, 1152, 1280, 1408, 1536, 1544, 1792, 2048, 2304, 2560,
          3072, 3584, 4096, 4864, 5120, 6144, 6272, 7168, 8192]


def say(msg):
    print(f"[sweep] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _cases():
    rng = np.random.default_rng(20250419)
    out = []
    for i in range(72):
        n = int(ORDERS[i % len(ORDERS)] if i < len(ORDERS) else rng.choice(ORDERS))
        kind = rng.integers(0, 4)
        if kind == 0:
            d = n
        elif kind == 1:
            d = n - 8 * int(rng.integers(1, max(2, n // 64)))
        elif kind == 2:
            d = int(rng.integers(max(1, n // 2), n + 1))            # any width, also odd ones
        else:
            d = n - 8
        d = max(1, d)
        rows = int(rng.choice([1, 2, 3, 5, 17, 64, 130, 333, 1500, 2300]))
        if n >= 4096:
            rows = min(rows, 333)
        dtype = str(rng.choice(["bf16", "bf16", "f16", "f32"]))
        pad = int(rng.choice([0, 0, 8, 24, 1]))                        # leading dimension beyond d
        b = int(rng.choice([3, 4]))
        clip = float(np.float32(rng.uniform(0.5, 1.0)))
        out.append((i, n, d, rows, dtype, pad, b, clip))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: f"{c[0]}-n{c[1]}-d{c[2]}-r{c[3]}-{c[4]}-ld+{c[5]}-b{c[6]}")
def test_random_shapes(torch, case):
    i, n, d, rows, dtype, pad, b, clip = case
    rng = np.random.default_rng(1000 + i)
    ld = d + pad
    full = rng.standard_t(3.0, size=(rows, ld)).astype(np.float32)
    full[:, rng.choice(d, min(3, d), replace=False)] *= 30
    if rows > 3:
        full[2] *= 200.0                       # a massive token
        full[3, :d] = 0.0                      # an all-zero row
    if dtype == "bf16":
        full = wl.f32_to_bf16_bits(full)
    elif dtype == "f16":
        full = np.clip(full, -6e4, 6e4).astype(np.float16)
    x = np.ascontiguousarray(full[:, :d])
    h = binding.hadamard_build(n)
    xt = parity.to_device(full)[:, :d]
    say(f"case {i}: n={n} d={d} rows={rows} {dtype} ld={ld} b={b} clip={clip:.4f}")
    codes, scales = binding.rotate_quantize(h, xt, b, clip)
    torch.cuda.synchronize()
    st = parity.check_rotate_quantize(x, n, b, clip, codes.cpu().numpy(), scales.cpu().numpy(),
                                      f"case {i} n={n} d={d} rows={rows} {dtype} ld={ld} b={b} [{h.last_kernel}]")
    say(f"  ok kernel={h.last_kernel} {st}")
    h.close()


def _other_cases():
    rng = np.random.default_rng(4201)
    out = []
    for i in range(30):
        n = int(rng.choice(ORDERS))
        d = n if rng.integers(0, 2) else n - 8 * int(rng.integers(1, max(2, n // 64)))
        rows = int(rng.choice([1, 3, 9, 40, 130, 700]))
        if n >= 4096:
            rows = min(rows, 130)
        dtype = str(rng.choice(["bf16", "f16", "f32"]))
        b = int(rng.choice([3, 4]))
        out.append((i, n, d, rows, dtype, b))
    return out


@pytest.mark.parametrize("case", _other_cases(), ids=lambda c: f"{c[0]}-n{c[1]}-d{c[2]}-r{c[3]}-{c[4]}-b{c[5]}")
def test_random_shapes_other_entry_points(torch, case):
    # the same kind of shapes through the asymmetric variant, the error objective, the plain
    # rotation and the way back from codes
    import rotq_oracle as oracle
    i, n, d, rows, dtype, b = case
    rng = np.random.default_rng(7000 + i)
    xf = (rng.standard_t(4.0, size=(rows, d)) + 0.3).astype(np.float32)
    xf[:, rng.choice(d, 2, replace=False)] *= 25
    x = wl.f32_to_bf16_bits(xf) if dtype == "bf16" else xf.astype(np.float16) if dtype == "f16" else xf
    h = binding.hadamard_build(n)
    xt = parity.to_device(x)
    say(f"case {i}: n={n} d={d} rows={rows} {dtype} b={b}")
    clips = [float(np.float32(c)) for c in rng.uniform(0.5, 1.0, size=3)]
    mse = binding.quant_error(h, xt, b, clips)
    torch.cuda.synchronize()
    parity.check_quant_error(x, n, b, clips, mse.cpu().numpy(), what=f"case {i} quant_error [{h.last_kernel}]")
    y = binding.rotate(h, xt)
    torch.cuda.synchronize()
    parity.check_float_rows(y.cpu().numpy(), oracle.rotate(x, n), what=f"case {i} rotate")
    codes, scales = binding.rotate_quantize(h, xt, b, clips[0])
    xb = binding.dequantize_rotate(h, codes, scales, b, d_out=d)
    torch.cuda.synchronize()
    # the way back is checked against the oracle's inverse of the GPU's own codes (the codes themselves
    # are checked by the other sweep): unpack, dequantize, rotate back
    qg = oracle.unpack_codes(codes.cpu().numpy(), b, n)
    yhat = qg.astype(np.float64) * scales.cpu().numpy().astype(np.float64)[:, None]
    parity.check_float_rows(xb.cpu().numpy(), oracle.rotate_back(yhat, n, d), what=f"case {i} dequantize_rotate")
    if n % 128 == 0:
        ca, sa, ma = binding.rotate_quantize_asym(h, xt, b, clips[1])
        torch.cuda.synchronize()
        parity.check_rotate_quantize_asym(x, n, b, clips[1], ca.cpu().numpy(), sa.cpu().numpy(), ma.cpu().numpy(),
                                          f"case {i} asym n={n} {dtype} [{h.last_kernel}]")
        mse = binding.quant_error(h, xt, b, clips, asym=True)
        torch.cuda.synchronize()
        parity.check_quant_error(x, n, b, clips, mse.cpu().numpy(), what=f"case {i} quant_error asym", asym=True)
    h.close()
