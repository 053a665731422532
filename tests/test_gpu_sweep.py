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
