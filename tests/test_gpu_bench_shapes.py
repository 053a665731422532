"""The launches bench.py times beyond rotate_quantize, at their full sizes and in the same launch
configuration (inputs tiled from a block of generated rows, as bench.py does): packed codes back to rows,
rotation alone on a Paley-block order, the rotated-domain dequantizer, the rotation-free quantizers on the
value cache and the whole-dimension Paley block.  The oracle cannot take millions of rows, so rows sampled
from the start, the middle and the ragged end of each launch are compared one by one."""
from __future__ import annotations

import sys

import numpy as np
import pytest

import parity
import rotq_oracle as oracle
from paper_2504_13989_amd import binding
from paper_2504_13989_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.skip("no GPU")
    return t


def tiled(torch, name, base_rows, rows):
    """bench.py's input: `base_rows` generated rows repeated to `rows` (device tensor and the host rows)."""
    w = wl.WORKLOADS[name]
    x = wl.generate(w.with_rows(base_rows))
    xt = parity.to_device(x).repeat(rows // base_rows, 1)
    return w, x, xt


def sample_rows(rows, base_rows, k=96):
    """Row numbers from the first rows, the middle and the end of the launch, and their rows in the base block."""
    pick = np.unique(np.r_[0:k, rows // 2 - k // 2:rows // 2 + k // 2, rows - k:rows])
    return pick, pick % base_rows


def bf16_close(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    amax = np.abs(want).max(axis=1, keepdims=True)
    lim = np.abs(want) * 2.0 ** -8 + 1e-5 * amax
    err = np.abs(got - want)
    assert np.all(err <= lim), f"{what}: max err {err.max():.3g} against a row maximum of {amax.max():.3g}"


def test_dequantize_rotate_kv_group_codes_full_size(torch):
    rows, base = 16 * 32 * 8192, 8192
    w, x, xt = tiled(torch, "kv_k", base, rows)
    h = binding.hadamard_build(w.n)
    say(f"dequantize_rotate kv group codes rows={rows}")
    codes, scales, mins = binding.rotate_quantize_asym(h, xt, 3, w.clip)
    y = torch.empty((rows, w.n), dtype=torch.bfloat16, device="cuda")
    binding.dequantize_rotate(h, codes, scales, 3, mins=mins, out=y)
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_dequant_rotate"
    pick, _ = sample_rows(rows, base)
    idx = torch.from_numpy(pick).cuda()
    q = oracle.unpack_codes(codes[idx].cpu().numpy(), 3, w.n, signed=False)
    d64 = scales[idx].cpu().numpy().astype(np.float64).reshape(len(pick), -1)
    l64 = mins[idx].cpu().numpy().astype(np.float64).reshape(len(pick), -1)
    want = oracle.rotate_back(oracle.dequantize_asym(q, d64, l64), w.n, w.n)
    bf16_close(y[idx].float().cpu().numpy(), want, "kv group codes -> bf16")


@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_dequantize_rotate_hidden_rows_full_size(torch, out):
    rows, base = 65536, 2048
    w, x, xt = tiled(torch, "llama_hidden", base, rows)
    h = binding.hadamard_build(w.n)
    say(f"dequantize_rotate llama rows={rows} -> {out}")
    codes, scales = binding.rotate_quantize(h, xt, 4, w.clip)
    y = torch.empty((rows, w.n), dtype=torch.bfloat16 if out == "bf16" else torch.float32, device="cuda")
    binding.dequantize_rotate(h, codes, scales, 4, out=y)
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_dequant_rotate"
    pick, _ = sample_rows(rows, base, 48)
    idx = torch.from_numpy(pick).cuda()
    q = oracle.unpack_codes(codes[idx].cpu().numpy(), 4, w.n)
    want = oracle.rotate_back(oracle.dequantize(q, scales[idx].cpu().numpy().astype(np.float64)), w.n, w.n)
    if out == "bf16":
        bf16_close(y[idx].float().cpu().numpy(), want, "llama codes -> bf16")
    else:
        parity.check_float_rows(y[idx].cpu().numpy(), want, what="llama codes -> fp32")
    # the rotated-domain dequantizer on the same launch: one exact-input fp32 product per value
    v = torch.empty((rows, w.n), dtype=torch.float32, device="cuda")
    binding.dequantize(h, codes, scales, 4, out=v)
    torch.cuda.synchronize()
    assert h.last_kernel == "dequantize"
    s32 = scales[idx].cpu().numpy()
    assert np.array_equal(v[idx].cpu().numpy(), (q.astype(np.float32) * s32[:, None]).astype(np.float32))


@pytest.mark.parametrize("transpose", [False, True])
def test_rotate_block_order_full_size(torch, transpose):
    rows, base = 73728, 2048
    w, x, xt = tiled(torch, "qwen_hidden", base, rows)
    h = binding.hadamard_build(w.n)
    say(f"rotate qwen rows={rows} transpose={transpose}")
    y = torch.empty_like(xt)
    binding.rotate(h, xt, transpose=transpose, out=y)
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_block_rotate"
    pick, src = sample_rows(rows, base, 32)
    xs = oracle.as_f64(x[src])
    want = oracle.rotate_back(xs, w.n, w.n) if transpose else oracle.rotate(x[src], w.n)
    bf16_close(y[torch.from_numpy(pick).cuda()].float().cpu().numpy(), want, f"rotate transpose={transpose}")


def test_rotation_free_quantizers_value_cache_full_size(torch):
    rows, base = 16 * 32 * 8192, 2048
    w, x, xt = tiled(torch, "kv_v", base, rows)
    b = w.bits[0]
    pick, src = sample_rows(rows, base)
    idx = torch.from_numpy(pick).cuda()
    say(f"rotation-free symmetric quantizer rows={rows} b={b}")
    codes, scales = binding.quantize(xt, b, w.clip)
    torch.cuda.synchronize()
    st = parity.check_quantize_plain(x[src], b, w.clip, codes[idx].cpu().numpy(), scales[idx].cpu().numpy(),
                                     "value cache, symmetric")
    say(f"  ok {st}")
    del codes, scales
    say(f"rotation-free asymmetric quantizer rows={rows} b={b}")
    ca, sa, ma = binding.quantize_asym(xt, b, w.clip)
    torch.cuda.synchronize()
    st = parity.check_rotate_quantize_asym(x[src], w.d, b, w.clip, ca[idx].cpu().numpy(), sa[idx].cpu().numpy(),
                                           ma[idx].cpu().numpy(), "value cache, asymmetric", rotate=False)
    say(f"  ok {st}")


def test_whole_dimension_paley_block_full_size(torch):
    n, rows = 1544, 16384
    rng = np.random.default_rng(1544)
    base = wl.f32_to_bf16_bits(rng.standard_t(3.0, size=(512, n)).astype(np.float32))
    xt = parity.to_device(base).repeat(rows // 512, 1)
    h = binding.hadamard_build(n)
    say(f"dense block n={n} rows={rows}")
    codes, scales = binding.rotate_quantize(h, xt, 4, 0.9)
    torch.cuda.synchronize()
    assert h.last_kernel == "dense_block"
    pick, src = sample_rows(rows, 512, 32)
    idx = torch.from_numpy(pick).cuda()
    st = parity.check_rotate_quantize(base[src], n, 4, 0.9, codes[idx].cpu().numpy(), scales[idx].cpu().numpy(),
                                      "1544 sampled")
    say(f"  ok {st}")
