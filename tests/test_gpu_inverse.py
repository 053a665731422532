"""GPU parity of the floating-point rotation entry points against the oracle: rq_rotate (offline
weight fusion, section 4.2 Eq. 2; inverse rotation) and rq_dequantize_rotate (codes back to the
original basis)."""
import sys

import numpy as np
import pytest

import parity
import rotq_oracle as oracle
from paper_2504_13989_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[inverse] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


_handles = {}


def handle(n):
    if n not in _handles:
        _handles[n] = binding.hadamard_build(n)
    return _handles[n]


CASES = [("tiny", 64), ("llama_hidden", 50), ("qwen_hidden", 40), ("ffn_expand", 30), ("ffn_down", 9),
         ("kv_k", 300)]


@pytest.mark.parametrize("name,rows", CASES)
def test_rotate_forward_and_back(torch, name, rows):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    h = handle(w.n)
    say(f"rotate {name} rows={rows} d={w.d} n={w.n}")
    xt = parity.to_device(x)
    y = binding.rotate(h, xt)
    torch.cuda.synchronize()
    want = oracle.rotate(x, w.n)
    parity.check_float_rows(y.cpu().numpy(), want, what=f"{name} forward")
    # H^T on the rotated rows gives the rows back (padding dropped)
    xb = binding.rotate(h, y, transpose=True, d_out=w.d)
    torch.cuda.synchronize()
    parity.check_float_rows(xb.cpu().numpy(), oracle.rotate_back(want, w.n, w.d), what=f"{name} back")
    parity.check_float_rows(xb.cpu().numpy(), oracle.as_f64(x), rtol=1e-5, what=f"{name} round trip")
    # transposed forward differs from forward exactly where the block is not symmetric
    yt = binding.rotate(h, xt, transpose=True)
    torch.cuda.synchronize()
    xp = np.zeros((rows, w.n))
    xp[:, : w.d] = oracle.as_f64(x)
    parity.check_float_rows(yt.cpu().numpy(), oracle.rotate_back(xp, w.n), what=f"{name} H^T forward")
    # bf16 output
    yb = binding.rotate(h, xt, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    parity.check_float_rows(yb.float().cpu().numpy(), want, what=f"{name} bf16 out", bf16=True)


def test_weight_fusion_preserves_the_product(torch):
    # a Linear-style weight [out, in] with in = 3000 expanded to 3072 (section 4.2): rows rotated
    rng = np.random.default_rng(31)
    d, n, out = 3000, 3072, 24
    wgt = rng.standard_normal((out, d)).astype(np.float32)
    x = rng.standard_normal((16, d)).astype(np.float32)
    h = handle(n)
    wf = binding.rotate(h, torch.from_numpy(wgt).cuda())               # [out, n] = (H pad(W^T))^T / sqrt(n)
    xr = binding.rotate(h, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    want_w = oracle.fuse_weight(wgt.T, n)                                # [n, out]
    parity.check_float_rows(wf.cpu().numpy(), want_w.T, what="fused weight")
    prod = xr.double().cpu().numpy() @ wf.double().cpu().numpy().T
    ref = x.astype(np.float64) @ wgt.astype(np.float64).T
    assert np.abs(prod - ref).max() <= 1e-4 * np.abs(ref).max()


@pytest.mark.parametrize("name,rows,b", [("tiny", 64, 3), ("llama_hidden", 50, 4), ("qwen_hidden", 40, 3),
                                         ("ffn_expand", 30, 3), ("ffn_down", 9, 3), ("kv_k", 300, 3)])
def test_dequantize_rotate(torch, name, rows, b):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    h = handle(w.n)
    say(f"dequantize_rotate {name} rows={rows} n={w.n} b={b}")
    # the oracle's codes and scales go to both sides: the comparison is of the inverse alone
    q, delta, _, y = oracle.rotate_quantize(x, w.n, b, w.clip)
    packed = oracle.pack_codes(q, b)
    scales32 = delta.astype(np.float32)
    out = binding.dequantize_rotate(h, torch.from_numpy(packed).cuda(), torch.from_numpy(scales32).cuda(), b,
                                    d_out=w.d)
    torch.cuda.synchronize()
    want = oracle.rotate_back(oracle.dequantize(q, scales32.astype(np.float64)), w.n, w.d)
    parity.check_float_rows(out.cpu().numpy(), want, what=f"{name} inverse")
    # end to end on the GPU: quantize there, come back, error in the original basis is bounded by
    # the error in the rotated basis (equal when nothing was padded)
    codes, scales = binding.rotate_quantize(h, parity.to_device(x), b, w.clip)
    xh = binding.dequantize_rotate(h, codes, scales, b, d_out=w.d)
    torch.cuda.synchronize()
    e_orig = np.linalg.norm(xh.double().cpu().numpy() - oracle.as_f64(x), axis=1)
    e_rot = np.linalg.norm(oracle.dequantize(q, delta) - y, axis=1)
    assert np.all(e_orig <= e_rot * (1 + 1e-3) + 1e-6 * np.abs(y).max())
    if w.d == w.n:
        assert np.allclose(e_orig, e_rot, rtol=1e-3, atol=1e-6 * np.abs(y).max())


@pytest.mark.parametrize("name,rows,b", [("kv_k", 300, 3), ("kv_v", 100, 4), ("llama_hidden", 20, 3)])
def test_dequantize_rotate_asym(torch, name, rows, b):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    h = handle(w.n)
    say(f"dequantize_rotate asym {name} rows={rows} n={w.n} b={b}")
    y = oracle.rotate(x, w.n)
    q, delta, lo, _ = oracle.quantize_asym(y, b, w.clip)
    packed = oracle.pack_codes(q, b)
    d32, l32 = delta.astype(np.float32), lo.astype(np.float32)
    out = binding.dequantize_rotate(h, torch.from_numpy(packed).cuda(), torch.from_numpy(d32).cuda(), b,
                                    mins=torch.from_numpy(l32).cuda(), d_out=w.d)
    torch.cuda.synchronize()
    want = oracle.rotate_back(oracle.dequantize_asym(q, d32.astype(np.float64), l32.astype(np.float64)), w.n, w.d)
    parity.check_float_rows(out.cpu().numpy(), want, what=f"{name} asym inverse")


@pytest.mark.parametrize("n,d,rows", [(128, 128, 1029), (128, 96, 7), (256, 256, 333), (512, 400, 65), (1024, 1024, 40),
                                      (2048, 2000, 9), (4096, 4096, 77), (8192, 8192, 5)])
@pytest.mark.parametrize("in_dtype", ["bf16", "f16"])
def test_rotate_on_the_wave_path(torch, n, d, rows, in_dtype):
    # Sylvester orders, 16-bit rows: the online rotation without a quantizer (e.g. the query heads),
    # every output type, a narrower output, a leading dimension beyond the width
    rng = np.random.default_rng(n + d + rows)
    xf = rng.standard_t(4.0, size=(rows, d + 8)).astype(np.float32)
    xf[:, 3] *= 30
    full = wl.f32_to_bf16_bits(xf) if in_dtype == "bf16" else xf.astype(np.float16)
    x = np.ascontiguousarray(full[:, :d])
    h = handle(n)
    xt = parity.to_device(full)[:, :d]
    want = oracle.rotate(x, n)
    for out_dtype, tol_bits in ((torch.float32, None), (torch.bfloat16, 8), (torch.float16, 11)):
        say(f"wave rotate n={n} d={d} rows={rows} {in_dtype} -> {out_dtype}")
        y = binding.rotate(h, xt, out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_rotate"
        got = y.double().cpu().numpy()
        amax = np.abs(want).max(axis=1, keepdims=True)
        if tol_bits is None:
            parity.check_float_rows(y.cpu().numpy(), want, what=f"n={n} f32")
        else:
            # one rounding to the output format on top of the fp32 result
            err = np.abs(got - want)
            assert np.all(err <= np.abs(want) * 2.0 ** -tol_bits + 1e-5 * amax + (6.2e-5 if tol_bits == 11 else 0.0)), \
                f"n={n} {out_dtype}: {err.max()}"
    # narrower output and a padded output row
    d_out = max(8, (d // 2) // 8 * 8)
    buf = torch.full((rows, d_out + 16), 7.0, dtype=torch.float32, device="cuda")
    binding.rotate(h, xt, d_out=d_out, out=buf[:, :d_out])
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_rotate"
    parity.check_float_rows(buf[:, :d_out].cpu().numpy(), want[:, :d_out], what=f"n={n} d_out={d_out}")
    assert bool((buf[:, d_out:] == 7.0).all())
    # H is symmetric for these orders: the transposed product is the same
    yt = binding.rotate(h, xt, transpose=True)
    torch.cuda.synchronize()
    parity.check_float_rows(yt.cpu().numpy(), want, what=f"n={n} transposed")


@pytest.mark.parametrize("name,rows,b", [("tiny", 64, 3), ("llama_hidden", 50, 4), ("qwen_hidden", 41, 3),
                                         ("ffn_expand", 30, 4), ("ffn_down", 9, 3), ("kv_k", 1029, 3)])
def test_dequantize_in_the_rotated_domain(torch, name, rows, b):
    """rq_dequantize (section 2.1, X^ = round(X / Delta) * Delta): one fp32 product per element, so the
    result equals the oracle's fp64 product of the same code and the same fp32 scale, rounded once."""
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    h = handle(w.n)
    say(f"dequantize {name} rows={rows} n={w.n} b={b}")
    q, delta, _, _ = oracle.rotate_quantize(x, w.n, b, w.clip)
    packed = oracle.pack_codes(q, b)
    scales32 = delta.astype(np.float32)
    out = binding.dequantize(h, torch.from_numpy(packed).cuda(), torch.from_numpy(scales32).cuda(), b)
    torch.cuda.synchronize()
    assert h.last_kernel == "dequantize"
    want = oracle.dequantize(q, scales32.astype(np.float64)).astype(np.float32)
    assert np.array_equal(out.cpu().numpy(), want), f"{name}: dequantized values differ"
    # the GPU's own codes and scales: the values the kernel chose, back in the rotated domain
    codes, scales = binding.rotate_quantize(h, parity.to_device(x), b, w.clip)
    yh = binding.dequantize(h, codes, scales, b)
    torch.cuda.synchronize()
    qg = oracle.unpack_codes(codes.cpu().numpy(), b, w.n)
    want = oracle.dequantize(qg, scales.cpu().numpy().astype(np.float64)).astype(np.float32)
    assert np.array_equal(yh.cpu().numpy(), want)


@pytest.mark.parametrize("n,rows", [(96, 1000), (160, 333), (896, 77), (1544, 13), (128, 600001), (1024, 70001)])
@pytest.mark.parametrize("b", [3, 4])
def test_dequantize_launch_shapes(torch, n, rows, b):
    """rq_dequantize on random codes: rows shorter than a workgroup that share one (row lengths that are not a
    power of two included), rows cut into segments, more row groups than the grid holds (the row loop), and an
    output that is not 16-byte aligned."""
    rng = np.random.default_rng(1000 * n + b)
    q = rng.integers(-(1 << (b - 1)), 1 << (b - 1), size=(rows, n), dtype=np.int64).astype(np.int8)
    packed = oracle.pack_codes(q, b)
    scales32 = rng.uniform(0.01, 3.0, size=rows).astype(np.float32)
    scales32[rows // 2] = 0.0
    h = handle(n)
    say(f"dequantize shapes n={n} rows={rows} b={b}")
    ct, st = torch.from_numpy(packed).cuda(), torch.from_numpy(scales32).cuda()
    out = binding.dequantize(h, ct, st, b)
    torch.cuda.synchronize()
    want = (q.astype(np.float32) * scales32[:, None]).astype(np.float32)       # one exact-input fp32 product each
    assert np.array_equal(out.cpu().numpy(), want)
    if rows <= 1000:
        buf = torch.full((rows * n + 8,), 7.0, dtype=torch.float32, device="cuda")
        view = buf[1:1 + rows * n].view(rows, n)                                # 4-byte aligned only
        binding.dequantize(h, ct, st, b, out=view)
        torch.cuda.synchronize()
        assert np.array_equal(view.cpu().numpy(), want)
        assert buf[0].item() == 7.0 and bool((buf[1 + rows * n:] == 7.0).all().item())


@pytest.mark.parametrize("name,rows,b", [("kv_k", 300, 3), ("kv_v", 1027, 4), ("llama_hidden", 20, 3)])
def test_dequantize_asym_in_the_rotated_domain(torch, name, rows, b):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    h = handle(w.n)
    say(f"dequantize asym {name} rows={rows} n={w.n} b={b}")
    y = oracle.rotate(x, w.n)
    q, delta, lo, _ = oracle.quantize_asym(y, b, w.clip)
    packed = oracle.pack_codes(q, b)
    d32, l32 = delta.astype(np.float32), lo.astype(np.float32)
    out = binding.dequantize(h, torch.from_numpy(packed).cuda(), torch.from_numpy(d32).cuda(), b,
                             mins=torch.from_numpy(l32).cuda())
    torch.cuda.synchronize()
    want = oracle.dequantize_asym(q, d32.astype(np.float64), l32.astype(np.float64))
    got = out.cpu().numpy().astype(np.float64)
    # one fused multiply-add in fp32: half an ulp of the result
    assert np.all(np.abs(got - want) <= 2.0 ** -24 * np.abs(want) + 1e-45), f"{name}: dequantized values differ"


@pytest.mark.parametrize("n,rows", [(128, 1029), (256, 333), (512, 65), (1024, 40), (2048, 9), (4096, 77), (8192, 5)])
@pytest.mark.parametrize("b", [3, 4])
def test_dequantize_rotate_on_the_wave_path(torch, n, rows, b):
    """Packed codes back to the original basis for Sylvester orders (sections 2.1, 2.3): every code value
    occurs, every output type, a narrower output, a padded output row, row counts that leave a ragged
    last pass."""
    rng = np.random.default_rng(7 * n + rows + b)
    _, qmin, qmax = oracle.quant_params(b)
    q = rng.integers(qmin, qmax + 1, size=(rows, n)).astype(np.int8)
    q[0] = qmin
    q[1 % rows] = qmax
    q[2 % rows] = 0
    scales32 = np.exp(rng.normal(0.0, 3.0, size=rows)).astype(np.float32)
    scales32[3 % rows] = 0.0
    packed = torch.from_numpy(oracle.pack_codes(q, b)).cuda()
    sc = torch.from_numpy(scales32).cuda()
    h = handle(n)
    want = oracle.rotate_back(oracle.dequantize(q, scales32.astype(np.float64)), n, n)
    for out_dtype, tol_bits in ((torch.float32, None), (torch.bfloat16, 8), (torch.float16, 11)):
        say(f"wave dequantize_rotate n={n} rows={rows} b={b} -> {out_dtype}")
        y = binding.dequantize_rotate(h, packed, sc, b, out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_dequant_rotate"
        got = y.double().cpu().numpy()
        amax = np.abs(want).max(axis=1, keepdims=True)
        if tol_bits is None:
            parity.check_float_rows(y.cpu().numpy(), want, what=f"n={n} b={b} f32")
        else:
            ok = np.isfinite(got) | (tol_bits == 11)            # large scales overflow fp16: not compared there
            err = np.abs(got - want)
            lim = np.abs(want) * 2.0 ** -tol_bits + 1e-5 * amax + (6.2e-5 if tol_bits == 11 else 0.0)
            fin = np.isfinite(got)
            assert np.all(err[fin] <= lim[fin]), f"n={n} b={b} {out_dtype}: {err[fin].max()}"
            assert ok.all()
    d_out = max(8, (n // 2 + 8) // 8 * 8)
    buf = torch.full((rows, d_out + 16), 7.0, dtype=torch.float32, device="cuda")
    binding.dequantize_rotate(h, packed, sc, b, d_out=d_out, out=buf[:, :d_out])
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_dequant_rotate"
    parity.check_float_rows(buf[:, :d_out].cpu().numpy(), want[:, :d_out], what=f"n={n} b={b} d_out={d_out}")
    assert bool((buf[:, d_out:] == 7.0).all())
    # H is symmetric for these orders: H and H^T give the same rows
    y0 = binding.dequantize_rotate(h, packed, sc, b, transpose=False)
    torch.cuda.synchronize()
    parity.check_float_rows(y0.cpu().numpy(), want, what=f"n={n} b={b} untransposed")


@pytest.mark.parametrize("rows", [1029, 3, 64])
@pytest.mark.parametrize("b", [3, 4])
def test_dequantize_rotate_group_codes_on_the_wave_path(torch, rows, b):
    """The asymmetric group codes of the KV-cache setting (section 5.1) with one group per head row."""
    n = 128
    rng = np.random.default_rng(rows + b)
    q = rng.integers(0, 1 << b, size=(rows, n)).astype(np.int8)
    q[0] = 0
    q[1 % rows] = (1 << b) - 1
    d32 = np.exp(rng.normal(0.0, 2.0, size=(rows, 1))).astype(np.float32)
    l32 = (rng.normal(0.0, 5.0, size=(rows, 1)) * d32).astype(np.float32)
    h = handle(n)
    want = oracle.rotate_back(oracle.dequantize_asym(q, d32.astype(np.float64), l32.astype(np.float64)), n, n)
    y = binding.dequantize_rotate(h, torch.from_numpy(oracle.pack_codes(q, b)).cuda(), torch.from_numpy(d32).cuda(), b,
                                  mins=torch.from_numpy(l32).cuda())
    torch.cuda.synchronize()
    assert h.last_kernel == "wave_dequant_rotate"
    parity.check_float_rows(y.cpu().numpy(), want, what=f"group codes rows={rows} b={b}")


@pytest.mark.parametrize("n,d,rows", [(3584, 3584, 41), (3072, 3000, 30), (1536, 1536, 77), (2560, 2400, 9), (1024 + 512, 1536, 3)])
@pytest.mark.parametrize("in_dtype", ["bf16", "f16"])
def test_rotate_block_orders_on_the_wave_path(torch, n, d, rows, in_dtype):
    """rq_rotate for Paley-block orders up to 32 x 128 (sections 2.3.3, 4.2): H_n and H_n^T (Paley I blocks are
    not symmetric), every output type, a narrower output."""
    rng = np.random.default_rng(n + d + rows)
    xf = rng.standard_t(4.0, size=(rows, d)).astype(np.float32)
    xf[:, 5] *= 25
    x = wl.f32_to_bf16_bits(xf) if in_dtype == "bf16" else xf.astype(np.float16)
    h = handle(n)
    xt = parity.to_device(x)
    xp = np.zeros((rows, n))
    xp[:, :d] = oracle.as_f64(x)
    for transpose, want in ((False, oracle.rotate(x, n)), (True, oracle.rotate_back(xp, n, n))):
        for out_dtype, tol_bits in ((torch.float32, None), (torch.bfloat16, 8), (torch.float16, 11)):
            say(f"wave block rotate n={n} d={d} rows={rows} {in_dtype} -> {out_dtype} transpose={transpose}")
            y = binding.rotate(h, xt, transpose=transpose, out_dtype=out_dtype)
            torch.cuda.synchronize()
            assert h.last_kernel == "wave_block_rotate"
            if tol_bits is None:
                parity.check_float_rows(y.cpu().numpy(), want, what=f"n={n} f32 transpose={transpose}")
            else:
                got = y.double().cpu().numpy()
                amax = np.abs(want).max(axis=1, keepdims=True)
                err = np.abs(got - want)
                assert np.all(err <= np.abs(want) * 2.0 ** -tol_bits + 1e-5 * amax + (6.2e-5 if tol_bits == 11 else 0.0))
        d_out = (n // 3) // 8 * 8
        buf = torch.full((rows, d_out + 8), 7.0, dtype=torch.float32, device="cuda")
        binding.rotate(h, xt, transpose=transpose, d_out=d_out, out=buf[:, :d_out])
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_block_rotate"
        parity.check_float_rows(buf[:, :d_out].cpu().numpy(), want[:, :d_out], what=f"n={n} d_out={d_out}")
        assert bool((buf[:, d_out:] == 7.0).all())
