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
