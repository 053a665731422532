"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Small cases compare every element; the full-size configurations run the launch the benchmark
times and compare either everything (when the oracle finishes in seconds) or sampled row
blocks (rows are independent, so a sampled row is checked exactly like any other).
"""
import sys

import numpy as np
import pytest

import parity
import rotq_oracle as oracle
from paper_2504_13989_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[parity] {msg}", flush=True)
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


def run_rq(torch, x_np, n, b, clip, variant=0, ld=None):
    h = handle(n)
    h.set_variant(variant)
    x = parity.to_device(x_np)
    if ld is not None:
        buf = torch.zeros((x.shape[0], ld), dtype=x.dtype, device="cuda")
        buf[:, : x.shape[1]] = x
        x = buf[:, : x.shape[1]]
    codes, scales = binding.rotate_quantize(h, x, b, clip)
    torch.cuda.synchronize()
    h.set_variant(0)
    return codes.cpu().numpy(), scales.cpu().numpy(), h.last_kernel


SMALL = [
    # workload, rows, variants
    ("tiny", 64), ("llama_hidden", 333), ("qwen_hidden", 333), ("ffn_expand", 333),
    ("ffn_down", 37), ("kv_k", 1029), ("kv_v", 515), ("calib", 130),
]


@pytest.mark.parametrize("variant", [0, 1], ids=["auto", "general"])
@pytest.mark.parametrize("name,rows", SMALL)
def test_small_cases(torch, name, rows, variant):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    for b in w.bits:
        say(f"small {name} rows={rows} n={w.n} b={b} variant={variant}")
        codes, scales, kern = run_rq(torch, x, w.n, b, w.clip, variant)
        st = parity.check_rotate_quantize(x, w.n, b, w.clip, codes, scales, f"{name} b={b} [{kern}]")
        say(f"  ok kernel={kern} {st}")


@pytest.mark.parametrize("n,d,dtype", [(256, 256, "f32"), (128, 100, "bf16"), (4096, 4000, "f32"),
                                       (3584, 3500, "bf16"), (3072, 3000, "f32"), (1536, 1536, "bf16"),
                                       (2048, 2048, "bf16"), (8192, 8192, "bf16"), (512, 512, "bf16"),
                                       (640, 640, "bf16"), (64, 64, "bf16"), (32, 20, "f32"),
                                       (2560, 2560, "bf16"), (2560, 2400, "bf16"), (5120, 5120, "bf16"),
                                       # blocks of 33 .. 64 on one wave: 36, 40, 48, 56
                                       (36 * 128, 36 * 128, "bf16"), (36 * 128, 4000, "bf16"), (5120, 5000, "bf16"),
                                       (48 * 128, 48 * 128, "bf16"), (56 * 128, 7000, "bf16"),
                                       # blocks above 32: 44 (q=43), 60 (II, q=29), 84, 108, 168, 200, 252
                                       (44 * 128, 44 * 128, "bf16"), (60 * 128, 7600, "bf16"),
                                       (84 * 128, 84 * 128, "bf16"), (108 * 128, 108 * 128, "bf16"),
                                       (168 * 128, 168 * 128, "bf16"), (200 * 128, 25000, "bf16"),
                                       (252 * 128, 252 * 128, "bf16"), (38 * 256, 38 * 256, "bf16"),
                                       # prime-power Paley blocks: 52 = 2 (25 + 1), 100 = 2 (49 + 1), 244 = 243 + 1
                                       (52 * 128, 52 * 128, "bf16"), (52 * 32, 1600, "bf16"), (100 * 64, 6400, "bf16"),
                                       (100 * 128, 12000, "bf16"), (244 * 128, 244 * 128, "bf16")])
@pytest.mark.parametrize("b", [3, 4])
def test_other_orders_and_padding(torch, n, d, dtype, b):
    rng = np.random.default_rng(n * 7 + d + b)
    x = rng.standard_t(3.0, size=(67 if n <= 8192 else 19, d)).astype(np.float32)
    x[:, rng.choice(d, 3, replace=False)] *= 40
    if dtype == "bf16":
        x = wl.f32_to_bf16_bits(x)
    say(f"order n={n} d={d} {dtype} b={b}")
    codes, scales, kern = run_rq(torch, x, n, b, 0.85)
    parity.check_rotate_quantize(x, n, b, 0.85, codes, scales, f"n={n} d={d} {dtype} b={b} [{kern}]")


@pytest.mark.parametrize("n,d,rows", [(28 * 32, 28 * 32, 67), (28 * 32, 800, 5), (12 * 32, 12 * 32, 1), (12 * 64, 12 * 64, 3),
                                      (20 * 64, 1200, 130), (76 * 64, 76 * 64, 67), (76 * 64, 4800, 2),
                                      (140 * 64, 140 * 64, 33), (44 * 32, 44 * 32, 10), (252 * 64, 16000, 9),
                                      (196 * 32, 6200, 6), (28 * 32, 28 * 32, 2101)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_short_sylvester_factor_blocks(torch, n, d, rows, dtype):
    # n = p 2^k with k = 5, 6: the block kernel lays 4 / 2 rows side by side; row counts that do not
    # fill the last pass, padded widths, a leading dimension beyond d
    rng = np.random.default_rng(n + 3 * d + rows)
    ld = d + 24
    full = rng.standard_t(3.0, size=(rows, ld)).astype(np.float32)
    full[:, rng.choice(d, 3, replace=False)] *= 40
    full = wl.f32_to_bf16_bits(full) if dtype == "bf16" else full.astype(np.float16)
    x = full[:, :d]
    h = handle(n)
    xt = parity.to_device(full)[:, :d]
    for b in (3, 4):
        say(f"short factor n={n} d={d} rows={rows} {dtype} b={b}")
        codes, scales = binding.rotate_quantize(h, xt, b, 0.85)
        torch.cuda.synchronize()
        assert h.last_kernel == "wg_block"
        st = parity.check_rotate_quantize(np.ascontiguousarray(x), n, b, 0.85, codes.cpu().numpy(),
                                          scales.cpu().numpy(), f"n={n} d={d} {dtype} b={b} [wg_block]")
        say(f"  ok {st}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_sylvester_orders_beyond_one_wave(torch, dtype):
    # n = 2^14 and 2^15 run on the block kernel with B = H_128 / H_256.  The oracle for 2^14 is the
    # dense product as always; for 2^15 the dense matrix (8 GiB as int64) is not built: Sylvester's
    # recursion (section 2.3.2, Eq. 1) H_2n = [[H_n, H_n], [H_n, -H_n]] is written out on the two
    # halves of the row with the oracle's own H_{2^14}.
    hs = oracle.sylvester(14).astype(np.float64)
    for n, d, rows in ((1 << 14, 1 << 14, 19), (1 << 14, 16000, 3), (1 << 15, 1 << 15, 11), (1 << 15, 30000, 4)):
        rng = np.random.default_rng(n + d)
        xf = rng.standard_t(3.0, size=(rows, d)).astype(np.float32)
        xf[:, rng.choice(d, 3, replace=False)] *= 40
        x = wl.f32_to_bf16_bits(xf) if dtype == "bf16" else xf.astype(np.float16)
        xp = np.zeros((rows, n))
        xp[:, :d] = oracle.as_f64(x)
        if n == 1 << 14:
            y = xp @ hs.T / np.sqrt(n)
        else:
            a, bb = xp[:, : n // 2] @ hs.T, xp[:, n // 2:] @ hs.T
            y = np.concatenate([a + bb, a - bb], axis=1) / np.sqrt(n)
        for b in (3, 4):
            say(f"long sylvester n={n} d={d} {dtype} b={b}")
            codes, scales, kern = run_rq(torch, x, n, b, 0.9)
            assert kern == "wg_block"
            st = parity.check_rotate_quantize(x, n, b, 0.9, codes, scales, f"n={n} d={d} {dtype} b={b}", rotated=y)
            say(f"  ok {st}")
    h = handle(1 << 14)
    clips = [0.6, 0.9, 1.0]
    xq = wl.f32_to_bf16_bits(np.random.default_rng(3).standard_normal((9, 1 << 14)).astype(np.float32))
    mse = binding.quant_error(h, parity.to_device(xq), 3, clips)
    torch.cuda.synchronize()
    assert h.last_kernel == "wg_block_quant_error"
    yq = oracle.as_f64(xq) @ hs.T / np.sqrt(1 << 14)
    want = [np.mean((oracle.dequantize(*oracle.quantize(yq, 3, c)[:2]) - yq) ** 2) for c in clips]
    assert np.allclose(mse.cpu().numpy(), want, rtol=1e-5, atol=0)


@pytest.mark.parametrize("n", [128, 512, 1536, 3584, 4096, 5120, 8960, 18944])
@pytest.mark.parametrize("scale", [1e-30, 1e30])
def test_rows_of_very_small_and_very_large_magnitude(torch, n, scale):
    # the scales' reciprocals, the fp32 butterflies and the reported Delta at both ends of the exponent
    # range (the rotated row stays finite: n * 30 * 1e30 < 3.4e38), through every kernel family
    rng = np.random.default_rng(n)
    xf = (np.clip(rng.standard_t(3.0, size=(19, n)), -30, 30) * scale).astype(np.float32)
    for dtype, x in (("bf16", wl.f32_to_bf16_bits(xf)), ("f32", xf)):
        if dtype == "f32" and n > 8960:
            continue                       # fp32 rows of this length do not fit the general kernel's LDS copy
        for b in (3, 4):
            say(f"magnitude n={n} scale={scale} {dtype} b={b}")
            codes, scales, kern = run_rq(torch, x, n, b, 0.9)
            st = parity.check_rotate_quantize(x, n, b, 0.9, codes, scales, f"n={n} scale={scale} {dtype} b={b} [{kern}]")
            say(f"  ok kernel={kern} {st}")
        if n % 128 == 0:
            h = handle(n)
            ca, sa, ma = binding.rotate_quantize_asym(h, parity.to_device(x), 3, 0.9)
            torch.cuda.synchronize()
            parity.check_rotate_quantize_asym(x, n, 3, 0.9, ca.cpu().numpy(), sa.cpu().numpy(), ma.cpu().numpy(),
                                              f"asym n={n} scale={scale} {dtype} [{h.last_kernel}]")


@pytest.mark.parametrize("variant", [2, 3, 4], ids=["one_wave", "split2", "split4"])
@pytest.mark.parametrize("n,d", [(2048, 2048), (4096, 4096), (4096, 4000), (8192, 8192), (8192, 6000)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_long_rows_split_over_waves(torch, n, d, variant, dtype):
    # the same rows through one wave per row and through 2 / 4 waves per row
    rng = np.random.default_rng(n + d)
    xf = rng.standard_t(3.0, size=(77, d)).astype(np.float32)
    xf[:, 5] *= 40.0
    x = wl.f32_to_bf16_bits(xf) if dtype == "bf16" else xf.astype(np.float16)
    for b in (3, 4):
        say(f"split n={n} d={d} b={b} variant={variant} {dtype}")
        codes, scales, kern = run_rq(torch, x, n, b, 0.9, variant)
        assert kern == "wave_sylvester"
        st = parity.check_rotate_quantize(x, n, b, 0.9, codes, scales, f"n={n} d={d} b={b} variant={variant}")
        say(f"  ok {st}")


@pytest.mark.parametrize("n,d,dtype", [(1544, 1544, "bf16"), (1544, 1536, "bf16"), (1544, 1536, "f32"),
                                       (3088, 3088, "bf16"), (3000, 3000, "bf16"), (56, 56, "f32"),
                                       (40, 33, "bf16")])
def test_large_blocks_and_byte_granular_rows(torch, n, d, dtype):
    # whole-dimension Paley blocks (1544 = 1543 + 1: the 1536 + 8 expansion of section 5.2.2) and
    # orders that are a multiple of 8 only; packed rows are then not a whole number of dwords
    rng = np.random.default_rng(n * 7 + d)
    xf = rng.standard_normal((21, d)).astype(np.float32)
    xf[:, 3] *= 25.0
    x = xf if dtype == "f32" else wl.f32_to_bf16_bits(xf)
    for b in (3, 4):
        for variant in (0, 1):
            say(f"large/odd order n={n} d={d} {dtype} b={b} variant={variant}")
            codes, scales, kern = run_rq(torch, x, n, b, 0.9, variant)
            dense = variant == 0 and dtype == "bf16" and d % 8 == 0
            assert kern == ("dense_block" if dense else "generic_lds")
            st = parity.check_rotate_quantize(x, n, b, 0.9, codes, scales, f"n={n} d={d} b={b} [{kern}]")
            say(f"  ok kernel={kern} {st}")
    h = handle(n)
    mse = binding.quant_error(h, parity.to_device(x), 3, [0.7, 1.0])
    torch.cuda.synchronize()
    parity.check_quant_error(x, n, 3, [0.7, 1.0], mse.cpu().numpy(), what=f"n={n}")
    # and back: codes -> original basis
    q, delta, _, y = oracle.rotate_quantize(x, n, 4, 0.9)
    out = binding.dequantize_rotate(h, torch.from_numpy(oracle.pack_codes(q, 4)).cuda(),
                                    torch.from_numpy(delta.astype(np.float32)).cuda(), 4, d_out=d)
    torch.cuda.synchronize()
    want = oracle.rotate_back(oracle.dequantize(q, delta.astype(np.float32).astype(np.float64)), n, d)
    parity.check_float_rows(out.cpu().numpy(), want, what=f"n={n} inverse")


@pytest.mark.parametrize("n,rows", [(32, 100), (64, 33), (96, 16), (104, 17), (1544, 333), (4080, 40), (4088, 5),
                                    # 32 rows per workgroup from 32 rows per CU on (ragged last group)
                                    (1544, 8192 + 21), (104, 9001),
                                    # the other register-tile sizes of the kernel (tiles per wave 5, 9, 14, 17)
                                    (568, 50), (1040, 37), (1784, 20), (2144, 18), (568, 8192 + 5)])
def test_dense_block_kernel_shapes(torch, n, rows):
    # orders below 128 and whole-dimension blocks on the matrix cores; ragged last group of 16 rows
    if oracle.factor_order(n) is None:
        pytest.skip(f"{n} is not a constructible order")
    rng = np.random.default_rng(n + rows)
    xf = rng.standard_t(3.0, size=(rows, n)).astype(np.float32)
    xf[rows // 2] = 0.0
    x = wl.f32_to_bf16_bits(xf)
    for b in (3, 4):
        say(f"dense n={n} rows={rows} b={b}")
        codes, scales, kern = run_rq(torch, x, n, b, 1.0)
        assert kern == "dense_block"
        st = parity.check_rotate_quantize(x, n, b, 1.0, codes, scales, f"dense n={n} b={b}")
        say(f"  ok {st}")


def test_leading_dimension_and_row_views(torch):
    w = wl.WORKLOADS["llama_hidden"].with_rows(70)
    x = wl.generate(w)
    say("ld > d")
    codes, scales, kern = run_rq(torch, x, w.n, 4, 0.9, ld=w.d + 24)
    parity.check_rotate_quantize(x, w.n, 4, 0.9, codes, scales, f"ld [{kern}]")
    w = wl.WORKLOADS["ffn_expand"].with_rows(70)
    x = wl.generate(w)
    codes, scales, kern = run_rq(torch, x, w.n, 3, 0.9, ld=w.d + 8)
    parity.check_rotate_quantize(x, w.n, 3, 0.9, codes, scales, f"ld [{kern}]")
    # dense-block kernel: rows narrower than the order inside a wider allocation (zero padding beyond d, the
    # loader's row pitch), a ragged last group of rows, degenerate rows
    rng = np.random.default_rng(15)
    xf = rng.standard_t(3.0, size=(70, 1536)).astype(np.float32)
    xf[5] = 0.0
    xf[6, :] = 0.0
    xf[6, 1535] = 4.0
    xd = wl.f32_to_bf16_bits(xf)
    for b in (3, 4):
        codes, scales, kern = run_rq(torch, xd, 1544, b, 0.9, ld=1600)
        assert kern == "dense_block"
        parity.check_rotate_quantize(xd, 1544, b, 0.9, codes, scales, f"dense ld [{kern}]")
        assert scales[5] == 0 and not codes[5].any()
    # 4-D KV view [B, H, S, 128]
    w = wl.WORKLOADS["kv_k"].with_rows(2 * 3 * 40)
    x = wl.generate(w)
    xt = parity.to_device(x).reshape(2, 3, 40, 128)
    codes, scales = binding.rotate_quantize(handle(128), xt, 3, 0.9)
    torch.cuda.synchronize()
    parity.check_rotate_quantize(x, 128, 3, 0.9, codes.cpu().numpy(), scales.cpu().numpy(), "kv view")


def test_degenerate_rows(torch):
    # empty input, single row, all-zero rows, one-hot rows (closed form: all codes at the range ends)
    h = handle(4096)
    x0 = torch.empty((0, 4096), dtype=torch.bfloat16, device="cuda")
    codes, scales = binding.rotate_quantize(h, x0, 4, 0.9)
    assert codes.shape == (0, 2048) and scales.shape == (0,)
    for n in (4096, 3584, 128, 256):
        x = np.zeros((5, n), dtype=np.float32)
        x[1, 7] = 12.0
        x[3, n - 1] = -3.0
        x[4, :] = 1.0
        for dtype in ("f32", "bf16"):
            xx = x if dtype == "f32" else wl.f32_to_bf16_bits(x)
            for b in (3, 4):
                say(f"degenerate n={n} {dtype} b={b}")
                codes, scales, kern = run_rq(torch, xx, n, b, 0.9)
                parity.check_rotate_quantize(xx, n, b, 0.9, codes, scales, f"degenerate n={n} [{kern}]")
                assert scales[0] == 0 and not codes[0].any()
                q = oracle.unpack_codes(codes, b, n)
                _, qmin, qmax = oracle.quant_params(b)
                assert set(np.unique(q[1])) <= {qmin, qmax}
                if n in (4096, 256, 128):   # Sylvester: closed-form scale c * clip / (sqrt(n) L)
                    want = float(np.float32(0.9)) * 12.0 / (np.sqrt(n) * ((1 << b) - 1))
                    assert abs(scales[1] - want) <= 1e-6 * want
        x1 = wl.generate(wl.WORKLOADS["calib"].with_rows(1)) if n == 4096 else None
        if x1 is not None:
            codes, scales, kern = run_rq(torch, x1, n, 4, 0.9)
            parity.check_rotate_quantize(x1, n, 4, 0.9, codes, scales, "single row")


def test_deterministic_and_output_bounds(torch):
    # two runs give identical bytes; bytes after the outputs stay untouched
    w = wl.WORKLOADS["qwen_hidden"].with_rows(257)
    x = parity.to_device(wl.generate(w))
    h = handle(w.n)
    nb = w.n * 3 // 8
    codes = torch.full((257 * nb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    scales = torch.full((257 + 16,), -7.0, dtype=torch.float32, device="cuda")
    binding.rotate_quantize(h, x, 3, 0.9, codes=codes[: 257 * nb].view(257, nb), scales=scales[:257])
    torch.cuda.synchronize()
    first = codes.clone(), scales.clone()
    binding.rotate_quantize(h, x, 3, 0.9, codes=codes[: 257 * nb].view(257, nb), scales=scales[:257])
    torch.cuda.synchronize()
    assert torch.equal(first[0], codes) and torch.equal(first[1], scales)
    assert bool((codes[257 * nb:] == 0xA5).all()) and bool((scales[257:] == -7.0).all())


# ------------------------------------------------------------------ full-size configurations

@pytest.mark.parametrize("name", ["tiny", "llama_hidden", "qwen_hidden", "ffn_expand"])
def test_full_size_all_rows(torch, name):
    w = wl.WORKLOADS[name]
    x = wl.generate(w)
    for b in w.bits:
        say(f"full {name} [{w.rows} x {w.d}] n={w.n} b={b}")
        codes, scales, kern = run_rq(torch, x, w.n, b, w.clip)
        st = parity.check_rotate_quantize(x, w.n, b, w.clip, codes, scales, f"{name} b={b} [{kern}]")
        say(f"  ok kernel={kern} {st}")


def _full_run_sampled_check(torch, name, blocks):
    w = wl.WORKLOADS[name]
    say(f"full {name} [{w.rows} x {w.d}] n={w.n}: generating")
    x = wl.generate(w)
    b = w.bits[0]
    say(f"full {name}: launching")
    h = handle(w.n)
    xt = parity.to_device(x)
    codes, scales = binding.rotate_quantize(h, xt, b, w.clip)
    torch.cuda.synchronize()
    rows = wl.block_row_index(blocks, w)
    idx = torch.from_numpy(rows).to("cuda")
    c = codes[idx].cpu().numpy()
    s = scales[idx].cpu().numpy()
    xs = wl.generate_blocks(w, blocks)
    assert np.array_equal(xs, x[rows])          # block regeneration gives the same rows
    st = parity.check_rotate_quantize(xs, w.n, b, w.clip, c, s, f"{name} sampled [{h.last_kernel}]")
    say(f"  ok kernel={h.last_kernel} sampled_rows={len(rows)} {st}")


def test_full_size_ffn_down_sampled(torch):
    _full_run_sampled_check(torch, "ffn_down", [0, 6, 15])


@pytest.mark.parametrize("name", ["kv_k", "kv_v"])
def test_full_size_kv_sampled(torch, name):
    nb = wl.n_blocks(wl.WORKLOADS[name])
    _full_run_sampled_check(torch, name, [0, 1, 31, 32, nb // 2 + 5, nb - 1])


# ------------------------------------------------------------------ quant_error

@pytest.mark.parametrize("variant", [0, 1], ids=["auto", "general"])
@pytest.mark.parametrize("name,rows,b", [("calib", 512, 3), ("calib", 77, 4), ("qwen_hidden", 50, 3),
                                         ("ffn_expand", 50, 3), ("tiny", 64, 3), ("kv_k", 300, 3),
                                         ("ffn_down", 9, 3), ("qwen_hidden", 700, 4), ("kv_v", 1031, 4),
                                         ("kv_k", 3, 3), ("kv_k", 5003, 3), ("kv_v", 4096 + 256, 4)])
def test_quant_error(torch, name, rows, b, variant):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    clips = wl.clip_grid()
    h = handle(w.n)
    h.set_variant(variant)
    say(f"quant_error {name} rows={rows} n={w.n} b={b} variant={variant}")
    mse = binding.quant_error(h, parity.to_device(x), b, clips)
    torch.cuda.synchronize()
    h.set_variant(0)
    rel = parity.check_quant_error(x, w.n, b, clips, mse.cpu().numpy(), what=f"{name} [{h.last_kernel}]")
    say(f"  ok kernel={h.last_kernel} max rel err {rel:.2e}")


@pytest.mark.parametrize("n,d", [(256, 256), (512, 500 // 8 * 8), (1536, 1536), (2560, 2400), (1024, 1024)])
def test_quant_error_other_orders(torch, n, d):
    rng = np.random.default_rng(n + d)
    xf = rng.standard_t(3.0, size=(45, d)).astype(np.float32)
    xf[:, 1] *= 30.0
    xf[7] = 0.0
    x = wl.f32_to_bf16_bits(xf)
    clips = [0.5, 0.77, 0.9, 1.0, 0.61]
    h = handle(n)
    for b in (3, 4):
        say(f"quant_error order n={n} d={d} b={b}")
        mse = binding.quant_error(h, parity.to_device(x), b, clips)
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_quant_error"
        parity.check_quant_error(x, n, b, clips, mse.cpu().numpy(), what=f"n={n} d={d} b={b}")


@pytest.mark.parametrize("n,d", [(896, 896), (4864, 4864), (8960, 8960), (8960, 8000), (1792, 1792), (640, 640),
                                 (2432, 2400)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_quant_error_orders_with_short_sylvester_factor(torch, n, d, dtype):
    # n = p * 64 or p * 32: several rows per pass of the workgroup kernel, sums per row of the pass;
    # row counts that leave the last pass ragged, 1 .. 32 clip ratios
    h = handle(n)
    rng = np.random.default_rng(n * 3 + d)
    for rows, k in ((1, 1), (7, 5), (66, 32), (301, 3)):
        xf = (rng.standard_t(3.0, size=(rows, d)) * rng.choice([0.1, 1.0, 20.0], size=(rows, 1))).astype(np.float32)
        if rows > 3:
            xf[2] = 0.0
        x = wl.f32_to_bf16_bits(xf) if dtype == "bf16" else np.clip(xf, -6e4, 6e4).astype(np.float16)
        clips = [float(np.float32(c)) for c in np.linspace(0.5, 1.0, k)]
        for b in (3, 4):
            say(f"quant_error short-factor order n={n} d={d} rows={rows} clips={k} {dtype} b={b}")
            mse = binding.quant_error(h, parity.to_device(x), b, clips)
            torch.cuda.synchronize()
            assert h.last_kernel == "wg_block_quant_error"
            parity.check_quant_error(x, n, b, clips, mse.cpu().numpy(), what=f"n={n} d={d} rows={rows} b={b} {dtype}")


def test_quant_error_consistent_with_rotate_quantize(torch):
    # the two entry points agree: mse[k] equals the error of dequantized rotate_quantize output
    w = wl.WORKLOADS["calib"].with_rows(64)
    x = wl.generate(w)
    xt = parity.to_device(x)
    h = handle(w.n)
    clips = np.array([0.6, 0.6, 0.95], dtype=np.float32)
    mse = binding.quant_error(h, xt, 3, clips).cpu().numpy()
    assert mse[0] == mse[1]
    y = oracle.rotate(x, w.n)
    for k in (0, 2):
        codes, scales = binding.rotate_quantize(h, xt, 3, float(clips[k]))
        q = oracle.unpack_codes(codes.cpu().numpy(), 3, w.n)
        err = np.mean((q * scales.cpu().numpy().astype(np.float64)[:, None] - y) ** 2)
        assert abs(err - mse[k]) <= 1e-5 * err
    # empty input -> zeros
    x0 = torch.empty((0, 4096), dtype=torch.bfloat16, device="cuda")
    assert not binding.quant_error(h, x0, 3, clips).cpu().numpy().any()


# ------------------------------------------------------------------ gradual binary search

@pytest.mark.parametrize("name,rows,b", [("calib", 512, 3), ("calib", 64, 4), ("qwen_hidden", 40, 3), ("tiny", 64, 3)])
def test_gbs_search_follows_algorithm_1(torch, name, rows, b):
    # the HIP-side search (host loop over rq_quant_error) against the oracle's Algorithm 1 with the
    # oracle's fp64 quant_error as objective: same probes in the same order, same result
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    eps = 1.0 / 64
    say(f"gbs {name} rows={rows} b={b}")
    clip, mse, trace = binding.gbs_search(handle(w.n), parity.to_device(x), b, eps)
    y = oracle.rotate(x, w.n)

    def f(c):
        q, delta, _ = oracle.quantize(y, b, np.float32(c))
        return float(np.mean((oracle.dequantize(q, delta) - y) ** 2))

    m, fm, otrace = oracle.gbs_search(f, eps)
    assert len(trace) == len(otrace)
    for (cg, fg), (co, fo) in zip(trace, otrace):
        assert cg == co, (trace, otrace)
        assert abs(fg - fo) <= 1e-5 * fo
    assert clip == m and abs(mse - fm) <= 1e-5 * fm
    # consistency with the grid: the found clip is no worse than the best of a 32-point grid
    # evaluated by the same entry point, up to the grid's own resolution
    grid = wl.clip_grid()
    gm = binding.quant_error(handle(w.n), parity.to_device(x), b, grid).cpu().numpy()
    assert mse <= gm.min() * 1.05
    say(f"  ok clip={clip} mse={mse:.4g} evals={len(trace)} grid argmin={grid[gm.argmin()]}")
