"""GPU parity of the widened entry points against the oracle: the asymmetric group-128 variant
(section 5.1, KV cache) and the rotation-free quantizer (section 2.1 alone)."""
import sys

import numpy as np
import pytest

import parity
from paper_2504_13989_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[variants] {msg}", flush=True)
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


def run_asym(torch, x_np, n, b, clip, variant=0):
    h = handle(n)
    h.set_variant(variant)
    codes, scales, mins = binding.rotate_quantize_asym(h, parity.to_device(x_np), b, clip)
    torch.cuda.synchronize()
    h.set_variant(0)
    return codes.cpu().numpy(), scales.cpu().numpy(), mins.cpu().numpy(), h.last_kernel


@pytest.mark.parametrize("variant", [0, 1], ids=["auto", "general"])
@pytest.mark.parametrize("name,rows", [("kv_k", 1029), ("kv_v", 515), ("tiny", 64), ("llama_hidden", 41),
                                       ("qwen_hidden", 23)])
@pytest.mark.parametrize("b", [3, 4])
def test_asym_small(torch, name, rows, b, variant):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    for clip in (1.0, 0.9):
        say(f"asym {name} rows={rows} n={w.n} b={b} clip={clip} variant={variant}")
        codes, scales, mins, kern = run_asym(torch, x, w.n, b, clip, variant)
        st = parity.check_rotate_quantize_asym(x, w.n, b, clip, codes, scales, mins, f"{name} b={b} [{kern}]")
        say(f"  ok kernel={kern} {st}")
        if variant == 0 and w.n == 128 and x.dtype == np.uint16:
            assert kern == "wave_short_asym"


def test_asym_shifted_and_degenerate_groups(torch):
    # rows far from zero (all-positive groups), constant rows, zero rows, a short ragged tail
    rng = np.random.default_rng(5)
    rows = 37
    xf = rng.standard_normal((rows, 128)).astype(np.float32)
    xf[3] = 0.0
    xf[4] = 2.5                      # constant input: rotated row is one spike, not a flat group
    xf[5, 1:] = 0.0                  # one non-zero input: rotated row has constant magnitude
    xf[6] += 40.0
    x = wl.f32_to_bf16_bits(xf)
    for b in (3, 4):
        for variant in (0, 1):
            say(f"asym degenerate b={b} variant={variant}")
            codes, scales, mins, kern = run_asym(torch, x, 128, b, 0.95, variant)
            parity.check_rotate_quantize_asym(x, 128, b, 0.95, codes, scales, mins, f"degenerate [{kern}]")
            assert scales[3, 0] == 0 and mins[3, 0] == 0 and not codes[3].any()
    # padded width
    say("asym d=100 of n=128")
    codes, scales, mins, kern = run_asym(torch, x[:, :100].copy(), 128, 3, 1.0)
    parity.check_rotate_quantize_asym(x[:, :100], 128, 3, 1.0, codes, scales, mins, f"padded [{kern}]")


@pytest.mark.parametrize("name", ["kv_k", "kv_v"])
def test_asym_full_size_kv_sampled(torch, name):
    w = wl.WORKLOADS[name]
    nb = wl.n_blocks(w)
    blocks = [0, 1, 31, nb // 2 + 5, nb - 1]
    say(f"asym full {name} [{w.rows} x {w.d}]: generating")
    x = wl.generate(w)
    b = w.bits[0]
    h = handle(w.n)
    say(f"asym full {name}: launching")
    codes, scales, mins = binding.rotate_quantize_asym(h, parity.to_device(x), b, w.clip)
    torch.cuda.synchronize()
    rows = wl.block_row_index(blocks, w)
    idx = torch.from_numpy(rows).to("cuda")
    st = parity.check_rotate_quantize_asym(x[rows], w.n, b, w.clip, codes[idx].cpu().numpy(),
                                           scales[idx].cpu().numpy(), mins[idx].cpu().numpy(),
                                           f"{name} asym sampled [{h.last_kernel}]")
    say(f"  ok kernel={h.last_kernel} sampled_rows={len(rows)} {st}")


@pytest.mark.parametrize("name,rows", [("tiny", 64), ("llama_hidden", 333), ("qwen_hidden", 100),
                                       ("ffn_down", 19), ("kv_k", 1029)])
@pytest.mark.parametrize("b", [3, 4])
def test_plain_quantize(torch, name, rows, b):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    if x.shape[1] % 32:
        x = np.ascontiguousarray(x[:, : x.shape[1] // 32 * 32])
    say(f"plain {name} rows={rows} d={x.shape[1]} b={b}")
    codes, scales = binding.quantize(parity.to_device(x), b, w.clip)
    torch.cuda.synchronize()
    st = parity.check_quantize_plain(x, b, w.clip, codes.cpu().numpy(), scales.cpu().numpy(), name)
    say(f"  ok {st}")


@pytest.mark.parametrize("d", [32, 64, 96, 128, 160, 256, 288, 512])
@pytest.mark.parametrize("b", [3, 4])
def test_plain_quantize_short_rows(torch, d, b):
    # head rows that arrive rotated: several rows per wave.  Row counts that leave the last pass and
    # the last iteration ragged; bf16 / fp16 values on their coarse grid (rounding ties are common),
    # fp32; an all-zero row; magnitudes at both ends of fp32; a view with a longer leading dimension
    rng = np.random.default_rng(100 * d + b)
    for rows in (1, 5, 67, 1030):
        xf = (rng.standard_t(3, size=(rows, d)) * rng.choice([1e-3, 1.0, 30.0], size=(rows, 1))).astype(np.float32)
        if rows > 4:
            xf[3] = 0.0
            xf[4, : d // 2] = 0.0
        cases = [("bf16", wl.f32_to_bf16_bits(xf)), ("fp16", np.clip(xf, -6e4, 6e4).astype(np.float16)), ("fp32", xf),
                 ("fp32 huge", np.clip(xf, -30, 30) * np.float32(1e37)), ("fp32 small", xf * np.float32(1e-30))]
        for label, xv in cases:
            for clip in (1.0, 0.9):
                say(f"plain short d={d} rows={rows} b={b} {label} clip={clip}")
                codes, scales = binding.quantize(parity.to_device(xv), b, clip)
                torch.cuda.synchronize()
                parity.check_quantize_plain(xv, b, clip, codes.cpu().numpy(), scales.cpu().numpy(),
                                            f"plain short d={d} rows={rows} {label} b={b}")
    xv = wl.f32_to_bf16_bits(rng.standard_normal((77, d)).astype(np.float32))
    buf = torch.zeros((77, d + 40), dtype=torch.bfloat16, device="cuda")
    buf[:, 8:d + 8] = parity.to_device(xv)
    codes, scales = binding.quantize(buf[:, 8:d + 8], b, 0.95)
    torch.cuda.synchronize()
    parity.check_quantize_plain(xv, b, 0.95, codes.cpu().numpy(), scales.cpu().numpy(), f"plain short view d={d}")


@pytest.mark.parametrize("n,rows", [(128, (1 << 20) + 37), (256, (1 << 19) + 11), (512, (1 << 18) + 3)])
def test_short_rows_large_inputs_ragged_end(torch, n, rows):
    # inputs of 2^27 elements and more take eight passes per wave: the first and the last rows (a ragged last
    # wave) against the oracle, symmetric and - for rows of 128 - asymmetric
    rng = np.random.default_rng(n)
    base = wl.f32_to_bf16_bits(rng.standard_t(3.0, size=(4096, n)).astype(np.float32))
    reps = (rows + 4095) // 4096
    x = np.tile(base, (reps, 1))[:rows]
    x[-300:] = wl.f32_to_bf16_bits((rng.standard_normal((300, n)) * 3).astype(np.float32))
    xt = parity.to_device(x)
    h = handle(n)
    pick = np.r_[0:64, rows - 300:rows]
    idx = torch.from_numpy(pick).to("cuda")
    for b in (3, 4):
        say(f"short rows, large input n={n} rows={rows} b={b}")
        codes, scales = binding.rotate_quantize(h, xt, b, 0.9)
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_sylvester"
        parity.check_rotate_quantize(x[pick], n, b, 0.9, codes[idx].cpu().numpy(), scales[idx].cpu().numpy(),
                                     f"large short n={n} b={b}")
        cp, sp = binding.quantize(xt, b, 0.9)              # the rotation-free quantizer's eight-pass launch
        torch.cuda.synchronize()
        parity.check_quantize_plain(x[pick], b, 0.9, cp[idx].cpu().numpy(), sp[idx].cpu().numpy(),
                                    f"large short plain n={n} b={b}")
        del cp, sp
        if n == 128:
            ca, sa, ma = binding.rotate_quantize_asym(h, xt, b, 0.9)
            torch.cuda.synchronize()
            parity.check_rotate_quantize_asym(x[pick], n, b, 0.9, ca[idx].cpu().numpy(), sa[idx].cpu().numpy(),
                                              ma[idx].cpu().numpy(), f"large short asym b={b}")


@pytest.mark.parametrize("b", [3, 4])
def test_plain_quantize_general_kernel(torch, b):
    # what neither the short-row nor the wave kernel takes: fp32 rows wider than 512, rows that do not
    # start on 16 bytes, a leading dimension that is not a multiple of 8, rows wider than 20480
    rng = np.random.default_rng(40 + b)
    xf = (rng.standard_t(3, size=(37, 1024)) * 3).astype(np.float32)
    xf[5] = 0.0
    cases = [("fp32 1024", xf, None), ("fp32 4096", np.tile(xf, (1, 4))[:9], None)]
    xb = wl.f32_to_bf16_bits(xf)
    cases += [("bf16 misaligned", xb[:, :992], (1, 1037)), ("fp16 odd ld", xf[:, :640].astype(np.float16), (0, 645))]
    wide = wl.f32_to_bf16_bits(rng.standard_normal((5, 28672)).astype(np.float32))
    cases += [("bf16 28672", wide, None)]
    cases += [("fp32 huge", np.clip(xf, -30, 30) * np.float32(1e37), None), ("fp32 small", xf * np.float32(1e-30), None),
              ("bf16 huge 4096", wl.f32_to_bf16_bits(np.tile(np.clip(xf, -30, 30) * np.float32(1e37), (1, 4))[:9]), None)]
    for label, xv, view in cases:
        say(f"plain general {label} b={b}")
        if view is None:
            xt = parity.to_device(xv)
        else:
            off, ld = view
            buf = parity.to_device(np.zeros((xv.shape[0], ld), dtype=xv.dtype))
            buf[:, off:off + xv.shape[1]] = parity.to_device(xv)
            xt = buf[:, off:off + xv.shape[1]]
        codes, scales = binding.quantize(xt, b, 0.9)
        torch.cuda.synchronize()
        parity.check_quantize_plain(xv, b, 0.9, codes.cpu().numpy(), scales.cpu().numpy(), f"plain general {label} b={b}")


def test_plain_quantize_views_and_zero_rows(torch):
    rng = np.random.default_rng(6)
    xf = rng.standard_normal((50, 96)).astype(np.float32)
    xf[7] = 0.0
    buf = torch.zeros((50, 160), dtype=torch.float32, device="cuda")
    buf[:, :96] = torch.from_numpy(xf).cuda()
    codes, scales = binding.quantize(buf[:, :96], 4, 0.8)
    torch.cuda.synchronize()
    parity.check_quantize_plain(xf, 4, 0.8, codes.cpu().numpy(), scales.cpu().numpy(), "ld view")
    assert scales[7].item() == 0 and not codes[7].any().item()
    c0, s0 = binding.quantize(buf[:0, :96], 4, 0.8)
    assert c0.shape[0] == 0


@pytest.mark.parametrize("variant", [0, 1], ids=["auto", "general"])
@pytest.mark.parametrize("name,rows,b", [("kv_k", 1029, 3), ("kv_v", 302, 4), ("kv_k", 3, 3), ("llama_hidden", 20, 3),
                                         ("tiny", 64, 4), ("kv_k", 4999, 3)])
def test_quant_error_asym(torch, name, rows, b, variant):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    clips = wl.clip_grid()
    h = handle(w.n)
    h.set_variant(variant)
    say(f"quant_error_asym {name} rows={rows} n={w.n} b={b} variant={variant}")
    mse = binding.quant_error(h, parity.to_device(x), b, clips, asym=True)
    torch.cuda.synchronize()
    h.set_variant(0)
    rel = parity.check_quant_error(x, w.n, b, clips, mse.cpu().numpy(), what=f"{name} [{h.last_kernel}]", asym=True)
    say(f"  ok kernel={h.last_kernel} max rel err {rel:.2e}")
    if variant == 0 and w.n == 128:
        assert h.last_kernel == "wave_quant_error_asym"


def test_gbs_search_asym_follows_algorithm_1(torch):
    import rotq_oracle as oracle
    w = wl.WORKLOADS["kv_k"].with_rows(2000)
    x = wl.generate(w)
    h = handle(w.n)
    clip, mse, trace = binding.gbs_search(h, parity.to_device(x), 3, 1.0 / 64, asym=True)
    m, fm, otrace = oracle.gbs_search(lambda c: oracle.quant_error_asym(x, w.n, 3, [np.float32(c)])[0], 1.0 / 64)
    say(f"gbs asym: clip {clip} after {len(trace)} probes (oracle {m})")
    assert [p for p, _ in trace] == [np.float32(p) for p, _ in otrace]
    assert clip == np.float32(m) and abs(mse - fm) <= 1e-5 * fm


@pytest.mark.parametrize("n,d", [(128, 128), (256, 200), (4096, 4096), (3584, 3584), (3072, 3000), (1544, 1544),
                                 (148 * 128, 148 * 128), (96, 96), (5120, 5120), (44 * 256, 11008),
                                 (36 * 128, 4600), (60 * 128, 60 * 128)])
def test_half_precision_input(torch, n, d):
    # IEEE fp16 rows (the paper's models run in FP16): every entry point that reads X
    rng = np.random.default_rng(n + d)
    x = (rng.standard_t(3.0, size=(37, d)) * 0.7).astype(np.float32)
    x[:, 2] *= 20.0
    x = x.astype(np.float16)
    h = handle(n)
    xt = parity.to_device(x)
    assert xt.dtype == torch.float16
    for b in (3, 4):
        say(f"fp16 n={n} d={d} b={b}")
        codes, scales = binding.rotate_quantize(h, xt, b, 0.9)
        torch.cuda.synchronize()
        st = parity.check_rotate_quantize(x, n, b, 0.9, codes.cpu().numpy(), scales.cpu().numpy(),
                                          f"fp16 n={n} b={b} [{h.last_kernel}]")
        say(f"  ok kernel={h.last_kernel} {st}")
        # the wave kernels take fp16 directly (fp16 matrix-core instruction, fp16 operand tiles)
        want = {128: "wave_sylvester", 4096: "wave_sylvester", 3584: "wave_block", 3072: "wave_block",
                148 * 128: "wg_block", 5120: "wave_block", 44 * 256: "wg_block", 36 * 128: "wave_block",
                60 * 128: "wave_block"}.get(n)
        if want and d % 8 == 0:
            assert h.last_kernel == want
    clips = [0.6, 0.85, 1.0]
    mse = binding.quant_error(h, xt, 3, clips)
    torch.cuda.synchronize()
    parity.check_quant_error(x, n, 3, clips, mse.cpu().numpy(), what=f"fp16 n={n}")
    want = {128: "wave_quant_error", 4096: "wave_quant_error", 3584: "wave_quant_error", 3072: "wave_quant_error",
            148 * 128: "wg_block_quant_error", 5120: "wg_block_quant_error"}.get(n)
    if want and d % 8 == 0:
        assert h.last_kernel == want
    if n == 128:
        mse = binding.quant_error(h, xt, 3, clips, asym=True)
        torch.cuda.synchronize()
        assert h.last_kernel == "wave_quant_error_asym"
        parity.check_quant_error(x, n, 3, clips, mse.cpu().numpy(), what=f"fp16 asym n={n}", asym=True)
    y = binding.rotate(h, xt)
    torch.cuda.synchronize()
    parity.check_float_rows(y.cpu().numpy(), __import__("rotq_oracle").rotate(x, n), what=f"fp16 rotate n={n}")
    if n % 128 == 0:
        codes, scales, mins = binding.rotate_quantize_asym(h, xt, 3, 1.0)
        torch.cuda.synchronize()
        parity.check_rotate_quantize_asym(x, n, 3, 1.0, codes.cpu().numpy(), scales.cpu().numpy(),
                                          mins.cpu().numpy(), f"fp16 asym n={n}")
    if d % 32 == 0:
        codes, scales = binding.quantize(xt, 4, 0.9)
        torch.cuda.synchronize()
        parity.check_quantize_plain(x, 4, 0.9, codes.cpu().numpy(), scales.cpu().numpy(), f"fp16 plain d={d}")


def test_graph_replay_and_side_stream(torch):
    """The hot-path calls allocate nothing and run on the caller's stream: captured in a HIP graph on a
    side stream and replayed several times with eager work in between, every replay must reproduce the
    eager result (codes, scales, mse)."""
    w = wl.WORKLOADS["llama_hidden"].with_rows(300)
    x = parity.to_device(wl.generate(w))
    wk = wl.WORKLOADS["kv_k"].with_rows(1000)
    xk = parity.to_device(wl.generate(wk))
    h, hk = handle(w.n), handle(wk.n)
    clips = [0.6, 0.8, 1.0]
    ref_c, ref_s = binding.rotate_quantize(h, x, 4, 0.9)
    ref_kc, ref_ks, ref_km = binding.rotate_quantize_asym(hk, xk, 3, 0.9)
    ref_m = binding.quant_error(h, x, 3, clips)
    torch.cuda.synchronize()
    codes, scales = torch.empty_like(ref_c), torch.empty_like(ref_s)
    kc, ks, km = torch.empty_like(ref_kc), torch.empty_like(ref_ks), torch.empty_like(ref_km)
    mse = torch.empty_like(ref_m)
    ws = torch.empty(binding.quant_error_workspace(300, 3) // 8, dtype=torch.float64, device="cuda")
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        # warm-up on the side stream, then capture
        binding.rotate_quantize(h, x, 4, 0.9, codes=codes, scales=scales)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=st):
            binding.rotate_quantize(h, x, 4, 0.9, codes=codes, scales=scales)
            binding.rotate_quantize_asym(hk, xk, 3, 0.9, codes=kc, scales=ks, mins=km)
            binding.quant_error(h, x, 3, clips, mse=mse, workspace=ws)
    for rep in range(4):
        for t in (codes, scales, kc, ks, km, mse):
            t.zero_()                                   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        say(f"graph replay {rep}")
        assert torch.equal(codes, ref_c) and torch.equal(scales, ref_s)
        assert torch.equal(kc, ref_kc) and torch.equal(ks, ref_ks) and torch.equal(km, ref_km)
        assert torch.equal(mse, ref_m)


@pytest.mark.parametrize("n,rows,b", [(4096, 77, 4), (4096, 5, 3), (1024, 300, 3), (8192, 9, 4)])
def test_stream_reference_moves_the_stated_bytes(torch, n, rows, b):
    # the measurement aid writes an xor fold of every 16-byte chunk where rotate_quantize writes that
    # chunk's codes: same loads, same stores, checkable bit for bit
    rng = np.random.default_rng(n + rows)
    bits16 = rng.integers(0, 1 << 16, size=(rows, n + 8), dtype=np.uint16)
    xt = parity.to_device(bits16)[:, :n]
    guard = 0xA5
    codes = torch.full((rows + 1, n * b // 8), guard, dtype=torch.uint8, device="cuda")
    scales = torch.zeros((rows,), dtype=torch.float32, device="cuda")
    binding.stream_reference(xt, b, codes=codes[:rows], scales=scales)
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    assert (got[rows] == guard).all()
    words = np.ascontiguousarray(bits16[:, :n]).view(np.uint32).reshape(rows, n // 8, 4)
    fold = words[:, :, 0] ^ words[:, :, 1] ^ words[:, :, 2] ^ words[:, :, 3]
    if b == 3:
        fold = fold.reshape(rows, n // 32, 4)[:, :, :3].reshape(rows, -1)
    assert np.array_equal(got[:rows].view(np.uint32).reshape(rows, -1), fold)


@pytest.mark.parametrize("name", ["llama_hidden", "qwen_hidden"])
def test_full_size_fp16(torch, name):
    # the configuration's rows on the fp16 grid with all 11 mantissa bits in use (the bf16 values
    # jittered by 0.2 %), every row compared: 8 and 15 million codes
    w = wl.WORKLOADS[name]
    xb = wl.generate(w)
    xf = (xb.astype(np.uint32) << 16).view(np.float32)
    rng = np.random.default_rng(5)
    x = np.clip(xf * (1 + rng.uniform(-2e-3, 2e-3, size=xf.shape).astype(np.float32)), -6e4, 6e4).astype(np.float16)
    h = handle(w.n)
    xt = parity.to_device(x)
    b = w.bits[0]
    say(f"full fp16 {name} [{w.rows} x {w.d}] b={b}")
    codes, scales = binding.rotate_quantize(h, xt, b, w.clip)
    torch.cuda.synchronize()
    st = parity.check_rotate_quantize(x, w.n, b, w.clip, codes.cpu().numpy(), scales.cpu().numpy(),
                                      f"{name} fp16 full [{h.last_kernel}]")
    say(f"  ok kernel={h.last_kernel} {st}")


@pytest.mark.parametrize("name,rows", [("kv_v", 1029), ("kv_k", 515), ("llama_hidden", 77), ("ffn_down", 9), ("tiny", 64)])
@pytest.mark.parametrize("b", [3, 4])
def test_plain_quantize_asym(torch, name, rows, b):
    # the asymmetric group-128 quantizer on rows as they are (value cache): bf16, fp16 and fp32 rows,
    # un-rotated values on their coarse grid (rounding ties are common), a view with a leading
    # dimension beyond the width and a misaligned view
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    d = w.d // 128 * 128
    x = np.ascontiguousarray(x[:, :d])
    variants = [("as generated", x)]
    if x.dtype == np.uint16:
        xf = (x.astype(np.uint32) << 16).view(np.float32)
        variants += [("fp16", np.clip(xf, -6e4, 6e4).astype(np.float16)), ("fp32", xf * np.float32(1.0009765625))]
    for label, xv in variants:
        say(f"plain asym {name} rows={rows} d={d} b={b} {label}")
        codes, scales, mins = binding.quantize_asym(parity.to_device(xv), b, 0.9)
        torch.cuda.synchronize()
        st = parity.check_rotate_quantize_asym(xv, d, b, 0.9, codes.cpu().numpy(), scales.cpu().numpy(),
                                               mins.cpu().numpy(), f"plain asym {name} {label} b={b}", rotate=False)
        say(f"  ok {st}")
    # leading dimension beyond d, and a row start that is not 16-byte aligned
    pad = np.zeros((rows, d + 9), dtype=x.dtype)
    pad[:, 1:d + 1] = x
    xt = parity.to_device(pad)[:, 1:d + 1]
    codes, scales, mins = binding.quantize_asym(xt, b, 1.0)
    torch.cuda.synchronize()
    parity.check_rotate_quantize_asym(x, d, b, 1.0, codes.cpu().numpy(), scales.cpu().numpy(), mins.cpu().numpy(),
                                      f"plain asym {name} view b={b}", rotate=False)


@pytest.mark.parametrize("b", [3, 4])
def test_plain_quantize_asym_groups_far_from_zero(torch, b):
    # groups whose offset is large against their range: fp32 cannot place the centre of such a group
    # to within the tie window, so these have to reach the exact quotient; also values at the edge of
    # the formats' ranges
    rng = np.random.default_rng(5 + b)
    base = rng.standard_normal((257, 384)).astype(np.float32)
    off = np.repeat(rng.choice([-1.0, 1.0], size=(257, 3)) * 10.0 ** rng.uniform(0, 4, size=(257, 3)), 128, axis=1)
    spread = np.repeat(10.0 ** rng.uniform(-3, 0, size=(257, 3)), 128, axis=1)
    xf = (off + off * spread * base * 0.1).astype(np.float32)
    cases = [("fp32", xf), ("bf16", wl.f32_to_bf16_bits(xf)), ("fp16", np.clip(xf, -6e4, 6e4).astype(np.float16))]
    big = (base * np.float32(6e37)).astype(np.float32)          # max - min beyond fp32 in some groups
    assert np.isfinite(big).all() and (big.max(axis=1) - big.min(axis=1) == np.inf).any()
    cases += [("fp32 huge", big), ("bf16 huge", wl.f32_to_bf16_bits(big)),
              ("fp32 small", (base * np.float32(1e-30)).astype(np.float32))]
    for label, xv in cases:
        for clip in (1.0, 0.85):
            say(f"plain asym offset groups {label} b={b} clip={clip}")
            codes, scales, mins = binding.quantize_asym(parity.to_device(xv), b, clip)
            torch.cuda.synchronize()
            st = parity.check_rotate_quantize_asym(xv, 384, b, clip, codes.cpu().numpy(), scales.cpu().numpy(),
                                                   mins.cpu().numpy(), f"plain asym offset {label} b={b}", rotate=False)
            say(f"  ok {st}")


def test_plain_quantize_asym_flat_groups_and_round_trip(torch):
    rng = np.random.default_rng(11)
    xf = rng.standard_normal((33, 256)).astype(np.float32)
    xf[3, :128] = 2.5                      # a constant group: Delta = 0, codes 0, lo = clip * value
    xf[4] = 0.0
    x = wl.f32_to_bf16_bits(xf)
    codes, scales, mins = binding.quantize_asym(parity.to_device(x), 4, 1.0)
    torch.cuda.synchronize()
    parity.check_rotate_quantize_asym(x, 256, 4, 1.0, codes.cpu().numpy(), scales.cpu().numpy(), mins.cpu().numpy(),
                                      "plain asym flat", rotate=False)
    s, m = scales.cpu().numpy(), mins.cpu().numpy()
    assert s[3, 0] == 0 and m[3, 0] == 2.5 and s[4, 0] == 0 and m[4, 1] == 0
    # zero rows: nothing written
    binding.quantize_asym(parity.to_device(x)[:0], 4, 1.0)
