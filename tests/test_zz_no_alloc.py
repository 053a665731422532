"""rq_quant_error_noalloc (the entry point for callers that cannot allocate device memory) against
rq_quant_error and the oracle: two calls in a row through the C ABI, the second on a smaller input,
so that whatever the first call left in the library's static scratch array is still there."""
import sys

import numpy as np
import pytest

import parity
from paper_2504_13989_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[noalloc] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _one_call(torch, h, name, rows, b, clips):
    w = wl.WORKLOADS[name].with_rows(rows)
    x = wl.generate(w)
    xt = parity.to_device(x)
    mse = torch.full((len(clips),), -1.0, dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    say(f"quant_error_noalloc {name} rows={rows} n={w.n} b={b} clips={len(clips)}")
    binding.quant_error_noalloc(h, xt, b, clips, mse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    kernel = h.last_kernel
    ref = binding.quant_error(h, xt, b, clips)
    torch.cuda.synchronize()
    assert h.last_kernel == kernel
    # same kernels, same fixed reduction order: the two entry points agree bit for bit
    assert np.array_equal(mse.cpu().numpy(), ref.cpu().numpy()), f"{name} rows={rows}: differs from rq_quant_error"
    rel = parity.check_quant_error(x, w.n, b, clips, mse.cpu().numpy(), what=f"{name} noalloc [{kernel}]")
    say(f"  ok kernel={kernel} max rel err {rel:.2e}")


@pytest.mark.parametrize("name,first,second,b", [("calib", 512, 77, 3), ("kv_k", 5003, 300, 3), ("qwen_hidden", 60, 7, 4),
                                                 ("ffn_down", 9, 2, 3), ("tiny", 64, 5, 3)])
def test_two_calls_in_a_row_second_smaller(torch, name, first, second, b):
    h = binding.hadamard_build(wl.WORKLOADS[name].n)
    clips = wl.clip_grid()
    _one_call(torch, h, name, first, b, clips)
    _one_call(torch, h, name, second, b, clips[:5])
    h.close()


def test_limit_and_empty_input(torch):
    h = binding.hadamard_build(128)
    clips = wl.clip_grid()
    rows = binding.RQ_NOALLOC_SCRATCH_BYTES // 8 // len(clips)
    x = torch.zeros((rows + 1, 128), dtype=torch.bfloat16, device="cuda")
    mse = torch.full((len(clips),), -1.0, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.RotqError) as e:
        binding.quant_error_noalloc(h, x, 3, clips, mse)
    assert e.value.code == binding.RQ_ERR_TOO_LARGE
    assert float(mse.min()) == -1.0                         # refused before anything ran
    binding.quant_error_noalloc(h, x[:rows], 3, clips, mse)  # exactly at the limit: all-zero rows, zero error
    torch.cuda.synchronize()
    assert float(mse.abs().max()) == 0.0
    mse.fill_(-1.0)
    binding.quant_error_noalloc(h, x[:0], 3, clips, mse)     # no rows: zeros
    torch.cuda.synchronize()
    assert float(mse.abs().max()) == 0.0
    h.close()
