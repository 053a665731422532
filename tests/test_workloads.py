"""CPU-only: the seeded input generators (shapes, determinism, bf16 rounding, structure)."""
import numpy as np

from paper_2504_13989_amd import workloads as wl


def test_bf16_rounding_ties_to_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is exactly halfway between bf16 1.0 (even) and 1.0078125 -> 1.0
    # 1.01171875 = 1 + 3*2^-8 is halfway between 1.0078125 (odd) and 1.015625 (even) -> 1.015625
    bits = wl.f32_to_bf16_bits(x)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert abs(back[4] - 3.0e38) / 3.0e38 < 2 ** -8


def test_shapes_and_determinism():
    for name in ("tiny", "calib"):
        w = wl.WORKLOADS[name]
        a = wl.generate(w)
        b = wl.generate(w)
        assert a.shape == (w.rows, w.d)
        assert a.dtype == (np.float32 if w.dtype == "f32" else np.uint16)
        assert np.array_equal(a, b)
    w = wl.WORKLOADS["llama_hidden"]
    blk = wl.generate_blocks(w, [3, 5])
    assert blk.shape == (2 * wl.BLOCK_ROWS, w.d)
    assert np.array_equal(wl.block_row_index([3, 5], w)[:2], [3 * wl.BLOCK_ROWS, 3 * wl.BLOCK_ROWS + 1])
    assert np.array_equal(blk[:wl.BLOCK_ROWS], wl.generate_blocks(w, [3]))


def test_outlier_structure():
    w = wl.WORKLOADS["tiny"]
    x = wl.generate(w)
    rms = np.sqrt((x.astype(np.float64) ** 2).mean(axis=0))
    assert (rms > 10).sum() == w.n_outlier_ch
    w = wl.WORKLOADS["calib"]
    x = (wl.generate(w).astype(np.uint32) << 16).view(np.float32)
    row_med = np.median(np.abs(x), axis=1)
    assert (row_med > 100 * np.median(row_med)).sum() == w.n_massive_rows


def test_kv_rows_and_clip_grid():
    w = wl.WORKLOADS["kv_k"]
    assert w.rows == 16 * 32 * 8192 and w.d == 128
    blk = wl.generate_blocks(w, [0, wl.n_blocks(w) - 1])
    assert blk.shape == (2 * wl.BLOCK_ROWS, 128)
    g = wl.clip_grid()
    assert g.dtype == np.float32 and len(g) == 32 and g[0] == 0.5 and g[-1] == 1.0
    assert np.all(np.diff(g) > 0)


def test_kv_rows_not_a_multiple_of_the_head_length():
    # a row count that ends inside a head still has outlier channels for that head
    w = wl.WORKLOADS["kv_k"].with_rows(8192 * 2 + 300)
    x = wl.generate(w)
    assert x.shape == (8192 * 2 + 300, 128)
    full = wl.generate(wl.WORKLOADS["kv_k"].with_rows(8192 * 3))
    assert np.array_equal(x[: 8192 * 2], full[: 8192 * 2])      # earlier heads do not depend on the row count
