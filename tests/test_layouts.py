"""Host-side checks of the library's internal memory layouts (no GPU needed): the tiled weight order,
the step-major activation order and the tiled value cache are bijections with the contiguity the
kernels rely on (one contiguous KiB per MFMA operand load)."""
import numpy as np
import pytest

from paper_2505_08600_amd import api


def test_tiled_weight_order_is_a_bijection_with_contiguous_operand_loads():
    N, K = 48, 384
    idx = np.array([[api.layout_index(0, n, k, K) for k in range(K)] for n in range(N)])
    assert sorted(idx.ravel().tolist()) == list(range(N * K))
    # one 16-row x 128-column step of a tile is 2048 contiguous elements; tiles of a row block follow along K
    for nt in range(N // 16):
        for ks in range(K // 128):
            blk = idx[nt * 16:(nt + 1) * 16, ks * 128:(ks + 1) * 128]
            base = (nt * (K // 128) + ks) * 2048
            assert blk.min() == base and blk.max() == base + 2047
            # load instruction i of a wave: lane 16*g + r holds row r, columns 32*i + 8*g .. +8, at 8 * lane
            for i in range(4):
                for g in range(4):
                    for r in range(16):
                        got = blk[r, 32 * i + 8 * g: 32 * i + 8 * g + 8]
                        want = base + i * 512 + (16 * g + r) * 8 + np.arange(8)
                        assert np.array_equal(got, want)
    assert api.layout_index(0, 0, 0, 100) == -1  # K must be a multiple of 128


def test_step_major_activation_order():
    rows, K = 7, 256
    idx = np.array([[api.layout_index(1, m, k, K, rows) for k in range(K)] for m in range(rows)])
    assert sorted(idx.ravel().tolist()) == list(range(rows * K))
    for m in range(rows):
        for ks in range(K // 128):
            seg = idx[m, ks * 128:(ks + 1) * 128]
            assert np.array_equal(seg, (ks * rows + m) * 128 + np.arange(128))  # rows of a step are adjacent
    assert api.layout_index(1, rows, 0, K, rows) == -1


@pytest.mark.parametrize("hd", [64, 128])
def test_value_cache_tiles(hd):
    T = 96
    idx = np.array([[api.layout_index(2, t, d, hd) for d in range(hd)] for t in range(T)])
    assert sorted(idx.ravel().tolist()) == list(range(T * hd))
    for tile in range(T // 32):
        blk = idx[tile * 32:(tile + 1) * 32]  # [token][dim]
        assert blk.min() == tile * 32 * hd and blk.max() == (tile + 1) * 32 * hd - 1
        # transposed inside the tile: 32 tokens of one dimension are contiguous
        for d in range(hd):
            assert np.array_equal(blk[:, d], tile * 32 * hd + d * 32 + np.arange(32))


@pytest.mark.parametrize("hd", [16, 32, 64, 128])
def test_key_cache_tiles_are_in_score_operand_order(hd):
    T = 64
    idx = np.array([[api.layout_index(3, t, d, hd) for d in range(hd)] for t in range(T)])
    assert sorted(idx.ravel().tolist()) == list(range(T * hd))
    G = min(hd, 32) // 8
    for tile in range(T // 32):
        base = tile * 32 * hd
        for c in range(max(1, hd // 32)):
            for ab in range(2):
                for g in range(G):
                    for i in range(16):
                        tok = 8 * (i // 4) + i % 4 + 4 * ab  # token held by row i of score operand a / b
                        got = idx[tile * 32 + tok, 32 * c + 8 * g: 32 * c + 8 * g + 8]
                        want = base + (((2 * c + ab) * G + g) * 16 + i) * 8 + np.arange(8)
                        assert np.array_equal(got, want)
