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


def test_row_blocked_gemm_plans_fit_the_busiest_die_in_one_round():
    """The launch plan of the row-blocked GEMM (host logic only).  Column tile t of a launch runs on die t mod 8 with
    all its row blocks and K splits, so the busiest die carries ceil(tiles / 8) * row blocks * splits blocks; K is
    split only as far as that die's 32 compute units (64 resident blocks for the 48-row shape) take in one round -
    counted over the whole chip instead, the 20 wide tiles of a 5120-wide projection would put 36 blocks on four
    dies.  Blocks cover the matrix, plain projections with few column tiles take the 128-column shape, and the shapes
    of the measured configurations keep the plans they were measured with."""
    for d, f in ((4096, 11008), (5120, 13824), (8192, 28672), (2048, 5632)):
        for m in list(range(33, 200, 7)) + [256, 288, 384, 512, 576, 640, 768, 1024, 2048]:
            for mode, n, k, seg in ((0, 3 * d, d, d), (0, d, d, d), (2, f, d, f), (0, d, f, d), (0, 32000, d, 32000)):
                plan = api.gemm_plan(mode, m, n, k, seg)
                assert plan is not None, (d, m, mode, n, k)
                cols, bm, ncol, nmb, ks, die = plan
                assert cols in (128, 192, 256) and bm in (48, 64, 96) and 1 <= ks <= 8
                assert ncol * cols >= n * (2 if mode == 2 else 1) > (ncol - 1) * cols
                assert nmb * bm >= m > (nmb - 1) * bm
                assert die == -(-ncol // 8) * nmb * ks
                if mode == 2:
                    assert ks == 1          # silu(gate) * up needs complete sums
                per_die = 64 if bm == 48 else 32
                if ks > 1:
                    # one round on the busiest die - unless not even the unsplit launch fits one round
                    assert die <= per_die or -(-ncol // 8) * nmb > per_die, (d, m, mode, n, k, plan)
                    assert k // 128 // ks >= 3      # no split shorter than about four K steps
    assert api.gemm_plan(0, 32, 4096, 4096) is None and api.gemm_plan(0, 192, 4096, 4000) is None
    # the shapes of config 3 (7B, M = 192) and config 4 (13B, M = 128 / 192 / 288)
    assert api.gemm_plan(0, 192, 4096, 4096) == (128, 96, 32, 2, 4, 32)         # O: 4 splits of 8 steps, not 8 of 4
    assert api.gemm_plan(0, 192, 4096, 11008) == (256, 96, 16, 2, 8, 32)        # down: the wide blocks
    assert api.gemm_plan(0, 192, 12288, 4096, 4096) == (192, 96, 64, 2, 2, 32)  # QKV
    assert api.gemm_plan(2, 192, 11008, 4096) == (192, 96, 115, 2, 1, 30)       # gate/up
    assert api.gemm_plan(0, 192, 5120, 13824)[4:] == (5, 30)                    # 20 tiles: 3 on a die, so 5 splits, not 6
    assert api.gemm_plan(0, 192, 5120, 5120)[0] == 128 and api.gemm_plan(0, 288, 5120, 13824)[0] == 128
    assert api.gemm_plan(0, 96, 4096, 11008)[:1] + api.gemm_plan(0, 96, 4096, 11008)[4:] == (128, 8, 32)   # M <= 96: twice the blocks
    # config 5 (7B, M = 576): the unsplit QKV launch is one and a half rounds, two splits make three full ones
    assert api.gemm_plan(0, 576, 12288, 4096, 4096) == (192, 96, 64, 6, 2, 96)
    assert api.gemm_plan(0, 768, 12288, 4096, 4096)[4] == 1 and api.gemm_plan(0, 1024, 12288, 4096, 4096)[4] == 1   # whole rounds: no split
