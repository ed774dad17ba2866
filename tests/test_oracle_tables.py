"""Pins for the min/max tables, tile classes, sparsity and FLOP counters (no GPU)."""
import os

import numpy as np
import pytest

import workloads
from oracle import flashmask_oracle as orc
from predicates import PREDICATES

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KINDS = sorted(PREDICATES) + ["random_intervals"]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n,bc", [(37, 8), (64, 16), (50, 64)])
def test_minmax_tables_brute_force(kind, n, bc):
    w = workloads.small_workload(kind, n, seed=n + bc)
    vec = w.vectors[0]
    t = orc.minmax_tables(*vec, bc)
    t_c = -(-n // bc)
    assert t.shape == (8, t_c) and t.dtype == np.int32
    for j in range(t_c):
        for a in range(4):
            block = np.asarray(vec[a])[j * bc:(j + 1) * bc]
            assert t[2 * a, j] == block.max() and t[2 * a + 1, j] == block.min()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n,br,bc", [(64, 8, 8), (61, 16, 8), (96, 32, 16), (40, 8, 64)])
def test_tile_classes_are_sound_and_fast_path_agrees(kind, n, br, bc):
    for seed in range(3):
        w = workloads.small_workload(kind, n, seed=100 * seed + n)
        vec = w.vectors[0]
        table = orc.minmax_tables(*vec, bc)
        cls = orc.classify_tiles(table, n, br, bc)
        assert np.array_equal(cls, orc.classify_tiles_fast(table, n, br, bc))
        masked = orc.expand_mask(*vec)
        lt_only = orc.expand_mask(vec[0], vec[1], np.zeros(n), np.zeros(n))
        ut_only = orc.expand_mask(np.zeros(n), np.zeros(n), vec[2], vec[3])
        for i in range(cls.shape[0]):
            for j in range(cls.shape[1]):
                tile = (slice(i * br, min((i + 1) * br, n)), slice(j * bc, min((j + 1) * bc, n)))
                kind_ = cls[i, j] & 3
                if kind_ == orc.FULLY:
                    assert masked[tile].all()
                    assert cls[i, j] == orc.FULLY
                elif kind_ == orc.UNMASKED:
                    assert not masked[tile].any()
                    assert cls[i, j] == orc.UNMASKED
                else:
                    assert cls[i, j] & (orc.NEED_LT | orc.NEED_UT)
                    # a pair whose NEED bit is clear masks nothing inside the tile
                    if not cls[i, j] & orc.NEED_LT:
                        assert not lt_only[tile].any()
                    if not cls[i, j] & orc.NEED_UT:
                        assert not ut_only[tile].any()


def test_causal_classes_are_the_textbook_triangle():
    n, b = 64, 8
    cls = orc.classify_tiles(orc.minmax_tables(*workloads.causal_mask(n), b), n, b, b)
    for i in range(n // b):
        for j in range(n // b):
            want = orc.UNMASKED if j < i else (orc.PARTIAL | orc.NEED_UT if j == i else orc.FULLY)
            assert cls[i, j] == want


def _golden_rows():
    rows = []
    for line in open(os.path.join(GOLDEN, "paper_kernel_table_d128.txt")):
        if line.startswith("#") or not line.strip():
            continue
        mask, n, bh, fw, bw, rho = line.split()
        rows.append((mask, int(n), int(bh), float(fw), float(bw), float(rho)))
    return rows


def _eviction_times(n):
    """Every other key (at random) is evicted at a random later row, the rest never: no 128-key block is
    ever evicted as a whole, which is what the printed Random Eviction rows (equal to Causal) imply."""
    rng = np.random.Generator(np.random.PCG64(n))
    return np.where(rng.random(n) < 0.5, n, np.arange(n) + 1 + rng.integers(0, n, size=n))


@pytest.mark.parametrize("mask,n,bh,fw,bw,rho", _golden_rows())
def test_paper_printed_sparsity_and_tflops(mask, n, bh, fw, bw, rho):
    """Tile counter + FLOP model reproduce the figures printed in the paper's
    kernel tables for the deterministic masks (128x128 accounting tiles)."""
    vec = {"full": lambda: workloads.full_mask(n),
           "causal": lambda: workloads.causal_mask(n),
           "sliding_window": lambda: workloads.sliding_window_mask(n, n // 16),
           "prefix_lm": lambda: workloads.prefix_lm_mask(n, n // 2),
           "global_sliding_window": lambda: workloads.global_sliding_window_mask(n, 128, n // 16),
           "random_eviction": lambda: workloads.random_eviction_mask(n, _eviction_times(n))}[mask]()
    cls = orc.classify_tiles_fast(orc.minmax_tables(*vec, 128), n, 128, 128)
    got_rho = orc.block_sparsity(cls)
    assert abs(got_rho - rho) <= 0.0051, (got_rho, rho)
    got_fw, got_bw = orc.flops_tile(cls, bh, 128)
    assert abs(got_fw / 1e12 - fw) <= 0.0101, (got_fw / 1e12, fw)
    assert abs(got_bw / 1e12 - bw) <= 0.0151, (got_bw / 1e12, bw)


@pytest.mark.parametrize("mask,n,bh,fw,bw,rho", [r for r in _golden_rows() if r[0] == "full"])
def test_elementwise_flop_model_reproduces_printed_full_mask_rows(mask, n, bh, fw, bw, rho):
    """flops_elem (the headline's numerator) on the Full mask, where every element is unmasked, must
    give the FW / BW TFLOPs the paper prints for its Full rows (d = 128 kernel tables): 17.59 / 43.98,
    70.37 / 175.92, 281.48 / 703.69 (printed to two decimals; 281.47 computed)."""
    vec = workloads.full_mask(n)
    unmasked = orc.count_unmasked_elements(*vec)
    assert unmasked == n * n
    got_fw, got_bw = orc.flops_elem(unmasked, bh, 128)
    assert abs(got_fw / 1e12 - fw) <= 0.0101, (got_fw / 1e12, fw)
    assert abs(got_bw / 1e12 - bw) <= 0.0151, (got_bw / 1e12, bw)
    assert got_bw == 2.5 * got_fw


def test_elementwise_flops_equal_tile_flops_where_no_tile_is_partial():
    """A mask whose boundaries all fall on multiples of 128 has no partially masked tile, so the
    element count and the tile count of the FLOP model agree exactly."""
    n = 2048
    vec = workloads.document_mask(n, workloads.spans_from_lengths([512, 256, 1024, 256]))
    cls = orc.classify_tiles(orc.minmax_tables(*vec, 128), n, 128, 128)
    assert not ((cls & 3) == orc.PARTIAL).any()
    assert orc.flops_elem(orc.count_unmasked_elements(*vec), 3, 128) == orc.flops_tile(cls, 3, 128)
    assert orc.count_unmasked_elements(*vec) == 512 ** 2 + 2 * 256 ** 2 + 1024 ** 2


def test_elementwise_flops_never_exceed_tile_flops():
    for name in ("4a", "4b"):
        w = workloads.config(name)
        vec = w.vectors[0]
        cls = orc.classify_tiles_fast(orc.minmax_tables(*vec, 128), w.N, 128, 128)
        f_tile, _ = orc.flops_tile(cls, w.B * w.H, w.d)
        f_elem, _ = orc.flops_elem(orc.count_unmasked_elements(*vec), w.B * w.H, w.d)
        assert f_elem <= f_tile
    # sliding window 1024 at N = 32768: 2268 live tiles of 65536
    w = workloads.config("4a")
    cls = orc.classify_tiles_fast(orc.minmax_tables(*w.vectors[0], 128), w.N, 128, 128)
    assert int(((cls & 3) != orc.FULLY).sum()) == 2268
