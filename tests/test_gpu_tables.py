"""GPU: preprocessing tables and tile classes are bit-exact vs the oracle."""
import numpy as np
import pytest
import torch

import workloads
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu

KINDS = ["full", "causal", "sliding_window", "document", "causal_document", "shared_question", "prefix_lm",
         "prefix_document", "global_sliding_window", "causal_blockwise", "random_eviction", "qk_sparse", "random_intervals"]


def _tables_equal(vecs_np, N, block_r, block_c):
    import paper_2410_01359_amd as fm
    dev = [torch.from_numpy(np.stack(v).astype(np.int32)).cuda() for v in zip(*vecs_np)]
    mm = fm.flashmask_preprocess(*dev, block_c)
    cls = fm.flashmask_classify(mm, N, block_r, block_c)
    torch.cuda.synchronize()
    mm, cls = mm.cpu().numpy(), cls.cpu().numpy()
    for b, v in enumerate(vecs_np):
        want = orc.minmax_tables(*v, block_c)
        assert np.array_equal(mm[b], want), f"min/max table differs (batch row {b})"
        assert np.array_equal(cls[b], orc.classify_tiles_fast(want, N, block_r, block_c)), f"classes differ (row {b})"


@pytest.mark.parametrize("kind", KINDS)
def test_tables_small_all_families(kind):
    for N, br, bc in ((256, 64, 32), (300, 32, 64), (1000, 128, 96)):   # ragged row and column tails too
        vecs = [workloads.small_workload(kind, N, seed=s).vectors[0] for s in (1, 2, 3)]
        _tables_equal(vecs, N, br, bc)


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_tables_at_config_sizes_and_kernel_tile_shapes(name):
    import paper_2410_01359_amd as fm
    w = workloads.config(name)
    for p in (fm.FM_PASS_FWD, fm.FM_PASS_BWD_DKDV, fm.FM_PASS_BWD_DQ):
        br, bc = fm.flashmask_tile_shape(p, w.d)
        _tables_equal(w.vectors, w.N, br, bc)
    _tables_equal(w.vectors, w.N, 128, 128)


def _check_unit_queues(w, pass_id):
    """Invariants of the tile scheduler's output (the library's own addition to the method):
    every unit exactly once, live ranges as Equation 4 gives them, queue membership by head,
    a queue's slices in groups, and within a group heavy units first and by falling work."""
    import paper_2410_01359_amd as fm
    vecs = tuple(torch.from_numpy(x).cuda() for x in w.stacked_vectors())
    rec = fm.flashmask_unit_queues(pass_id, *vecs, w.H, w.d)
    torch.cuda.synchronize()
    rec = rec.cpu().numpy()
    br, bc = fm.flashmask_tile_shape(pass_id, w.d)
    rows = pass_id != fm.FM_PASS_BWD_DKDV
    T = w.N // (br if rows else bc)
    units = w.B * w.H * T
    assert rec.shape[0] % 8 == 0 and rec.shape[0] >= units
    ids = rec[:, 0]
    assert np.array_equal(np.sort(ids[ids >= 0]), np.arange(units)), "every unit exactly once"
    assert np.all(rec[ids < 0, 1:] == 0) and np.all(rec[:, 3] == 0)
    # live range and work of every unit from the oracle's tile classes
    lo_ref, hi_ref, work_ref = (np.zeros((w.B, T), dtype=np.int64) for _ in range(3))
    for b, v in enumerate(w.vectors):
        live = orc.tile_kind(orc.classify_tiles_fast(orc.minmax_tables(*v, bc), w.N, br, bc)) != orc.FULLY
        live = live if rows else live.T                     # [unit block, scanned block]
        work_ref[b] = live.sum(axis=1)
        any_live = work_ref[b] > 0
        lo_ref[b] = np.where(any_live, live.argmax(axis=1), 0)
        hi_ref[b] = np.where(any_live, live.shape[1] - live[:, ::-1].argmax(axis=1), 0)
    slot = np.nonzero(ids >= 0)[0]
    u = ids[slot].astype(np.int64)
    bh, blk = u // T, u % T
    b = bh // w.H
    assert np.array_equal(rec[slot, 1], lo_ref[b, blk]) and np.array_equal(rec[slot, 2], hi_ref[b, blk])
    # Queue of every unit: slices (batch row, head) go to queues whole, slice s to queue s % 8, while they
    # fill rounds of 8; the r slices left over are shared block by block, four of them between 2 queues
    # each, two between 4 queues each, one between all 8 (r = 4a + 2b + c).
    slices = w.B * w.H
    whole, r = slices // 8 * 8, slices % 8
    j = bh - whole
    in4 = (r & 4 != 0) & (j < 4)
    j2 = j - (4 if r & 4 else 0)
    in2 = ~in4 & (r & 2 != 0) & (j2 >= 0) & (j2 < 2)
    shared_q = np.where(in4, 2 * j + (blk & 1), np.where(in2, 4 * j2 + (blk & 3), blk & 7))
    assert np.array_equal(slot % 8, np.where(bh < whole, bh % 8, shared_q)), "queue of every unit"
    max_work = w.N // (bc if rows else br)
    chunk = 2                      # whole slices of a queue that are ranked together (FM_QUEUE_CHUNK)
    n_groups = -(-(whole // 8) // chunk)
    group = np.where(bh < whole, (bh // 8) // chunk, n_groups)     # the shared slices form the last group
    for q in range(8):
        in_q = slot % 8 == q
        pos = slot[in_q] // 8
        order_q = np.argsort(pos)
        pos, work_q, group_q = pos[order_q], work_ref[b[in_q], blk[in_q]][order_q], group[in_q][order_q]
        assert np.array_equal(pos, np.arange(pos.size)), "a queue has no holes"
        assert np.all(np.diff(group_q) >= 0), "a queue's groups of slices, one after the other"
        whole_q = group_q < n_groups
        assert np.array_equal(pos[whole_q] // (chunk * T), group_q[whole_q])
        for sg in np.unique(group_q):
            work = work_q[group_q == sg]
            heavy = work * 8 >= max_work
            if heavy.any():
                assert not heavy[np.argmin(heavy):].any() or heavy.all(), "heavy units come first"
                hw = work[heavy]
                level = max(1, -(-7 * max_work // (8 * 383)))   # work span of one of the 384 fine ranks
                assert np.all(hw[:-1] + level >= hw[1:]), "heavy units by falling work (to the rank's resolution)"
            light = work[~heavy]
            if light.size:
                octave = np.floor(np.log2(max_work / (8.0 * np.maximum(light, 1)))).clip(0, 7)
                assert np.all(np.diff(octave) >= 0), "lighter units by falling octave of work"


@pytest.mark.parametrize("name", ["1", "2", "3", "4a", "4b", "5"])
def test_unit_queues_at_config_sizes(name):
    import paper_2410_01359_amd as fm
    w = workloads.config(name)
    for p in (fm.FM_PASS_FWD, fm.FM_PASS_BWD_DQ, fm.FM_PASS_BWD_DKDV):
        _check_unit_queues(w, p)


@pytest.mark.parametrize("kind", ["full", "document", "random_intervals", "global_sliding_window"])
def test_unit_queues_small_families(kind):
    import paper_2410_01359_amd as fm
    w = workloads.small_workload(kind, 1536, seed=11, B=3, H=5, d=64)    # B * H not a multiple of 8
    for p in (fm.FM_PASS_FWD, fm.FM_PASS_BWD_DQ, fm.FM_PASS_BWD_DKDV):
        _check_unit_queues(w, p)


@pytest.mark.parametrize("B,H,N", [(5, 8, 2048), (3, 16, 2048), (1, 8, 2048), (1, 1, 1152), (1, 2, 1152), (3, 1, 1152),
                                   (1, 4, 1152), (5, 1, 1152), (2, 3, 1152), (1, 7, 1152), (3, 5, 1152), (1, 12, 2048),
                                   (23, 1, 384), (3, 20, 640)])
def test_unit_queues_many_slices(B, H, N):
    """Slice counts that give a queue several groups of whole slices (the last one partial) and every
    number of shared slices, with block counts that do not divide by the sharing."""
    import paper_2410_01359_amd as fm
    w = workloads.small_workload("causal_document", N, seed=13, B=B, H=H, d=128)
    for p in (fm.FM_PASS_FWD, fm.FM_PASS_BWD_DQ, fm.FM_PASS_BWD_DKDV):
        _check_unit_queues(w, p)
