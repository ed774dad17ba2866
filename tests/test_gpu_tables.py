"""GPU: preprocessing tables and tile classes are bit-exact vs the oracle."""
import numpy as np
import pytest
import torch

import workloads
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu

KINDS = ["full", "causal", "sliding_window", "document", "causal_document", "shared_question", "prefix_lm",
         "prefix_document", "global_sliding_window", "causal_blockwise", "random_eviction", "random_intervals"]


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
