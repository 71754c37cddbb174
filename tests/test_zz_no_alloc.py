"""The selection entry point that allocates nothing (its scratch is a static device array)
against the ordinary one, through the C ABI: ids and scores bit for bit, on two calls in a
row, the second on a smaller input (the shared array then still holds the first call's
scores, histogram state and chunk counts)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import DEV, GpuRun, dev_f32
from paper_2405_14852_amd import PVError

pytestmark = pytest.mark.gpu


def _both(run, T, W, k, want_scores):
    N = run.lay.num_groups
    out = []
    for name in ("pv_select_topk_groups", "pv_select_topk_groups_noalloc"):
        idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device=DEV)
        sc = torch.full((N,), -1.0, dtype=torch.float32, device=DEV) if want_scores else None
        getattr(run.ctx, name)(run.lay, T, W, k, idx, sc)
        torch.cuda.synchronize()
        out.append((idx[:k].cpu().numpy(), None if sc is None else sc.cpu().numpy()))
    return out


@pytest.mark.parametrize("want_scores", [False, True])
def test_noalloc_selection_equals_the_ordinary_one_twice_in_a_row(want_scores):
    shapes = [((512, 4096), 8, 0.05), ((96, 1000), 4, 0.3)]      # the second is smaller and ragged
    for (o, i), g, tau in shapes:
        wl = workloads.make(o, i, g, 1, 8, seed=3, sigma_g=1e-3, tau=tau)
        run = GpuRun(wl)
        T = run.targets()
        (ref_idx, ref_sc), (got_idx, got_sc) = _both(run, T, run.W, wl.k, want_scores)
        assert len(got_idx) == wl.k and np.array_equal(got_idx, ref_idx)
        if want_scores:
            assert np.array_equal(got_sc.view(np.uint32), ref_sc.view(np.uint32))
    # planted ties across the threshold and k = N, k = 1, k = 0 on the small shape
    Tt = run.W.clone()
    Tt[::3] += 1.0
    for k in (run.lay.num_groups, 1, 0, 1234):
        (ref_idx, _), (got_idx, _) = _both(run, Tt, run.W, k, False)
        assert np.array_equal(got_idx, ref_idx)


def test_noalloc_selection_rejects_sizes_beyond_its_static_array():
    wl = workloads.make(8, 64, 8, 1, 4, seed=1)
    run = GpuRun(wl)
    big = type(run.lay)(4096, 8200, 8, 1, 4)         # 4 198 400 groups > 4 194 304
    idx = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(PVError) as e:
        run.ctx.pv_select_topk_groups_noalloc(big, run.W, run.W, 1, idx)
    assert e.value.status == 3 and "static" in str(e.value)
