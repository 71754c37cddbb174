"""GPU parity of the scalar uniform-grid representation (App. K): dequantise and the
round-to-nearest V step, bit-exact against the CPU oracle, with targets and selection taken
through the ordinary calls at group size 1."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DEV, dev_f32, dev_i32
from paper_2405_14852_amd import Layout, PVContext, PVError

pytestmark = pytest.mark.gpu


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(DEV)


@pytest.mark.parametrize("shape,block,nbits", [((64, 512), 128, 2), ((33, 96), 16, 3), ((7, 60), 6, 4),
                                               ((16, 256), 8, 8), ((5, 7), 7, 1)])
@pytest.mark.parametrize("frac", [0.05, 1.0])
def test_scalar_v_step_matches_oracle(shape, block, nbits, frac):
    W0, G, codes, sc, zp = workloads.make_scalar(shape[0], shape[1], block, nbits, seed=95)
    ctx = PVContext(0)
    o, i = shape
    n = o * i
    k = max(1, int(frac * n))
    lay1 = Layout(o, i, 1, 1, 8)                       # group size 1: the unit is a weight
    cd, sd, zd = dev_u8(codes), dev_f32(sc), dev_f32(zp)
    Wd = torch.empty(o, i, dtype=torch.float32, device=DEV)
    ctx.pv_dequantize_scalar(o, i, block, nbits, cd, sd, zd, Wd)
    W_ref = oracle.dequantize_scalar(codes, sc, zp, block, nbits)
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W_ref.view(np.uint32))
    Gd = dev_f32(G * 20)
    Td = torch.empty_like(Wd)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    ctx.pv_encode_targets_select(lay1, Wd, Gd, 1.0, Td, k, idx)
    T_ref = oracle.encode_targets(W_ref, G * 20, 1.0)
    idx_ref = oracle.select_topk_groups(T_ref, W_ref, 1, k)
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    nch = torch.full((1,), -3, dtype=torch.int64, device=DEV)
    ctx.pv_reencode_scalar(o, i, block, nbits, Td, sd, zd, idx, k, cd, nch)
    torch.cuda.synchronize()
    want, changed = oracle.reencode_scalar(T_ref, sc, zp, idx_ref, codes, block, nbits)
    assert np.array_equal(cd.cpu().numpy(), want)
    assert int(nch.item()) == changed
    assert changed > 0 or n < 100
    ctx.pv_dequantize_scalar(o, i, block, nbits, cd, sd, zd, Wd)
    assert np.array_equal(Wd.cpu().numpy(), oracle.dequantize_scalar(want, sc, zp, block, nbits))
    ctx.close()


def test_scalar_tie_rule_empty_list_and_errors():
    ctx = PVContext(0)
    sc, zp = dev_f32(np.array([[1.0]], np.float32)), dev_f32(np.array([[0.0]], np.float32))
    codes = dev_u8(np.array([[2, 1, 0, 3]], np.uint8))
    T = dev_f32(np.array([[1.5, 1.5, 7.0, 100.0]], np.float32))
    nch = torch.zeros(1, dtype=torch.int64, device=DEV)
    ctx.pv_reencode_scalar(1, 4, 4, 2, T, sc, zp, dev_i32(np.array([0, 1, 2], np.int32)), 3, codes, nch)
    torch.cuda.synchronize()
    assert list(codes.cpu().numpy()[0]) == [2, 1, 3, 3] and int(nch.item()) == 1
    ctx.pv_reencode_scalar(1, 4, 4, 2, T, sc, zp, None, 0, codes, nch)          # k = 0: a no-op
    torch.cuda.synchronize()
    assert int(nch.item()) == 0
    for args in ((1, 4, 3, 2), (1, 4, 4, 9), (1, 4, 4, 0)):                      # bad block size / bits
        with pytest.raises(PVError):
            ctx.pv_reencode_scalar(*args, T, sc, zp, dev_i32(np.array([0], np.int32)), 1, codes, nch)
    with pytest.raises(PVError):
        ctx.pv_reencode_scalar(1, 4, 4, 2, T, sc, zp, dev_i32(np.array([0], np.int32)), 5, codes, nch)
    ctx.close()
