"""GPU parity of pv_codebook_grads (Alg. 3, P step) against the CPU oracle.

Codebook gradients: bit-exact when no codeword is shared by more than 128 groups (the GPU
then adds in the oracle's order); otherwise, and for the scale gradients (tree sum against a
sequential sum, both in double, rounded to fp32 once), within 2 fp32 ulps of the value plus
1e-12 of the sum of magnitudes.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DEV, GpuRun, dev_f32, dev_u16

pytestmark = pytest.mark.gpu


def run_case(wl, want_scales=True):
    run = GpuRun(wl)
    gc = torch.full(tuple(wl.codebooks.shape), 7.0, dtype=torch.float32, device=DEV)
    gs = torch.full((wl.layout.out_features,), 7.0, dtype=torch.float32, device=DEV) if want_scales else None
    run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
    torch.cuda.synchronize()
    gc_ref, gs_ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
    return gc.cpu().numpy(), (gs.cpu().numpy() if want_scales else None), gc_ref, gs_ref


def close_sum(got, want, mag):
    tol = 2 * np.spacing(np.abs(want).astype(np.float32)) + 1e-12 * mag
    return (np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol).all()


@pytest.mark.parametrize("g,M,B,shape", [(8, 1, 8, (64, 512)), (8, 2, 5, (33, 256)), (16, 1, 9, (48, 512)),
                                         (4, 1, 4, (40, 256)), (6, 3, 4, (20, 36)), (1, 1, 2, (9, 31)),
                                         (8, 1, 16, (128, 1024))])
def test_codebook_grads_match_oracle(g, M, B, shape):
    wl = workloads.make(shape[0], shape[1], g, M, B, seed=81, sigma_g=1e-2)
    gc, gs, gc_ref, gs_ref = run_case(wl)
    counts = [np.bincount(wl.codes[..., m].ravel(), minlength=1 << B).max() for m in range(M)]
    if max(counts) <= 128:
        assert np.array_equal(gc.view(np.uint32), gc_ref.view(np.uint32))
    else:
        assert close_sum(gc, gc_ref, np.abs(wl.G).sum() * np.abs(wl.scales).max())
    q = oracle.dequantize(wl.codes, wl.codebooks, np.ones_like(wl.scales))
    assert close_sum(gs, gs_ref, np.abs(wl.G * q).sum(axis=1))


def test_codebook_grads_popular_codewords():
    """Most groups share three codewords (segments of tens of thousands), the rest are spread."""
    wl = workloads.make(96, 2048, 8, 1, 8, seed=82, sigma_g=1e-2)
    rng = np.random.default_rng(82)
    hot = rng.random(wl.codes.shape) < 0.9
    wl.codes[hot] = rng.choice(np.array([3, 77, 200], dtype=np.uint16), size=int(hot.sum()))
    gc, gs, gc_ref, gs_ref = run_case(wl)
    mag = np.abs(wl.G).sum() * np.abs(wl.scales).max()
    assert close_sum(gc, gc_ref, mag)
    cold = np.ones(256, bool)
    cold[[3, 77, 200]] = False
    assert np.array_equal(gc[0, cold].view(np.uint32), gc_ref[0, cold].view(np.uint32))
    assert np.abs(gc_ref[0, [3, 77, 200]]).max() > 0


def test_codebook_grads_unused_codewords_and_no_scales():
    wl = workloads.make(8, 64, 8, 1, 10, seed=83, sigma_g=1e-2)      # 64 groups, 1024 codewords
    gc, gs, gc_ref, _ = run_case(wl, want_scales=False)
    assert gs is None and np.array_equal(gc, gc_ref)
    used = np.zeros(1024, bool)
    used[np.unique(wl.codes)] = True
    assert (gc[0, ~used] == 0).all() and np.abs(gc[0, used]).max() > 0


def test_codebook_grads_second_call_and_errors():
    from paper_2405_14852_amd import PVError
    wl = workloads.make(16, 128, 8, 2, 6, seed=84, sigma_g=1e-2)
    run = GpuRun(wl)
    gc = torch.empty(tuple(wl.codebooks.shape), dtype=torch.float32, device=DEV)
    gs = torch.empty(16, dtype=torch.float32, device=DEV)
    ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
    for _ in range(2):                              # outputs are overwritten, not accumulated
        run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
    torch.cuda.synchronize()
    assert np.array_equal(gc.cpu().numpy(), ref[0])
    with pytest.raises((PVError, TypeError)):       # the binding refuses a missing output itself
        run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, None, gs)
    from paper_2405_14852_amd import Layout
    with pytest.raises(PVError):
        run.ctx.pv_codebook_grads(Layout(16, 2048, 128, 2, 6), run.G, run.codes, run.cb, run.sc, gc, gs)


def test_codebook_grads_long_buckets_sorted_in_lds_and_in_global_memory():
    """The bucketed route (the table of sums does not fit LDS) with one codeword held by more than
    8192 groups, one by a few thousand, one by just over 128 and the rest spread thinly: the three
    ways a bucket is put into group order.  Thin buckets are bit-exact, the long ones within the
    tolerance of a different association, and a second run repeats the first bit for bit."""
    wl = workloads.make(64, 4096, 8, 1, 11, seed=85, sigma_g=1e-2)       # 32768 groups, 2048 codewords
    rng = np.random.default_rng(85)
    u = rng.random(wl.codes.shape)
    wl.codes[u < 0.5] = 1234
    wl.codes[(u >= 0.5) & (u < 0.6)] = 7
    flat = wl.codes.reshape(-1)
    free = np.nonzero((flat != 1234) & (flat != 7))[0]
    flat[free[:150]] = 2000
    counts = np.bincount(flat, minlength=2048)
    assert counts[1234] > 8192 and 128 < counts[7] <= 8192 and 128 < counts[2000] < 400
    gc, gs, gc_ref, gs_ref = run_case(wl)
    mag = np.abs(wl.G).sum() * np.abs(wl.scales).max()
    assert close_sum(gc, gc_ref, mag)
    thin = counts <= 128
    assert thin.sum() > 1900
    assert np.array_equal(gc[0, thin].view(np.uint32), gc_ref[0, thin].view(np.uint32))
    again, _, _, _ = run_case(wl)
    assert np.array_equal(gc.view(np.uint32), again.view(np.uint32))


@pytest.mark.parametrize("g,M,B,shape", [(8, 1, 16, (256, 2048)), (16, 1, 12, (128, 2048)), (8, 2, 8, (512, 4096)),
                                         (8, 1, 8, (64, 512))])
def test_codebook_grads_repeat_bit_for_bit(g, M, B, shape):
    wl = workloads.make(shape[0], shape[1], g, M, B, seed=86, sigma_g=1e-2)
    a = run_case(wl)
    b = run_case(wl)
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32))
    assert np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_codebook_grads_rejects_misaligned_pointers():
    from paper_2405_14852_amd import PVError
    wl = workloads.make(16, 128, 8, 1, 6, seed=87)
    run = GpuRun(wl)
    gc = torch.empty(tuple(wl.codebooks.shape), dtype=torch.float32, device=DEV)
    big = torch.zeros(16 * 128 + 4, dtype=torch.float32, device=DEV)
    with pytest.raises(PVError):
        run.ctx.pv_codebook_grads(run.lay, big[1:1 + 16 * 128].view(16, 128), run.codes, run.cb, run.sc, gc, None)


def test_codebook_grads_small_codebook_route_is_close_to_the_exact_sum_and_flags_non_finite_input():
    """The fixed-point route (the table of sums fits LDS): its sums are exact up to 2^-39 of the
    largest term, so they agree with the oracle's double loop to the last fp32 bit almost always;
    a gradient that is not finite turns the whole result into NaN."""
    wl = workloads.make(256, 2048, 8, 2, 6, seed=88, sigma_g=1e-2)       # 65536 groups, 64 codewords
    gc, gs, gc_ref, gs_ref = run_case(wl)
    assert (gc.view(np.uint32) != gc_ref.view(np.uint32)).mean() < 0.01
    assert close_sum(gc, gc_ref, 1e-3 * np.abs(wl.G).sum() * np.abs(wl.scales).max())
    wl.G[5, 17] = np.inf
    gc, gs, _, _ = run_case(wl)
    assert np.isnan(gc).all()
    wl.G[5, 17] = 0.0
    wl.G *= 0
    gc, gs, _, _ = run_case(wl)
    assert (gc == 0).all() and (gs == 0).all()


@pytest.mark.parametrize("g,M,B,shape", [(16, 1, 6, (128, 2048)), (16, 2, 8, (512, 4096)), (12, 1, 5, (96, 1536)),
                                         (8, 3, 5, (128, 1024)), (4, 2, 4, (64, 512)), (8, 1, 6, (100, 1000)),
                                         (8, 2, 8, (1031, 1160)),
                                         # codebooks of fewer than 4 g codewords with several codebooks:
                                         # the row permutation must use the code within its codebook
                                         (8, 3, 4, (40, 840)), (16, 2, 4, (54, 1120)), (16, 3, 5, (64, 2048)),
                                         (8, 2, 3, (64, 512)), (16, 2, 2, (32, 512)), (8, 4, 1, (32, 256))])
def test_codebook_grads_small_codebook_route_shapes(g, M, B, shape):
    """The fixed-point route over the group sizes it has a kernel for (4, 8, 16 and the general
    one), more than two codebooks, and block ranges that start in the middle of a row."""
    wl = workloads.make(shape[0], shape[1], g, M, B, seed=89, sigma_g=1e-2)
    gc, gs, gc_ref, gs_ref = run_case(wl)
    assert (gc.view(np.uint32) != gc_ref.view(np.uint32)).mean() < 0.01
    assert close_sum(gc, gc_ref, 1e-3 * np.abs(wl.G).sum() * np.abs(wl.scales).max())
    q = oracle.dequantize(wl.codes, wl.codebooks, np.ones_like(wl.scales))
    assert close_sum(gs, gs_ref, np.abs(wl.G * q).sum(axis=1))
    again, gs2, _, _ = run_case(wl)
    assert np.array_equal(gc.view(np.uint32), again.view(np.uint32))
    assert np.array_equal(gs.view(np.uint32), gs2.view(np.uint32))


def test_codebook_grads_of_an_empty_matrix_are_zero():
    from paper_2405_14852_amd import Layout, PVContext
    ctx = PVContext(0)
    lay = Layout(0, 64, 8, 1, 6)
    gc = torch.full((1, 64, 8), 3.0, dtype=torch.float32, device=DEV)
    G = torch.zeros((1, 64), dtype=torch.float32, device=DEV)          # never read
    codes = torch.zeros((1, 8, 1), dtype=torch.int16, device=DEV).view(torch.uint16)
    cb = torch.zeros((1, 64, 8), dtype=torch.float32, device=DEV)
    sc = torch.zeros((1,), dtype=torch.float32, device=DEV)
    ctx.pv_codebook_grads(lay, G, codes, cb, sc, gc, None)
    torch.cuda.synchronize()
    assert (gc == 0).all()
    ctx.close()
