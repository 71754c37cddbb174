"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  Targets, scores-derived selection and
dequantised weights are compared in full (bit-exact); the search is compared on
every selected group where the oracle finishes in seconds (4096 x 4096, 1x16)
and on a seeded sample of selected groups otherwise (the oracle re-encodes the
sampled groups one by one; the GPU re-encodes all of them).  Properties that
hold at any size are checked on everything: unselected codes untouched, codes
in range, selection size and order.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import GpuRun, check_codes_on, dev_f32, host_u16

pytestmark = pytest.mark.gpu


def run_config(name, sample):
    wl = workloads.make_config(name, seed=0)
    lay = wl.layout
    g, M = lay.group_size, lay.num_codebooks
    run = GpuRun(wl)
    T = run.targets()
    T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    assert np.array_equal(T.cpu().numpy().view(np.uint32), T_ref.view(np.uint32))
    idx = run.select(T, wl.k)
    idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, wl.k)
    assert len(idx) == wl.k and np.array_equal(idx, idx_ref)
    got, nch = run.reencode(T, idx)
    stats = run.ctx.pv_reencode_stats()
    # properties on everything
    g2 = got.reshape(-1, M)
    mask = np.ones(lay.num_groups, bool)
    mask[idx] = False
    assert np.array_equal(g2[mask], wl.codes.reshape(-1, M)[mask])
    assert int(g2.max()) < lay.codebook_size
    assert nch == int((g2[idx] != wl.codes.reshape(-1, M)[idx]).any(1).sum())
    # the oracle on all / a seeded sample of the selected groups
    if sample is None or sample >= wl.k:
        sub = idx
    else:
        sub = np.sort(np.random.default_rng(123).choice(idx, size=sample, replace=False))
    want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, sub, wl.codes,
                                        beam_width=wl.beam_width)
    w2 = want.reshape(-1, M)
    diff = np.nonzero((g2[sub] != w2[sub]).any(1))[0]
    if len(diff):
        pos = np.searchsorted(sub, sub[diff])
        assert info["near_tie"][pos].all(), f"{len(diff)} differing groups outside near-ties"
        obj = oracle.group_objective(T_ref, wl.codebooks, wl.scales, sub[diff], g2[sub[diff]])
        assert (np.abs(obj - info["obj_new"][pos]) <= 1e-6 * info["obj_new"][pos]).all()
    assert (info["obj_new"] <= info["obj_prev"]).all()
    # dequantise the GPU's codes on both sides
    W2 = run.dequantize(got)
    W2_ref = oracle.dequantize(got, wl.codebooks, wl.scales)
    assert np.array_equal(W2.view(np.uint32), W2_ref.view(np.uint32))
    return stats


def test_c2_full_every_group():
    stats = run_config("c2_4096x4096_1x16", None)
    assert stats["filtered"] + stats["fallback"] == 20971
    assert stats["fallback"] < 0.02 * 20971      # the certificate holds for nearly every group


def test_c3_full_beam_every_group():
    stats = run_config("c3_11008x4096_2x8", None)
    assert stats["filtered"] + stats["fallback"] == 281804
    assert stats["fallback"] < 0.01 * 281804     # the certificates hold for nearly every group


@pytest.mark.parametrize("name", ["c5a_14336x4096_1x16g16", "c5b_4096x14336_1x16g16"])
def test_c5_full_group16_sampled(name):
    stats = run_config(name, 1024)
    assert stats["filtered"] + stats["fallback"] == 183500


def test_c4_block_matrices_sampled():
    """Three of the seven matrices of one decoder block of the 32-layer stack (square,
    tall, wide), each as one V-step call with its own codebook."""
    for proj in ("q_proj", "up_proj", "down_proj"):
        wl = workloads.make_block_matrix(3, proj, seed=0)
        run = GpuRun(wl)
        T = run.targets()
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx = run.select(T, wl.k)
        assert np.array_equal(idx, oracle.select_topk_groups(T_ref, wl.W, 8, wl.k))
        got, _ = run.reencode(T, idx)
        sub = np.sort(np.random.default_rng(7).choice(idx, size=2048, replace=False))
        want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, sub, wl.codes)
        check_codes_on(wl, T_ref, sub, got, want, info)


def test_c4_two_contexts_on_two_streams_concurrently():
    """The stack sweep as bench.py runs it: independent matrices dealt to several contexts,
    each on a stream of its own, nothing waiting in between.  Four matrices of one decoder
    block (all three shapes) go through the whole step (targets + selection in one sweep,
    re-encode, dequantize) on two contexts whose calls are enqueued alternately; everything
    is compared with the oracle afterwards: ids in full, codes on every selected group of the
    square matrix and on 4096 sampled groups of the others, dequantised weights in full."""
    from gpu_util import DEV, dev_i32, lay_of
    from paper_2405_14852_amd import PVContext
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    ctxs = [PVContext(0, s) for s in streams]
    jobs = []
    for slot, proj in enumerate(("q_proj", "up_proj", "down_proj", "k_proj")):
        wl = workloads.make_block_matrix(5, proj, seed=0)
        jobs.append({"wl": wl, "ctx": slot % 2})
    torch.cuda.synchronize()
    # device copies first (on the default stream), then a barrier, then the two queues
    for job in jobs:
        wl = job["wl"]
        job["run"] = GpuRun(wl, ctx=ctxs[job["ctx"]])
        job["T"] = torch.empty_like(job["run"].W)
        job["idx"] = torch.empty(wl.k, dtype=torch.int32, device=DEV)
        job["codes"] = job["run"].codes.clone()
        job["W2"] = torch.empty_like(job["run"].W)
        job["nch"] = torch.zeros(1, dtype=torch.int64, device=DEV)
    torch.cuda.synchronize()
    for rep in range(2):            # the second round re-uses every context's scratch at another shape
        for job in jobs:
            run, wl, c = job["run"], job["wl"], ctxs[job["ctx"]]
            if rep == 1:
                job["codes"].copy_(run.codes)
                torch.cuda.synchronize()
            c.pv_encode_targets_select(run.lay, run.W, run.G, wl.alpha, job["T"], wl.k, job["idx"])
            c.pv_reencode_groups(run.lay, job["T"], run.cb, run.sc, job["idx"], wl.k, 1,
                                 job["codes"], job["nch"])
            c.pv_dequantize(run.lay, job["codes"], run.cb, run.sc, job["W2"])
        torch.cuda.synchronize()
        for job in jobs:
            wl = job["wl"]
            T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
            assert np.array_equal(job["T"].cpu().numpy().view(np.uint32), T_ref.view(np.uint32))
            idx = job["idx"].cpu().numpy()
            assert np.array_equal(idx, oracle.select_topk_groups(T_ref, wl.W, 8, wl.k))
            got = host_u16(job["codes"])
            mask = np.ones(wl.layout.num_groups, bool)
            mask[idx] = False
            assert np.array_equal(got.reshape(-1)[mask], wl.codes.reshape(-1)[mask])
            if wl.name.endswith("q_proj"):
                sub = idx
            else:
                sub = np.sort(np.random.default_rng(11 + rep).choice(idx, size=4096, replace=False))
            want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, sub, wl.codes)
            ndiff = check_codes_on(wl, T_ref, sub, got, want, info)
            if sub is idx:
                assert abs(int(job["nch"].item()) - info["num_changed"]) <= ndiff
            W2_ref = oracle.dequantize(got, wl.codebooks, wl.scales)
            assert np.array_equal(job["W2"].cpu().numpy().view(np.uint32), W2_ref.view(np.uint32))
    for c in ctxs:
        c.close()


def test_c2_full_trust_ratio():
    """The trust-ratio call at the benchmark shape, x^k = the dequantised current codes, all
    20 971 candidates ranked and re-encoded, against the oracle's chunked procedure."""
    from gpu_util import DEV
    wl = workloads.make_config("c2_4096x4096_1x16", seed=0)
    wl.W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
    # a gradient large enough that codes move: the update norm is then comparable to the
    # distance between neighbouring codewords
    wl.G = wl.G * np.float32(40.0)
    T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    run = GpuRun(wl)
    k_max, chunk = wl.k, wl.k // 10
    for ratio in (0.01, 0.03):
        codes = run.codes.clone()
        rank = torch.empty(k_max, dtype=torch.int32, device=DEV)
        napp = torch.zeros(1, dtype=torch.int64, device=DEV)
        stats = torch.zeros(2, dtype=torch.float64, device=DEV)
        run.ctx.pv_reencode_trust_ratio(run.lay, dev_f32(T_ref), run.W, run.cb, run.sc, k_max,
                                        chunk, ratio, 1, codes, rank, napp, stats)
        torch.cuda.synchronize()
        want, info = oracle.reencode_trust_ratio(T_ref, wl.W, wl.codebooks, wl.scales, wl.codes,
                                                 k_max, chunk, ratio)
        assert np.array_equal(rank.cpu().numpy(), info["rank_idx"])
        assert int(napp.item()) == info["num_applied"]
        assert 1 < info["num_applied"]
        st = stats.cpu().numpy()
        assert st[0] == pytest.approx(info["change_sq"], rel=1e-12)
        assert st[1] == pytest.approx(info["norm_sq"], rel=1e-12)
        assert np.array_equal(host_u16(codes), want)


def _grads_on_gpu(wl):
    run = GpuRun(wl)
    gc = torch.full(tuple(wl.codebooks.shape), 7.0, dtype=torch.float32, device="cuda:0")
    gs = torch.full((wl.layout.out_features,), 7.0, dtype=torch.float32, device="cuda:0")
    run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
    torch.cuda.synchronize()
    first = (gc.cpu().numpy(), gs.cpu().numpy())
    gc.fill_(-3.0)
    gs.fill_(-3.0)
    run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
    torch.cuda.synchronize()
    # a second call on the same context returns the same bits
    assert np.array_equal(first[0].view(np.uint32), gc.cpu().numpy().view(np.uint32))
    assert np.array_equal(first[1].view(np.uint32), gs.cpu().numpy().view(np.uint32))
    return first


def _close(got, want, mag):
    tol = 2 * np.spacing(np.abs(want).astype(np.float32)) + 1e-12 * mag
    return np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol


@pytest.mark.parametrize("name", ["c2_4096x4096_1x16", "c3_11008x4096_2x8", "c5a_14336x4096_1x16g16"])
def test_pstep_gradients_full_size(name):
    """Codebook and scale gradients of the P step at the benchmark sizes, every entry against
    the oracle's sequential double sums: the sorted route (c2: segments of about 32 groups, the
    same sum in the same order, so nearly every entry has the same bits) and the fixed-point
    tables (c3: 22 000 terms per codeword)."""
    wl = workloads.make_config(name, seed=0)
    gc, gs = _grads_on_gpu(wl)
    gc_ref, gs_ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
    mag = float(np.abs(wl.G).max() * np.abs(wl.scales).max()) * wl.layout.num_groups
    assert _close(gc, gc_ref, mag * 1e-3).all()
    same = (gc.view(np.uint32) == gc_ref.view(np.uint32)).mean()
    assert same > 0.99, same
    q = oracle.dequantize(wl.codes, wl.codebooks, np.ones_like(wl.scales))
    assert _close(gs, gs_ref, np.abs(wl.G * q).sum(axis=1)).all()
    # every weight of a group pulls on its codeword with the row's scale: the gradients of
    # one codebook add up to the sum of s_o * G over the matrix, element by element
    g = wl.layout.group_size
    total = (wl.G.astype(np.float64) * wl.scales.astype(np.float64)[:, None]).reshape(-1, g).sum(axis=0)
    for m in range(wl.layout.num_codebooks):
        assert np.allclose(gc[m].astype(np.float64).sum(axis=0), total, rtol=0, atol=1e-6 * np.abs(total).max() + 1e-9)


@pytest.mark.parametrize("name,sample", [("c2_4096x4096_1x16", 4096), ("c5a_14336x4096_1x16g16", 1024)])
def test_stochastic_rounding_full_size_sampled(name, sample):
    """pv_reencode_groups_stochastic at the benchmark sizes (power 5, as App. K's temperature
    gives): all selected groups are rounded on the GPU, a seeded sample of them by the oracle."""
    from gpu_util import dev_i32, dev_u16, lay_of
    wl = workloads.make_config(name, seed=0)
    M = wl.layout.num_codebooks
    run = GpuRun(wl)
    T = run.targets()
    T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    idx = run.select(T, wl.k)
    assert np.array_equal(idx, oracle.select_topk_groups(T_ref, wl.W, wl.layout.group_size, wl.k))
    codes = dev_u16(wl.codes)
    nch = torch.full((1,), -1, dtype=torch.int64, device="cuda:0")
    seed = 20240528
    run.ctx.pv_reencode_groups_stochastic(lay_of(wl), T, run.cb, run.sc, dev_i32(idx), len(idx), 5, seed,
                                          codes, nch)
    torch.cuda.synchronize()
    got = host_u16(codes).reshape(-1)
    rest = np.ones(wl.layout.num_groups, bool)
    rest[idx] = False
    assert np.array_equal(got[rest], wl.codes.reshape(-1)[rest])
    assert int(nch.item()) == int((got[idx] != wl.codes.reshape(-1)[idx]).sum())
    sub = np.sort(np.random.default_rng(321).choice(idx, size=sample, replace=False))
    want, info = oracle.reencode_stochastic(T_ref, wl.codebooks, wl.scales, sub, wl.codes, power=5, seed=seed)
    differ = np.nonzero(got[sub] != want.reshape(-1)[sub])[0]
    assert info["near_tie"][differ].all(), (len(differ), differ[:5])
    # the second nearest is taken in a noticeable share of the groups, never in most
    second = (want.reshape(-1)[sub] == info["nearest_two"][:, 1]).mean()
    assert 0.01 < second < 0.5, second
    stats = run.ctx.pv_reencode_stats()
    assert stats["filtered"] + stats["fallback"] == wl.k


def test_c2_full_adam_direction_then_search():
    """Sec. 3.4's Adam direction at the benchmark size: the fused sweep (moments, targets, scores,
    selection) bit for bit against the oracle at step 3 with moments in flight, then the search on
    the selected groups of those targets."""
    from gpu_util import dev_i32
    wl = workloads.make_config("c2_4096x4096_1x16", seed=0)
    g = wl.layout.group_size
    shape = wl.W.shape
    rng = np.random.default_rng(91)
    m = (rng.standard_normal(shape) * 1e-4).astype(np.float32)
    v = (rng.random(shape) * 1e-8).astype(np.float32)
    run = GpuRun(wl)
    md, vd = dev_f32(m), dev_f32(v)
    T = torch.empty_like(run.W)
    idx = torch.empty(wl.k, dtype=torch.int32, device="cuda:0")
    run.ctx.pv_encode_targets_adam_select(run.lay, run.W, run.G, md, vd, 3, 3e-3, 0.9, 0.95, 1e-8, T, wl.k, idx)
    torch.cuda.synchronize()
    T_ref, m_ref, v_ref = oracle.encode_targets_adam(wl.W, wl.G, m, v, 3, 3e-3, 0.9, 0.95, 1e-8)
    assert np.array_equal(T.cpu().numpy().view(np.uint32), T_ref.view(np.uint32))
    assert np.array_equal(md.cpu().numpy().view(np.uint32), m_ref.view(np.uint32))
    assert np.array_equal(vd.cpu().numpy().view(np.uint32), v_ref.view(np.uint32))
    idx_np = idx.cpu().numpy()
    assert np.array_equal(idx_np, oracle.select_topk_groups(T_ref, wl.W, g, wl.k))
    got, _ = run.reencode(T, idx_np)
    sub = np.sort(np.random.default_rng(92).choice(idx_np, size=4096, replace=False))
    want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, sub, wl.codes)
    check_codes_on(wl, T_ref, sub, got, want, info)


def test_c2_full_straight_through_step():
    """App. E at the benchmark size: the gradient step goes to the buffer (targets written over
    W), the subspace is chosen from buffer against the dequantised codes, the codes follow the
    buffer.  Buffer and subspace bit for bit, codes by the per-group rule."""
    from gpu_util import dev_u16, lay_of
    wl = workloads.make_config("c2_4096x4096_1x16", seed=0)
    lay = lay_of(wl)
    run = GpuRun(wl)
    codes = dev_u16(wl.codes)
    buf = torch.empty_like(run.W)
    run.ctx.pv_dequantize(lay, codes, run.cb, run.sc, buf)
    Wq = buf.clone()
    idx = torch.empty(wl.k, dtype=torch.int32, device="cuda:0")
    nch = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    alpha = 40.0                                          # updates of a fraction of the codeword spacing
    run.ctx.pv_encode_targets(lay, buf, run.G, alpha, buf)
    run.ctx.pv_select_topk_groups(lay, buf, Wq, wl.k, idx)
    run.ctx.pv_reencode_groups(lay, buf, run.cb, run.sc, idx, wl.k, 1, codes, nch)
    torch.cuda.synchronize()
    buf0 = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
    buf_ref, want, info = oracle.ste_step(buf0, wl.G, alpha, wl.codebooks, wl.scales, wl.codes.copy(), k=wl.k)
    assert np.array_equal(buf.cpu().numpy().view(np.uint32), buf_ref.view(np.uint32))
    assert np.array_equal(idx.cpu().numpy(), info["group_idx"])
    got = host_u16(codes)
    ndiff = check_codes_on(wl, buf_ref, info["group_idx"], got, want, info)
    assert abs(int(nch.item()) - info["num_changed"]) <= ndiff
    assert info["num_changed"] > 0
