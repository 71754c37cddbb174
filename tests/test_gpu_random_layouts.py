"""Seeded random layouts through every call of the library against the oracle.

The hand-picked cases of the other files cover the shapes somebody thought of; this file draws
layouts (group size, number and size of codebooks, matrix shape, fraction selected, beam width,
search mode) and value scales (weights, gradients, scales of mixed sign and magnitude) from a
seeded generator and applies the same acceptance rules: targets, moments, selected ids and
weights bit for bit; codes by the per-group rule (a differing group must be one the oracle flags
as a near-tie, with an objective within 1e-6 relative); gradients within 2 ulp; the trust-ratio
prefix and its codes identical.  (A permuted read-out of the small-codebook gradient tables for
several codebooks of fewer than 4 g codewords was found this way.)"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DEV, GpuRun, check_codes_on, dev_f32, dev_i32, dev_u16, host_u16
from paper_2405_14852_amd import Layout, PVContext

pytestmark = pytest.mark.gpu

CASES_PER_SEED = 24


def draw_case(rng):
    g = int(rng.choice([4, 8, 8, 8, 16, 16, 12, 2]))
    M = int(rng.choice([1, 1, 1, 2, 2, 3]))
    B = int(rng.integers(1, 17)) if M == 1 else int(rng.choice([2, 4, 5, 6, 8, 8]))
    big = rng.random() < 0.25
    out = int(rng.integers(200, 1200)) if big else int(rng.integers(3, 200))
    gpr = int(rng.integers(64, 600)) if big else int(rng.integers(1, 120))
    beam = 1 if M == 1 else int(rng.choice([1, 2, 4, 8]))
    tau = float(rng.choice([0.01, 0.1, 0.5, 1.0]))
    # keep the oracle's search within a second or so
    tau = max(min(tau, 2e7 / (out * gpr * (1 << B) * beam)), 1.5 / (out * gpr))
    wl = workloads.make(out, gpr * g, g, M, B, seed=int(rng.integers(1 << 30)),
                        sigma_g=float(10 ** rng.uniform(-5, -1.5)), sigma_w=float(10 ** rng.uniform(-3, 0)),
                        tau=tau, beam_width=beam)
    if rng.random() < 0.3:      # scales of mixed sign and magnitude
        wl.scales = (wl.scales * rng.choice([-1.0, 1.0], size=wl.scales.shape)
                     * 10 ** rng.uniform(-2, 2, size=wl.scales.shape)).astype(np.float32)
    return wl, int(rng.integers(0, 2))


def close(got, want, mag):
    tol = 2 * np.spacing(np.abs(want).astype(np.float32)) + 1e-9 * mag
    return (np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol).all()


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_layouts_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for case in range(CASES_PER_SEED):
        wl, mode = draw_case(rng)
        lay = wl.layout
        g, M, beam, k = lay.group_size, lay.num_codebooks, wl.beam_width, wl.k
        tag = (seed, case, lay.out_features, lay.in_features, g, M, lay.nbits, beam, k, mode)
        run = GpuRun(wl)
        run.ctx.pv_set_search_mode(mode)

        # targets + selection in one sweep, search, dequantize
        T, idx = run.targets_select(k)
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, k)
        assert np.array_equal(T.cpu().numpy().view(np.uint32), T_ref.view(np.uint32)), tag
        assert np.array_equal(idx, idx_ref), tag
        got, nch = run.reencode(T, idx)
        want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, idx_ref, wl.codes, beam_width=beam)
        ndiff = check_codes_on(wl, T_ref, idx_ref, got, want, info)
        assert abs(nch - info["num_changed"]) <= ndiff, tag
        W2 = run.dequantize(got)
        W2_ref = oracle.dequantize(got, wl.codebooks, wl.scales)
        assert np.array_equal(W2.view(np.uint32), W2_ref.view(np.uint32)), tag

        # the re-encoded groups only, into the old weights
        Wd = dev_f32(oracle.dequantize(wl.codes, wl.codebooks, wl.scales))
        run.ctx.pv_dequantize_groups(run.lay, dev_u16(got), run.cb, run.sc, dev_i32(idx_ref), k, Wd)
        torch.cuda.synchronize()
        assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W2_ref.view(np.uint32)), tag

        # the selection that allocates nothing
        if lay.num_groups <= (1 << 22):
            ib = torch.empty(max(k, 1), dtype=torch.int32, device=DEV)
            run.ctx.pv_select_topk_groups_noalloc(run.lay, T, run.W, k, ib)
            torch.cuda.synchronize()
            assert np.array_equal(ib.cpu().numpy()[:k], idx_ref), tag

        # Adam direction fused with the selection
        step = int(rng.integers(1, 60))
        lr = float(10 ** rng.uniform(-4, -2))
        m0 = (rng.standard_normal(wl.W.shape) * 1e-4).astype(np.float32) if step > 1 else np.zeros(wl.W.shape, np.float32)
        v0 = (rng.random(wl.W.shape) * 1e-8).astype(np.float32) if step > 1 else np.zeros(wl.W.shape, np.float32)
        md, vd = dev_f32(m0), dev_f32(v0)
        Ta = torch.empty_like(run.W)
        ia = torch.empty(max(k, 1), dtype=torch.int32, device=DEV)
        run.ctx.pv_encode_targets_adam_select(run.lay, run.W, run.G, md, vd, step, lr, 0.9, 0.95, 1e-8, Ta, k, ia)
        torch.cuda.synchronize()
        Tr, mr, vr = oracle.encode_targets_adam(wl.W, wl.G, m0, v0, step, lr, 0.9, 0.95, 1e-8)
        assert np.array_equal(Ta.cpu().numpy().view(np.uint32), Tr.view(np.uint32)), tag
        assert np.array_equal(md.cpu().numpy().view(np.uint32), mr.view(np.uint32)), tag
        assert np.array_equal(vd.cpu().numpy().view(np.uint32), vr.view(np.uint32)), tag
        assert np.array_equal(ia.cpu().numpy()[:k], oracle.select_topk_groups(Tr, wl.W, g, k)), tag

        # trust-ratio step from the dequantised codes
        codes = dev_u16(wl.codes)
        rank = torch.empty(max(k, 1), dtype=torch.int32, device=DEV)
        napp = torch.zeros(1, dtype=torch.int64, device=DEV)
        Wq = torch.empty_like(run.W)
        run.ctx.pv_dequantize(run.lay, run.codes, run.cb, run.sc, Wq)
        Tq = torch.empty_like(run.W)
        run.ctx.pv_encode_targets(run.lay, Wq, run.G, 40.0, Tq)
        ratio = float(10 ** rng.uniform(-3, -0.5))
        chunk = max(1, k // int(rng.integers(1, 20)))
        run.ctx.pv_reencode_trust_ratio(run.lay, Tq, Wq, run.cb, run.sc, k, chunk, ratio, beam, codes, rank, napp)
        torch.cuda.synchronize()
        Wq_ref = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
        Tq_ref = oracle.encode_targets(Wq_ref, wl.G, 40.0)
        new_ref, ti = oracle.reencode_trust_ratio(Tq_ref, Wq_ref, wl.codebooks, wl.scales, wl.codes, k, chunk,
                                                  ratio, beam_width=beam)
        assert int(napp.item()) == ti["num_applied"], tag
        assert np.array_equal(rank.cpu().numpy()[:k], ti["rank_idx"]), tag
        assert np.array_equal(host_u16(codes).reshape(-1), new_ref.reshape(-1)), tag

        # P-step gradients
        gc = torch.full(tuple(wl.codebooks.shape), 7.0, dtype=torch.float32, device=DEV)
        gs = torch.full((lay.out_features,), 7.0, dtype=torch.float32, device=DEV)
        run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
        torch.cuda.synchronize()
        gc_ref, gs_ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
        assert close(gc.cpu().numpy(), gc_ref, np.abs(wl.G).sum() * np.abs(wl.scales).max()), tag
        q = oracle.dequantize(wl.codes, wl.codebooks, np.ones_like(wl.scales))
        assert close(gs.cpu().numpy(), gs_ref, np.abs(wl.G * q).sum(axis=1)), tag

        # stochastic rounding (defined for one codebook)
        if M == 1:
            codes = dev_u16(wl.codes)
            n2 = torch.zeros(1, dtype=torch.int64, device=DEV)
            rseed = int(rng.integers(1 << 40))
            power = int(rng.choice([1, 5]))
            run.ctx.pv_reencode_groups_stochastic(run.lay, T, run.cb, run.sc, dev_i32(idx_ref), k, power, rseed,
                                                  codes, n2)
            torch.cuda.synchronize()
            w2, i2 = oracle.reencode_stochastic(T_ref, wl.codebooks, wl.scales, idx_ref, wl.codes, power=power,
                                                seed=rseed)
            differ = np.nonzero(host_u16(codes).reshape(-1)[idx_ref] != w2.reshape(-1)[idx_ref])[0]
            assert i2["near_tie"][differ].all(), tag
        run.ctx.close()


@pytest.mark.parametrize("seed", [201, 202])
def test_random_scalar_grids_match_the_oracle(seed):
    """The scalar uniform-grid representation (App. K): dequantise, targets and selection at group
    size 1, round to the nearest grid value; every array bit for bit."""
    rng = np.random.default_rng(seed)
    for case in range(CASES_PER_SEED):
        block = int(rng.choice([1, 3, 6, 8, 16, 32, 64, 128]))
        blocks = int(rng.integers(1, 40))
        o, i = int(rng.integers(1, 300)), block * blocks
        nbits = int(rng.integers(1, 9))
        n = o * i
        k = max(1, int(float(rng.choice([0.01, 0.2, 1.0])) * n))
        sw = float(10 ** rng.uniform(-3, 0))
        W0, G, codes, sc, zp = workloads.make_scalar(o, i, block, nbits, seed=int(rng.integers(1 << 30)), sigma_w=sw,
                                                     sigma_g=sw * float(10 ** rng.uniform(-2, 0)))
        if rng.random() < 0.3:
            sc = (sc * rng.choice([-1.0, 1.0], size=sc.shape)).astype(np.float32)
        tag = (seed, case, o, i, block, nbits, k)
        ctx = PVContext(0)
        lay1 = Layout(o, i, 1, 1, 8)
        cd = torch.from_numpy(codes).to(DEV)
        sd, zd = dev_f32(sc), dev_f32(zp)
        Wd = torch.empty(o, i, dtype=torch.float32, device=DEV)
        ctx.pv_dequantize_scalar(o, i, block, nbits, cd, sd, zd, Wd)
        W_ref = oracle.dequantize_scalar(codes, sc, zp, block, nbits)
        assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W_ref.view(np.uint32)), tag
        Td = torch.empty_like(Wd)
        idx = torch.empty(k, dtype=torch.int32, device=DEV)
        ctx.pv_encode_targets_select(lay1, Wd, dev_f32(G), 3.0, Td, k, idx)
        T_ref = oracle.encode_targets(W_ref, G, 3.0)
        idx_ref = oracle.select_topk_groups(T_ref, W_ref, 1, k)
        assert np.array_equal(idx.cpu().numpy(), idx_ref), tag
        nch = torch.zeros(1, dtype=torch.int64, device=DEV)
        ctx.pv_reencode_scalar(o, i, block, nbits, Td, sd, zd, idx, k, cd, nch)
        torch.cuda.synchronize()
        want, changed = oracle.reencode_scalar(T_ref, sc, zp, idx_ref, codes, block, nbits)
        assert np.array_equal(cd.cpu().numpy(), want), tag
        assert int(nch.item()) == changed, tag
        ctx.close()


@pytest.mark.parametrize("seed", [301, 302])
def test_random_large_layouts_match_the_oracle(seed):
    """Large odd shapes with thousands of selected groups: the matrix-core scoring and the beam
    filter over many tiles and ragged tails, in both regimes of W (the configuration's dense
    Gaussian, and the dequantised current codes as in a real step)."""
    rng = np.random.default_rng(seed)
    for case in range(6):
        kind = int(rng.integers(0, 4))
        if kind == 0:
            g, M, B, beam = 8, 1, int(rng.integers(11, 17)), 1
        elif kind == 1:
            g, M, B, beam = 16, 1, int(rng.integers(11, 17)), 1
        elif kind == 2:
            g, M, B, beam = 8, 2, 8, int(rng.choice([4, 8, 16]))
        else:
            g, M, B, beam = int(rng.choice([4, 8, 16])), int(rng.choice([2, 3])), int(rng.choice([6, 8])), 8
        out, gpr = int(rng.integers(500, 3000)), int(rng.integers(100, 1000))
        N = out * gpr
        budget = 2e9 if M == 1 else 3e8              # the oracle's search stays near a second
        tau = max(min(float(rng.choice([0.01, 0.05, 0.3])), budget / (N * (1 << B) * beam * M)), 1.5 / N)
        wl = workloads.make(out, gpr * g, g, M, B, seed=int(rng.integers(1 << 30)),
                            sigma_g=float(10 ** rng.uniform(-4.5, -2)), sigma_w=0.02, tau=tau, beam_width=beam)
        structured = rng.random() < 0.5
        if structured:
            wl.W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
        tag = (seed, case, out, gpr * g, g, M, B, beam, wl.k, structured)
        run = GpuRun(wl)
        T, idx = run.targets_select(wl.k)
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, wl.k)
        assert np.array_equal(T.cpu().numpy().view(np.uint32), T_ref.view(np.uint32)), tag
        assert np.array_equal(idx, idx_ref), tag
        got, nch = run.reencode(T, idx)
        want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, idx_ref, wl.codes, beam_width=beam)
        ndiff = check_codes_on(wl, T_ref, idx_ref, got, want, info)
        assert abs(nch - info["num_changed"]) <= ndiff, tag
        assert np.array_equal(run.dequantize(got).view(np.uint32),
                              oracle.dequantize(got, wl.codebooks, wl.scales).view(np.uint32)), tag
        gc = torch.empty(tuple(wl.codebooks.shape), dtype=torch.float32, device=DEV)
        gs = torch.empty((out,), dtype=torch.float32, device=DEV)
        run.ctx.pv_codebook_grads(run.lay, run.G, run.codes, run.cb, run.sc, gc, gs)
        torch.cuda.synchronize()
        gc_ref, gs_ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
        assert close(gc.cpu().numpy(), gc_ref, np.abs(wl.G).sum() * np.abs(wl.scales).max()), tag
        q = oracle.dequantize(wl.codes, wl.codebooks, np.ones_like(wl.scales))
        assert close(gs.cpu().numpy(), gs_ref, np.abs(wl.G * q).sum(axis=1)), tag
        run.ctx.close()
