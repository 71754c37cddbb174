"""The V step under HIP graph capture: the library launches kernels on the context's stream and
nothing else once its scratch buffers exist (no allocation, no memset node, no copy back to the
host), so a caller may capture a step and replay it.  Every replay is compared with the eager
result, with eager work and synchronisations of the same context between the replays."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DEV, dev_f32, lay_of
from paper_2405_14852_amd import PVContext

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,g,M,B,beam", [((128, 1024), 8, 1, 16, 1), ((64, 1024), 16, 1, 12, 1),
                                             ((96, 512), 8, 2, 8, 8), ((48, 384), 8, 1, 7, 1)])
def test_captured_step_replays_like_the_eager_one(shape, g, M, B, beam):
    wl = workloads.make(shape[0], shape[1], g, M, B, beam_width=beam, tau=0.1, sigma_g=5e-3, seed=700 + B)
    lay = lay_of(wl)
    k = wl.k
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ctx = PVContext(0, stream=side)
        W, G = dev_f32(wl.W), dev_f32(wl.G)
        cb, sc = dev_f32(wl.codebooks), dev_f32(wl.scales)
        codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(DEV)
        codes = codes0.clone()
        T, Wq = torch.empty_like(W), torch.empty_like(W)
        idx = torch.empty(k, dtype=torch.int32, device=DEV)
        nch = torch.zeros(1, dtype=torch.int64, device=DEV)

        def step():
            codes.copy_(codes0)
            cu = codes.view(torch.uint16)
            ctx.pv_dequantize(lay, cu, cb, sc, Wq)
            ctx.pv_encode_targets_select(lay, W, G, wl.alpha, T, k, idx)
            ctx.pv_reencode_groups(lay, T, cb, sc, idx, k, beam, cu, nch)
            ctx.pv_dequantize(lay, cu, cb, sc, Wq)

        step()                                    # the first call sizes the scratch buffers
        step()
        side.synchronize()
        want = (codes.clone(), Wq.clone(), idx.clone(), int(nch.item()))
        # the eager result is the oracle's
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, k)
        assert np.array_equal(want[2].cpu().numpy(), idx_ref)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        side.synchronize()
        for rep in range(4):
            codes.fill_(0)
            Wq.zero_()
            idx.zero_()
            nch.fill_(-7)
            if rep % 2:                           # eager calls of the same context in between
                step()
                codes.fill_(0)
                Wq.zero_()
            side.synchronize()
            graph.replay()
            side.synchronize()
            assert torch.equal(codes, want[0]), rep
            assert torch.equal(Wq, want[1]), rep
            assert torch.equal(idx, want[2]), rep
            assert int(nch.item()) == want[3], rep
        ctx.close()


@pytest.mark.parametrize("factor", [2.0, 0.25])
def test_captured_step_follows_a_codebook_that_changes_between_replays(factor):
    """A P step rewrites the codebook in place between two V steps: the replayed graph must see
    the new codebook's statistics (largest entry, norms, rounding error), not what an earlier
    replay left behind."""
    wl = workloads.make(128, 1024, 8, 1, 16, tau=0.1, sigma_g=5e-3, seed=731)
    lay = lay_of(wl)
    k = wl.k
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ctx = PVContext(0, stream=side)
        W, G = dev_f32(wl.W), dev_f32(wl.G)
        cb, sc = dev_f32(wl.codebooks), dev_f32(wl.scales)
        codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(DEV)
        codes = codes0.clone()
        T = torch.empty_like(W)
        idx = torch.empty(k, dtype=torch.int32, device=DEV)
        nch = torch.zeros(1, dtype=torch.int64, device=DEV)

        def step():
            codes.copy_(codes0)
            ctx.pv_encode_targets_select(lay, W, G, wl.alpha, T, k, idx)
            ctx.pv_reencode_groups(lay, T, cb, sc, idx, k, 1, codes.view(torch.uint16), nch)

        step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        side.synchronize()
        graph.replay()
        graph.replay()
        side.synchronize()
        cb.mul_(factor)                            # the codebook changes in place
        side.synchronize()
        graph.replay()
        side.synchronize()
        got = codes.clone()
        stats = ctx.pv_reencode_stats()
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, 8, k)
        new_cb = (wl.codebooks * np.float32(factor)).astype(np.float32)
        want, info = oracle.reencode_groups(T_ref, new_cb, wl.scales, idx_ref, wl.codes)
        g2 = got.cpu().numpy().view(np.uint16).reshape(-1)
        differ = np.nonzero(g2[idx_ref] != want.reshape(-1)[idx_ref])[0]
        assert info["near_tie"][differ].all(), (len(differ), differ[:5])
        # the filter still decides nearly every group itself
        assert stats["fallback"] < 0.05 * k, stats
        ctx.close()


def test_captured_step_forgets_the_statistics_of_the_last_replay():
    """The codebook statistics of a call are accumulated with atomics in a slot that eager calls
    alternate; a replayed graph keeps its slot, so the call clears it first when it is being
    captured.  Seen from outside: a codebook with a non-finite entry switches the filter off (every
    group is scanned exactly); once the entry is repaired in place the next replay must use the
    filter again."""
    wl = workloads.make(128, 1024, 8, 1, 16, tau=0.1, sigma_g=5e-3, seed=733)
    lay = lay_of(wl)
    k = wl.k
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ctx = PVContext(0, stream=side)
        W, G = dev_f32(wl.W), dev_f32(wl.G)
        cb, sc = dev_f32(wl.codebooks), dev_f32(wl.scales)
        good = float(cb[0, 77, 3].item())
        cb[0, 77, 3] = float("inf")
        codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(DEV)
        codes = codes0.clone()
        T = torch.empty_like(W)
        idx = torch.empty(k, dtype=torch.int32, device=DEV)
        nch = torch.zeros(1, dtype=torch.int64, device=DEV)

        def step():
            codes.copy_(codes0)
            ctx.pv_encode_targets_select(lay, W, G, wl.alpha, T, k, idx)
            ctx.pv_reencode_groups(lay, T, cb, sc, idx, k, 1, codes.view(torch.uint16), nch)

        step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        side.synchronize()
        graph.replay()
        side.synchronize()
        assert ctx.pv_reencode_stats()["fallback"] == k       # the filter is off
        cb[0, 77, 3] = good
        side.synchronize()
        graph.replay()
        side.synchronize()
        stats = ctx.pv_reencode_stats()
        assert stats["filtered"] + stats["fallback"] == k and stats["fallback"] < 0.05 * k, stats
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, 8, k)
        want, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, idx_ref, wl.codes)
        g2 = codes.cpu().numpy().view(np.uint16).reshape(-1)
        differ = np.nonzero(g2[idx_ref] != want.reshape(-1)[idx_ref])[0]
        assert info["near_tie"][differ].all(), (len(differ), differ[:5])
        ctx.close()


def _replays_equal_eager(side, run_once, outputs, scramble):
    """Captures run_once on `side`, replays it three times (outputs scrambled before each, an eager
    call in between) and compares the outputs with those of an eager call."""
    run_once()
    run_once()
    side.synchronize()
    want = [o.clone() for o in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_once()
    side.synchronize()
    for rep in range(3):
        scramble()
        if rep == 1:
            run_once()
            scramble()
        side.synchronize()
        graph.replay()
        side.synchronize()
        for o, w in zip(outputs, want):
            assert torch.equal(o.view(torch.uint8), w.view(torch.uint8)), rep


def test_captured_trust_ratio_step_replays_like_the_eager_one():
    wl = workloads.make(128, 1024, 8, 1, 12, tau=0.1, sigma_g=4e-3, seed=741)
    lay = lay_of(wl)
    k = wl.k
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ctx = PVContext(0, stream=side)
        G = dev_f32(wl.G)
        cb, sc = dev_f32(wl.codebooks), dev_f32(wl.scales)
        codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(DEV)
        codes = codes0.clone()
        Wq = torch.empty(wl.W.shape, dtype=torch.float32, device=DEV)
        T = torch.empty_like(Wq)
        rank = torch.empty(k, dtype=torch.int32, device=DEV)
        napp = torch.zeros(1, dtype=torch.int64, device=DEV)
        sums = torch.zeros(2, dtype=torch.float64, device=DEV)

        def run_once():
            codes.copy_(codes0)
            cu = codes.view(torch.uint16)
            ctx.pv_dequantize(lay, cu, cb, sc, Wq)
            ctx.pv_encode_targets(lay, Wq, G, 40.0, T)
            ctx.pv_reencode_trust_ratio(lay, T, Wq, cb, sc, k, max(1, k // 10), 0.01, 1, cu, rank, napp, sums)

        def scramble():
            codes.fill_(0)
            rank.zero_()
            napp.fill_(-3)
            sums.fill_(-1.0)

        _replays_equal_eager(side, run_once, [codes, rank, napp, sums], scramble)
        assert int(napp.item()) > 0
        ctx.close()


@pytest.mark.parametrize("g,M,B,shape", [(8, 1, 16, (128, 1024)), (8, 2, 8, (256, 2048)), (16, 1, 10, (64, 1024))])
def test_captured_p_step_and_stochastic_rounding_replay_like_the_eager_ones(g, M, B, shape):
    wl = workloads.make(shape[0], shape[1], g, M, B, tau=0.1, sigma_g=5e-3, seed=751 + B)
    lay = lay_of(wl)
    k = wl.k
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ctx = PVContext(0, stream=side)
        W, G = dev_f32(wl.W), dev_f32(wl.G)
        cb, sc = dev_f32(wl.codebooks), dev_f32(wl.scales)
        codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(DEV)
        codes = codes0.clone()
        gcb, gsc = torch.empty_like(cb), torch.empty_like(sc)

        def p_step():
            ctx.pv_codebook_grads(lay, G, codes0.view(torch.uint16), cb, sc, gcb, gsc)

        def scramble_p():
            gcb.fill_(9.0)
            gsc.fill_(9.0)

        _replays_equal_eager(side, p_step, [gcb, gsc], scramble_p)
        if M == 1:
            T = torch.empty_like(W)
            idx = torch.empty(k, dtype=torch.int32, device=DEV)
            nch = torch.zeros(1, dtype=torch.int64, device=DEV)

            def rounding():
                codes.copy_(codes0)
                ctx.pv_encode_targets_select(lay, W, G, wl.alpha, T, k, idx)
                ctx.pv_reencode_groups_stochastic(lay, T, cb, sc, idx, k, 5, 99, codes.view(torch.uint16), nch)

            def scramble_r():
                codes.fill_(0)
                nch.fill_(-1)

            _replays_equal_eager(side, rounding, [codes, nch], scramble_r)
        ctx.close()
