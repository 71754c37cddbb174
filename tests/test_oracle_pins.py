"""Pins for the CPU oracle: every routine is checked against something other
than itself -- the paper's worked example, closed forms in exact rational
arithmetic, brute force over all code tuples, library nearest-neighbour
routines, and the invariants the paper proves.  None of these needs a GPU.
"""
from fractions import Fraction
from itertools import product
from pathlib import Path

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle
import workloads

GOLDEN = Path(__file__).resolve().parent / "golden"


# ----------------------------------------------------------------- helpers

def f32_round(fr: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) fp32 value of a rational."""
    if fr == 0:
        return np.float32(0.0)
    c = np.float32(float(fr))          # at most one ulp off after double rounding
    cands = {c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))}
    best = None
    for v in cands:
        if not np.isfinite(v):
            continue
        err = abs(Fraction(float(v)) - fr)
        even = (np.array(v, dtype=np.float32).view(np.uint32) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, v)
    return best[1]


def fr(x) -> Fraction:
    return Fraction(float(x))


def exact_objective(cbs, tup, s, t) -> Fraction:
    """|| s * sum_m C_m[b_m] - t ||^2 in exact rational arithmetic."""
    tot = Fraction(0)
    for i in range(len(t)):
        acc = sum(fr(cbs[m][tup[m]][i]) for m in range(len(tup)))
        r = fr(s) * acc - fr(t[i])
        tot += r * r
    return tot


def tiny_problem(seed, out_f, in_f, g, M, B, scales="uniform"):
    wl = workloads.make(out_f, in_f, g, M, B, sigma_g=5e-3, scales=scales, seed=seed,
                        tau=1.0, beam_width=1)
    T = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    return wl, T


# ------------------------------------------------------------- O1: targets

def test_targets_exact_single_rounding():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((7, 24)).astype(np.float32) * np.float32(0.02)
    G = rng.standard_normal((7, 24)).astype(np.float32) * np.float32(1e-3)
    for alpha in (1.0, 0.3, 3e-3, -0.75):
        T = oracle.encode_targets(W, G, alpha)
        a = np.float32(alpha)
        for w, g_, t in zip(W.ravel(), G.ravel(), T.ravel()):
            assert t == f32_round(fr(w) - fr(a) * fr(g_))


def test_targets_special_cases():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((16, 64)).astype(np.float32)
    G = rng.standard_normal((16, 64)).astype(np.float32)
    assert np.array_equal(oracle.encode_targets(W, G, 0.0).view(np.uint32), W.view(np.uint32))
    assert np.array_equal(oracle.encode_targets(W, np.zeros_like(G), 0.7).view(np.uint32),
                          W.view(np.uint32))
    assert np.array_equal(oracle.encode_targets(W, G, 1.0), W - G)
    assert np.array_equal(oracle.encode_targets(W, G, -1.0), W + G)


# ----------------------------------------------------------- O2: selection

def test_selection_scores_exact_chain():
    rng = np.random.default_rng(3)
    g = 8
    W = rng.standard_normal((4, 32)).astype(np.float32) * np.float32(0.02)
    T = W + rng.standard_normal((4, 32)).astype(np.float32) * np.float32(1e-3)
    _, scores = oracle.select_topk_groups(T, W, g, 3, return_scores=True)
    Tg, Wg = T.reshape(-1, g), W.reshape(-1, g)
    for n in range(Tg.shape[0]):
        s = np.float32(0)
        for i in range(g):
            d = np.float32(Tg[n, i] - Wg[n, i])
            s = f32_round(fr(d) * fr(d) + fr(s))
        assert scores[n] == s
    # and it is the squared update norm up to fp32 rounding
    ref = ((Tg.astype(np.float64) - Wg.astype(np.float64)) ** 2).sum(1)
    assert np.allclose(scores, ref, rtol=1e-5)


@pytest.mark.parametrize("k", [0, 1, 5, 37, 96])
def test_selection_matches_full_sort(k):
    rng = np.random.default_rng(4)
    g = 4
    W = rng.standard_normal((8, 48)).astype(np.float32)
    T = W + rng.standard_normal((8, 48)).astype(np.float32)
    # plant exact score ties, some straddling the cut
    T.reshape(-1, g)[10] = W.reshape(-1, g)[10] + (T.reshape(-1, g)[3] - W.reshape(-1, g)[3])
    idx, scores = oracle.select_topk_groups(T, W, g, k, return_scores=True)
    N = scores.shape[0]
    order = np.lexsort((np.arange(N), -scores.astype(np.float64)))   # score desc, id asc
    assert np.array_equal(idx, np.sort(order[:k]).astype(np.int32))
    if 0 < k < N:
        sel = np.zeros(N, bool)
        sel[idx] = True
        assert scores[sel].min() >= scores[~sel].max()


def test_selection_special_cases():
    rng = np.random.default_rng(5)
    g = 8
    W = rng.standard_normal((8, 64)).astype(np.float32)
    T = W + rng.standard_normal((8, 64)).astype(np.float32)
    N = 64
    assert np.array_equal(oracle.select_topk_groups(T, W, g, N), np.arange(N, dtype=np.int32))
    sc = ((T - W).astype(np.float64) ** 2).reshape(N, g).sum(1)
    assert oracle.select_topk_groups(T, W, g, 1)[0] == int(np.argmax(sc))
    # all scores equal: the first k ids
    W2 = np.zeros_like(W)
    T2 = W2 + np.float32(0.5)
    assert np.array_equal(oracle.select_topk_groups(T2, W2, g, 9), np.arange(9, dtype=np.int32))
    # two equal maxima: lowest id wins at k = 1
    T3 = W.copy()
    T3.reshape(N, g)[[20, 41], 0] += np.float32(2.0)
    W3 = W.copy()
    W3.reshape(N, g)[[20, 41], 0] = 0
    T3.reshape(N, g)[[20, 41], 0] = 2.0
    assert oracle.select_topk_groups(T3, W3, g, 1)[0] == 20
    with pytest.raises(ValueError):
        oracle.select_topk_groups(T, W, g, N + 1)


# ------------------------------------------- O3: nearest codeword (M = 1)

def _read_golden():
    vals = {}
    for line in (GOLDEN / "app_p_vstep_example.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [float(v) for v in rest]
    return vals


def test_paper_worked_vstep_example():
    """App. P: xstar={2,10,0,11}, y0={2,5,5,11} -> x1={2,11,2,11}."""
    gold = _read_golden()
    xstar = np.array(gold["xstar"], np.float32)[None, :]
    y0 = np.array(gold["y0"], np.float32)[None, :]
    values = gold["values"]
    cb = np.array(values + [1.0e6], np.float32).reshape(1, 4, 1)     # pad to 2^2 codewords
    scales = np.ones(1, np.float32)
    codes0 = np.array([values.index(v) for v in gold["y0"]], np.uint16).reshape(1, 4, 1)
    assert np.array_equal(oracle.dequantize(codes0, cb, scales), y0)
    grad = 2.0 * (y0 - xstar)                    # gradient of sum (x - xstar)^2 at y0
    T = oracle.encode_targets(y0, grad, 0.5)     # 1/L with L = 2
    assert np.array_equal(T, xstar)
    idx = oracle.select_topk_groups(T, y0, 1, 4)
    new, info = oracle.reencode_groups(T, cb, scales, idx, codes0)
    x1 = oracle.dequantize(new, cb, scales)
    assert x1.ravel().tolist() == gold["x1"]
    assert info["num_changed"] == 2
    # restricted to the two coordinates with the largest update only those may move
    idx2 = oracle.select_topk_groups(T, y0, 1, 2)
    assert idx2.tolist() == [1, 2]
    new2, _ = oracle.reencode_groups(T, cb, scales, idx2, codes0)
    assert np.array_equal(new2, new)


def test_scalar_case_is_binary_search_in_sorted_values():
    """g = 1: nearest value of a sorted codebook (Sec. 3.2, scalar case; Alg. 6)."""
    rng = np.random.default_rng(6)
    B = 5
    vals = np.sort(rng.standard_normal(1 << B).astype(np.float32))
    cb = vals.reshape(1, -1, 1)
    T = rng.standard_normal((6, 40)).astype(np.float32) * np.float32(1.5)
    scales = np.ones(6, np.float32)
    codes0 = rng.integers(0, 1 << B, size=(6, 40, 1)).astype(np.uint16)
    new, _ = oracle.reencode_groups(T, cb, scales, np.arange(240), codes0)
    t = T.ravel().astype(np.float64)
    v = vals.astype(np.float64)
    hi = np.clip(np.searchsorted(v, t), 1, len(v) - 1)
    lo = hi - 1
    ref = np.where(np.abs(t - v[lo]) <= np.abs(v[hi] - t), lo, hi)
    assert np.array_equal(new.ravel(), ref.astype(np.uint16))


@pytest.mark.parametrize("g,B", [(8, 6), (16, 5), (4, 8), (2, 3)])
def test_m1_equals_library_nearest_neighbour(g, B):
    wl, T = tiny_problem(7 + g, 12, 8 * g, g, 1, B, scales="ones")
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes)
    D = cdist(T.reshape(-1, g).astype(np.float64), wl.codebooks[0].astype(np.float64),
              "sqeuclidean")
    assert np.array_equal(new.ravel(), D.argmin(1).astype(np.uint16))
    assert np.allclose(info["obj_new"], D.min(1), rtol=1e-9, atol=0)


def test_m1_with_scales_exact_rational_argmin():
    wl, T = tiny_problem(11, 6, 16, 4, 1, 4)
    wl.scales[2] = np.float32(-0.8)            # a negative scale is legal
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes)
    gpr = wl.layout.groups_per_row
    for n in idx:
        t = T.reshape(-1, 4)[n]
        s = wl.scales[n // gpr]
        objs = [exact_objective(wl.codebooks, (c,), s, t) for c in range(16)]
        assert new.reshape(-1)[n] == int(np.argmin(objs))
        assert abs(info["obj_new"][n] - float(min(objs))) <= 1e-12 * float(min(objs))


def test_m1_tie_rule_previous_code_then_lowest_index():
    g = 2
    cb = np.array([[[1, 0], [0, 1], [1, 0], [0, 1], [5, 5], [5, 5], [-3, 2], [1, 0]]], np.float32)
    scales = np.ones(1, np.float32)
    T = np.array([[1, 0, 1, 0, 0, 1, 5, 5]], np.float32)     # four groups
    codes0 = np.array([2, 4, 6, 5], np.uint16).reshape(1, 4, 1)
    new, info = oracle.reencode_groups(T, cb, scales, np.arange(4), codes0)
    # group0: minimisers {0,2,7}, previous 2 kept; group1: minimisers {0,2,7}, previous 4 not
    # one -> lowest (0); group2: minimisers {1,3} -> 1; group3: minimisers {4,5}, previous 5 kept
    assert new.ravel().tolist() == [2, 0, 1, 5]
    assert info["near_tie"].all()
    assert info["num_changed"] == 2


@pytest.mark.parametrize("ulps,flagged", [(0, True), (2, True), (4, True), (5, False), (8, False),
                                          (1000, False)])
def test_m1_near_tie_flag_is_the_stated_relative_tolerance(ulps, flagged):
    """The flag that excuses a differing code: best two objectives closer than 1e-6 RELATIVE.
    One weight per group, target 0, scale 1: the objectives are the squared codewords.  With
    codewords 1 and 1 + ulps * 2^-23 the relative gap of the objectives is about
    ulps * 2.38e-7: 4 ulps = 9.5e-7 (flagged), 5 ulps = 1.19e-6 (not flagged).  A tolerance off
    by a factor of two in either direction, or an absolute one, fails a case."""
    hi = np.float32(1.0) + np.float32(ulps) * np.float32(2.0 ** -23)
    for scale_pow in (0, -20, 20):      # the rule is relative: the flag must not depend on magnitude
        unit = np.float32(2.0 ** scale_pow)
        cb = np.array([[[1.0 * unit], [hi * unit], [3.0 * unit], [-2.5 * unit]]], np.float32)
        T = np.zeros((1, 1), np.float32)
        codes0 = np.array([2], np.uint16).reshape(1, 1, 1)
        new, info = oracle.reencode_groups(T, cb, np.ones(1, np.float32), np.arange(1), codes0)
        assert new.ravel().tolist() == [0]
        lo_obj, hi_obj = float(unit) ** 2, (float(hi) * float(unit)) ** 2
        assert info["obj_new"][0] == lo_obj
        assert ((hi_obj - lo_obj) < 1e-6 * hi_obj or hi_obj == lo_obj) == flagged   # the case is what it claims
        assert bool(info["near_tie"][0]) == flagged


@pytest.mark.parametrize("ulps,flagged", [(2, True), (4, True), (5, False), (8, False)])
def test_beam_near_tie_flag_at_the_prune_boundary(ulps, flagged):
    """Beam 1 over two codebooks of two codewords: at the first codebook the kept candidate
    (objective 1) and the dropped one (objective (1 + ulps * 2^-23)^2) are the only boundary
    in the run that is close: the second step's candidates are far apart and the winner is the
    previous tuple.  The flag must follow that one boundary."""
    hi = np.float32(1.0) + np.float32(ulps) * np.float32(2.0 ** -23)
    cb = np.array([[[1.0], [hi]], [[0.0], [5.0]]], np.float32)        # [M=2, 2, g=1]
    T = np.zeros((1, 1), np.float32)
    codes0 = np.array([0, 0], np.uint16).reshape(1, 1, 2)
    new, info = oracle.reencode_groups(T, cb, np.ones(1, np.float32), np.arange(1), codes0,
                                       beam_width=1)
    assert new.ravel().tolist() == [0, 0] and info["num_changed"] == 0
    assert info["obj_new"][0] == 1.0
    assert bool(info["near_tie"][0]) == flagged
    # the final best two (1 against 36) and the keep-or-replace decision are not close: with a
    # beam that drops nothing at the first step the same inputs are flagged only through the
    # final pair (1, hi^2)
    new2, info2 = oracle.reencode_groups(T, cb, np.ones(1, np.float32), np.arange(1), codes0,
                                         beam_width=2)
    assert new2.ravel().tolist() == [0, 0]
    assert bool(info2["near_tie"][0]) == flagged


@pytest.mark.parametrize("M,B", [(1, 3), (2, 2), (1, 15)])
def test_reencode_rejects_a_stored_code_outside_the_codebook(M, B):
    """A stored code >= 2^B is not an index into the codebook; the oracle refuses the call (as
    its dequantiser does) instead of reading outside the table.  Unlisted groups are not looked at."""
    rng = np.random.default_rng(5)
    g = 2
    cb = rng.standard_normal((M, 1 << B, g)).astype(np.float32)
    T = rng.standard_normal((2, 4 * g)).astype(np.float32)
    codes0 = rng.integers(0, 1 << B, size=(2, 4, M)).astype(np.uint16)
    oracle.reencode_groups(T, cb, np.ones(2, np.float32), np.arange(8), codes0, beam_width=2)
    bad = codes0.copy()
    bad[1, 2, M - 1] = 1 << B
    with pytest.raises(ValueError):
        oracle.reencode_groups(T, cb, np.ones(2, np.float32), np.arange(8), bad, beam_width=2)
    listed = np.array([0, 1, 2, 3, 4, 5, 7])      # group 6 = (1, 2) is not listed
    new, _ = oracle.reencode_groups(T, cb, np.ones(2, np.float32), listed, bad, beam_width=2)
    assert new[1, 2, M - 1] == 1 << B


def test_lemma_3_1_quadratic_model_brute_force():
    """argmin over all code tuples of <grad, x-y> + L/2 ||x-y||^2 equals the
    nearest representable point to y - grad/L (Lemma 3.1)."""
    rng = np.random.default_rng(8)
    g, B, ngroups, L = 2, 2, 4, 3.0
    cb = rng.standard_normal((1, 1 << B, g)).astype(np.float32)
    scales = np.ones(1, np.float32)
    codes0 = rng.integers(0, 1 << B, size=(1, ngroups, 1)).astype(np.uint16)
    y = oracle.dequantize(codes0, cb, scales)
    grad = rng.standard_normal(y.shape).astype(np.float32)
    best, best_tup = None, None
    for tup in product(range(1 << B), repeat=ngroups):
        x = cb[0][list(tup)].reshape(1, -1).astype(np.float64)
        val = float((grad * (x - y)).sum() + 0.5 * L * ((x - y) ** 2).sum())
        if best is None or val < best:
            best, best_tup = val, tup
    T = oracle.encode_targets(y, grad, 1.0 / L)
    new, _ = oracle.reencode_groups(T, cb, scales, np.arange(ngroups), codes0)
    assert tuple(int(c) for c in new.ravel()) == best_tup


def test_app_d_identity_argmin_without_target_norm():
    """||c - x||^2 = ||c||^2 - 2<c,x> + ||x||^2: dropping ||x||^2 keeps the argmin (App. D)."""
    wl, T = tiny_problem(13, 8, 64, 8, 1, 7, scales="ones")
    new, _ = oracle.reencode_groups(T, wl.codebooks, wl.scales,
                                    np.arange(wl.layout.num_groups), wl.codes)
    C = wl.codebooks[0].astype(np.float64)
    X = T.reshape(-1, 8).astype(np.float64)
    score = (C * C).sum(1)[None, :] - 2.0 * X @ C.T
    assert np.array_equal(new.ravel(), score.argmin(1).astype(np.uint16))


# --------------------------------------------------- O4: beam search (M >= 2)

def brute_force_tuples(cbs, s, t):
    M, csize, _ = cbs.shape
    best = None
    for tup in product(range(csize), repeat=M):
        o = exact_objective(cbs, tup, s, t)
        if best is None or o < best[0]:
            best = (o, tup)
    return best


@pytest.mark.parametrize("M,B,beam", [(2, 3, 8), (2, 4, 16), (2, 2, 64), (3, 2, 16)])
def test_wide_beam_equals_brute_force(M, B, beam):
    """A beam at least as wide as everything it can hold is exhaustive."""
    wl, T = tiny_problem(17 + M + B, 3, 16, 4, M, B)
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes, beam_width=beam)
    gpr = wl.layout.groups_per_row
    need = (1 << B) ** (M - 1)
    assert beam >= need
    for n in idx:
        t = T.reshape(-1, 4)[n]
        s = wl.scales[n // gpr]
        o, tup = brute_force_tuples(wl.codebooks, s, t)
        got = tuple(int(c) for c in new.reshape(-1, M)[n])
        assert exact_objective(wl.codebooks, got, s, t) == o
        assert abs(info["obj_new"][n] - float(o)) <= 1e-12 * float(o)


@pytest.mark.parametrize("beam", [1, 2, 8])
def test_beam_bounds_optimum_and_previous(beam):
    """brute-force optimum <= obj(result) <= obj(previous) (Lemma 3.2: y is feasible)."""
    wl, T = tiny_problem(23, 4, 32, 8, 2, 4)
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes, beam_width=beam)
    gpr = wl.layout.groups_per_row
    for n in idx:
        t = T.reshape(-1, 8)[n]
        s = wl.scales[n // gpr]
        o_best, _ = brute_force_tuples(wl.codebooks, s, t)
        o_new = exact_objective(wl.codebooks, tuple(new.reshape(-1, 2)[n]), s, t)
        o_old = exact_objective(wl.codebooks, tuple(wl.codes.reshape(-1, 2)[n]), s, t)
        assert o_best <= o_new <= o_old
    assert (info["obj_new"] <= info["obj_prev"]).all()


def test_beam_with_one_codebook_is_the_definition():
    wl, T = tiny_problem(29, 8, 64, 8, 1, 6)
    idx = np.arange(wl.layout.num_groups)
    a, ia = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes)
    for beam in (1, 3, 8):
        b, ib = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes,
                                       beam_width=beam, use_beam=True)
        assert np.array_equal(a, b)
        assert np.array_equal(ia["obj_new"], ib["obj_new"])


def test_beam_one_is_greedy_single_index_descent():
    """beam 1 = one pass of App. D's local search: fix all codes but one, take the best."""
    wl, T = tiny_problem(31, 4, 32, 4, 3, 3)
    idx = np.arange(wl.layout.num_groups)
    new, _ = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes, beam_width=1)
    gpr = wl.layout.groups_per_row
    for n in idx:
        t = T.reshape(-1, 4)[n]
        s = wl.scales[n // gpr]
        prev = [int(c) for c in wl.codes.reshape(-1, 3)[n]]
        cur = list(prev)
        for m in range(3):
            objs = []
            for c in range(8):
                trial = list(cur)
                trial[m] = c
                objs.append(exact_objective(wl.codebooks, trial, s, t))
            # ties: the lexicographically first tuple = lowest code at this position
            cur[m] = int(np.argmin(objs))
        if not exact_objective(wl.codebooks, cur, s, t) < exact_objective(wl.codebooks, prev, s, t):
            cur = prev
        assert [int(c) for c in new.reshape(-1, 3)[n]] == cur


def _python_beam(cbs, s, t, prev, beam):
    """Independent restatement of the beam reading in exact arithmetic (a cross-check against
    slips in the C code; the reading itself is only pinned by the bounds above)."""
    M, csize, _ = cbs.shape
    cur = [(exact_objective(cbs, prev, s, t), tuple(prev))]
    for m in range(M):
        pool = []
        for _, tup in cur:
            for c in range(csize):
                q = list(tup)
                q[m] = c
                pool.append((exact_objective(cbs, q, s, t), tuple(q)))
        pool.sort()
        cur = pool[:beam]
    o_prev = exact_objective(cbs, prev, s, t)
    return list(cur[0][1]) if cur[0][0] < o_prev else list(prev)


@pytest.mark.parametrize("beam", [2, 3, 8])
def test_beam_cross_check_exact_arithmetic(beam):
    wl, T = tiny_problem(37, 3, 32, 8, 2, 4)
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes, beam_width=beam)
    gpr = wl.layout.groups_per_row
    for n in idx:
        if info["near_tie"][n]:
            continue
        ref = _python_beam(wl.codebooks, wl.scales[n // gpr], T.reshape(-1, 8)[n],
                           [int(c) for c in wl.codes.reshape(-1, 2)[n]], beam)
        assert [int(c) for c in new.reshape(-1, 2)[n]] == ref


# -------------------------------------------------------- O5: dequantize

@pytest.mark.parametrize("M", [1, 2, 3])
def test_dequantize_definition(M):
    wl = workloads.make(10, 48, 8, M, 5, seed=41)
    W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
    acc = wl.codebooks[0][wl.codes[..., 0]]
    for m in range(1, M):
        acc = acc + wl.codebooks[m][wl.codes[..., m]]
    ref = (wl.scales[:, None, None] * acc).reshape(10, 48)
    assert W.dtype == np.float32 and np.array_equal(W, ref)
    # one hand-computed entry
    o, j, i = 3, 2, 5
    v = sum(float(wl.codebooks[m][wl.codes[o, j, m]][i]) for m in range(M)) * float(wl.scales[o])
    assert abs(W[o, j * 8 + i] - v) <= 1e-6 * abs(v)


def test_dequantize_rejects_out_of_range_code():
    wl = workloads.make(2, 16, 8, 1, 3, seed=43)
    wl.codes[1, 1, 0] = 9
    with pytest.raises(ValueError):
        oracle.dequantize(wl.codes, wl.codebooks, wl.scales)


# ---------------------------------------------------------- whole path

@pytest.mark.parametrize("M,B,beam", [(1, 8, 1), (2, 4, 4)])
def test_round_trip_is_a_fixed_point(M, B, beam):
    """If the target is the current point (zero update), no code changes (Sec. 3.2,
    'the optimal solution is often y itself')."""
    wl = workloads.make(16, 64, 8, M, B, seed=47, beam_width=beam)
    W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
    T = oracle.encode_targets(W, wl.G, 0.0)
    idx = np.arange(wl.layout.num_groups)
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes, beam_width=beam)
    assert np.array_equal(new, wl.codes) and info["num_changed"] == 0


@pytest.mark.parametrize("name,shape", [("c1_256x256_1x8", (64, 128)),
                                        ("c3_11008x4096_2x8", (32, 64))])
def test_path_invariants(name, shape):
    wl = workloads.make_config(name, seed=3, out_features=shape[0], in_features=shape[1], tau=0.1)
    g = wl.layout.group_size
    T = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    idx = oracle.select_topk_groups(T, wl.W, g, wl.k)
    assert len(idx) == wl.k and (np.diff(idx) > 0).all()
    new, info = oracle.reencode_groups(T, wl.codebooks, wl.scales, idx, wl.codes,
                                       beam_width=wl.beam_width)
    M = wl.layout.num_codebooks
    mask = np.ones(wl.layout.num_groups, bool)
    mask[idx] = False
    # codes outside the chosen subspace are untouched (Eq. 7)
    assert np.array_equal(new.reshape(-1, M)[mask], wl.codes.reshape(-1, M)[mask])
    # the re-encoded point is never worse than the previous one (Lemma 3.2)
    assert (info["obj_new"] <= info["obj_prev"]).all()
    obj = oracle.group_objective(T, wl.codebooks, wl.scales, idx, new.reshape(-1, M)[idx])
    assert np.array_equal(obj, info["obj_new"])
    W2 = oracle.dequantize(new, wl.codebooks, wl.scales)
    err_new = ((W2 - T).astype(np.float64) ** 2).reshape(-1, g).sum(1)[idx]
    assert np.allclose(err_new, info["obj_new"], rtol=1e-4)


# ---------------------------------------------- trust-ratio subspace size (Sec. 4.3, App. K)

def _tr_case(seed, M=1, B=5, beam=1, shape=(24, 128), g=8, sigma_g=1e-2):
    wl = workloads.make(shape[0], shape[1], g, M, B, seed=seed, sigma_g=sigma_g, beam_width=beam)
    # current weights = the dequantised codes, as in a real V step (the generator leaves W dense)
    wl.W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
    T = oracle.encode_targets(wl.W, wl.G, wl.alpha)
    return wl, T


def _rank_order(T, W, g, k):
    """Selection order (largest score first, lower id first) written out with numpy."""
    d = (T - W).reshape(-1, g).astype(np.float32)
    s = np.zeros(d.shape[0], dtype=np.float32)
    for i in range(g):
        s = np.float32(d[:, i]) * np.float32(d[:, i]) + s     # exact product + one rounding = fma
        # (products of fp32 are exact in double; emulate the fused op in double then round)
    s64 = np.zeros(d.shape[0], dtype=np.float64)
    acc = np.zeros(d.shape[0], dtype=np.float32)
    for i in range(g):
        acc = (d[:, i].astype(np.float64) ** 2 + acc.astype(np.float64)).astype(np.float32)
    del s, s64
    order = np.lexsort((np.arange(len(acc)), -acc.astype(np.float64)))
    return order[:k].astype(np.int32)


@pytest.mark.parametrize("seed,M,B,beam", [(31, 1, 5, 1), (32, 2, 3, 4), (33, 1, 8, 1)])
@pytest.mark.parametrize("ratio", [0.02, 0.1, 0.2])
def test_trust_ratio_is_the_largest_feasible_prefix(seed, M, B, beam, ratio):
    """Brute force over every prefix length, through independent routines: plain re-encode of
    the top-L groups, dequantise, Frobenius norms by numpy."""
    wl, T = _tr_case(seed, M=M, B=B, beam=beam)
    g = wl.layout.group_size
    k_max = 60
    new, info = oracle.reencode_trust_ratio(T, wl.W, wl.codebooks, wl.scales, wl.codes, k_max,
                                            chunk=7, ratio=ratio, beam_width=beam)
    rank = _rank_order(T, wl.W, g, k_max)
    assert np.array_equal(info["rank_idx"], rank)
    x0 = oracle.dequantize(wl.codes, wl.codebooks, wl.scales).astype(np.float64)
    feas, moved = [], []
    for L in range(k_max + 1):
        cL, _ = oracle.reencode_groups(T, wl.codebooks, wl.scales, np.sort(rank[:L]), wl.codes,
                                       beam_width=beam)
        xL = oracle.dequantize(cL, wl.codebooks, wl.scales).astype(np.float64)
        feas.append(np.linalg.norm(xL - x0) / np.linalg.norm(x0) < ratio)
        moved.append(int((cL != wl.codes).any(-1).sum()))
    best = max(L for L in range(k_max + 1) if feas[L])
    assert all(feas[: best + 1]), "change must grow with the prefix"
    if moved[best] == 0 and best < k_max:
        # the bound fails before any code has moved: one moved group is kept all the same
        # (it lies in the chunk the procedure was working on)
        first = min(L for L in range(k_max + 1) if moved[L] > 0)
        assert first <= (best // 7 + 1) * 7
        best = first
    want, _ = oracle.reencode_groups(T, wl.codebooks, wl.scales, np.sort(rank[:best]), wl.codes,
                                     beam_width=beam)
    assert np.array_equal(new, want)
    xb = oracle.dequantize(new, wl.codebooks, wl.scales).astype(np.float64)
    assert info["change_sq"] == pytest.approx(np.sum((xb - x0) ** 2), rel=1e-12)
    assert info["norm_sq"] == pytest.approx(np.sum(x0 ** 2), rel=1e-12)


def test_trust_ratio_closed_form_scalar_case():
    """g = 1, codebook {1, 2}, every weight at 1: a flipped weight changes by exactly 1, so with
    N = 100 and ratio 0.25 the bound 0.0625 * 100 admits exactly 6 flips (6 < 6.25 < 7)."""
    N = 100
    cb = np.array([[[1.0], [2.0]]], dtype=np.float32)
    scales = np.ones(1, dtype=np.float32)
    codes = np.zeros((1, N, 1), dtype=np.uint16)
    W = np.ones((1, N), dtype=np.float32)
    T = W.copy()
    movers = [5, 17, 3, 42, 99, 60, 8, 77, 23, 11]           # update sizes decrease in this order
    for r, n in enumerate(movers):
        T[0, n] = 1.0 + 0.95 - 0.03 * r                      # all nearer to 2 than to 1
    T[0, 50] = 1.2                                            # moves, but stays nearest to 1
    new, info = oracle.reencode_trust_ratio(T, W, cb, scales, codes, k_max=20, chunk=4, ratio=0.25)
    assert info["num_applied"] == 6
    assert list(info["rank_idx"][:11]) == movers + [50]
    flipped = np.nonzero(new[0, :, 0])[0]
    assert sorted(flipped) == sorted(movers[:6])
    assert info["change_sq"] == 6.0 and info["norm_sq"] == 100.0


@pytest.mark.parametrize("ratio", [0.03, 0.1])
def test_trust_ratio_does_not_depend_on_the_chunk_size(ratio):
    wl, T = _tr_case(34, B=6)
    ref = None
    for chunk in (1, 3, 7, 16, 50, 1000):
        new, info = oracle.reencode_trust_ratio(T, wl.W, wl.codebooks, wl.scales, wl.codes, 50,
                                                chunk=chunk, ratio=ratio)
        cur = (new.tobytes(), info["num_applied"], info["change_sq"])
        ref = ref or cur
        assert cur == ref


def test_trust_ratio_limits():
    wl, T = _tr_case(35, B=6)
    g = wl.layout.group_size
    k_max = 40
    rank = _rank_order(T, wl.W, g, k_max)
    # no bound: the plain V step on the k_max best groups
    new, info = oracle.reencode_trust_ratio(T, wl.W, wl.codebooks, wl.scales, wl.codes, k_max,
                                            chunk=9, ratio=1e30)
    want, winfo = oracle.reencode_groups(T, wl.codebooks, wl.scales, np.sort(rank), wl.codes)
    assert info["num_applied"] == k_max and np.array_equal(new, want)
    # bound zero: exactly one group changes, the first in selection order whose code moves
    new0, info0 = oracle.reencode_trust_ratio(T, wl.W, wl.codebooks, wl.scales, wl.codes, k_max,
                                              chunk=9, ratio=0.0)
    changed = np.nonzero((new0 != wl.codes).any(-1).ravel())[0]
    moved_in_order = [n for n in rank if (want.reshape(-1, 1)[n] != wl.codes.reshape(-1, 1)[n]).any()]
    first_chunk = list(rank[:9])
    if moved_in_order and moved_in_order[0] in first_chunk:
        assert list(changed) == [moved_in_order[0]]
        assert info0["num_applied"] == list(rank).index(moved_in_order[0]) + 1
    else:
        assert len(changed) == 0 and info0["num_applied"] == 0


def test_trust_ratio_bound_is_tight():
    wl, T = _tr_case(36, B=7, shape=(32, 256))
    k_max = 100
    new, info = oracle.reencode_trust_ratio(T, wl.W, wl.codebooks, wl.scales, wl.codes, k_max,
                                            chunk=10, ratio=0.1)
    L = info["num_applied"]
    assert 1 < L < k_max
    bound = 0.1 ** 2 * info["norm_sq"]
    assert info["change_sq"] < bound
    # one more group in selection order breaks the bound
    nxt = np.sort(info["rank_idx"][: L + 1])
    c2, _ = oracle.reencode_groups(T, wl.codebooks, wl.scales, nxt, wl.codes)
    x0 = oracle.dequantize(wl.codes, wl.codebooks, wl.scales).astype(np.float64)
    x2 = oracle.dequantize(c2, wl.codebooks, wl.scales).astype(np.float64)
    assert np.sum((x2 - x0) ** 2) >= bound


# ------------------------------------------------- Adam update as the direction (Sec. 3.4)

def _sqrt_f32(fr_val: Fraction) -> np.float32:
    """Correctly rounded fp32 square root of a non-negative rational (integer arithmetic)."""
    if fr_val == 0:
        return np.float32(0.0)
    import math
    scale = 1 << 200
    root = math.isqrt(fr_val.numerator * scale * scale // fr_val.denominator)   # floor(sqrt(x) * 2^200)
    lo = f32_round(Fraction(root, scale))
    # candidates around the truncated root; pick the one whose square is nearest in the sense of
    # |c - sqrt(x)|, decided exactly through the midpoints
    cands = sorted({lo, np.nextafter(lo, np.float32(np.inf)), np.nextafter(lo, np.float32(0))})
    best = None
    for c in cands:
        err = abs(Fraction(float(c)) - Fraction(root, scale))
        if best is None or err < best[0]:
            best = (err, c)
    return best[1]


def _adam_exact(w, g, m, v, t, lr, b1, b2, eps):
    """The oracle's operation sequence in exact rational arithmetic, rounding where it rounds."""
    F = Fraction
    b1f, b2f, lrf, epsf = (F(float(np.float32(x))) for x in (b1, b2, lr, eps))
    omb1 = f32_round(1 - b1f)
    omb2 = f32_round(1 - b2f)

    def powi_double(b, n):          # IEEE double multiplications, as the oracle does
        r, b = 1.0, float(b)
        while n > 0:
            if n & 1:
                r = r * b
            b = b * b
            n >>= 1
        return r
    c1 = np.float32(1.0 - powi_double(np.float32(b1), t))
    c2 = np.float32(1.0 - powi_double(np.float32(b2), t))
    mi = f32_round(b1f * F(float(m)) + F(float(f32_round(F(float(omb1)) * F(float(g))))))
    g2 = f32_round(F(float(g)) * F(float(g)))
    vi = f32_round(b2f * F(float(v)) + F(float(f32_round(F(float(omb2)) * F(float(g2))))))
    mhat = f32_round(F(float(mi)) / F(float(c1)))
    vhat = f32_round(F(float(vi)) / F(float(c2)))
    den = f32_round(F(float(_sqrt_f32(F(float(vhat))))) + epsf)
    upd = f32_round(F(float(mhat)) / F(float(den)))
    T = f32_round(F(float(w)) - lrf * F(float(upd)))
    return T, mi, vi


@pytest.mark.parametrize("t", [1, 2, 7, 1000])
def test_adam_targets_exact_rational(t):
    rng = np.random.default_rng(50 + t)
    n = 24
    W = (rng.standard_normal((2, n)) * 0.02).astype(np.float32)
    G = (rng.standard_normal((2, n)) * 1e-3).astype(np.float32)
    m = (rng.standard_normal((2, n)) * 1e-3).astype(np.float32) if t > 1 else np.zeros((2, n), np.float32)
    v = (rng.random((2, n)) * 1e-6).astype(np.float32) if t > 1 else np.zeros((2, n), np.float32)
    G[0, 0] = 0.0                                  # zero gradient, zero moments at t = 1
    T, m2, v2 = oracle.encode_targets_adam(W, G, m, v, t, 3e-3, 0.9, 0.95, 1e-8)
    for idx in np.ndindex(W.shape):
        want = _adam_exact(W[idx], G[idx], m[idx], v[idx], t, 3e-3, 0.9, 0.95, 1e-8)
        assert (T[idx], m2[idx], v2[idx]) == want, idx


def test_adam_targets_follow_a_library_optimiser():
    """Five consecutive updates against torch.optim.Adam (same rule, different rounding)."""
    import torch
    rng = np.random.default_rng(60)
    W0 = (rng.standard_normal((8, 32)) * 0.02).astype(np.float32)
    p = torch.nn.Parameter(torch.from_numpy(W0.copy()))
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8)
    W = W0.copy()
    m = np.zeros_like(W)
    v = np.zeros_like(W)
    for t in range(1, 6):
        G = (rng.standard_normal(W.shape) * 1e-3).astype(np.float32)
        p.grad = torch.from_numpy(G.copy())
        opt.step()
        T, m, v = oracle.encode_targets_adam(W, G, m, v, t, 3e-3, 0.9, 0.95, 1e-8)
        ref = p.detach().numpy()
        assert np.allclose(T, ref, rtol=0, atol=3e-3 * 2e-5), t     # a few 1e-5 of one step
        assert np.abs(T - W).max() > 1e-4                            # the steps are not trivial
        W = T.copy()


def test_adam_first_step_is_a_sign_step():
    rng = np.random.default_rng(61)
    W = (rng.standard_normal((4, 16)) * 0.02).astype(np.float32)
    G = (rng.standard_normal((4, 16)) * 1e-3).astype(np.float32)
    z = np.zeros_like(W)
    T, m, v = oracle.encode_targets_adam(W, G, z, z, 1, 1e-2, 0.9, 0.95, 1e-12)
    assert np.allclose(T, W - 1e-2 * np.sign(G), rtol=0, atol=1e-2 * 1e-5)
    assert np.allclose(m, 0.1 * G, rtol=1e-6) and np.allclose(v, 0.05 * G * G, rtol=1e-6)
    # selection then ranks by the size of the Adam update, as Sec. 3.4 prescribes
    idx = oracle.select_topk_groups(T, W, 8, 3)
    assert len(idx) == 3


# ------------------------------------------------ P-step gradients (Alg. 3, P step)

def _torch_dequantize(codes, cb, sc):
    """An independent dequantiser written with torch indexing (float64, differentiable)."""
    import torch
    M = cb.shape[0]
    idx = torch.from_numpy(codes.astype(np.int64))
    w = sum(cb[m][idx[..., m]] for m in range(M))            # [out, in/g, g]
    return (sc[:, None, None] * w).reshape(codes.shape[0], -1)


@pytest.mark.parametrize("g,M,B,shape", [(8, 1, 4, (12, 64)), (4, 2, 3, (9, 40)), (1, 1, 2, (5, 7)),
                                         (8, 3, 2, (6, 32))])
def test_codebook_grads_equal_automatic_differentiation(g, M, B, shape):
    import torch
    wl = workloads.make(shape[0], shape[1], g, M, B, seed=70, sigma_g=1e-2)
    cb = torch.tensor(wl.codebooks, dtype=torch.float64, requires_grad=True)
    sc = torch.tensor(wl.scales, dtype=torch.float64, requires_grad=True)
    W = _torch_dequantize(wl.codes, cb, sc)
    (W * torch.from_numpy(wl.G.astype(np.float64))).sum().backward()   # d/dW of <G, W> is G
    gc, gs = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
    assert np.allclose(gc, cb.grad.numpy(), rtol=1e-6, atol=1e-9)
    assert np.allclose(gs, sc.grad.numpy(), rtol=1e-6, atol=1e-9)
    # codewords nobody uses get exactly zero
    used = np.zeros((M, 1 << B), bool)
    for m in range(M):
        used[m, np.unique(wl.codes[..., m])] = True
    assert (gc[~used] == 0).all()


def test_codebook_grads_by_finite_differences_of_a_quadratic_loss():
    """phi(W) = 0.5 ||W - Z||^2 has dphi/dW = W - Z; central differences in double are exact for
    a quadratic up to rounding."""
    wl = workloads.make(6, 32, 8, 2, 3, seed=71)
    Z = wl.W.astype(np.float64)
    cb0, sc0 = wl.codebooks.astype(np.float64), wl.scales.astype(np.float64)

    def deq(cb, sc):
        w = sum(cb[m][wl.codes[..., m].astype(np.int64)] for m in range(cb.shape[0]))
        return (sc[:, None, None] * w).reshape(6, 32)

    def phi(cb, sc):
        return 0.5 * np.sum((deq(cb, sc) - Z) ** 2)
    G = (deq(cb0, sc0) - Z).astype(np.float32)
    gc, gs = oracle.codebook_grads(G, wl.codes, wl.codebooks, wl.scales)
    h = 1e-4
    rng = np.random.default_rng(71)
    for _ in range(25):
        m, c, i = rng.integers(2), rng.integers(8), rng.integers(8)
        e = np.zeros_like(cb0)
        e[m, c, i] = h
        fd = (phi(cb0 + e, sc0) - phi(cb0 - e, sc0)) / (2 * h)
        assert gc[m, c, i] == pytest.approx(fd, rel=1e-4, abs=1e-7)
    for o in range(6):
        e = np.zeros_like(sc0)
        e[o] = h
        fd = (phi(cb0, sc0 + e) - phi(cb0, sc0 - e)) / (2 * h)
        assert gs[o] == pytest.approx(fd, rel=1e-4, abs=1e-7)


def test_codebook_grads_exact_small_case():
    """One row, scale 2, codes [1, 0, 1]: dC[1] = 2 (G_0 + G_2), dC[0] = 2 G_1, ds = <G, q>."""
    cb = np.array([[[1.0, -1.0], [0.5, 4.0]]], dtype=np.float32)
    codes = np.array([[[1], [0], [1]]], dtype=np.uint16)
    G = np.array([[1.0, 2.0, 3.0, 4.0, 5.0, 6.0]], dtype=np.float32)
    gc, gs = oracle.codebook_grads(G, codes, cb, np.array([2.0], np.float32))
    assert np.array_equal(gc[0, 1], [2 * (1 + 5), 2 * (2 + 6)])
    assert np.array_equal(gc[0, 0], [2 * 3, 2 * 4])
    assert gs[0] == 1 * 0.5 + 2 * 4 + 3 * 1 + 4 * -1 + 5 * 0.5 + 6 * 4


# --------------------------------------- scalar uniform grid (App. K, "GPTQ" representation)

@pytest.mark.parametrize("nbits,block", [(2, 128), (3, 16), (4, 32), (8, 8)])
def test_scalar_reencode_is_rounding_to_the_nearest_grid_value(nbits, block):
    W, G, codes, sc, zp = workloads.make_scalar(6, 256, block, nbits, seed=90)
    T = oracle.encode_targets(oracle.dequantize_scalar(codes, sc, zp, block, nbits), G * 20, 1.0)
    idx = np.arange(T.size, dtype=np.int32)
    new, changed = oracle.reencode_scalar(T, sc, zp, idx, codes, block, nbits)
    # closed form: q = clip(rint(t / s + z)); compare where the target is not near a half-way point
    s_full = np.repeat(sc, block, axis=1).astype(np.float64)
    z_full = np.repeat(zp, block, axis=1).astype(np.float64)
    u = T.astype(np.float64) / s_full + z_full
    q = np.clip(np.rint(u), 0, (1 << nbits) - 1).astype(np.uint8)
    safe = np.abs(u - np.floor(u) - 0.5) > 1e-3
    assert safe.mean() > 0.9 and np.array_equal(new[safe], q[safe])
    assert changed == int((new != codes).sum()) and changed > 0
    # bisection in the sorted grid of each block: the same nearest value
    for o, i in [(0, 0), (3, 77), (5, 255), (2, 128)]:
        vals = (sc[o, i // block] * (np.arange(1 << nbits, dtype=np.float32) - zp[o, i // block])).astype(np.float32)
        order = np.argsort(vals, kind="stable")
        pos = np.searchsorted(vals[order], T[o, i])
        cand = [order[max(pos - 1, 0)], order[min(pos, len(order) - 1)]]
        near = min(cand, key=lambda c: (abs(float(vals[c]) - float(T[o, i])), c))
        if abs(abs(float(vals[cand[0]]) - float(T[o, i])) - abs(float(vals[cand[1]]) - float(T[o, i]))) > 1e-9:
            assert new[o, i] == near


def test_scalar_reencode_tie_rule_and_untouched_weights():
    sc = np.array([[1.0]], np.float32)
    zp = np.array([[0.0]], np.float32)
    codes = np.array([[2, 1, 0, 3]], np.uint8)
    T = np.array([[1.5, 1.5, 7.0, 100.0]], np.float32)          # half-way between 1 and 2
    new, changed = oracle.reencode_scalar(T, sc, zp, np.array([0, 1, 2], np.int32), codes, 4, 2)
    assert list(new[0]) == [2, 1, 3, 3]      # ties keep the previous code; 7 clips to 3; weight 3 not listed
    assert changed == 1
    new2, _ = oracle.reencode_scalar(T, sc, zp, np.array([0], np.int32), np.array([[0, 1, 0, 3]], np.uint8), 4, 2)
    assert new2[0, 0] == 1                   # previous code 0 is no minimiser: the lower of the tied values


def test_scalar_dequantize_definition():
    W, G, codes, sc, zp = workloads.make_scalar(5, 64, 16, 3, seed=91)
    got = oracle.dequantize_scalar(codes, sc, zp, 16, 3)
    want = np.repeat(sc, 16, axis=1) * (codes.astype(np.float32) - np.repeat(zp, 16, axis=1))
    assert np.array_equal(got, want.astype(np.float32))
