"""Pins for the oracle's two variants of the V step that the paper compares against and
combines with: the straight-through buffer (App. E) and stochastic rounding over the two nearest
codewords (App. F, temperature of App. K).  Each is checked against hand cases, exact
probabilities in rational arithmetic, brute force and the properties App. E / App. F state.
None of these needs a GPU.
"""
from fractions import Fraction
from math import sqrt

import numpy as np
import pytest

import oracle


# ------------------------------------------------------------ the generator

def test_generator_reproduces_the_published_first_outputs_of_splitmix64():
    # seed 0: the state after one increment is the increment itself; these are the first outputs
    # of the reference generator that every implementation's self-test lists
    assert oracle.random_bits(0, 0) == 0xE220A8397B1DCDAF
    assert oracle.random_bits(0, 1) == 0x6E789E6AA1B965F4
    assert oracle.random_bits(0, 2) == 0x06C45D188009454F


def test_generator_written_out_again_in_python_integers():
    mask = 2 ** 64 - 1

    def bits(seed, n):
        z = (seed + (n + 1) * 0x9E3779B97F4A7C15) & mask
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        return z ^ (z >> 31)

    rng = np.random.default_rng(3)
    for seed, n in zip(rng.integers(0, 2 ** 63, 50), rng.integers(0, 2 ** 31, 50)):
        assert oracle.random_bits(int(seed), int(n)) == bits(int(seed), int(n))
        assert oracle.uniform(int(seed), int(n)) == (bits(int(seed), int(n)) >> 11) / 2.0 ** 53


def test_variates_are_uniform_and_differ_between_seeds():
    u = np.array([oracle.uniform(11, n) for n in range(20000)])
    assert 0.0 <= u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4 * sqrt(1 / 12 / len(u))
    hist = np.histogram(u, bins=20, range=(0, 1))[0]
    chi2 = ((hist - 1000.0) ** 2 / 1000.0).sum()
    assert chi2 < 50.0            # 19 degrees of freedom: the 99.99 % point is 50.8
    v = np.array([oracle.uniform(12, n) for n in range(20000)])
    assert abs(np.corrcoef(u, v)[0, 1]) < 0.03


# --------------------------------------------------- stochastic rounding (App. F)

def two_point(target, n_groups, power, seed, grid=(0.0, 1.0), scale=1.0):
    cb = np.array([[[grid[0]], [grid[1]]]], np.float32)
    T = np.full((1, n_groups), target, np.float32)
    codes = np.zeros((1, n_groups, 1), np.uint16)
    new, info = oracle.reencode_stochastic(T, cb, np.array([scale], np.float32), np.arange(n_groups),
                                           codes, power=power, seed=seed)
    return new.reshape(-1), info


@pytest.mark.parametrize("power,exact", [(1, Fraction(3, 4)), (2, Fraction(9, 10)),
                                         (5, Fraction(243, 244))])
def test_probability_of_the_nearer_grid_point_is_the_inverse_distance_rule(power, exact):
    # target 1/4 between 0 and 1: distances 1/4 and 3/4, p(0) = (1/4)^-n / ((1/4)^-n + (3/4)^-n)
    # = 3^n / (1 + 3^n); all three operands are exact in binary
    n = 200000
    new, info = two_point(0.25, n, power, seed=5)
    assert abs(info["p_nearest"][0] - float(exact)) < 1e-15
    assert (info["nearest_two"] == [0, 1]).all()
    p = float(exact)
    freq = (new == 0).mean()
    assert abs(freq - p) < 4.5 * sqrt(p * (1 - p) / n)
    # the decision itself: nearest exactly where the variate is below p
    assert ((new == 0) == (info["variate"] < info["p_nearest"])).all()
    assert info["num_changed"] == int((new != 0).sum())


def test_scalar_rounding_with_power_one_is_unbiased():
    # App. F: with the two neighbours on either side and p inversely proportional to the distance,
    # the expectation of the rounded value is the target
    n = 200000
    for target in (0.125, 0.4, 0.75):
        new, _ = two_point(target, n, 1, seed=17)
        mean = new.astype(np.float64).mean()        # grid values are 0 and 1: the code is the value
        assert abs(mean - target) < 4.5 * sqrt(target * (1 - target) / n)


def test_both_nearest_on_one_side_gives_the_biased_rounding_app_f_describes():
    # codewords 1 and 1.25 both lie above the target 0: the expectation cannot be the target;
    # p(1) = 1.25 / (1 + 1.25) = 5/9 exactly
    n = 100000
    new, info = two_point(0.0, n, 1, seed=2, grid=(1.0, 1.25))
    assert abs(info["p_nearest"][0] - 5.0 / 9.0) < 1e-15
    freq = (new == 0).mean()
    assert abs(freq - 5.0 / 9.0) < 4.5 * sqrt(20.0 / 81.0 / n)
    mean_value = 1.0 * freq + 1.25 * (1 - freq)
    assert mean_value > 1.0


def test_target_on_a_codeword_and_single_codeword_leave_no_choice():
    new, info = two_point(1.0, 1000, 1, seed=9)
    assert (new == 1).all() and (info["p_nearest"] == 1.0).all()
    cb = np.array([[[0.5, -0.5]]], np.float32)              # 2^0 = 1 codeword is not a valid B
    with pytest.raises(Exception):
        oracle.reencode_stochastic(np.zeros((1, 2), np.float32), cb, np.ones(1, np.float32), [0],
                                   np.zeros((1, 1, 1), np.uint16))


def test_two_nearest_and_their_probability_by_brute_force():
    rng = np.random.default_rng(21)
    out_f, in_f, g, B = 6, 24, 4, 5
    cb = rng.normal(size=(1, 1 << B, g)).astype(np.float32)
    cb[0, 7] = cb[0, 3]                                      # duplicates: equal objectives, index order
    sc = (rng.random(out_f) + 0.5).astype(np.float32)
    T = rng.normal(size=(out_f, in_f)).astype(np.float32)
    codes = rng.integers(0, 1 << B, (out_f, in_f // g, 1)).astype(np.uint16)
    idx = np.arange(out_f * in_f // g)
    for power in (1, 3, 5):
        new, info = oracle.reencode_stochastic(T, cb, sc, idx, codes, power=power, seed=99)
        for j, n in enumerate(idx):
            t = T.reshape(-1, g)[n].astype(np.float64)
            s = float(sc[n // (in_f // g)])
            d2 = [sum((s * float(cb[0, c, i]) - t[i]) ** 2 for i in range(g)) for c in range(1 << B)]
            order = sorted(range(1 << B), key=lambda c: (d2[c], c))
            assert list(info["nearest_two"][j]) == order[:2]
            w1, w2 = sqrt(d2[order[0]]) ** -power, sqrt(d2[order[1]]) ** -power
            assert abs(info["p_nearest"][j] - w1 / (w1 + w2)) < 1e-12
            u = oracle.uniform(99, int(n))
            assert info["variate"][j] == u
            want = order[0] if u < info["p_nearest"][j] else order[1]
            assert new.reshape(-1)[n] == want


def test_unlisted_groups_keep_their_codes_and_large_power_approaches_the_nearest_codeword():
    rng = np.random.default_rng(4)
    out_f, in_f, g, B = 8, 64, 8, 6
    cb = rng.normal(size=(1, 1 << B, g)).astype(np.float32)
    sc = np.ones(out_f, np.float32)
    T = rng.normal(size=(out_f, in_f)).astype(np.float32)
    codes = rng.integers(0, 1 << B, (out_f, in_f // g, 1)).astype(np.uint16)
    idx = np.arange(0, 64, 3)
    new, info = oracle.reencode_stochastic(T, cb, sc, idx, codes, power=64, seed=1)
    rest = np.setdiff1d(np.arange(64), idx)
    assert (new.reshape(-1)[rest] == codes.reshape(-1)[rest]).all()
    det, _ = oracle.reencode_groups(T, cb, sc, idx, codes)
    sure = info["p_nearest"] > 1 - 1e-6
    assert sure.sum() >= 3        # in 8 dimensions the two nearest are often almost equally far
    assert (new.reshape(-1)[idx][sure] == det.reshape(-1)[idx][sure]).all()


def test_near_flag_marks_a_variate_at_the_probability_and_a_contested_second_place():
    # second and third codeword at the same distance up to 1e-9 relative: which one is "second" is
    # a matter of rounding
    cb = np.array([[[0.0], [1.0], [-1.0 - 1e-7], [5.0]]], np.float32)
    T = np.full((1, 4), 0.25, np.float32)
    _, info = oracle.reencode_stochastic(T, cb, np.ones(1, np.float32), np.arange(4),
                                         np.zeros((1, 4, 1), np.uint16), power=1, seed=0)
    assert not info["near_tie"].any()                 # 0.75 against 1.25: well separated
    cb[0, 2, 0] = np.nextafter(np.float32(-0.5), np.float32(-1))      # |t - c| = 0.75 + 1 ulp
    _, info = oracle.reencode_stochastic(T, cb, np.ones(1, np.float32), np.arange(4),
                                         np.zeros((1, 4, 1), np.uint16), power=1, seed=0)
    assert info["near_tie"].all()


# ------------------------------------------------ straight-through buffer (App. E)

def test_ste_buffer_accumulates_updates_that_the_plain_v_step_rounds_away():
    # one weight, grid {0, 1}, the weight sits at 0 and every step's gradient asks for +0.2:
    # the plain V step rounds 0 + 0.2 back to 0 for ever (the stalling of Sec. 3.3); the buffer
    # reaches 0.6 > 1/2 on the third step and the code flips (App. E)
    cb = np.array([[[0.0], [1.0]]], np.float32)
    sc = np.ones(1, np.float32)
    codes = np.zeros((1, 1, 1), np.uint16)
    G = np.full((1, 1), -1.0, np.float32)
    alpha = 0.2

    y = codes.copy()
    for _ in range(10):
        W = oracle.dequantize(y, cb, sc)
        T = oracle.encode_targets(W, G, alpha)
        y, _ = oracle.reencode_groups(T, cb, sc, [0], y)
    assert y[0, 0, 0] == 0

    buf = oracle.dequantize(codes, cb, sc)
    y = codes.copy()
    seen = []
    for _ in range(4):
        buf, y, _ = oracle.ste_step(buf, G, alpha, cb, sc, y)
        seen.append((round(float(buf[0, 0]), 6), int(y[0, 0, 0])))
    assert seen == [(0.2, 0), (0.4, 0), (0.6, 1), (0.8, 1)]


def test_ste_step_is_the_gradient_step_on_the_buffer_followed_by_the_l2_projection():
    rng = np.random.default_rng(8)
    out_f, in_f, g, B = 4, 32, 4, 4
    cb = rng.normal(size=(1, 1 << B, g)).astype(np.float32)
    sc = (rng.random(out_f) + 0.5).astype(np.float32)
    codes = rng.integers(0, 1 << B, (out_f, in_f // g, 1)).astype(np.uint16)
    buf = oracle.dequantize(codes, cb, sc)
    G = rng.normal(size=(out_f, in_f)).astype(np.float32)
    nb, nc, info = oracle.ste_step(buf, G, 0.3, cb, sc, codes)
    want_buf = (buf.astype(np.float64) - np.float64(np.float32(0.3)) * G).astype(np.float32)
    assert np.array_equal(nb, want_buf)
    # projection: every group of the new codes is a nearest codeword of the buffer (scipy-free brute force)
    tb = nb.reshape(-1, g).astype(np.float64)
    for n in range(tb.shape[0]):
        s = float(sc[n // (in_f // g)])
        d = ((s * cb[0].astype(np.float64) - tb[n]) ** 2).sum(1)
        assert d[nc.reshape(-1)[n]] == d.min()


def test_subspace_ste_moves_only_the_groups_farthest_from_the_quantised_weights():
    rng = np.random.default_rng(9)
    out_f, in_f, g, B = 4, 64, 8, 5
    cb = rng.normal(size=(1, 1 << B, g)).astype(np.float32)
    sc = np.ones(out_f, np.float32)
    codes = rng.integers(0, 1 << B, (out_f, in_f // g, 1)).astype(np.uint16)
    Wq = oracle.dequantize(codes, cb, sc)
    buf = Wq.copy()
    G = rng.normal(size=(out_f, in_f)).astype(np.float32)
    nb, nc, info = oracle.ste_step(buf, G, 0.5, cb, sc, codes, k=5)
    dist = ((nb.astype(np.float64) - Wq) ** 2).reshape(-1, g).sum(1)
    assert set(info["group_idx"]) == set(np.argsort(-dist, kind="stable")[:5])
    moved = np.nonzero(nc.reshape(-1) != codes.reshape(-1))[0]
    assert set(moved) <= set(info["group_idx"])
