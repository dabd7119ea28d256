"""Pins for the quantiser oracle (Algorithm 1 of section 3.2 with the building blocks of section 2.2).

The oracle is checked against things other than itself: the q = 1 closed form and the greedy
recurrence of section 2.2 written out with numpy, numpy's least-squares routine, brute-force
nearest-level search, exhaustive search of ALL code assignments on tiny groups, the textbook
monotonicity of alternating minimisation, matrices that are exactly representable, the claims
that planes are shared/frozen and that the error does not grow with p, and exact symmetries
(power-of-two scaling, negation, column permutation, shift with an offset).
"""
import itertools

import numpy as np
import pytest

import oracle
import synthetic_inputs as syn


def rebuild(q, p, group, w_shape):
    """W_p from the oracle's codes and scale set p (numpy, float64)."""
    W = np.zeros(w_shape, dtype=np.float64)
    for i in range(p):
        W += np.repeat(q["scales"][p][i], group, axis=1) * q["codes"][i]
    if q["offsets"] is not None:
        W += np.repeat(q["offsets"][p], group, axis=1)
    return W


def group_err(w, W, group):
    d = (w.astype(np.float64) - W) ** 2
    return d.reshape(w.shape[0], -1, group).sum(axis=2)


def sign1(v):
    return np.where(v >= 0, 1.0, -1.0)


def gauss(m, n, seed):
    return syn.make_weights(m, n, seed=(90, seed))


# ----------------------------------------------------------------------------------------------
# section 2.2: q = 1 and the greedy recurrence
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cycles", [0, 1, 5])
def test_one_bit_closed_form(cycles):
    """q = 1: B = sign(W), alpha = <W, B> / |B|^2 = mean |w| per group; further cycles change nothing."""
    w = gauss(6, 256, 1)
    q = oracle.quantize(w, 1, 1, cycles, group=128)
    wd = w.astype(np.float64)
    assert np.array_equal(q["codes"][0], sign1(wd).astype(np.int8))
    alpha = np.abs(wd).reshape(6, 2, 128).mean(axis=2)
    np.testing.assert_allclose(q["scales"][1][0], alpha, rtol=1e-13)


def greedy_numpy(wd, p, group):
    """b_i = sign(r_{i-1}), a_i = <r_{i-1}, b_i> / g, r_i = r_{i-1} - a_i b_i, written with numpy."""
    m, n = wd.shape
    r = wd.copy()
    codes, alphas = [], []
    for _ in range(p):
        b = sign1(r)
        a = (r * b).reshape(m, -1, group).mean(axis=2)
        r = r - np.repeat(a, group, axis=1) * b
        codes.append(b)
        alphas.append(a)
    return np.stack(codes), np.stack(alphas)


@pytest.mark.parametrize("p", [2, 3, 4])
def test_greedy_recurrence(p):
    """T = 0 leaves the greedy initialisation: residual signs and mean absolute residuals."""
    w = gauss(5, 384, 2)
    q = oracle.quantize(w, p, p, 0, group=128)
    codes, alphas = greedy_numpy(w.astype(np.float64), p, 128)
    assert np.array_equal(q["codes"], codes.astype(np.int8))
    np.testing.assert_allclose(q["scales"][p], alphas, rtol=1e-12)


# ----------------------------------------------------------------------------------------------
# one cycle of the base stage: LS against numpy's routine, BS against brute force
# ----------------------------------------------------------------------------------------------
def lstsq_groups(B, wd, group, with_offset=False):
    """numpy.linalg.lstsq per (row, group); B is [p][m][n] of +-1."""
    p, m, n = B.shape
    out = np.zeros((p + int(with_offset), m, n // group))
    for r in range(m):
        for G in range(n // group):
            cols = [B[i, r, G * group:(G + 1) * group] for i in range(p)]
            if with_offset:
                cols.append(np.ones(group))
            A = np.stack(cols, axis=1).astype(np.float64)
            sol = np.linalg.lstsq(A, wd[r, G * group:(G + 1) * group], rcond=None)[0]
            out[:, r, G] = sol
    return out


def nearest_codes(wd, alpha, group, z=None):
    """Brute force: for every weight the +-1 combination whose level is nearest (numpy argmin)."""
    p, m, ng = alpha.shape
    combos = np.array(list(itertools.product([-1.0, 1.0], repeat=p)))          # plane 1 varies slowest
    codes = np.zeros((p, m, ng * group))
    for r in range(m):
        for G in range(ng):
            lev = combos @ alpha[:, r, G] + (0.0 if z is None else z[r, G])
            seg = wd[r, G * group:(G + 1) * group]
            best = np.argmin(np.abs(seg[:, None] - lev[None, :]), axis=1)
            codes[:, r, G * group:(G + 1) * group] = combos[best].T
    return codes


@pytest.mark.parametrize("p", [2, 3])
def test_first_cycle_ls_then_bs(p):
    """T = 1 at the base precision: scales = lstsq(greedy codes, w), codes = nearest level of those scales."""
    w = gauss(4, 256, 3)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, p, p, 1, group=128)
    g_codes, _ = greedy_numpy(wd, p, 128)
    alpha = lstsq_groups(g_codes, wd, 128)
    np.testing.assert_allclose(q["scales"][p], alpha, rtol=1e-9, atol=1e-15)
    assert np.array_equal(q["codes"], nearest_codes(wd, q["scales"][p], 128).astype(np.int8))


@pytest.mark.parametrize("cycles", [1, 3, 20])
def test_codes_are_nearest_levels_of_output_scales(cycles):
    """The base stage ends with BS: its codes are the nearest levels under the scales it returns."""
    w = gauss(4, 256, 4)
    q = oracle.quantize(w, 2, 2, cycles, group=128)
    assert np.array_equal(q["codes"], nearest_codes(w.astype(np.float64), q["scales"][2], 128).astype(np.int8))


def test_alternating_never_increases_error():
    """Textbook property of alternating minimisation: LS and BS each cannot raise the error, so the
    error after T cycles is non-increasing in T, and never above the greedy one."""
    w = gauss(8, 256, 5)
    errs = []
    for cycles in range(0, 8):
        q = oracle.quantize(w, 2, 2, cycles, group=128)
        errs.append(group_err(w, rebuild(q, 2, 128, w.shape), 128))
    for a, b in zip(errs, errs[1:]):
        assert np.all(b <= a * (1 + 1e-12) + 1e-18)
    assert np.any(errs[-1] < errs[0] * 0.99)        # and it does improve on greedy


def test_exhaustive_optimum_on_tiny_groups():
    """g = 6, q = 2: enumerate all 2^12 code assignments with least-squares scales.  The alternating
    result lies between that optimum and the greedy error."""
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((6, 6)) * 0.05).astype(np.float16)
    wd = w.astype(np.float64)
    q0 = oracle.quantize(w, 2, 2, 0, group=6)
    q = oracle.quantize(w, 2, 2, 20, group=6)
    e0 = group_err(w, rebuild(q0, 2, 6, w.shape), 6)[:, 0]
    e = group_err(w, rebuild(q, 2, 6, w.shape), 6)[:, 0]
    signs = np.array(list(itertools.product([-1.0, 1.0], repeat=6)))
    for r in range(6):
        best = np.inf
        for b1 in signs:
            for b2 in signs:
                A = np.stack([b1, b2], axis=1)
                sol, *_ = np.linalg.lstsq(A, wd[r], rcond=None)
                best = min(best, float(np.sum((wd[r] - A @ sol) ** 2)))
        assert best <= e[r] * (1 + 1e-9) + 1e-18
        assert e[r] <= e0[r] * (1 + 1e-12) + 1e-18


# ----------------------------------------------------------------------------------------------
# progressive expansion (Algorithm 1, the branch p > p_L)
# ----------------------------------------------------------------------------------------------
def test_planes_are_frozen_and_shared():
    """Section 3.2: codes of earlier precisions stay fixed; the 2-bit model inside a 2..4-bit model is
    the 2-bit model, and the 3-bit one inside it is the 2..3-bit one."""
    w = gauss(6, 256, 6)
    q24 = oracle.quantize(w, 2, 4, 7)
    q23 = oracle.quantize(w, 2, 3, 7)
    q22 = oracle.quantize(w, 2, 2, 7)
    assert np.array_equal(q24["codes"][:2], q22["codes"])
    assert np.array_equal(q24["codes"][:3], q23["codes"])
    assert np.array_equal(q24["scales"][2], q22["scales"][2])
    assert np.array_equal(q24["scales"][3], q23["scales"][3])
    # a set per precision: the first two scales of set 3 are not those of set 2
    assert not np.allclose(q24["scales"][3][:2], q24["scales"][2])


def test_new_plane_is_sign_of_residual_first_cycle():
    """T = 1: plane p = sign(w - W_{p-1}) with the scale set of p-1, then LS over all p planes."""
    w = gauss(4, 256, 7)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, 2, 4, 1)
    for p in (3, 4):
        prev = {"codes": q["codes"], "scales": q["scales"], "offsets": None}
        R = wd - rebuild(prev, p - 1, 128, w.shape)
        assert np.array_equal(q["codes"][p - 1], sign1(R).astype(np.int8))
        alpha = lstsq_groups(q["codes"][:p].astype(np.float64), wd, 128)
        np.testing.assert_allclose(q["scales"][p], alpha, rtol=1e-9, atol=1e-15)


def test_expansion_cycles_replayed_with_numpy():
    """T = 3 at 3 bits, replayed with numpy: every cycle takes the residual after the two frozen planes
    under the CURRENT 3-bit scales (not those of the 2-bit set), re-signs plane 3 and refits all scales."""
    w = gauss(3, 256, 18)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, 2, 3, 3)
    B = q["codes"].astype(np.float64)
    alpha = np.concatenate([q["scales"][2], np.zeros((1, 3, 2))])
    for _ in range(3):
        R = wd - sum(np.repeat(alpha[i], 128, axis=1) * B[i] for i in range(2))
        B[2] = sign1(R)
        alpha = lstsq_groups(B, wd, 128)
    assert np.array_equal(q["codes"][2], B[2].astype(np.int8))
    np.testing.assert_allclose(q["scales"][3], alpha, rtol=1e-8, atol=1e-14)


@pytest.mark.parametrize("p_high,cycles", [(3, 3), (4, 2), (4, 5)])
def test_listing_residual_cycles_replayed_with_numpy(p_high, cycles):
    """The expansion loop exactly as Algorithm 1 prints it (literal_residual=True), replayed with numpy: every cycle
    takes R = W - Dequant over ALL p planes with the current scales -- the new plane included, zero with a zero
    scale in the first cycle -- re-signs the new plane with sign(R) and refits all p scales by least squares."""
    w = gauss(3, 256, 19)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, 2, p_high, cycles, literal_residual=True)
    B = q["codes"].astype(np.float64).copy()
    alpha = q["scales"][2]
    for p in range(3, p_high + 1):
        alpha = np.concatenate([alpha, np.zeros((1, 3, 2))])           # alpha^p starts as [alpha^(p-1), 0]
        Bp = B[:p].copy()
        Bp[p - 1] = 0.0                                                # B_p starts as 0
        for _ in range(cycles):
            R = wd - sum(np.repeat(alpha[i], 128, axis=1) * Bp[i] for i in range(p))
            Bp[p - 1] = sign1(R)
            alpha = lstsq_groups(Bp, wd, 128)
        assert np.array_equal(q["codes"][p - 1], Bp[p - 1].astype(np.int8)), f"plane {p} differs from the replay"
        np.testing.assert_allclose(q["scales"][p], alpha, rtol=1e-8, atol=1e-14)
        assert np.array_equal(q["codes"][:p - 1], B[:p - 1].astype(np.int8))      # frozen planes untouched


def test_listing_residual_differs_from_the_default_from_the_second_cycle_on():
    """Both forms agree after one cycle and part ways from the second (the new plane enters its own residual)."""
    w = gauss(4, 256, 20)
    a1, b1 = oracle.quantize(w, 2, 3, 1), oracle.quantize(w, 2, 3, 1, literal_residual=True)
    assert np.array_equal(a1["codes"], b1["codes"])
    a2, b2 = oracle.quantize(w, 2, 3, 2), oracle.quantize(w, 2, 3, 2, literal_residual=True)
    assert np.array_equal(a2["codes"][:2], b2["codes"][:2])
    assert not np.array_equal(a2["codes"][2], b2["codes"][2])


@pytest.mark.parametrize("cycles", [2, 20])
def test_expansion_ends_with_least_squares(cycles):
    """Each expansion stage ends with LS: its scale set is numpy's least-squares solution for its planes."""
    w = gauss(4, 256, 8)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, 2, 4, cycles)
    for p in (3, 4):
        alpha = lstsq_groups(q["codes"][:p].astype(np.float64), wd, 128)
        np.testing.assert_allclose(q["scales"][p], alpha, rtol=1e-8, atol=1e-14)


def test_error_does_not_grow_with_precision():
    """Abstract / section 3.2: each added plane refines the model; per group err_2 >= err_3 >= err_4,
    because LS at p bits can always fall back to [alpha^(p-1), 0]."""
    w = syn.make_weights(16, 512, seed=(90, 9), heavy_tail=False)
    q = oracle.quantize(w, 2, 4, 20)
    e = [group_err(w, rebuild(q, p, 128, w.shape), 128) for p in (2, 3, 4)]
    assert np.all(e[1] <= e[0] * (1 + 1e-12))
    assert np.all(e[2] <= e[1] * (1 + 1e-12))
    rel = [float(x.sum() / (w.astype(np.float64) ** 2).sum()) for x in e]
    # Gaussian weights: near the distortion of the optimal 2/3/4-bit scalar quantiser of a Gaussian
    # (0.1175, 0.0345, 0.0095 of the variance); the shared, frozen planes cost a little at 3 and 4 bits
    assert 0.09 < rel[0] < 0.14 and 0.03 < rel[1] < 0.05 and 0.009 < rel[2] < 0.025


def test_listing_residual_reading_is_worse():
    """The listing's residual (new plane included in its own residual from the second cycle on) flips
    every code whose residual is below the new scale and does not settle; the reading taken (residual
    after the frozen planes) gives a clearly smaller 3- and 4-bit error.  Same result at T = 1."""
    w = gauss(16, 512, 10)
    q = oracle.quantize(w, 2, 4, 20)
    ql = oracle.quantize(w, 2, 4, 20, literal_residual=True)
    for p in (3, 4):
        e = group_err(w, rebuild(q, p, 128, w.shape), 128).sum()
        el = group_err(w, rebuild(ql, p, 128, w.shape), 128).sum()
        assert e < 0.7 * el
    q1 = oracle.quantize(w, 2, 4, 1)
    ql1 = oracle.quantize(w, 2, 4, 1, literal_residual=True)
    assert np.array_equal(q1["codes"], ql1["codes"])
    for p in (2, 3, 4):
        assert np.array_equal(q1["scales"][p], ql1["scales"][p])


# ----------------------------------------------------------------------------------------------
# exactly representable matrices, degenerate groups
# ----------------------------------------------------------------------------------------------
def test_exact_two_bit_matrix_is_recovered():
    """w = +-0.5 +- 0.25 with all four levels equally frequent: greedy already finds the codes,
    LS the scales (0.5, 0.25); error 0 at every precision."""
    rng = np.random.default_rng(5)
    m, n = 4, 256
    b1 = np.tile(np.array([1.0, 1.0, -1.0, -1.0]), (m, n // 4))
    b2 = np.tile(np.array([1.0, -1.0, 1.0, -1.0]), (m, n // 4))
    perm = rng.permutation(128)
    b1 = np.concatenate([b1[:, :128][:, perm], b1[:, 128:][:, perm]], axis=1)
    b2 = np.concatenate([b2[:, :128][:, perm], b2[:, 128:][:, perm]], axis=1)
    w = (0.5 * b1 + 0.25 * b2).astype(np.float16)
    q = oracle.quantize(w, 2, 4, 3)
    assert np.array_equal(q["codes"][0], b1.astype(np.int8))
    assert np.array_equal(q["codes"][1], b2.astype(np.int8))
    np.testing.assert_allclose(q["scales"][2][0], 0.5, rtol=1e-14)
    np.testing.assert_allclose(q["scales"][2][1], 0.25, rtol=1e-14)
    for p in (2, 3, 4):
        assert np.all(group_err(w, rebuild(q, p, 128, w.shape), 128) < 1e-28)


def test_zero_and_constant_groups():
    """A zero group: all levels tie, so BS picks the first enumerated one (every base code -1), and
    later planes are sign(0) = +1; dependent planes get scale 0; nothing is NaN."""
    w = np.zeros((2, 256), dtype=np.float16)
    w[1, :128] = 0.375                                  # a constant group
    w[1, 128:] = -0.375
    q = oracle.quantize(w, 2, 4, 4)
    assert np.all(np.abs(q["codes"]) == 1)
    assert np.all(q["codes"][:2, 0, :] == -1) and np.all(q["codes"][2:, 0, :] == 1)
    for p in (2, 3, 4):
        assert np.all(np.isfinite(q["scales"][p]))
        assert np.all(q["scales"][p][:, 0, :] == 0.0)
        assert np.all(group_err(w, rebuild(q, p, 128, w.shape), 128) < 1e-28)
    assert np.all(q["codes"][0, 1, :128] == 1) and np.all(q["codes"][0, 1, 128:] == -1)
    np.testing.assert_allclose(q["scales"][2][0, 1], 0.375, rtol=1e-14)
    assert np.all(q["scales"][2][1, 1] == 0.0)          # second plane equals +-first: dependent


# ----------------------------------------------------------------------------------------------
# exact symmetries
# ----------------------------------------------------------------------------------------------
def test_power_of_two_scaling_is_exact():
    w = gauss(4, 256, 12)
    q = oracle.quantize(w, 2, 4, 6)
    q4 = oracle.quantize((w.astype(np.float32) * 4).astype(np.float16), 2, 4, 6)
    assert np.array_equal(q["codes"], q4["codes"])
    for p in (2, 3, 4):
        assert np.array_equal(q["scales"][p] * 4.0, q4["scales"][p])


def test_negation_negates_codes():
    w = gauss(4, 256, 13)
    assert not np.any(w == 0)
    q = oracle.quantize(w, 2, 4, 6)
    qn = oracle.quantize(-w, 2, 4, 6)
    assert np.array_equal(q["codes"], -qn["codes"])
    for p in (2, 3, 4):
        np.testing.assert_allclose(q["scales"][p], qn["scales"][p], rtol=1e-12)


def test_column_permutation_inside_groups_permutes_codes():
    """Sums of binary16 values are exact in double, so the order inside a group cannot matter."""
    w = gauss(4, 256, 14)
    rng = np.random.default_rng(3)
    perm = np.concatenate([rng.permutation(128), 128 + rng.permutation(128)])
    q = oracle.quantize(w, 2, 4, 6)
    qp = oracle.quantize(np.ascontiguousarray(w[:, perm]), 2, 4, 6)
    assert np.array_equal(q["codes"][:, :, perm], qp["codes"])
    for p in (2, 3, 4):
        np.testing.assert_allclose(q["scales"][p], qp["scales"][p], rtol=1e-12)


def test_group_size_is_respected():
    """Groups are independent: quantising two groups at once equals quantising each alone."""
    w = gauss(3, 256, 15)
    q = oracle.quantize(w, 2, 4, 5)
    for G in range(2):
        qg = oracle.quantize(np.ascontiguousarray(w[:, G * 128:(G + 1) * 128]), 2, 4, 5)
        assert np.array_equal(q["codes"][:, :, G * 128:(G + 1) * 128], qg["codes"])
        for p in (2, 3, 4):
            assert np.array_equal(q["scales"][p][:, :, G:G + 1], qg["scales"][p])


# ----------------------------------------------------------------------------------------------
# asymmetric scheme (section 4.1): the offset as one more least-squares unknown
# ----------------------------------------------------------------------------------------------
def test_offset_is_least_squares_with_a_ones_column():
    w = gauss(4, 256, 16)
    wd = w.astype(np.float64)
    q = oracle.quantize(w, 2, 4, 5, with_offset=True)
    for p in (3, 4):
        sol = lstsq_groups(q["codes"][:p].astype(np.float64), wd, 128, with_offset=True)
        np.testing.assert_allclose(q["scales"][p], sol[:p], rtol=1e-8, atol=1e-14)
        np.testing.assert_allclose(q["offsets"][p], sol[p], rtol=1e-7, atol=1e-12)
    assert np.array_equal(q["codes"][:2], nearest_codes(wd, q["scales"][2], 128, z=q["offsets"][2]).astype(np.int8))


def test_offset_absorbs_a_shift():
    """Weights k / 256 and the same plus 1.0 (both exact in binary16): same codes, same scales,
    offsets 1.0 apart; and the offset never makes the error worse than the symmetric fit."""
    rng = np.random.default_rng(8)
    k = np.clip(np.round(rng.standard_normal((4, 256)) * 40), -200, 200)
    w0 = (k / 256.0).astype(np.float16)
    w1 = (k / 256.0 + 1.0).astype(np.float16)
    assert np.array_equal(w1.astype(np.float64), w0.astype(np.float64) + 1.0)
    q0 = oracle.quantize(w0, 2, 4, 6, with_offset=True)
    q1 = oracle.quantize(w1, 2, 4, 6, with_offset=True)
    assert np.array_equal(q0["codes"], q1["codes"])
    for p in (2, 3, 4):
        np.testing.assert_allclose(q0["scales"][p], q1["scales"][p], rtol=1e-9, atol=1e-13)
        np.testing.assert_allclose(q0["offsets"][p] + 1.0, q1["offsets"][p], rtol=1e-11)
    qs = oracle.quantize(w1, 2, 4, 6)
    for p in (2, 3, 4):
        assert group_err(w1, rebuild(q1, p, 128, w1.shape), 128).sum() < 0.5 * group_err(w1, rebuild(qs, p, 128, w1.shape), 128).sum()


def test_bad_arguments():
    w = gauss(2, 256, 17)
    for args in [(0, 2, 1), (3, 2, 1), (2, 5, 1), (2, 3, 0), (2, 2, -1)]:
        with pytest.raises(ValueError):
            oracle.quantize(w, *args)
    with pytest.raises(ValueError):
        oracle.quantize(w, 2, 2, 1, group=96)
