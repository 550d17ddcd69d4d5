"""Pins for the oracle's quantiser primitives, the 3-sigma mask and SQC (Eq. 1, Eq. 2, Eq. 5,
Alg. 2 SQC).  Expected values are worked out by hand or by brute force written independently
of the oracle."""
import itertools
import os

import numpy as np
import pytest

from oracle import slim_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            key, *vals = line.split()
            out[key] = vals
    return out


def test_tau_grid_matches_paper_constants():
    g = _golden()
    lam, n = float(g["sqc_lambda"][0]), int(g["sqc_n"][0])
    tau = orc.tau_grid(lam, n)
    assert tau.shape == (int(g["sqc_candidates"][0]),)
    assert tau[0] == pytest.approx(1 - lam, abs=1e-15)
    assert tau[n] == 1.0                                   # tau = 1 is on the grid
    assert np.all(np.diff(tau) > 0) and np.allclose(np.diff(tau), lam / n, rtol=1e-9)
    assert tau[-1] < 1 + lam and tau[-1] == pytest.approx(1 + lam - lam / n, abs=1e-12)


def test_eq1_worked_example_by_hand():
    # w in [-1, 2], N = 2: s = (2 - (-1)) / 3 = 1, z = -round(-1/1) = 1.
    # round half to even: round(-0.5) = -0, round(0.5) = 0, round(1.5) = 2.
    w = np.array([-1.0, -0.5, 0.0, 0.5, 1.0, 1.5, 2.0])
    delta0, z = orc.minmax_params(w, 2)
    assert (delta0, z) == (1.0, 1.0)
    q = orc.quantize_affine(w, delta0, z, 2)
    assert q.tolist() == [0, 1, 1, 1, 2, 3, 3]
    assert orc.dequantize(q, delta0, z).tolist() == [-1, 0, 0, 0, 1, 2, 2]
    # clamp: values outside the calibrated range saturate
    assert orc.quantize_affine(np.array([-7.0, 9.0]), 1.0, 1.0, 2).tolist() == [0, 3]
    # 3 bits: 8 levels; s = 7/7 = 1, z = -round(-3) = 3
    w3 = np.array([-3.0, 4.0, 0.4, -2.6])
    d3, z3 = orc.minmax_params(w3, 3)
    assert (d3, z3) == (1.0, 3.0)
    assert orc.quantize_affine(w3, d3, z3, 3).tolist() == [0, 7, 3, 0]


def test_eq2_sign_quantiser_by_hand():
    w = np.array([[0.5, -1.5, 0.0, 2.0]])
    out = orc.rtn_fakequant(w, np.array([1]), 4)
    # alpha = (0.5 + 1.5 + 0 + 2) / 4 = 1; sign(0) = +1
    assert out.tolist() == [[1.0, -1.0, 1.0, 1.0]]


def test_degenerate_ranges():
    # constant group: range widened to include 0, value reproduced exactly at tau = 1
    assert orc.minmax_params(np.full(4, 0.75), 2) == (0.25, 0.0)
    d, z = orc.minmax_params(np.full(4, -0.75), 2)
    assert (d, z) == (0.25, 3.0)
    out = orc.rtn_fakequant(np.array([[0.75] * 4 + [-0.75] * 4 + [0.0] * 4]), np.array([2, 2, 3]), 4)
    assert out.tolist() == [[0.75] * 4 + [-0.75] * 4 + [0.0] * 4]
    assert orc.minmax_params(np.zeros(4), 3) == (1.0, 0.0)
    tau = orc.tau_grid()
    s, zz, c, losses = orc.sqc_search(np.full(8, 0.3), 2, tau, np.ones(8))
    assert c == 50 and losses[c] == 0.0 and s * (3 - zz) == pytest.approx(0.3, rel=1e-15)


def test_rtn_nearest_level_brute_force():
    # for fixed (delta, z) the code of Eq. 1 is the nearest representable level
    rng = np.random.default_rng(0)
    for bits in (2, 3, 4):
        w = rng.standard_normal(50)
        delta0, z = orc.minmax_params(w, bits)
        for tau in (0.9, 1.0, 1.07):
            delta = tau * delta0
            q = orc.quantize_affine(w, delta, z, bits)
            levels = delta * (np.arange(2 ** bits) - z)
            brute = np.argmin(np.abs(w[:, None] - levels[None, :]), axis=1)
            assert np.array_equal(q.astype(int), brute)


def test_fast_fakequant_equals_loop_form():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((9, 32)) * 0.02
    W[3, 8:16] = 0.0
    W[4, 16:24] = 0.01
    bits = np.array([1, 2, 3, 4], dtype=np.uint8)
    for q1 in (orc.Q1_SIGN, orc.Q1_AFFINE):
        assert np.array_equal(orc.rtn_fakequant(W, bits, 8, q1), orc.rtn_fakequant_fast(W, bits, 8, q1))


def test_three_sigma_mask_fraction_and_scope():
    rng = np.random.default_rng(2)
    blk = rng.standard_normal((2048, 128))
    frac = orc.block_mask(blk).mean()
    assert 0.0020 < frac < 0.0034          # two-sided 3 sigma of a Gaussian: 0.27 %
    # by hand: one far outlier in an otherwise tight block
    b = np.zeros((2, 8))
    b[0, :] = [1, -1, 1, -1, 1, -1, 1, -1]
    b[1, :] = [1, -1, 1, -1, 1, -1, 1, 40]
    m = orc.block_mask(b)
    assert m.sum() == 1 and m[1, 7]
    mrow = orc.block_mask(b, orc.SCOPE_ROW)   # per row: sigma of row 1 is ~13.6, 40 is < 3 sigma away
    assert mrow.sum() == 0


def _plain_grid_search(w, bits, tau):
    """Independent plain min-error grid search with Python scalars."""
    qmax = 2 ** bits - 1
    lo, hi = min(w), max(w)
    d0 = (hi - lo) / qmax
    z = -round(lo / d0)          # Python round is half-to-even as well
    best, best_c = None, None
    for c, t in enumerate(tau):
        d = t * d0
        loss = 0.0
        for x in w:
            q = min(max(round(x / d) + z, 0), qmax)
            loss += (x - d * (q - z)) ** 2
        if best is None or loss < best:
            best, best_c = loss, c
    return best_c, best, d0, z


def test_sqc_uniform_is_plain_grid_search():
    rng = np.random.default_rng(3)
    tau = orc.tau_grid()
    for bits in (2, 3, 4):
        for _ in range(6):
            w = (rng.standard_t(4, 32) * 0.02)
            c_ref, loss_ref, d0, z = _plain_grid_search([float(x) for x in w], bits, [float(t) for t in tau])
            s, zz, c, losses = orc.sqc_search(w, bits, tau, np.ones(32))
            assert c == c_ref and zz == z
            assert losses[c] == pytest.approx(loss_ref, rel=1e-12)
            assert s == tau[c] * d0
            assert losses[c] <= losses[50]          # tau = 1 is a candidate: never worse than min-max


def test_sqc_per_candidate_optimal_codes_brute_force():
    # tiny group: for each candidate the loss equals the minimum over ALL code assignments
    rng = np.random.default_rng(4)
    tau = orc.tau_grid()
    w = rng.standard_normal(4)
    omega = np.array([1.0, 3.0, 0.5, 2.0])
    s, z, c, losses = orc.sqc_search(w, 2, tau, omega)
    d0, z0 = orc.minmax_params(w, 2)
    for ci in (0, 17, 50, 99):
        d = tau[ci] * d0
        brute = min(sum(omega[j] * (w[j] - d * (q[j] - z0)) ** 2 for j in range(4))
                    for q in itertools.product(range(4), repeat=4))
        assert losses[ci] == pytest.approx(brute, rel=1e-12)
    assert c == int(np.argmin(losses))


def test_sqc_weight_modes_reduce_to_uniform():
    rng = np.random.default_rng(5)
    tau = orc.tau_grid()
    blk = rng.uniform(-1, 1, (16, 32))      # bounded: nothing beyond 3 sigma, mask empty
    assert orc.block_mask(blk).sum() == 0
    su, zu, cu, _ = orc.sqc_calibrate(blk, 3, tau, orc.WEIGHT_UNIFORM)
    sm, zm, cm, _ = orc.sqc_calibrate(blk, 3, tau, orc.WEIGHT_MASK_MEAN)
    assert np.array_equal(cu, cm) and np.array_equal(su, sm) and np.array_equal(zu, zm)
    # constant element salience => ELEMENT weighting is uniform up to a factor: use |w| = const
    sgn = np.where(rng.standard_normal((16, 32)) > 0, 1.0, -1.0) * 0.5
    d = np.ones(32)
    se, ze, ce, _ = orc.sqc_calibrate(sgn, 2, tau, orc.WEIGHT_ELEMENT, d=d)
    s1, z1, c1, _ = orc.sqc_calibrate(sgn, 2, tau, orc.WEIGHT_UNIFORM)
    assert np.array_equal(ce, c1)


def test_sqc_element_weights_by_hand():
    """ELEMENT loss weights are the element salience of Def. 1, omega_j = w_j^2 / d_j^2 with d = diag(H^-1):
    numbers worked by hand with a non-constant w and a non-unit d, so that a wrong exponent on either fails."""
    w = np.array([0.5, -1.0, 2.0, 0.25])
    d = np.array([0.5, 2.0, 1.0, 0.25])
    # w^2 = [0.25, 1, 4, 0.0625];  d^2 = [0.25, 4, 1, 0.0625]
    assert orc.sqc_weights(w, None, orc.WEIGHT_ELEMENT, d).tolist() == [1.0, 0.25, 4.0, 1.0]
    blk = np.stack([w, 2.0 * w])
    assert orc._omega_rows(blk, orc.WEIGHT_ELEMENT, orc.SCOPE_BLOCK, d).tolist() == [[1.0, 0.25, 4.0, 1.0],
                                                                                    [4.0, 1.0, 16.0, 4.0]]
    # the loss of the tau = 1 candidate at 2 bits: range [-1, 2], delta0 = 1, z = 1;
    # round(w) = [0 (tie to even), -1, 2, 0] -> q = [1, 0, 3, 1] -> w_hat = [0, -1, 2, 0]; errors [0.5, 0, 0, 0.25]
    # L = 1.0 * 0.25 + 1.0 * 0.0625 = 0.3125   (w^2/d would give 0.140625, |w|/d^2 0.75, uniform 0.3125 + 0 ...)
    tau = orc.tau_grid()
    om = orc.sqc_weights(w, None, orc.WEIGHT_ELEMENT, d)
    _, z, _, losses = orc.sqc_search(w, 2, tau, om)
    assert z == 1.0 and losses[50] == 0.3125
    # a second vector where the weights change the winner: the heavy element decides the step
    w2 = np.array([0.0, 0.3, 0.6, 0.95, 3.0, 1.5, 2.1, 2.7])
    d2 = np.array([1.0, 1.0, 1.0, 0.05, 1.0, 1.0, 1.0, 1.0])
    om2 = orc.sqc_weights(w2, None, orc.WEIGHT_ELEMENT, d2)
    assert om2[3] == pytest.approx(0.95 ** 2 / 0.05 ** 2, rel=1e-15)
    s_e, _, c_e, L_e = orc.sqc_search(w2, 2, tau, om2)
    s_u, _, c_u, L_u = orc.sqc_search(w2, 2, tau, np.ones(8))
    # element 3 carries 361 of the weight: its error (0.95 - q * delta)^2 must be near its minimum at the winner
    e3 = np.array([(0.95 - t * np.clip(np.rint(0.95 / t), 0, 3)) ** 2 for t in tau])
    assert e3[c_e] <= e3.min() + 1e-4 and c_e != c_u
    # and through the block interface, with d handed over per column
    se, ze, ce, _ = orc.sqc_calibrate(np.stack([w2, w2]), 2, tau, orc.WEIGHT_ELEMENT, d=d2)
    assert ce.tolist() == [c_e, c_e] and se[0] == s_e


def test_sqc_mask_mean_by_hand():
    # one masked element with a large error dominates under MASK_MEAN, not under UNIFORM
    w = np.array([0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 3.0])
    mask = np.zeros(8, bool)
    mask[7] = True
    om = orc.sqc_weights(w, mask, orc.WEIGHT_MASK_MEAN)
    assert om.tolist() == [1 / 7] * 7 + [1.0]
    assert orc.sqc_weights(w, np.zeros(8, bool), orc.WEIGHT_MASK_MEAN).tolist() == [1 / 8] * 8
    assert orc.sqc_weights(w, np.ones(8, bool), orc.WEIGHT_MASK_MEAN).tolist() == [1 / 8] * 8
    tau = orc.tau_grid()
    _, _, c_u, Lu = orc.sqc_search(w, 2, tau, np.ones(8))
    _, _, c_m, Lm = orc.sqc_search(w, 2, tau, om)
    # loss is the weighted sum: recompute candidate 50 (tau = 1, delta = 1, z = 0) by hand
    # codes: round(w) clipped to [0,3] -> [0,0,0,0,0,0(0.5->0),1,3]; errors w - q
    err = w - np.array([0, 0, 0, 0, 0, 0, 1, 3.0])
    assert Lu[50] == pytest.approx(np.sum(err ** 2), rel=1e-13)
    assert Lm[50] == pytest.approx(np.sum(err[:7] ** 2) / 7 + err[7] ** 2, rel=1e-13)


def test_sqc_sign_uniform_optimum_is_tau_one():
    # alpha = mean|w| is the least-squares scale of sign(w): with uniform weights tau = 1 wins
    rng = np.random.default_rng(6)
    tau = orc.tau_grid()
    for _ in range(5):
        w = rng.standard_normal(64)
        s, z, c, losses = orc.sqc_search(w, 1, tau, np.ones(64))
        assert c == 50 and z == 0.5 and s == pytest.approx(2 * np.mean(np.abs(w)), rel=1e-15)
        # closed form: L(tau) = sum w^2 - 2 tau alpha sum|w| + 64 tau^2 alpha^2
        a = np.mean(np.abs(w))
        closed = np.sum(w * w) - 2 * tau * a * np.sum(np.abs(w)) + 64 * (tau * a) ** 2
        assert np.allclose(losses, closed, rtol=1e-11)


def test_sqc_fast_rows_equal_per_row_search():
    rng = np.random.default_rng(7)
    tau = orc.tau_grid()
    blk = rng.standard_t(4, (24, 32)) * 0.02
    blk[5] = 0.0
    blk[6] = 0.013
    for bits in (1, 2, 3):
        for mode in (orc.WEIGHT_MASK_MEAN, orc.WEIGHT_UNIFORM):
            s, z, c, mg = orc.sqc_calibrate(blk, bits, tau, mode)
            om = orc._omega_rows(blk, mode, orc.SCOPE_BLOCK, None)
            s2, z2, c2, _ = orc._sqc_rows_fast(blk, bits, tau, om, orc.Q1_SIGN)
            assert np.array_equal(c, c2) and np.array_equal(s, s2) and np.array_equal(z, z2)
