"""Pins for the oracle's CSER routines (Algorithms 2 and 3, PSync, implementation II).

The paper prints no numeric trace, so the oracle is pinned by what the paper and the
mathematics fix: exact rational brute force on tiny dyadic inputs, Lemma 1, the reductions the
paper states (identity compressor = synchronous momentum SGD, one worker = plain SGD, C_step = 0
with H = 1 = CSEA, C_step = 0 = CSER-PL, C_reset = identity on top = local SGD, beta = 0 =
Algorithm 2), the closed form of the mean model from the proofs, the closed form of the residual,
the agreement of implementations I and II, the communication-ratio formula of Section 5.1 with
the printed rows of Table 4, and the bound of Lemma 3.
"""
from fractions import Fraction
import os

import numpy as np
import pytest

from oracle import reference as R
from tests import _np_models as M

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _grads(rng, T, W, d, scale=1.0):
    return [rng.standard_normal((W, d)) * scale for _ in range(T)]


def _masks(seed, stream, T, B, k):
    return {t: R.select_blocks(seed, stream, t, B, k)[1] for t in range(1, T + 1)}


def _run(oracle, grads):
    for g in grads:
        oracle.step(g)
    return oracle


# ---------------------------------------------------------------- exact brute force (tiny inputs)
@pytest.mark.parametrize("W,d,block,R_step,R_reset,H,T", [
    (2, 12, 4, 2, 2, 2, 4),      # B = 3 full blocks
    (4, 11, 3, 2, 1, 3, 6),      # ragged tail block, full reset
    (4, 10, 4, 3, 2, 1, 3),      # reset after every step
    (2, 7, 2, 0, 2, 2, 4),       # per-step compressor keeps nothing
    (2, 9, 3, 1, 3, 2, 4),       # per-step compressor is the identity
])
def test_algorithm3_matches_exact_rational_arithmetic(W, d, block, R_step, R_reset, H, T):
    """All inputs are small dyadic rationals, lr = beta = 1/2 and W is a power of two, so every
    float32 operation of the oracle is exact and must equal the Fraction evaluation of
    Algorithm 3 bit for bit -- a dropped term, a wrong sign or a wrong index cannot survive."""
    rng = np.random.default_rng(100 + d)
    seed = 77
    B = -(-d // block)
    x0 = rng.integers(-8, 9, size=d) / 4.0
    grads = [rng.integers(-8, 9, size=(W, d)) / 8.0 for _ in range(T)]
    smask = _masks(seed, 0, T, B, R.blocks_kept(B, R_step))
    rmask = _masks(seed, 1, T, B, R.blocks_kept(B, R_reset))
    xe, ee, me = M.mcser_exact([Fraction(float(v)) for v in x0],
                               [[[Fraction(float(v)) for v in row] for row in g] for g in grads],
                               smask, rmask, H, Fraction(1, 2), Fraction(1, 2), block)
    for dtype in (np.float32, np.float64):
        o = R.OracleCSER(d, W, block, R_step, R_reset, H, 0.5, 0.5, seed, x0, dtype=dtype)
        residual_seen = 0.0
        for g in grads:
            o.step(g)
            residual_seen = max(residual_seen, np.abs(o.e).max())
        for got, want in ((o.x, xe), (o.e, ee), (o.m, me)):
            want = np.array([[float(v) for v in row] for row in want])
            assert np.array_equal(got.astype(np.float64), want)
        # the test is not vacuous: something was synchronised and something was left local
        if 0 < R_step and R.blocks_kept(B, R_step) < B:
            assert any(m.sum() > 0 for m in smask.values()) and residual_seen > 0


def test_non_power_of_two_worker_count_against_exact_arithmetic():
    W, d, block, T, H = 3, 10, 2, 5, 2
    rng = np.random.default_rng(5)
    x0 = rng.integers(-8, 9, size=d) / 4.0
    grads = [rng.integers(-8, 9, size=(W, d)) / 8.0 for _ in range(T)]
    B = 5
    smask, rmask = _masks(9, 0, T, B, 2), _masks(9, 1, T, B, 3)
    xe, ee, me = M.mcser_exact([Fraction(float(v)) for v in x0],
                               [[[Fraction(float(v)) for v in row] for row in g] for g in grads],
                               smask, rmask, H, Fraction(1, 2), Fraction(1, 2), block)
    o = _run(R.OracleCSER(d, W, block, 3, 2, H, 0.5, 0.5, 9, x0, dtype=np.float64), grads)
    assert R.blocks_kept(B, 3) == 2 and R.blocks_kept(B, 2) == 3
    for got, want in ((o.x, xe), (o.e, ee), (o.m, me)):
        want = np.array([[float(v) for v in row] for row in want])
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- Lemma 1
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-13), (np.float32, 2e-5)])
def test_lemma1_model_minus_residual_is_common_to_all_workers(dtype, tol):
    rng = np.random.default_rng(1)
    W, d, T = 5, 300, 40
    o = R.OracleCSER(d, W, 16, 4, 2, 4, 0.1, 0.9, 3, rng.standard_normal(d), dtype=dtype)
    for g in _grads(rng, T, W, d):
        o.step(g)
        z = o.x.astype(np.float64) - o.e.astype(np.float64)
        assert np.abs(z - z[0]).max() <= tol * max(1.0, np.abs(o.x).max())
    assert np.abs(o.e).max() > 0.1      # the workers really did drift apart


# ---------------------------------------------------------------- identity compressor = synchronous momentum SGD
def test_identity_step_compressor_is_fully_synchronous_nesterov_sgd():
    rng = np.random.default_rng(2)
    W, d, T = 4, 257, 25
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = _run(R.OracleCSER(d, W, 8, 1, 3, 5, 0.05, 0.9, 1, x0, dtype=np.float64), grads)
    assert not o.e.any()                                           # nothing is ever left local
    assert all(np.array_equal(o.x[0], o.x[i]) for i in range(W))   # bitwise equal local models
    xs, ms = M.nesterov_sgd(x0, [g.mean(axis=0) for g in grads], 0.05, 0.9)
    np.testing.assert_allclose(o.x[0], xs, rtol=0, atol=1e-13)     # = SGD on the averaged gradient
    np.testing.assert_allclose(o.m.mean(axis=0), ms, rtol=0, atol=1e-13)
    o32 = _run(R.OracleCSER(d, W, 8, 1, 3, 5, 0.05, 0.9, 1, x0, dtype=np.float32), grads)
    assert not o32.e.any() and all(np.array_equal(o32.x[0], o32.x[i]) for i in range(W))
    np.testing.assert_allclose(o32.x[0], xs, rtol=0, atol=2e-5)


# ---------------------------------------------------------------- full reset
def test_full_error_reset_makes_local_models_coincide():
    rng = np.random.default_rng(3)
    W, d, H = 6, 130, 7
    x0 = rng.standard_normal(d)
    grads = _grads(rng, H, W, d)
    o = R.OracleCSER(d, W, 4, 8, 1, H, 0.1, 0.9, 2, x0, dtype=np.float64)
    for g in grads[:-1]:
        o.step(g)
    assert np.abs(o.x - o.x[0]).max() > 1e-3                       # models bifurcated before the reset
    o.step(grads[-1])                                              # t = H: step, then reset with C = identity
    assert not o.e.any() and np.all(np.signbit(o.e) == False)      # e is exactly +0
    assert np.abs(o.x - o.x[0]).max() < 1e-14
    # and the common model is synchronous-SGD's: mean of momentum updates
    z = x0.copy()
    m = np.zeros((W, d))
    for g in grads:
        m = 0.9 * m + g
        z = z - (0.1 * (0.9 * m + g)).mean(axis=0)
    np.testing.assert_allclose(o.x[0], z, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- error reset, block by block, in float32
def test_error_reset_touches_only_the_blocks_it_chose_and_follows_the_written_formula_there():
    """Algorithm 3's reset branch in float32 on non-dyadic values, where (x - e) + e != x in general.

    Off the blocks C_reset chose, Algorithm PSync gives C(e_i) = 0 on every worker, hence e'_i = 0 + r_i = e_i
    exactly and the correction -e_i + e'_i of the model is identically zero: x and e must come out
    bit-identical (implementation II of Appendix A.4, which the paper states to be equivalent, does not visit
    those blocks either).  On the chosen blocks r_i = 0, e'_i = ebar, so x_i <- (x_i - e_i) + ebar with ebar
    the left-to-right float32 sum over the workers divided by n, and e_i <- +0."""
    rng = np.random.default_rng(31)
    W, d, block, seed, T = 5, 203, 8, 19, 7           # ragged last block of 3 columns, n not a power of two
    B = -(-d // block)
    x0 = (rng.standard_normal(d) / 3.0).astype(np.float32)
    o = R.OracleCSER(d, W, block, 4, 3, 0, 0.1, 0.9, seed, x0, dtype=np.float32)    # H = 0: no automatic reset
    for g in _grads(rng, T, W, d, 0.1):
        o.step(g.astype(np.float32))
    x_before, e_before = o.x.copy(), o.e.copy()
    o.error_reset()
    cols = M.column_mask(R.select_blocks(seed, 1, T, B, R.blocks_kept(B, 3))[1], d, block)
    assert 0 < cols.sum() < d
    # unchosen blocks: nothing moves, not even by a rounding
    assert np.array_equal(o.x[:, ~cols].view(np.uint32), x_before[:, ~cols].view(np.uint32))
    assert np.array_equal(o.e[:, ~cols].view(np.uint32), e_before[:, ~cols].view(np.uint32))
    # the literal (x - e) + e would have moved some of them: the test separates the two readings
    literal = (x_before - e_before) + e_before
    assert (literal[:, ~cols] != x_before[:, ~cols]).any()
    # chosen blocks: the written formula, float32 operation by operation
    ebar = e_before[0].copy()
    for i in range(1, W):
        ebar = ebar + e_before[i]
    ebar = ebar / np.float32(W)
    want = (x_before - e_before) + ebar[None, :]
    assert want.dtype == np.float32
    assert np.array_equal(o.x[:, cols].view(np.uint32), want[:, cols].view(np.uint32))
    assert not o.e[:, cols].any() and not np.signbit(o.e[:, cols]).any()
    assert np.abs(e_before[:, cols]).max() > 1e-3     # there was a residual to reset


# ---------------------------------------------------------------- one worker = plain SGD
@pytest.mark.parametrize("R_step,R_reset,H", [(4, 2, 3), (0, 1, 1), (1, 5, 2), (7, 7, 0)])
def test_single_worker_is_plain_momentum_sgd(R_step, R_reset, H):
    rng = np.random.default_rng(4)
    d, T = 100, 20
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, 1, d)
    o = _run(R.OracleCSER(d, 1, 8, R_step, R_reset, H, 0.1, 0.8, 5, x0, dtype=np.float64), grads)
    xs, ms = M.nesterov_sgd(x0, [g[0] for g in grads], 0.1, 0.8)
    np.testing.assert_allclose(o.x[0], xs, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o.m[0], ms, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- implementation I vs II
@pytest.mark.parametrize("R_step,R_reset,H,beta", [(4, 2, 3, 0.9), (0, 2, 1, 0.0), (0, 4, 4, 0.9), (16, 16, 8, 0.5)])
def test_implementations_one_and_two_give_the_same_models(R_step, R_reset, H, beta):
    rng = np.random.default_rng(6)
    W, d, T = 4, 203, 33
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    a = _run(R.OracleCSER(d, W, 8, R_step, R_reset, H, 0.1, beta, 8, x0, dtype=np.float64), grads)
    b = _run(R.OracleCSER(d, W, 8, R_step, R_reset, H, 0.1, beta, 8, x0, dtype=np.float64, with_error=False), grads)
    np.testing.assert_allclose(a.x, b.x, rtol=0, atol=1e-12)
    assert np.abs(a.x - a.x[0]).max() > 1e-3


# ---------------------------------------------------------------- mean model closed form
@pytest.mark.parametrize("R_step,R_reset,H,block", [(4, 2, 3, 8), (0, 3, 5, 1), (32, 1, 2, 64), (2, 2, 0, 7)])
def test_mean_model_moves_by_the_mean_update_whatever_the_compressors(R_step, R_reset, H, block):
    rng = np.random.default_rng(7)
    W, d, T = 4, 150, 30
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = _run(R.OracleCSER(d, W, block, R_step, R_reset, H, 0.07, 0.9, 4, x0, dtype=np.float64), grads)
    m = np.zeros((W, d))
    xbar = x0.copy()
    for g in grads:                      # xbar_t = xbar_{t-1} - (1/n) sum_i p_i, from g alone
        m = 0.9 * m + g
        xbar -= (0.07 * (0.9 * m + g)).mean(axis=0)
    np.testing.assert_allclose(o.x.mean(axis=0), xbar, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- residual closed form
def test_residual_is_minus_the_unsynchronised_updates_since_the_blocks_last_reset():
    rng = np.random.default_rng(8)
    W, d, T, block, H, R_step, R_reset, seed = 3, 96, 24, 8, 4, 3, 2, 6
    B = d // block
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = R.OracleCSER(d, W, block, R_step, R_reset, H, 0.1, 0.9, seed, x0, dtype=np.float64)
    m = np.zeros((W, d))
    acc = np.zeros((W, d))                                         # expected residual
    for t, g in enumerate(grads, start=1):
        o.step(g)
        m = 0.9 * m + g
        p = 0.1 * (0.9 * m + g)
        step_cols = M.column_mask(R.select_blocks(seed, 0, t, B, R.blocks_kept(B, R_step))[1], d, block)
        acc[:, ~step_cols] -= p[:, ~step_cols]
        if t % H == 0:
            reset_cols = M.column_mask(R.select_blocks(seed, 1, t, B, R.blocks_kept(B, R_reset))[1], d, block)
            acc[:, reset_cols] = 0.0
            assert not o.e[:, reset_cols].any()
        np.testing.assert_allclose(o.e, acc, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- named special cases, re-coded from their boxes
def test_beta_zero_is_algorithm_2():
    rng = np.random.default_rng(9)
    W, d, T, block, H, seed = 4, 77, 18, 5, 3, 12
    B = -(-d // block)
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = _run(R.OracleCSER(d, W, block, 4, 2, H, 0.1, 0.0, seed, x0, dtype=np.float64), grads)
    x, e = M.alg2_cser(x0, grads, _masks(seed, 0, T, B, R.blocks_kept(B, 4)),
                       _masks(seed, 1, T, B, R.blocks_kept(B, 2)), H, 0.1, block)
    np.testing.assert_allclose(o.x, x, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o.e, e, rtol=0, atol=1e-13)


def test_no_step_sync_and_reset_every_iteration_is_csea():
    rng = np.random.default_rng(10)
    W, d, T, block, seed = 4, 60, 15, 4, 13
    B = d // block
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = _run(R.OracleCSER(d, W, block, 0, 4, 1, 0.1, 0.0, seed, x0, dtype=np.float64), grads)
    x, e = M.csea_impl1(x0, grads, _masks(seed, 1, T, B, R.blocks_kept(B, 4)), 0.1, block)
    np.testing.assert_allclose(o.x, x, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o.e, e, rtol=0, atol=1e-13)


def test_no_step_sync_is_cser_pl_and_with_identity_reset_is_local_sgd():
    rng = np.random.default_rng(11)
    W, d, T, block, H, seed = 4, 60, 16, 4, 4, 14
    B = d // block
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = _run(R.OracleCSER(d, W, block, 0, 4, H, 0.1, 0.0, seed, x0, dtype=np.float64), grads)
    x, e = M.cser_pl_impl1(x0, grads, _masks(seed, 1, T, B, R.blocks_kept(B, 4)), H, 0.1, block)
    np.testing.assert_allclose(o.x, x, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o.e, e, rtol=0, atol=1e-13)
    o1 = _run(R.OracleCSER(d, W, block, 0, 1, H, 0.1, 0.0, seed, x0, dtype=np.float64), grads)
    np.testing.assert_allclose(o1.x, M.local_sgd(x0, grads, H, 0.1), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- communication budget (Section 5.1, Table 4)
def test_overall_ratio_formula_on_the_printed_table4_rows_and_on_synced_element_counts():
    rows = [tuple(int(v) for v in l.split()) for l in open(os.path.join(GOLDEN, "table4_cser_rows.txt"))
            if l.strip() and l[0] != "#"]
    assert len(rows) == 10
    for overall, r_step, r_reset, H in rows:
        assert Fraction(1) / (Fraction(1, r_step) + Fraction(1, r_reset * H)) == overall
    # the oracle's selection lists reproduce that budget: elements synchronised per worker over T steps
    overall, r_step, r_reset, H = rows[3]          # 16 = (32, 8, 4)
    block, B = 2, 512
    d, T = block * B, 40
    sent = 0
    for t in range(1, T + 1):
        sent += int(R.select_blocks(1, 0, t, B, R.blocks_kept(B, r_step))[1].sum()) * block
        if t % H == 0:
            sent += int(R.select_blocks(1, 1, t, B, R.blocks_kept(B, r_reset))[1].sum()) * block
    assert Fraction(T * d, sent) == overall


# ---------------------------------------------------------------- Lemma 3 (bound on the residual after a reset)
def test_residual_after_reset_obeys_lemma3_bound():
    rng = np.random.default_rng(12)
    W, d, block, H, R_step, R_reset, lr, sigma = 4, 4096, 16, 4, 4, 2, 0.1, 0.5
    B = d // block
    o = R.OracleCSER(d, W, block, R_step, R_reset, H, lr, 0.0, 21, np.zeros(d), dtype=np.float64)
    delta1, delta2 = R.blocks_kept(B, R_reset) / B, R.blocks_kept(B, R_step) / B
    V2 = d * sigma ** 2                                            # E||g||^2 for g ~ N(0, sigma^2 I)
    bound = (1 - delta2) * (1 - delta1) * lr ** 2 * H ** 2 * V2 / (1 - np.sqrt(1 - delta1)) ** 2
    worst = 0.0
    for t in range(1, 20 * H + 1):
        o.step(rng.standard_normal((W, d)) * sigma)
        if t % H == 0:
            worst = max(worst, (o.e ** 2).sum(axis=1).mean())
    assert 0 < worst <= bound


# ---------------------------------------------------------------- slices and precision
def test_a_block_slice_evolves_exactly_as_in_the_full_run():
    rng = np.random.default_rng(13)
    W, d, block, T = 4, 1000, 16, 12       # B = 63, ragged tail of 8
    x0 = rng.standard_normal(d).astype(np.float32)
    grads = [g.astype(np.float32) for g in _grads(rng, T, W, d)]
    full = _run(R.OracleCSER(d, W, block, 4, 2, 3, 0.1, 0.9, 17, x0), grads)
    for b0, b1 in [(0, 5), (20, 41), (60, 63)]:
        c0, c1 = b0 * block, min(d, b1 * block)
        part = R.OracleCSER(d, W, block, 4, 2, 3, 0.1, 0.9, 17, x0[c0:c1], b0=b0, b1=b1)
        for g in grads:
            part.step(g[:, c0:c1])
        for name in ("x", "e", "m"):
            assert np.array_equal(getattr(part, name), getattr(full, name)[:, c0:c1])


def test_float32_run_stays_within_rounding_of_the_float64_run():
    rng = np.random.default_rng(14)
    W, d, T = 8, 2048, 100
    x0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    grads = [(g * 0.1).astype(np.float32) for g in _grads(rng, T, W, d)]
    a = _run(R.OracleCSER(d, W, 64, 8, 4, 4, 0.1, 0.9, 0, x0, dtype=np.float32), grads)
    b = _run(R.OracleCSER(d, W, 64, 8, 4, 4, 0.1, np.float32(0.9), 0, x0, dtype=np.float64), grads)
    # one rounding of about 2^-24 |value| per statement and step, accumulating like a random walk
    for name in ("x", "e", "m"):
        va, vb = getattr(a, name).astype(np.float64), getattr(b, name)
        assert np.abs(va - vb).max() < 100 * 2.0 ** -24 * max(1.0, np.abs(vb).max())
        assert np.abs(va - vb).max() > 0


def test_step_size_can_change_between_iterations():
    rng = np.random.default_rng(15)
    W, d, T = 2, 64, 10
    x0 = rng.standard_normal(d)
    grads = _grads(rng, T, W, d)
    o = R.OracleCSER(d, W, 8, 2, 2, 3, 0.1, 0.9, 3, x0, dtype=np.float64)
    m = np.zeros((W, d))
    xbar = x0.copy()
    for t, g in enumerate(grads, start=1):
        lr = 0.1 / t
        o.set_lr(lr)
        o.step(g)
        m = 0.9 * m + g
        xbar -= (lr * (0.9 * m + g)).mean(axis=0)
    np.testing.assert_allclose(o.x.mean(axis=0), xbar, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- the worked numbers of Section 4.2
def test_compression_error_term_reproduces_the_numbers_printed_in_section_4_2():
    """Theorem 1's compression-error factor [4(1-d1)/d1^2 + 1](1-d2) H^2 (constants dropped, as the text does)
    against the four numbers the paper prints; the same (d1, d2, H) reading drives test_residual_after_reset_obeys_lemma3_bound."""
    def cser_term(d1, d2, H):
        return (Fraction(4) * (1 - d1) / d1 ** 2 + 1) * (1 - d2) * H ** 2

    def qsparse_term(d1, H):
        return (Fraction(4) * (1 - d1 ** 2) / d1 ** 2 + 1) * H ** 2

    half = Fraction(1, 2)
    assert qsparse_term(half, 8) == 832 and cser_term(half, 0, 8) == 576          # Remark 1's example
    assert cser_term(Fraction(1, 3), 0, 4) == 400                                   # all budget on the reset
    moved = cser_term(Fraction(7, 8), Fraction(1, 96), 12)                          # some budget moved to the step
    assert 235 < moved < 236
    # "the overall compression budget remains the same": delta_1 / H + delta_2 is 1/12 in both settings
    assert Fraction(1, 3) / 4 == Fraction(7, 8) / 12 + Fraction(1, 96)
