"""Pins for the oracle's shared-seed block selector (GRBS, Definition 2 of the paper).

The paper fixes no concrete random lists, so the selector is pinned by what the definition and
the mathematics fix: the published known answers of its generator, that it is a bijection
(brute force), that it picks exactly k distinct blocks, that each block and each pair of blocks
is picked with the frequency uniform sampling without replacement has, and that the resulting
compressor is a k/B-approximate one in expectation.
"""
import os

import numpy as np
import pytest

from oracle import reference as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for row in rows:
        w = [int(v, 16) for v in row]
        got = R.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in got] == w[6:10]


@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1000, 1672, 4096, 6240])
def test_permutation_is_bijection_and_inverse_matches(B):
    for (seed, stream, t) in [(0, 0, 1), (12345678901234567, 1, 2**40 + 3)]:
        fwd = np.array([R.block_perm(seed, stream, t, B, v) for v in range(B)])
        assert fwd.min() >= 0 and fwd.max() < B
        assert np.array_equal(np.sort(fwd), np.arange(B))          # brute force: a permutation
        inv = np.array([R.block_perm_inverse(seed, stream, t, B, int(b)) for b in fwd])
        assert np.array_equal(inv, np.arange(B))                   # inverse network undoes it


@pytest.mark.parametrize("B,R_", [(256, 8), (256, 4), (1672, 32), (1672, 8), (24959, 256), (24959, 16),
                                  (6240, 2), (99833, 1024), (81788, 512), (10, 0), (10, 1), (1, 1), (1, 0), (7, 100)])
def test_exactly_k_distinct_blocks_and_mask_agrees(B, R_):
    k = R.blocks_kept(B, R_)
    assert k == (0 if R_ == 0 else -(-B // R_))                    # ceil(B / R); R = 0 keeps nothing
    idx, mask = R.select_blocks(7, 0, 11, B, k)
    assert len(idx) == k and len(set(idx.tolist())) == k
    assert (idx < B).all() if k else True
    assert int(mask.sum()) == k
    assert set(np.nonzero(mask)[0].tolist()) == set(idx.tolist())
    assert set(np.unique(mask).tolist()) <= {0, 1}
    # draw order is pi(0), pi(1), ...
    for j in range(min(k, 5)):
        assert R.block_perm(7, 0, 11, B, j) == idx[j]


def test_blocks_kept_on_the_named_workloads():
    # B = ceil(d / block); k = ceil(B / R)
    assert R.blocks_kept(256, 8) == 32 and R.blocks_kept(256, 4) == 64
    assert -(-855770 // 512) == 1672 and R.blocks_kept(1672, 32) == 53 and R.blocks_kept(1672, 8) == 209
    assert -(-25557032 // 1024) == 24959 and R.blocks_kept(24959, 256) == 98 and R.blocks_kept(24959, 16) == 1560
    assert -(-335000000 // 4096) == 81788 and R.blocks_kept(81788, 512) == 160 and R.blocks_kept(81788, 32) == 2556
    assert R.blocks_kept(5, 1) == 5            # ratio 1 is the identity compressor


def test_selection_depends_on_seed_stream_and_iteration():
    B, k = 4096, 64
    base = set(R.select_blocks(1, 0, 5, B, k)[0].tolist())
    for other in [R.select_blocks(2, 0, 5, B, k), R.select_blocks(1, 1, 5, B, k), R.select_blocks(1, 0, 6, B, k),
                  R.select_blocks(1, 0, 5 + 2**32, B, k), R.select_blocks(1 + 2**32, 0, 5, B, k)]:
        s = set(other[0].tolist())
        # two independent uniform k-subsets of 4096 share k*k/B = 1 block on average
        assert len(base & s) < 12
    again = set(R.select_blocks(1, 0, 5, B, k)[0].tolist())
    assert again == base                                           # a pure function of its arguments


def _chi2_ok(chi2, dof, sigmas=5.0):
    return abs(chi2 - dof) < sigmas * np.sqrt(2.0 * dof)


@pytest.mark.parametrize("B,k", [(64, 8), (37, 5), (5, 2), (3, 1)])
def test_each_block_is_picked_with_frequency_k_over_B(B, k):
    T = 20000
    counts = np.zeros(B)
    for t in range(1, T + 1):
        counts += R.select_blocks(99, 0, t, B, k)[1]
    p = k / B
    # sampling k of B without replacement: counts sum to kT, each has mean pT and variance T p (1-p);
    # sum_b (c_b - pT)^2 / (T p (1-p)) has mean B - 1 (one linear constraint)
    chi2 = ((counts - p * T) ** 2).sum() / (T * p * (1 - p))
    assert counts.sum() == k * T
    assert _chi2_ok(chi2 * (B - 1) / B, B - 1), (chi2, B)


def test_pairs_of_blocks_are_picked_together_with_the_hypergeometric_rate():
    B, k, T = 16, 4, 30000
    pair = np.zeros((B, B))
    for t in range(1, T + 1):
        m = R.select_blocks(3, 1, t, B, k)[1].astype(np.float64)
        pair += np.outer(m, m)
    q = k * (k - 1) / (B * (B - 1))                                # P(both b and b' chosen)
    iu = np.triu_indices(B, 1)
    obs = pair[iu]
    assert obs.sum() == T * k * (k - 1) / 2
    chi2 = ((obs - q * T) ** 2 / (q * T)).sum()
    # the pair indicators are weakly dependent, so allow a generous band round the 119 dof
    assert 60 < chi2 < 200, chi2
    assert abs(obs.mean() / T - q) < 1e-12 + 0.0                   # exact by counting
    assert obs.min() / T > q * 0.8 and obs.max() / T < q * 1.2


def test_consecutive_iterations_look_independent():
    B, k, T = 32, 8, 20000
    prev = R.select_blocks(5, 0, 0, B, k)[1].astype(np.float64)
    both = 0.0
    for t in range(1, T + 1):
        cur = R.select_blocks(5, 0, t, B, k)[1].astype(np.float64)
        both += (prev * cur).sum()
        prev = cur
    # E |S_t & S_{t+1}| = k^2 / B for independent draws; hypergeometric variance < k^2/B
    mean_overlap = both / T
    assert abs(mean_overlap - k * k / B) < 5 * np.sqrt((k * k / B) / T)


def test_grbs_is_a_k_over_B_approximate_compressor_in_expectation():
    # E || C(v) - v ||^2 = (1 - k/B) ||v||^2 for any fixed v  (Definition 2 / Section 4.2)
    rng = np.random.default_rng(0)
    B, k, block, T = 40, 5, 3, 8000
    d = B * block - 1                                              # ragged last block
    v = rng.standard_normal(d) * np.linspace(0.1, 3.0, d)
    block_energy = np.add.reduceat(v * v, np.arange(0, d, block))
    acc = 0.0
    for t in range(1, T + 1):
        mask = R.select_blocks(11, 0, t, B, k)[1]
        acc += block_energy[mask == 0].sum()
    expected = (1 - k / B) * (v * v).sum()
    # Var per draw is at most ||v||^4; T draws
    assert abs(acc / T - expected) < 5 * (v * v).sum() * np.sqrt((k / B) * (1 - k / B) / T) + 1e-9
