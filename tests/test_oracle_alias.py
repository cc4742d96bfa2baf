"""Pins for the oracle's alias table (P(i) ~ degree^0.75) and its draws.

The table is pinned by what the mathematics fixes: the probability a table implies is an exact
integer identity over its entries and must equal deg^0.75 / sum (computed here with numpy's pow, a
different route from the oracle's sqrt*sqrt(sqrt)); 10^7 draws must match those probabilities; and
the special cases have known answers.
"""
import numpy as np
import pytest

import oracle

TWO32 = 1 << 32


def implied_mass(thr, alias):
    """n * 2^32 * P(i) as exact Python integers, by enumerating every (slot, accept/reject) outcome."""
    n = len(thr)
    mass = [0] * n
    for s in range(n):
        mass[s] += int(thr[s])
        mass[int(alias[s])] += TWO32 - int(thr[s])
    return mass


def true_prob(deg):
    w = np.asarray(deg, dtype=np.float64) ** 0.75
    return w / w.sum()


@pytest.mark.parametrize("n,seed", [(1, 0), (2, 1), (3, 2), (4, 3), (17, 4), (1000, 5), (4099, 6)])
def test_alias_identity(n, seed):
    rng = np.random.default_rng(seed)
    deg = (rng.pareto(1.2, n) * 3).astype(np.uint32)
    deg[rng.integers(0, n)] += 1           # at least one non-zero
    if n > 4:
        deg[rng.integers(0, n, n // 5)] = 0
        deg[0] += 1
    thr, alias, prob = oracle.build_alias(deg)
    p = true_prob(deg)
    np.testing.assert_allclose(prob, p, rtol=1e-12, atol=0)
    mass = implied_mass(thr, alias)
    assert sum(mass) == n * TWO32
    fan_in = np.bincount(alias, minlength=n)
    for i in range(n):
        want = p[i] * n * TWO32
        # one quantisation unit per entry that feeds i, plus fp64 rounding of the running p_l
        tol = fan_in[i] + 2 + 1e-9 * want
        assert abs(mass[i] - want) <= tol, (i, mass[i], want)
        if deg[i] == 0:
            assert mass[i] == 0


def test_alias_special_cases():
    thr, alias, _ = oracle.build_alias(np.full(64, 7, dtype=np.uint32))
    assert (thr == TWO32 - 1).all() and (alias == np.arange(64)).all()
    deg = np.zeros(50, dtype=np.uint32)
    deg[31] = 9
    thr, alias, _ = oracle.build_alias(deg)
    neg = oracle.sample_negatives(3, 0, 20000, 5, thr, alias)
    assert (neg == 31).all()
    with pytest.raises(ValueError):
        oracle.build_alias(np.zeros(5, dtype=np.uint32))


def test_alias_draw_mapping_matches_big_integers():
    """slot = floor(((r0<<32)|r1) * n / 2^64); accept iff r2 < thr_q[slot]; id = base + result."""
    rng = np.random.default_rng(11)
    n = 37
    deg = rng.integers(0, 50, n).astype(np.uint32)
    thr, alias, _ = oracle.build_alias(deg)
    seed, base_id, sb = 0x123456789ABCDEF, 1000, (1 << 33) + 5
    B, K = 300, 4
    neg = oracle.sample_negatives(seed, sb, B, K, thr, alias, base=base_id)
    for b in range(B):
        idx = sb + b
        for k in range(K):
            r = [int(v) for v in oracle.philox4x32_10([idx & 0xFFFFFFFF, idx >> 32, k, 0],
                                                      [seed & 0xFFFFFFFF, seed >> 32])]
            slot = (((r[0] << 32) | r[1]) * n) >> 64
            want = slot if r[2] < int(thr[slot]) else int(alias[slot])
            assert neg[b, k] == base_id + want


def test_alias_frequencies_1e7_draws():
    rng = np.random.default_rng(7)
    n = 500
    deg = (rng.pareto(1.0, n) * 4).astype(np.uint32)
    deg[:5] = [0, 1, 2, 10000, 0]
    thr, alias, _ = oracle.build_alias(deg)
    p = true_prob(deg)
    draws = 10_000_000
    K = 5
    neg = oracle.sample_negatives(42, 0, draws // K, K, thr, alias)
    cnt = np.bincount(neg.reshape(-1), minlength=n).astype(np.float64)
    assert (cnt[p == 0] == 0).all()
    freq = cnt / draws
    sd = np.sqrt(p * (1 - p) / draws)
    live = p > 0
    assert np.all(np.abs(freq - p)[live] <= 5 * sd[live] + 1e-12)
    exp = p[live] * draws
    chi2 = ((cnt[live] - exp) ** 2 / exp).sum()
    dof = live.sum() - 1
    z = (chi2 - dof) / np.sqrt(2 * dof)
    assert abs(z) < 3.3        # two-sided p about 0.001
    # each of the K draw slots has the same distribution (the k counter word is used)
    for k in range(K):
        ck = np.bincount(neg[:, k], minlength=n) / (draws / K)
        assert np.abs(ck - p).max() < 6 * np.sqrt(p.max() * K / draws) + 1e-4


def test_negative_streams_are_counter_addressed():
    """Draw (sample, k) does not depend on batch boundaries: [0,B) equals [0,B1) ++ [B1,B)."""
    deg = np.arange(1, 300, dtype=np.uint32)
    thr, alias, _ = oracle.build_alias(deg)
    a = oracle.sample_negatives(9, 100, 1000, 5, thr, alias)
    b = np.concatenate([oracle.sample_negatives(9, 100, 400, 5, thr, alias),
                        oracle.sample_negatives(9, 500, 600, 5, thr, alias)])
    assert (a == b).all()
    c = oracle.sample_negatives(10, 100, 1000, 5, thr, alias)
    assert (a != c).mean() > 0.5
