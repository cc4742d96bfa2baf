"""Host-side check of the hash that the exact step's duplicate detection uses (ne_hash_position).

The detection stores each row key at its home position and resolves collisions by linear probing at load
<= 1/2.  That only stays cheap if the home positions use the whole table: with B = 2^22 pairs and K = 10
negatives a batch has 5e7 references and 2^27 positions.  The checks: the exported function equals the
stated formula; for a 100 M-node id sample of that size the home positions cover the table evenly and a
linear-probing insertion of all keys (simulated here, no GPU) has short probe sequences.  A hash of fixed
width (for comparison: 25 bits, as an earlier version had) fails the same check by orders of magnitude.
"""
import numpy as np
import pytest

import paper_2005_13789_amd as ne

C = np.uint32(0x9E3779B1)


def home_positions(keys: np.ndarray, positions: int) -> np.ndarray:
    k = int(positions).bit_length() - 1
    return (keys.astype(np.uint32) * C) >> np.uint32(32 - k)


def probe_displacements(home: np.ndarray, positions: int) -> np.ndarray:
    """Displacement of every key after inserting all of them with linear probing (the set of occupied
    positions does not depend on the insertion order; wrap-around ignored: the table's end stays far)."""
    h = np.sort(home.astype(np.int64))
    idx = np.arange(h.size, dtype=np.int64)
    final = np.maximum.accumulate(h - idx) + idx
    return final - h


def test_export_equals_formula():
    rng = np.random.default_rng(0)
    keys = rng.integers(0, 2**32, 2000, dtype=np.uint64).astype(np.uint32)
    for positions in (2, 2048, 1 << 20, 1 << 25, 1 << 27, 1 << 29, 1 << 31):
        want = home_positions(keys, positions)
        got = np.array([ne.ne_hash_position(int(k), positions) for k in keys], dtype=np.uint32)
        assert np.array_equal(got, want), positions
        assert got.max() < positions
    for bad in (0, 1, 3, 2049, (1 << 31) + 1):
        assert ne.ne_hash_position(5, bad) == 0xFFFFFFFF


@pytest.mark.parametrize("dist", ["uniform", "skewed"])
def test_large_batch_keys_spread_over_the_whole_table(dist):
    V, refs = 100_000_000, (1 << 22) * 12          # B = 2^22, K = 10
    positions = 1 << 27                            # smallest power of two >= 2 * refs
    assert positions >= 2 * refs > positions // 2
    rng = np.random.default_rng(1)
    n = 40_000_000                                 # distinct rows such a batch can name (more than 2^25)
    if dist == "uniform":
        ids = rng.choice(V, n, replace=False).astype(np.uint32)
    else:                                          # heavy tail folded into the id range, then made distinct
        ids = np.unique((rng.pareto(0.7, 2 * n) * 1000).astype(np.uint64) % V).astype(np.uint32)
    keys = ids | np.uint32(0x80000000)             # context rows
    home = home_positions(keys, positions)
    # every 1/1024th of the table gets its share
    hist = np.bincount(home >> np.uint32(17), minlength=1024)
    assert hist.min() > 0.8 * keys.size / 1024 and hist.max() < 1.2 * keys.size / 1024
    disp = probe_displacements(home, positions)
    assert disp.mean() < 1.0 and disp.max() < 100, (disp.mean(), disp.max())
    # a 25-bit hash in the same table: all homes in its first quarter, probe sequences of millions
    narrow = ((keys * C) >> np.uint32(7)) & np.uint32(positions - 1)
    assert narrow.max() < (1 << 25)
    if keys.size > (1 << 25):
        assert probe_displacements(narrow, positions).mean() > 100_000


def test_small_tables_unchanged_in_quality():
    rng = np.random.default_rng(2)
    ids = rng.choice(25_000_000, 300_000, replace=False).astype(np.uint32)
    for positions in (1 << 20, 1 << 21):
        disp = probe_displacements(home_positions(ids, positions), positions)
        assert disp.max() < 64
