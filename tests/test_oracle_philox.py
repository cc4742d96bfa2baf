"""Pins for the oracle's Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).

1. Library pin: rocRAND's public Philox4x32-10 engine is callable on the host; a small helper
   compiled here calls it and every output block must agree with the oracle.
2. Big-integer pin: one round written with Python integers (mulhi/mullo by plain 64-bit products).
3. Statistical sanity of the outputs the method consumes.
"""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _philox_bigint(ctr, key):
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    c = list(ctr)
    k = list(key)
    mask = 0xFFFFFFFF
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & mask, (p0 >> 32) ^ c[3] ^ k[1], p0 & mask]
        k = [(k[0] + W0) & mask, (k[1] + W1) & mask]
    return c


def test_philox_matches_bigint():
    rng = np.random.default_rng(1)
    for _ in range(2000):
        ctr = [int(v) for v in rng.integers(0, 2**32, 4)]
        key = [int(v) for v in rng.integers(0, 2**32, 2)]
        assert list(map(int, oracle.philox4x32_10(ctr, key))) == _philox_bigint(ctr, key)
    for ctr, key in ([0, 0, 0, 0], [0, 0]), ([2**32 - 1] * 4, [2**32 - 1] * 2):
        assert list(map(int, oracle.philox4x32_10(ctr, key))) == _philox_bigint(ctr, key)


@pytest.fixture(scope="module")
def rocrand_host(tmp_path_factory):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("rr") / "librocrand_philox_host.so"
    src = os.path.join(HERE, "helpers", "rocrand_philox_host.cpp")
    subprocess.run(["hipcc", "-O1", "-shared", "-fPIC", "--offload-arch=gfx950", "-x", "hip", src,
                    "-o", str(out)], check=True, capture_output=True)
    lib = ctypes.CDLL(str(out))
    lib.rocrand_philox_block.argtypes = [ctypes.c_ulonglong] * 3 + [ctypes.c_void_p]
    lib.rocrand_philox_block.restype = None
    return lib


def test_philox_matches_rocrand_host_engine(rocrand_host):
    """key = seed (lo, hi); counter = (offset/4 lo, hi, subsequence lo, hi)."""
    rng = np.random.default_rng(0)
    out = np.zeros(4, dtype=np.uint32)
    cases = [(0, 0, 0), (2**64 - 1, 2**64 - 1, 2**62 - 1), (1, 0, 0), (0, 1, 0), (0, 0, 1)]
    for _ in range(3000):
        cases.append((int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2)),
                      int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2)),
                      int(rng.integers(0, 2**62))))
    m = 0xFFFFFFFF
    for seed, sub, c in cases:
        rocrand_host.rocrand_philox_block(seed, sub, c, out.ctypes.data_as(ctypes.c_void_p))
        mine = oracle.philox4x32_10([c & m, c >> 32, sub & m, sub >> 32], [seed & m, seed >> 32])
        assert (mine == out).all(), (seed, sub, c)


def test_philox_outputs_look_uniform():
    """Bytes of 2.5e5 consecutive-counter outputs: chi-square over 256 bins; bit balance; lag-1."""
    n = 60000
    words = np.empty((n, 4), dtype=np.uint32)
    for i in range(n):
        words[i] = oracle.philox4x32_10([i, 0, i % 5, 0], [0, 0])
    b = words.view(np.uint8).reshape(-1)
    cnt = np.bincount(b, minlength=256).astype(np.float64)
    e = b.size / 256
    chi2 = ((cnt - e) ** 2 / e).sum()
    assert 160 < chi2 < 370          # 255 dof: mean 255, sd 22.6  (about +-4.5 sd)
    bits = np.unpackbits(b).mean()
    assert abs(bits - 0.5) < 4 * 0.5 / np.sqrt(b.size * 8)
    u = words[:, 0].astype(np.float64) / 2**32
    r = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(r) < 4 / np.sqrt(n)
