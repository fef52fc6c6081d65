"""Pins for oracle.philox: the authors' published known-answer vectors, and the
vectorised routine against the plain-int one on random inputs."""
import os
import random

import numpy as np

from oracle.philox import philox4x32_10, philox4x32_10_scalar


def _load_kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_kat_vectorised(golden_dir):
    rows = _load_kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = philox4x32_10(*ctr, *key)
        assert [int(g) for g in got] == want


def test_kat_scalar(golden_dir):
    for ctr, key, want in _load_kat(golden_dir):
        assert list(philox4x32_10_scalar(ctr, key)) == want


def test_kat_in_a_batch(golden_dir):
    """All vectors at once, to exercise broadcasting."""
    rows = _load_kat(golden_dir)
    ctr = np.array([r[0] for r in rows], dtype=np.uint64)
    key = np.array([r[1] for r in rows], dtype=np.uint64)
    got = philox4x32_10(ctr[:, 0], ctr[:, 1], ctr[:, 2], ctr[:, 3], key[:, 0], key[:, 1])
    got = np.stack(got, axis=1)
    assert got.dtype == np.uint32
    assert got.tolist() == [r[2] for r in rows]


def test_vectorised_equals_scalar_on_random_inputs():
    rnd = random.Random(7)
    n = 200
    ctr = [[rnd.getrandbits(32) for _ in range(4)] for _ in range(n)]
    key = [[rnd.getrandbits(32) for _ in range(2)] for _ in range(n)]
    c = np.array(ctr, dtype=np.uint64)
    k = np.array(key, dtype=np.uint64)
    got = np.stack(philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], k[:, 0], k[:, 1]), axis=1)
    for i in range(n):
        assert tuple(int(x) for x in got[i]) == philox4x32_10_scalar(ctr[i], key[i])


def test_is_a_bijection_on_a_sample():
    """Distinct counters under one key must give distinct 128-bit outputs."""
    c0 = np.arange(4096, dtype=np.uint64)
    r = np.stack(philox4x32_10(c0, 3, 1, 0, 0xDEADBEEF, 0x1234), axis=1)
    assert len({tuple(row) for row in r.tolist()}) == 4096


def test_output_bits_are_balanced():
    """Each of the 128 output bits is set about half the time (avalanche)."""
    c0 = np.arange(1 << 16, dtype=np.uint64)
    r = np.stack(philox4x32_10(c0, 0, 0, 0, 1, 2), axis=1)           # (65536, 4)
    bits = (r[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1
    frac = bits.reshape(-1, 128).mean(axis=0)
    assert np.all(np.abs(frac - 0.5) < 5 * 0.5 / np.sqrt(1 << 16))
