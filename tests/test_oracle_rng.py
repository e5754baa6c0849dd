"""Pins for the oracle's counter-based generator, weight generator and bf16 rounding."""
import os

import numpy as np
import torch

import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        yield w[0:4], w[4:6], w[6:10]


def py_philox(ctr, key):
    """Second, independent implementation (python ints) of Philox4x32-10."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        hi0, lo0 = divmod(0xD2511F53 * c[0], 1 << 32)
        hi1, lo1 = divmod(0xCD9E8D57 * c[2], 1 << 32)
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers():
    rows = list(_kat_rows())
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert [int(x) for x in O.philox(ctr, key)] == out
        assert py_philox(ctr, key) == out


def test_philox_two_implementations_agree():
    rng = np.random.default_rng(7)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        assert [int(x) for x in O.philox(ctr, key)] == py_philox(ctr, key)


def test_weight_generator_matches_independent_formula():
    # sum of the eight 16-bit halves, centred, times one fp32 constant
    seed, tid, layer = 0x1234567ABCDEF, 11, 3
    got = O.weight_fill(seed, tid, layer, 5, 64, 0)
    c = np.float32(0.02 / np.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0))
    for i in range(64):
        e = 5 + i
        o = py_philox([e & 0xFFFFFFFF, e >> 32, tid, layer], [seed & 0xFFFFFFFF, seed >> 32])
        s = sum((x & 0xFFFF) + (x >> 16) for x in o)
        assert got[i] == np.float32(s - 262140) * c


def test_weight_generator_bf16_values_are_bf16():
    w32 = O.weight_fill(9, 18, 1, 0, 4096, 0)
    w16 = O.weight_fill(9, 18, 1, 0, 4096, 1)
    ref = torch.from_numpy(w32).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(w16, ref)


def test_weight_generator_moments():
    w = O.weight_fill(42, 0, 0, 0, 1 << 21, 0).astype(np.float64)
    assert abs(w.mean()) < 5e-5
    assert abs(w.std() - 0.02) < 1e-4
    kurt = ((w / w.std()) ** 4).mean()
    assert abs(kurt - (3.0 - 1.2 / 8.0)) < 0.02     # Irwin-Hall(8): excess kurtosis -6/(5*8)
    assert np.abs(w).max() <= 0.02 * 4.9 + 1e-6
    # different tensors / layers / seeds are different streams
    a = O.weight_fill(42, 0, 0, 0, 1024, 0)
    assert not np.array_equal(a, O.weight_fill(42, 1, 0, 0, 1024, 0))
    assert not np.array_equal(a, O.weight_fill(42, 0, 1, 0, 1024, 0))
    assert not np.array_equal(a, O.weight_fill(43, 0, 0, 0, 1024, 0))
    # windows of one stream are consistent
    assert np.array_equal(a[100:200], O.weight_fill(42, 0, 0, 100, 100, 0))


def np_round_bf16(x):
    """Independent bit-level round-to-nearest-even of float64 to 8 significant bits."""
    b = np.asarray(x, dtype=np.float64).view(np.uint64)
    drop = np.uint64(52 - 7)
    lsb = (b >> drop) & np.uint64(1)
    r = b + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + lsb
    r &= ~((np.uint64(1) << drop) - np.uint64(1))
    return r.view(np.float64)


def test_bf16_rounding():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [1.0, -1.0, 0.0, 1.00390625, 1.01171875, 255.5, 3.0e-5]])
    got = np.array([O.round_bf16(v) for v in x])
    assert np.array_equal(got, np_round_bf16(x))
    # on fp32 inputs it is the library's float -> bfloat16 conversion
    xf = x.astype(np.float32)
    lib = torch.from_numpy(xf).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(np.array([O.round_bf16(float(v)) for v in xf]), lib)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert O.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
