"""Pins for the dropout-mask generator of the oracle.

The paper fixes only the mask's distribution (Sec. 3.3: every entry dropped with
probability p); the generator (Philox4x32-10, Salmon et al., SC'11) is this build's
contract.  The stream is pinned to an independent implementation, rocRAND's Philox4x32-10
engine run on the host (tests/philox_rocrand_host.cpp, built by the test with hipcc's host
pass), and by what mathematics fixes: the closed forms of the Weyl key increments, the
bijectivity of a round, a scalar big-integer evaluation of the same rounds, avalanche, and
the statistics of the keep bits.
"""
import math
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import tempo_oracle as O

M32 = 0xFFFFFFFF


@pytest.fixture(scope="module")
def rocrand_philox(tmp_path_factory):
    """Path of the host program over rocRAND's engine; skipped where the ROCm toolchain or the
    rocRAND headers are missing."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc) or not os.path.exists("/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"):
        pytest.skip("hipcc or the rocRAND headers are not installed")
    src = os.path.join(os.path.dirname(__file__), "philox_rocrand_host.cpp")
    exe = str(tmp_path_factory.mktemp("philox") / "philox_rocrand_host")
    r = subprocess.run([hipcc, "--cuda-host-only", "-O1", "-o", exe, src], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]

    def run(seed, subsequence, offset, count):
        out = subprocess.run([exe, str(seed), str(subsequence), str(offset), str(count)],
                             capture_output=True, text=True, timeout=60, check=True)
        return np.array(out.stdout.split(), dtype=np.uint64)
    return run


def test_stream_equals_rocrand_engine(rocrand_philox):
    # counter (g_lo, g_hi, offset_lo, offset_hi), key (seed_lo, seed_hi): the engine's
    # subsequence is the upper half of the counter, its offset counts single outputs
    rng = np.random.default_rng(2022)
    cases = [(0, 0, 0), (1, 0, 0), (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFFFFFFFFFF, (1 << 61) - 3),
             (0x5EED0001, 0, 12345), (0x0123456789ABCDEF, 1 << 33, (1 << 32) - 2)]
    cases += [(int(rng.integers(0, 1 << 63)) * 2 + 1, int(rng.integers(0, 1 << 63)),
               int(rng.integers(0, 1 << 60))) for _ in range(6)]
    for seed, offset, g in cases:
        blocks = 5
        ref = rocrand_philox(seed, offset, 4 * g, 4 * blocks).reshape(blocks, 4)
        gs = np.arange(g, g + blocks, dtype=np.uint64)
        got = O.philox4x32_10((gs & np.uint64(M32), gs >> np.uint64(32), np.uint64(offset & M32),
                               np.uint64(offset >> 32)), (seed & M32, seed >> 32))
        got = np.stack([np.broadcast_to(w, gs.shape) for w in got], axis=1)
        assert np.array_equal(got, ref), (hex(seed), hex(offset), hex(g))


def test_keep_bits_from_the_rocrand_stream(rocrand_philox):
    # the dropout contract on top of the independent stream: element e takes 16-bit lane
    # (e & 7) of group e >> 3 (low half of a word first) and is kept iff lane < T16
    seed, offset, start, n = 0x5EED0000ABCDEF01, 77, 8 * 1000 + 3, 501
    p = np.float32(0.1)
    first, last = start >> 3, (start + n - 1) >> 3
    wordsr = rocrand_philox(seed, offset, 4 * first, 4 * (last - first + 1))
    lanes = np.stack([wordsr & np.uint64(0xFFFF), wordsr >> np.uint64(16)], axis=1).reshape(-1)
    keep_ref = lanes[start - 8 * first: start - 8 * first + n] < O.keep_threshold16(p)
    assert np.array_equal(O.dropout_keep(n, p, seed, offset, start=start), keep_ref)


def test_weyl_constants_closed_form():
    # key increments: 2^32 / golden ratio and 2^32 (sqrt(3) - 1), truncated (integer sqrt: exact)
    golden = (math.isqrt(5 << 64) - (1 << 32)) // 2          # 2^32 (sqrt5 - 1)/2
    assert int(O._PHILOX_W0) == golden
    assert int(O._PHILOX_W1) == math.isqrt(3 << 64) - (1 << 32)
    # multipliers must be odd (invertible mod 2^32) for the round to be a bijection
    assert int(O._PHILOX_M0) & 1 and int(O._PHILOX_M1) & 1


def _scalar_philox(ctr, key, rounds=10):
    c = [int(v) & M32 for v in ctr]
    k = [int(v) & M32 for v in key]
    m0, m1 = int(O._PHILOX_M0), int(O._PHILOX_M1)
    for r in range(rounds):
        if r:
            k = [(k[0] + int(O._PHILOX_W0)) & M32, (k[1] + int(O._PHILOX_W1)) & M32]
        p0, p1 = m0 * c[0], m1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M32, (p0 >> 32) ^ c[3] ^ k[1], p0 & M32]
    return c


def test_vectorised_rounds_equal_big_integer_rounds():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 1 << 32, size=(50, 4), dtype=np.uint64)
    key = (0x12345678, 0x9ABCDEF0)
    out = O.philox4x32_10(tuple(ctr[:, i] for i in range(4)), key)
    for n in range(50):
        assert [int(w[n]) for w in out] == _scalar_philox(ctr[n], key)
    # extreme words exercise the 64-bit products
    out = O.philox4x32_10((np.uint64(M32),) * 4, (M32, M32))
    assert [int(w) for w in out] == _scalar_philox([M32] * 4, [M32, M32])


def test_round_is_a_bijection():
    rng = np.random.default_rng(1)
    c = [rng.integers(0, 1 << 32, size=1000, dtype=np.uint64) for _ in range(4)]
    k0, k1 = np.uint64(0xDEADBEEF), np.uint64(0x0BADF00D)
    o = O.philox_round(*c, k0, k1)
    inv0 = pow(int(O._PHILOX_M0), -1, 1 << 32)
    inv1 = pow(int(O._PHILOX_M1), -1, 1 << 32)
    m = np.uint64(M32)
    c0 = (o[3] * np.uint64(inv0)) & m
    c2 = (o[1] * np.uint64(inv1)) & m
    hi0 = (O._PHILOX_M0 * c0) >> np.uint64(32)
    hi1 = (O._PHILOX_M1 * c2) >> np.uint64(32)
    c1 = o[0] ^ hi1 ^ k0
    c3 = o[2] ^ hi0 ^ k1
    for a, b in zip((c0, c1, c2, c3), c):
        assert np.array_equal(a, b)


def test_avalanche():
    # flipping any single counter or key bit flips about half of the 128 output bits
    rng = np.random.default_rng(2)
    n = 400
    base_c = [rng.integers(0, 1 << 32, size=n, dtype=np.uint64) for _ in range(4)]
    key = (123, 456)
    base = np.stack(O.philox4x32_10(base_c, key))
    popc = lambda a: np.array([bin(int(v)).count("1") for v in a.reshape(-1)]).reshape(a.shape)
    for word in range(4):
        for bit in (0, 7, 16, 31):
            c = [x.copy() for x in base_c]
            c[word] ^= np.uint64(1 << bit)
            flipped = popc(np.stack(O.philox4x32_10(c, key)) ^ base).sum(0)
            assert 58 < flipped.mean() < 70, (word, bit, flipped.mean())
    for kw in range(2):
        k = list(key)
        k[kw] ^= 1 << 5
        flipped = popc(np.stack(O.philox4x32_10(base_c, k)) ^ base).sum(0)
        assert 58 < flipped.mean() < 70


def test_threshold():
    assert O.keep_threshold16(0.1) == 58982      # (1 - float32(0.1)) * 65536 rounded
    assert O.keep_threshold16(0.0) == 65536
    assert O.keep_threshold16(0.5) == 32768
    assert O.keep_threshold16(np.float32(0.99999)) == 1


@pytest.mark.parametrize("p", [0.1, 0.5, 0.9])
def test_keep_bits_statistics(p):
    n = 1 << 21
    K = O.dropout_keep(n, p, seed=0x5EED0001, offset=0)
    q = O.keep_threshold16(p) / 65536.0
    sigma = math.sqrt(q * (1 - q) / n)
    assert abs(K.mean() - q) < 4 * sigma
    # every one of the eight 16-bit lanes of a group is balanced
    lanes = K.reshape(-1, 8).mean(0)
    assert np.all(np.abs(lanes - q) < 4.5 * sigma * math.sqrt(8))
    # neighbouring elements, neighbouring rows of 128 and of 512 are uncorrelated
    k = K.astype(np.float64) - K.mean()
    for lag in (1, 2, 8, 32, 128, 512):
        corr = float((k[:-lag] * k[lag:]).mean() / k.var())
        assert abs(corr) < 4.5 / math.sqrt(n), (lag, corr)


def test_keep_bits_are_a_function_of_seed_offset_index():
    a = O.dropout_keep(1000, 0.1, 9, 5)
    assert np.array_equal(a, O.dropout_keep(1000, 0.1, 9, 5))
    # any window equals the same window of a longer stream (launch geometry cannot matter)
    assert np.array_equal(O.dropout_keep(100, 0.1, 9, 5, start=333), a[333:433])
    assert not np.array_equal(a, O.dropout_keep(1000, 0.1, 10, 5))
    assert not np.array_equal(a, O.dropout_keep(1000, 0.1, 9, 6))
    assert not np.array_equal(a, O.dropout_keep(1000, 0.1, 9 + (1 << 32), 5))   # high seed word is used
    assert not np.array_equal(a, O.dropout_keep(1000, 0.1, 9, 5 + (1 << 32)))   # high offset word is used
    assert O.dropout_keep(64, 0.0, 1, 0).all()
    assert O.dropout_keep(0, 0.1, 1, 0).size == 0


def test_bit_packing_layout():
    bits = np.zeros(70, dtype=bool)
    bits[[0, 2, 31, 32, 69]] = True
    w = O.pack_bits(bits)
    assert w.dtype == np.uint32 and w.tolist() == [(1 << 0) | (1 << 2) | (1 << 31), 1, 1 << 5]
    assert np.array_equal(O.unpack_bits(w, 70), bits)
    rnd = np.random.default_rng(3).random(1000) < 0.5
    assert np.array_equal(O.unpack_bits(O.pack_bits(rnd), 1000), rnd)
    # little-endian bytes of the words are the bytes of numpy's little-bit-order packing
    assert np.array_equal(O.pack_bits(rnd).view(np.uint8)[:125], np.packbits(rnd, bitorder="little"))
