"""Pins for the oracle's arithmetic layer: random streams, noise, negacyclic products,
gadget decomposition, modulus switch, accumulator initialisation.

Each check compares the oracle with something fixed outside it: a published test
vector, a library routine on a special case, a closed form or an algebraic law.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")
M32 = (1 << 32) - 1


def rnd_u32(rng, n):
    return rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)


# --------------------------------------------------------------------------- streams
def test_splitmix64_published_vector(orc):
    want = [int(l) for l in open(os.path.join(GOLD, "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    got = [orc.rand(1234567, "RAW", i) for i in range(len(want))]
    assert got == want


def test_domain_streams_are_reseeded_splitmix(orc):
    # domain d >= 1 is the generator seeded with output d of the seed's own generator
    for seed in (0, 1, 0xDEADBEEF, 2**64 - 1):
        for d in (1, 2, 5, 8):
            sub = orc.rand(seed, "RAW", d - 1)
            for i in (0, 1, 17, 10**9):
                assert orc.rand(seed, d, i) == orc.rand(sub, "RAW", i)


def test_uniform_words_are_balanced(orc):
    v = np.array([orc.rand(99, "ENC_A", i) >> 32 for i in range(40000)], dtype=np.float64)
    assert abs(v.mean() / 2**32 - 0.5) < 0.01
    assert abs(v.std() / 2**32 - 12 ** -0.5) < 0.01
    top = np.array([orc.rand(99, "LWE_SK", i) >> 63 for i in range(40000)])
    assert abs(top.mean() - 0.5) < 0.01


@pytest.mark.parametrize("log2", [-15, -25])
def test_noise_moments(orc, log2):
    e = np.array([orc.noise(5, "ENC_E", i, log2) for i in range(60000)], dtype=np.float64)
    sigma = 2.0 ** (32 + log2)
    assert abs(e.mean()) < 4 * sigma / 60000 ** 0.5
    assert abs(e.std() / sigma - 1) < 0.01
    assert np.abs(e).max() <= 6 * sigma + 1          # Irwin-Hall(12) support
    # excess kurtosis of a sum of 12 uniforms is -0.1
    k = ((e - e.mean()) ** 4).mean() / e.var() ** 2 - 3
    assert abs(k + 0.1) < 0.08


def test_noise_is_rounded_sum_of_twelve_words(orc):
    from fractions import Fraction
    import math
    for idx in range(200):
        G = sum(orc.rand(11, "BK_E", 12 * idx + j) >> 32 for j in range(12)) - 6 * 2**32
        for log2 in (-15, -25, -3):
            want = math.floor(Fraction(G, 2 ** -log2) + Fraction(1, 2))
            assert orc.noise(11, "BK_E", idx, log2) == want
    assert all(orc.noise(11, "BK_E", i, -40) == 0 for i in range(100))
    assert all(orc.noise(11, "BK_E", i, -60) == 0 for i in range(100))


# --------------------------------------------------------------------------- products
@pytest.mark.parametrize("N", [2, 4, 8, 16, 64, 256])
def test_three_products_agree(orc, N):
    rng = np.random.default_rng(N)
    for _ in range(5):
        a, b = rnd_u32(rng, N), rnd_u32(rng, N)
        d = orc.negacyclic(a, b, "definition")
        assert np.array_equal(d, orc.negacyclic(a, b, "schoolbook"))
        assert np.array_equal(d, orc.negacyclic(a, b, "karatsuba"))


def test_products_agree_at_ring_size(orc):
    rng = np.random.default_rng(1024)
    a, b = rnd_u32(rng, 1024), rnd_u32(rng, 1024)
    s = orc.negacyclic(a, b, "schoolbook")
    assert np.array_equal(s, orc.negacyclic(a, b, "karatsuba"))
    assert np.array_equal(s, orc.negacyclic(a, b, "definition"))


@pytest.mark.parametrize("N", [4, 16, 128, 1024])
@pytest.mark.parametrize("method", ["definition", "schoolbook", "karatsuba"])
def test_product_against_numpy_convolution(orc, N, method):
    """Small operands: the integer convolution of numpy, folded with X^N = -1."""
    rng = np.random.default_rng(7 * N)
    a = rng.integers(-512, 512, N)
    b = rng.integers(-2**20, 2**20, N)
    lin = np.convolve(a.astype(np.int64), b.astype(np.int64))
    want = lin[:N].copy()
    want[:N - 1] -= lin[N:]
    got = orc.negacyclic((a & M32).astype(np.uint32), (b & M32).astype(np.uint32), method)
    assert np.array_equal(got, (want & M32).astype(np.uint32))


@pytest.mark.parametrize("N", [8, 64])
def test_ring_laws(orc, N):
    rng = np.random.default_rng(3)
    p, q, r = rnd_u32(rng, N), rnd_u32(rng, N), rnd_u32(rng, N)
    mul = lambda x, y: orc.negacyclic(x, y, "karatsuba")
    assert np.array_equal(mul(p, q), mul(q, p))
    assert np.array_equal(mul(mul(p, q), r), mul(p, mul(q, r)))
    assert np.array_equal(mul(p, (q + r).astype(np.uint32)), (mul(p, q) + mul(p, r)).astype(np.uint32))
    one = np.zeros(N, np.uint32); one[0] = 1
    assert np.array_equal(mul(p, one), p)
    c = np.zeros(N, np.uint32); c[0] = 12345
    assert np.array_equal(mul(p, c), (p * np.uint32(12345)).astype(np.uint32))
    # X^N = -1:  X^(N-1) * X = -1
    x1 = np.zeros(N, np.uint32); x1[1] = 1
    xl = np.zeros(N, np.uint32); xl[N - 1] = 1
    minus_one = np.zeros(N, np.uint32); minus_one[0] = M32
    assert np.array_equal(mul(x1, xl), minus_one)


@pytest.mark.parametrize("N", [4, 32])
def test_monomial_is_signed_rotation(orc, N):
    rng = np.random.default_rng(5)
    p = rnd_u32(rng, N)
    for a in range(2 * N):
        got = orc.mul_by_xpow(p, a)
        # by hand: coefficient j moves to j + a; every wrap past N flips the sign
        want = np.zeros(N, np.uint32)
        for j in range(N):
            e = j + a
            want[e % N] = p[j] if (e // N) % 2 == 0 else (0 - int(p[j])) & M32
        assert np.array_equal(got, want)
        mono = np.zeros(N, np.uint32)
        mono[a % N] = 1 if a < N else M32
        assert np.array_equal(got, orc.negacyclic(p, mono, "definition"))
    assert np.array_equal(orc.mul_by_xpow(orc.mul_by_xpow(p, 3), 2 * N - 3), p)


# --------------------------------------------------------------------------- decomposition
@pytest.mark.parametrize("l,bg", [(2, 10), (3, 7), (1, 8), (2, 8), (3, 10)])
def test_decomposition_reconstructs_with_bounded_residue(orc, l, bg):
    P = orc.Params(8, 16, 1, l, bg, 8, 2, -15, -25)
    K = orc.Keys(P, 1, cloud=False)
    rng = np.random.default_rng(l * 100 + bg)
    low = 32 - l * bg                       # bits below the last digit
    edge = [0, 1, M32, 1 << 31, (1 << 31) - 1, (1 << 31) + 1,
            (1 << (low - 1)) - 1, 1 << (low - 1), (1 << (low - 1)) + 1, (1 << low) - 1, 1 << low]
    xs = edge + [int(v) for v in rnd_u32(rng, 3000)]
    for x in xs:
        d = K.decompose(x)
        assert d.min() >= -(1 << (bg - 1)) and d.max() < (1 << (bg - 1))
        approx = sum(int(d[j]) << (32 - bg * (j + 1)) for j in range(l))
        res = (x - approx) & M32
        res = res - (1 << 32) if res >= (1 << 31) else res
        assert -(1 << (low - 1)) <= res < (1 << (low - 1)), (x, d, res)
    assert list(K.decompose(0)) == [0] * l


def test_decomposition_default_offset_constant(orc):
    # at l=2, Bgbit=10 the digits are ((x + 2^31 + 2^21 + 2^11) >> {22,12} & 1023) - 512
    K = orc.Keys(orc.default_params(), 1, cloud=False)
    rng = np.random.default_rng(0)
    for x in rnd_u32(rng, 2000):
        xp = (int(x) + 2**31 + 2**21 + 2**11) & M32
        assert list(K.decompose(x)) == [((xp >> 22) & 1023) - 512, ((xp >> 12) & 1023) - 512]


# --------------------------------------------------------------------------- modswitch / acc
def test_modswitch_rounds_half_up_to_2N(orc):
    P = orc.default_params()
    K = orc.Keys(P, 1, cloud=False)
    c = np.zeros(P.n + 1, np.uint32)
    cases = {0: 0, 1: 0, (1 << 20) - 1: 0, 1 << 20: 1, 1 << 21: 1, (1 << 21) + (1 << 20) - 1: 1,
             (1 << 21) + (1 << 20): 2, 1023 << 21: 1023, 1 << 31: 1024, M32: 0,
             M32 - (1 << 20): 2047, M32 - (1 << 20) + 1: 0, (2047 << 21) + (1 << 20) - 1: 2047}
    for k, (x, want) in enumerate(cases.items()):
        c[k] = x
    bar = K.modswitch(c)
    for k, (x, want) in enumerate(cases.items()):
        assert bar[k] == want, (hex(x), bar[k], want)
    # against float rounding for random words
    rng = np.random.default_rng(1)
    c = rnd_u32(rng, P.n + 1)
    want = np.floor(c.astype(np.float64) * 2048 / 2**32 + 0.5).astype(np.int64) % 2048
    assert np.array_equal(K.modswitch(c), want.astype(np.uint32))


def test_modswitch_other_ring_size(orc):
    P = orc.Params(4, 64, 1, 2, 10, 8, 2, -15, -25)
    K = orc.Keys(P, 1, cloud=False)
    rng = np.random.default_rng(2)
    c = rnd_u32(rng, 5)
    want = np.floor(c.astype(np.float64) * 128 / 2**32 + 0.5).astype(np.int64) % 128
    assert np.array_equal(K.modswitch(c), want.astype(np.uint32))


@pytest.mark.parametrize("N", [16, 1024])
def test_acc_init_closed_form(orc, N):
    """X^(-b) * (1/8)(1 + X + ... + X^(N-1)): +1/8 below N-b, -1/8 from N-b on (b < N);
    the negated pattern for b >= N."""
    P = orc.Params(4, N, 1, 2, 10, 8, 2, -15, -25)
    K = orc.Keys(P, 1, cloud=False)
    mu = 1 << 29
    for b in [0, 1, 2, N // 2, N - 1, N, N + 1, 2 * N - 1]:
        acc = K.acc_init(b)
        assert not acc[:N].any()
        bb, sgn = (b, 1) if b < N else (b - N, -1)
        want = np.where(np.arange(N) < N - bb, sgn * mu, -sgn * mu) & M32
        assert np.array_equal(acc[N:], want.astype(np.uint32)), b
