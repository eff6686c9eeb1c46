"""Pure-Python brute-force checkers (unbounded integers, exact rationals).

These restate the definitions a second time, in a different language and with
exact arithmetic, for tiny problem sizes.  They check the C oracle; they are
never used by the product.
"""
from fractions import Fraction
from itertools import permutations

# Philox round constants by word width (Salmon et al., SC'11, Table 2).
PHILOX_CONSTANTS = {
    32: dict(M0=0xD2511F53, M1=0xCD9E8D57, W0=0x9E3779B9, W1=0xBB67AE85),
    64: dict(M0=0xD2E7470EE14C6C93, M1=0xCA5A826395121157, W0=0x9E3779B97F4A7C15, W1=0xBB67AE8584CAA73B),
}


def philox4(ctr, key, width=32, rounds=10):
    """Philox-4xW with `rounds` rounds on Python integers."""
    cst = PHILOX_CONSTANTS[width]
    mask = (1 << width) - 1
    c = [int(w) & mask for w in ctr]
    k = [int(w) & mask for w in key]
    for r in range(rounds):
        if r:
            k = [(k[0] + cst["W0"]) & mask, (k[1] + cst["W1"]) & mask]
        p0 = cst["M0"] * c[0]
        p1 = cst["M1"] * c[2]
        c = [(p1 >> width) ^ c[1] ^ k[0], p1 & mask, (p0 >> width) ^ c[3] ^ k[1], p0 & mask]
    return tuple(c)


def u01_fraction(r):
    """The open-interval uniform as an exact rational: (2 b + 1) / 2^24, b = top 23 bits."""
    return Fraction(2 * (r >> 9) + 1, 1 << 24)


def make_perm(seed, step, k, stream_perm=5):
    """Fisher-Yates from the top of the array down, index by multiply-shift."""
    key = (seed & 0xFFFFFFFF, seed >> 32)
    p = list(range(k))
    for i in range(k - 1, 0, -1):
        r = philox4((i, 0, step, stream_perm), key)[0]
        j = (r * (i + 1)) >> 32
        p[i], p[j] = p[j], p[i]
    return p


def is_permutation(p):
    return sorted(p) == list(range(len(p)))


def all_permutations(k):
    return [list(p) for p in permutations(range(k))]


def gossip_mix_exact(xp, peer, beta):
    """theta_i <- theta'_i - beta (theta'_i - theta'_peer(i)) on exact rationals.
    xp: list over replicas of lists over columns."""
    b = Fraction(beta)
    return [[xi - b * (xi - xp[peer[i]][j]) for j, xi in enumerate(row)] for i, row in enumerate(xp)]


def consensus_distance(x):
    k = len(x)
    n = len(x[0])
    tot = Fraction(0)
    for j in range(n):
        mean = sum(Fraction(x[i][j]) for i in range(k)) / k
        tot += sum((Fraction(x[i][j]) - mean) ** 2 for i in range(k))
    return tot


# --------------------------------------------------------------------------
# fp32 rounding of exact rationals: lets a test replay an fp32 computation one
# rounding at a time without using any floating-point hardware.

def nearest_f32(q):
    """Round an exact rational to the nearest IEEE binary32 value (ties to
    even), returned as an exact Fraction.  Subnormals handled; no overflow
    expected for the magnitudes the tests use."""
    q = Fraction(q)
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = -q if q < 0 else q
    # exponent e with 2^23 <= a / 2^e < 2^24, clamped at the subnormal exponent
    e = a.numerator.bit_length() - a.denominator.bit_length() - 24
    while a >= Fraction(2) ** (e + 24):
        e += 1
    while a < Fraction(2) ** (e + 23):
        e -= 1
    e = max(e, -149)
    scaled = a / Fraction(2) ** e
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return sign * n * Fraction(2) ** e


def f32_fma(a, b, c):
    return nearest_f32(Fraction(a) * Fraction(b) + Fraction(c))


def f32_mul(a, b):
    return nearest_f32(Fraction(a) * Fraction(b))


def f32_add(a, b):
    return nearest_f32(Fraction(a) + Fraction(b))


def f32_sub(a, b):
    return nearest_f32(Fraction(a) - Fraction(b))


SQRT3_F32 = Fraction(14529495, 1 << 23)   # the binary32 value nearest to sqrt(3)


def uniform_noise_exact(word):
    """sqrt(3) (2u - 1) as the method's fp32 arithmetic produces it."""
    w = 2 * u01_fraction(word) - 1          # exact in fp32
    return f32_mul(SQRT3_F32, w)
