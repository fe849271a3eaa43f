"""Range arguments of the integer butterflies, replayed with Python integers (no GPU).

The HIP kernels keep lazy values in 64-bit words: the twiddle product estimates its quotient from three of the four
32 x 32 partial products (result below 4q), 60-bit primes use Harvey-style butterflies on [0,8q) / [0,4q), primes below
2^52 never correct on the way forward and let sums double on the way back. These tests follow the same recurrences at
the largest moduli each form accepts and check that nothing reaches 2^64 and that every value stays congruent to the
exact product. They model the arithmetic statement, not the kernels' code: bit-exactness of the kernels themselves is
what the GPU parity tests check.
"""
import random

M64 = (1 << 64) - 1


def approx_product(x, w, ws, m):
    """x * w - qt * m modulo 2^64, qt = top partial product + high words of the two middle ones of x * ws."""
    x0, x1, p0, p1 = x & 0xFFFFFFFF, x >> 32, ws & 0xFFFFFFFF, ws >> 32
    qt = x1 * p1 + ((x1 * p0) >> 32) + ((x0 * p1) >> 32)
    assert qt <= M64
    return (x * w - qt * m) & M64


def top_prime_like(bits):
    # any odd modulus just below 2^bits exercises the bounds (primality plays no part in them)
    return (1 << bits) - 59


def test_approximate_product_is_below_4m_and_congruent():
    rng = random.Random(11)
    for bits in (60, 59, 52, 51, 50):
        m = top_prime_like(bits)
        for _ in range(4000):
            w = rng.randrange(m)
            ws = (w << 64) // m
            x = rng.choice([M64, M64 - rng.getrandbits(12), rng.getrandbits(64), rng.getrandbits(40), 16 * m - 1 if 16 * m <= M64 else M64])
            r = approx_product(x, w, ws, m)
            assert r < 4 * m
            assert r % m == (x * w) % m


def _stage(values, m, corrected, rng, forward):
    """One butterfly stage on a list of (value, bound) pairs; returns the new pairs and checks the 64-bit words."""
    out = []
    q4 = 4 * m
    for k in range(0, len(values), 2):
        (X, bx), (Y, by) = values[k], values[k + 1]
        w = rng.randrange(m)
        ws = (w << 64) // m
        if forward:
            if corrected:
                assert bx <= 8 * m
                X = X - q4 if X >= q4 else X
                bx = q4
            T = approx_product(Y, w, ws, m)
            assert X + q4 <= M64
            out += [(X + T, bx + q4), (X + q4 - T, bx + q4)]
        else:
            c = q4 if corrected else max(bx, by)
            assert c % m == 0 and by <= c
            S, D = X + Y, X + c - Y
            assert S <= M64 and D <= M64
            if corrected:
                S = S - c if S >= c else S
                out += [(S, c), (approx_product(D, w, ws, m), q4)]
            else:
                out += [(S, 2 * c), (approx_product(D, w, ws, m), q4)]
    for v, b in out:
        assert v < b <= M64 + 1
    return out


def test_forward_ranges():
    rng = random.Random(5)
    for bits, corrected, stages in ((60, True, 16), (52, False, 16), (52, False, 17)):
        m = top_prime_like(bits)
        vals = [(m - 1, m)] * 32          # canonical inputs at the maximum
        for _ in range(stages):
            rng.shuffle(vals)
            vals = _stage(vals, m, corrected, rng, True)
        bound = max(b for _, b in vals)
        assert bound <= (8 * m if corrected else (1 + 4 * stages) * m)


def test_inverse_ranges():
    rng = random.Random(6)
    # 60-bit primes: inputs below 4q stay below 4q through any number of stages
    m = top_prime_like(60)
    vals = [(4 * m - 1, 4 * m)] * 32
    for _ in range(16):
        rng.shuffle(vals)
        vals = _stage(vals, m, True, rng, False)
    assert max(b for _, b in vals) <= 4 * m
    # primes below 2^52: sums double for the 8 stages of a pass, from inputs below 4q
    m = top_prime_like(52)
    vals = [(4 * m - 1, 4 * m)] * 32
    for _ in range(8):
        vals = sorted(vals, key=lambda vb: -vb[1])    # pair the largest bounds with each other: the worst case
        vals = _stage(vals, m, False, rng, False)
    assert max(b for _, b in vals) <= 1024 * m < (1 << 62)
