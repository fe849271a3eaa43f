"""Pins for CRT, base conversion and ModDown, against Python's exact integers (CPU only)."""
import math

import numpy as np
import pytest

from ckks_inputs import make_params
from oracle import ref


def prod(xs):
    r = 1
    for x in xs:
        r *= int(x)
    return r


def residues(vals, moduli):
    return np.array([[v % m for v in vals] for m in moduli], dtype=np.uint64)


def centre(v, m):
    v %= m
    return v - m if v > m // 2 else v


@pytest.fixture(scope="module")
def ctx():
    p = make_params(4, 6, 50, 3, 60, 2)      # alpha = 3, K = 3
    return p, ref.RefContext(p)


def test_crt_reconstruction_and_rns_product(ctx):
    p, _ = ctx
    rng = np.random.default_rng(0)
    Q = prod(p.q)
    xs = [int.from_bytes(rng.bytes(48), "little") % Q for _ in range(16)]
    ys = [int.from_bytes(rng.bytes(48), "little") % Q for _ in range(16)]
    rec = ref.crt_centred(residues(xs, p.q), p.q)
    assert rec == [centre(x, Q) for x in xs]
    L = ref.lib()
    pr = np.array([[L.ref_mulmod(x % m, y % m, m) for x, y in zip(xs, ys)] for m in p.q], dtype=np.uint64)
    assert ref.crt_centred(pr, p.q) == [centre(x * y, Q) for x, y in zip(xs, ys)]


@pytest.mark.parametrize("src", [[0, 1, 2], [3, 4, 5], [6, 7, 8], [1], [4, 5]])
def test_bconv_value_is_centred_lift_plus_small_multiple(ctx, src):
    p, c = ctx
    mod = p.moduli
    dst = [i for i in range(len(mod)) if i not in src]
    C = prod(mod[i] for i in src)
    rng = np.random.default_rng(len(src))
    xs = [int.from_bytes(rng.bytes(40), "little") % C for _ in range(61)] + [0, 1, C - 1, C // 2, C // 2 + 1]
    out = c.bconv(residues(xs, [mod[i] for i in src]), src, dst)
    # the target basis is wide enough to recover the integer V the conversion represents
    D = prod(mod[i] for i in dst)
    assert D > 4 * len(src) * C
    V = ref.crt_centred(out, [mod[i] for i in dst])
    n = len(src)
    for x, v in zip(xs, V):
        assert (v - x) % C == 0
        u = (v - centre(x, C)) // C
        assert abs(u) <= math.ceil(n / 2)
        if n == 1:
            assert v == centre(x, C)             # single-prime source: exact centred lift


def test_bconv_is_exactly_the_centred_sum_formula(ctx):
    """V = sum_i centred([x_i * (C/c_i)^-1]_{c_i}) * (C/c_i), evaluated here with Python integers."""
    p, c = ctx
    mod = p.moduli
    src, dst = [3, 4, 5], [0, 1, 2, 6, 7, 8]
    cs = [mod[i] for i in src]
    C = prod(cs)
    rng = np.random.default_rng(9)
    xs = [int.from_bytes(rng.bytes(40), "little") % C for _ in range(32)]
    out = c.bconv(residues(xs, cs), src, dst)
    for k, x in enumerate(xs):
        V = 0
        for ci in cs:
            h = C // ci
            V += centre((x % ci) * pow(h, -1, ci), ci) * h
        for t, j in enumerate(dst):
            assert int(out[t, k]) == V % mod[j]


@pytest.mark.parametrize("shape", [(6, 3), (4, 3), (2, 1), (5, 2)])
def test_moddown_is_rounded_division_by_P(shape):
    nq, K = shape
    p = make_params(4, nq, 50, K, 60, 2)
    c = ref.RefContext(p)
    Q, P = prod(p.q), prod(p.p)
    rng = np.random.default_rng(nq * 10 + K)
    Xs = [centre(int.from_bytes(rng.bytes(80), "little"), P * Q) for _ in range(40)]
    Xs += [P * centre(int.from_bytes(rng.bytes(80), "little"), Q) for _ in range(8)]     # exact multiples of P
    Xs += [0, 1, -1, P // 2, P // 2 + 1, -(P // 2) - 1]
    Xs = (Xs + [0] * 16)[:((len(Xs) + 15) // 16) * 16]
    out = c.moddown_coeff(residues(Xs, p.moduli), nq)
    got = ref.crt_centred(out, p.q)
    for X, g in zip(Xs, got):
        r = X - P * ((2 * X + P) // (2 * P))      # X = P*round(X/P) + r
        rounded = (X - r) // P
        diff = centre(g - rounded, Q)
        assert abs(diff) <= math.ceil(K / 2)
        if X % P == 0:
            assert diff == 0
        if K == 1:
            assert diff == 0


def test_rescale_is_exact_rounded_division_by_last_prime():
    """CRT(rescale(c)) = round(c / q_L) on the centred integers, every coefficient (coefficient domain via INTT)."""
    p = make_params(4, 4, 50, 1, 60, 2)
    c = ref.RefContext(p)
    rng = np.random.default_rng(5)
    nl = 4
    ids = list(range(nl))
    Q, qL = prod(p.q), p.q[-1]
    vals = [[centre(int.from_bytes(rng.bytes(32), "little"), Q) for _ in range(p.N)] for _ in range(2)]
    vals[0][0], vals[0][1], vals[0][2] = 0, qL // 2, -(qL // 2) - 1
    coeff = np.stack([residues(v, p.q) for v in vals])[None]                 # [1][2][nl][N] coefficient domain
    ct = c.ntt(coeff.reshape(2, nl, p.N), ids).reshape(1, 2, nl, p.N)
    out = c.rescale(ct)
    back = c.intt(out.reshape(2, nl - 1, p.N), ids[:-1])
    Qp = Q // qL
    for comp in range(2):
        got = ref.crt_centred(back[comp], p.q[:-1])
        for x, g in zip(vals[comp], got):
            want = (x - centre(x, qL)) // qL
            assert (g - want) % Qp == 0
