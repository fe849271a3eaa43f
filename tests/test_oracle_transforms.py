"""Pins for the oracle's modular arithmetic, transforms and automorphisms (CPU only).

Nothing here compares the oracle with itself through the same formula: the pins are Python's
exact integers, closed forms, the convolution theorem against the schoolbook product, and
group laws of the Galois maps.
"""
import numpy as np
import pytest

from ckks_inputs import make_params
from oracle import ref


def brev(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2) if bits else 0


@pytest.fixture(scope="module")
def small():
    p = make_params(5, 3, 50, 2, 60, 2)
    return p, ref.RefContext(p)


def rand_poly(rng, q, n):
    return np.array([int(rng.integers(0, 2**62)) % q for _ in range(n)], dtype=np.uint64)


def test_mulmod_powmod_against_python_ints():
    rng = np.random.default_rng(1)
    L = ref.lib()
    for bits in (40, 50, 60, 62):
        m = (1 << bits) - int(rng.integers(1, 1000)) * 2 - 1
        for a, b in [(0, 0), (1, m - 1), (m - 1, m - 1), (m - 1, 2)] + \
                [(int(rng.integers(0, m)), int(rng.integers(0, m))) for _ in range(200)]:
            assert L.ref_mulmod(a, b, m) == a * b % m
            assert L.ref_powmod(a, b, m) == pow(a, b, m)


def test_schoolbook_hand_example_and_numpy():
    q = 97
    n = 8
    a = np.zeros(n, dtype=np.uint64); a[0] = 1; a[1] = 1        # 1 + x
    b = np.zeros(n, dtype=np.uint64); b[n - 1] = 1              # x^(n-1)
    c = ref.schoolbook(a, b, q)                                 # = x^(n-1) + x^n = x^(n-1) - 1
    exp = np.zeros(n, dtype=np.uint64); exp[n - 1] = 1; exp[0] = q - 1
    assert (c == exp).all()
    rng = np.random.default_rng(2)
    q = 12289
    for n in (4, 16, 64):
        a = rng.integers(0, q, n).astype(np.uint64)
        b = rng.integers(0, q, n).astype(np.uint64)
        full = np.convolve(a.astype(object), b.astype(object))  # library polynomial product, exact ints
        folded = [(int(full[k]) - (int(full[k + n]) if k + n < len(full) else 0)) % q for k in range(n)]
        assert ref.schoolbook(a, b, q).tolist() == folded


def test_ntt_closed_forms(small):
    p, c = small
    N, logN = p.N, p.logN
    for lid, (q, psi) in enumerate(zip(p.moduli, p.psi)):
        one = np.zeros((1, 1, N), dtype=np.uint64); one[0, 0, 0] = 1
        assert (c.ntt(one, [lid]) == 1).all()                   # NTT(1) = all ones
        x = np.zeros((1, 1, N), dtype=np.uint64); x[0, 0, 1] = 1
        exp = [pow(psi, 2 * brev(k, logN) + 1, q) for k in range(N)]   # NTT(X)[k] = evaluation point itself
        assert c.ntt(x, [lid])[0, 0].tolist() == exp
        assert c.ntt_definition(x[0, 0], lid).tolist() == exp
        xm = np.zeros((1, 1, N), dtype=np.uint64); xm[0, 0, N - 1] = 1
        exp = [pow(psi, (2 * brev(k, logN) + 1) * (N - 1), q) for k in range(N)]
        assert c.ntt(xm, [lid])[0, 0].tolist() == exp


def test_ntt_is_evaluation_by_horner(small):
    p, c = small
    rng = np.random.default_rng(3)
    for lid, (q, psi) in enumerate(zip(p.moduli, p.psi)):
        a = rand_poly(rng, q, p.N)
        got = c.ntt(a.reshape(1, 1, -1), [lid])[0, 0].tolist()
        for k in range(p.N):
            x = pow(psi, 2 * brev(k, p.logN) + 1, q)
            acc = 0
            for coef in reversed(a.tolist()):
                acc = (acc * x + coef) % q
            assert got[k] == acc


@pytest.mark.parametrize("logN", [2, 3, 6, 10])
def test_fast_transform_equals_definition_and_inverts(logN):
    p = make_params(logN, 2, 50, 1, 60, 1)
    c = ref.RefContext(p)
    rng = np.random.default_rng(logN)
    for lid, q in enumerate(p.moduli):
        a = rand_poly(rng, q, p.N)
        f = c.ntt(a.reshape(1, 1, -1), [lid])
        assert (f[0, 0] == c.ntt_definition(a, lid)).all()
        assert (c.intt(f, [lid])[0, 0] == a).all()
        assert (c.ntt(c.intt(a.reshape(1, 1, -1), [lid]), [lid])[0, 0] == a).all()


@pytest.mark.parametrize("logN", [2, 4, 6])
def test_convolution_theorem_against_schoolbook(logN):
    p = make_params(logN, 2, 50, 1, 60, 1)
    c = ref.RefContext(p)
    rng = np.random.default_rng(10 + logN)
    for lid, q in enumerate(p.moduli):
        a = rand_poly(rng, q, p.N)
        b = rand_poly(rng, q, p.N)
        fa = c.ntt(a.reshape(1, 1, -1), [lid])
        fb = c.ntt(b.reshape(1, 1, -1), [lid])
        prod = c.pointwise(fa, fb, [lid], "mul")
        assert (c.intt(prod, [lid])[0, 0] == ref.schoolbook(a, b, q)).all()


def test_ntt_linearity_and_multi_limb_layout(small):
    p, c = small
    rng = np.random.default_rng(4)
    ids = [3, 0, 4]
    a = np.stack([np.stack([rand_poly(rng, p.moduli[i], p.N) for i in ids]) for _ in range(2)])
    b = np.stack([np.stack([rand_poly(rng, p.moduli[i], p.N) for i in ids]) for _ in range(2)])
    lhs = c.ntt(c.pointwise(a, b, ids, "add"), ids)
    rhs = c.pointwise(c.ntt(a, ids), c.ntt(b, ids), ids, "add")
    assert (lhs == rhs).all()
    for k, i in enumerate(ids):          # each (poly, limb) row uses its own modulus
        assert (c.ntt(a[1:2, k:k + 1], [i]) == c.ntt(a, ids)[1:2, k:k + 1]).all()


# ---------------- automorphisms ----------------
def test_automorph_closed_form_and_group_law(small):
    p, c = small
    N = p.N
    rng = np.random.default_rng(5)
    ids = [0, 4]
    a = np.stack([rand_poly(rng, p.moduli[i], N) for i in ids]).reshape(1, 2, N)
    assert (c.automorph(a, ids, 1, False) == a).all()
    inv = c.automorph(c.automorph(a, ids, 2 * N - 1, False), ids, 2 * N - 1, False)
    assert (inv == a).all()
    for g in (3, 5, 25, 2 * N - 1, N + 1):
        x = np.zeros((1, 1, N), dtype=np.uint64); x[0, 0, 1] = 1
        out = c.automorph(x, [0], g, False)[0, 0]
        exp = np.zeros(N, dtype=np.uint64)
        if g < N:
            exp[g] = 1
        else:
            exp[g - N] = p.moduli[0] - 1                       # X^g = -X^(g-N)
        assert (out == exp).all()
        for h in (5, 7, 2 * N - 3):
            lhs = c.automorph(c.automorph(a, ids, h, False), ids, g, False)
            assert (lhs == c.automorph(a, ids, g * h % (2 * N), False)).all()
            lhs = c.automorph(c.automorph(a, ids, h, True), ids, g, True)
            assert (lhs == c.automorph(a, ids, g * h % (2 * N), True)).all()


def test_automorph_is_ring_homomorphism(small):
    p, c = small
    rng = np.random.default_rng(6)
    q = p.moduli[1]
    a = rand_poly(rng, q, p.N)
    b = rand_poly(rng, q, p.N)
    g = 5
    sa = c.automorph(a.reshape(1, 1, -1), [1], g, False)[0, 0]
    sb = c.automorph(b.reshape(1, 1, -1), [1], g, False)[0, 0]
    sab = c.automorph(ref.schoolbook(a, b, q).reshape(1, 1, -1), [1], g, False)[0, 0]
    assert (ref.schoolbook(sa, sb, q) == sab).all()


def test_eval_domain_automorph_is_the_index_permutation(small):
    """In the bit-reversed evaluation order, sigma_g is out[k] = in[k'] with
    2*brev(k')+1 = (2*brev(k)+1)*g mod 2N."""
    p, c = small
    N, logN = p.N, p.logN
    rng = np.random.default_rng(7)
    ids = [2, 3]
    a = np.stack([rand_poly(rng, p.moduli[i], N) for i in ids]).reshape(1, 2, N)
    for g in (5, 25, 2 * N - 1, 3):
        out = c.automorph(a, ids, g, True)
        perm = [brev((((2 * brev(k, logN) + 1) * g) % (2 * N) - 1) // 2, logN) for k in range(N)]
        assert (out == a[..., perm]).all()


def test_signed_helpers():
    a = np.array([1, -2, 0, 3], dtype=np.int64)
    b = np.array([0, 1, 0, 0], dtype=np.int64)               # X
    assert ref.negacyclic_signed(a, b).tolist() == [-3, 1, -2, 0]
    assert ref.automorph_signed(a, 3).tolist() == [1, 3, 0, -2]    # N=4: -2X -> -2X^3, 3X^3 -> 3X^9 = 3X (X^8 = 1)
