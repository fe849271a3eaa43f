"""Parameter selection for the synthetic RNS-CKKS workloads.

The paper fixes only the ring (Z_q[x]/(x^N+1), Sec. 2.1) and the shape of its
parameter set (Sec. 5.1 "Encryption Parameters"); it does not say which primes or
which roots of unity are used. The deterministic rules below are this build's
reading; the values they produce are passed as plain inputs to both the CPU oracle
and the HIP library, and each of those validates them on its own.
"""
from dataclasses import dataclass, field
from typing import List

_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)  # deterministic for n < 3.3e24


def is_prime(n: int) -> bool:
    if n < 2:
        return False
    for b in _MR_BASES:
        if n % b == 0:
            return n == b
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in _MR_BASES:
        x = pow(a, d, n)
        if x == 1 or x == n - 1:
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def find_ntt_primes(bits: int, count: int, logN: int, exclude=()) -> List[int]:
    """`count` primes q = 1 (mod 2N), scanning downward from 2^bits - 1; first found is first returned."""
    two_n = 2 << logN
    out = []
    q = ((1 << bits) - 1) // two_n * two_n + 1
    while len(out) < count:
        if q < (1 << (bits - 1)):
            raise ValueError("ran out of %d-bit primes = 1 mod %d" % (bits, two_n))
        if q not in exclude and is_prime(q):
            out.append(q)
        q -= two_n
    return out


def find_psi(q: int, logN: int) -> int:
    """Primitive 2N-th root of unity: g^((q-1)/2N) for the smallest quadratic non-residue g >= 2."""
    two_n = 2 << logN
    assert (q - 1) % two_n == 0
    g = 2
    while pow(g, (q - 1) // 2, q) != q - 1:
        g += 1
    psi = pow(g, (q - 1) // two_n, q)
    assert pow(psi, two_n // 2, q) == q - 1
    return psi


@dataclass
class CkksParams:
    logN: int
    q: List[int]            # L+1 main primes
    p: List[int]            # K special primes
    dnum: int
    psi: List[int] = field(default_factory=list)   # one primitive 2N-th root per modulus, q first then p

    @property
    def N(self):
        return 1 << self.logN

    @property
    def moduli(self):
        return list(self.q) + list(self.p)

    @property
    def alpha(self):
        return -(-len(self.q) // self.dnum)

    def beta(self, nlimbs):
        return -(-nlimbs // self.alpha)


def make_params(logN, nq, q_bits, np_, p_bits, dnum) -> CkksParams:
    q = find_ntt_primes(q_bits, nq, logN)
    p = find_ntt_primes(p_bits, np_, logN, exclude=set(q))
    psi = [find_psi(m, logN) for m in q + p]
    return CkksParams(logN=logN, q=q, p=p, dnum=dnum, psi=psi)
