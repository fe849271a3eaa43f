"""Python face of the CPU oracle. TEST INFRASTRUCTURE ONLY: imported by tests, the smoke
check and the benchmark's CPU-baseline leg, never by the product path.

The heavy integer arithmetic lives in ref_ckks.cpp (plain C++, __int128 and `%`). This
module adds what is easiest to state with Python's exact integers and numpy:

* CRT reconstruction of RNS residues into centred big integers (Sec. 2.2 of the paper:
  every coefficient c in Z_Q is stored as {c mod q_i});
* the CKKS canonical-embedding encode/decode for S = N/2 slots (Sec. 2.1), using
  numpy's FFT as a library step; it is pinned against the O(N*S) definition in the tests;
* convenience wrappers that assemble keys and ciphertexts from seeded arrays.

Readings taken where the paper is silent are listed in the design document.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None
u64p = C.POINTER(C.c_uint64)
i64p = C.POINTER(C.c_int64)
u32p = C.POINTER(C.c_uint32)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.ref_last_error.restype = C.c_char_p
        L.ref_mulmod.restype = C.c_uint64
        L.ref_mulmod.argtypes = [C.c_uint64] * 3
        L.ref_powmod.restype = C.c_uint64
        L.ref_powmod.argtypes = [C.c_uint64] * 3
        _lib = L
    return _lib


def _u64(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return a, a.ctypes.data_as(u64p)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(i64p)


def _ids(ids):
    a = np.ascontiguousarray(ids, dtype=np.uint32)
    return a, a.ctypes.data_as(u32p), C.c_uint32(len(a))


def _check(rc):
    if rc != 0:
        raise RuntimeError("oracle: " + lib().ref_last_error().decode())


def set_threads(n):
    lib().ref_set_threads(C.c_int(int(n)))


class RefContext:
    """Oracle context for one parameter set (ckks_inputs.CkksParams)."""

    def __init__(self, params):
        self.params = params
        self.N = params.N
        self.logN = params.logN
        self.nq, self.np_ = len(params.q), len(params.p)
        self.nm = self.nq + self.np_
        self.moduli = params.moduli
        q, qp = _u64(params.q)
        p, pp = _u64(params.p if params.p else [0])
        psi, psip = _u64(params.psi)
        self._h = C.c_void_p()
        _check(lib().ref_ctx_create(C.byref(self._h), C.c_uint32(params.logN), qp, C.c_uint32(self.nq), pp,
                                    C.c_uint32(self.np_), C.c_uint32(params.dnum), psip))

    def __del__(self):
        # at interpreter shutdown the module globals may already be gone; the process is ending anyway
        if getattr(self, "_h", None) and lib is not None:
            try:
                lib().ref_ctx_destroy(self._h)
            except Exception:
                pass
            self._h = None

    # ---- transforms (return new arrays) ----
    def ntt_definition(self, a, limb_id):
        a, p = _u64(np.array(a, dtype=np.uint64, copy=True))
        _check(lib().ref_ntt_definition(self._h, p, C.c_uint32(limb_id)))
        return a

    def _xform(self, fn, data, limb_ids):
        data = np.array(data, dtype=np.uint64, copy=True)
        nl = len(limb_ids)
        assert data.shape[-1] == self.N and data.shape[-2] == nl
        npoly = int(np.prod(data.shape[:-2], dtype=np.int64))
        _, ip, n = _ids(limb_ids)
        _check(fn(self._h, data.ctypes.data_as(u64p), C.c_uint32(npoly), ip, n))
        return data

    def ntt(self, data, limb_ids):
        return self._xform(lib().ref_ntt, data, limb_ids)

    def intt(self, data, limb_ids):
        return self._xform(lib().ref_intt, data, limb_ids)

    def automorph(self, data, limb_ids, g, eval_domain):
        data, dp = _u64(data)
        out = np.empty_like(data)
        npoly = int(np.prod(data.shape[:-2], dtype=np.int64))
        _, ip, n = _ids(limb_ids)
        _check(lib().ref_automorph(self._h, out.ctypes.data_as(u64p), dp, C.c_uint32(npoly), ip, n, C.c_uint32(g),
                                   C.c_int(1 if eval_domain else 0)))
        return out

    def pointwise(self, a, b, limb_ids, op):
        a, ap = _u64(a)
        b, bp = _u64(b)
        out = np.empty_like(a)
        npoly = int(np.prod(a.shape[:-2], dtype=np.int64))
        b_npoly = int(np.prod(b.shape[:-2], dtype=np.int64))
        assert b_npoly in (1, npoly)
        _, ip, n = _ids(limb_ids)
        _check(lib().ref_pointwise(self._h, out.ctypes.data_as(u64p), ap, bp, C.c_uint32(npoly), C.c_uint32(b_npoly),
                                   ip, n, C.c_int({"add": 0, "sub": 1, "mul": 2}[op])))
        return out

    def signed_to_rns(self, v, limb_ids):
        v, vp = _i64(v)
        out = np.empty((len(limb_ids), self.N), dtype=np.uint64)
        _, ip, n = _ids(limb_ids)
        _check(lib().ref_signed_to_rns(self._h, out.ctypes.data_as(u64p), vp, ip, n))
        return out

    def bconv(self, x, src_ids, dst_ids):
        x, xp = _u64(x)
        ncoef = x.shape[-1]
        out = np.empty((len(dst_ids), ncoef), dtype=np.uint64)
        _, sp, ns = _ids(src_ids)
        _, dp, nd = _ids(dst_ids)
        _check(lib().ref_bconv(self._h, out.ctypes.data_as(u64p), xp, sp, ns, dp, nd, C.c_uint32(ncoef)))
        return out

    def moddown_coeff(self, x, nlimbs):
        x, xp = _u64(x)
        ncoef = x.shape[-1]
        assert x.shape[0] == nlimbs + self.np_
        out = np.empty((nlimbs, ncoef), dtype=np.uint64)
        _check(lib().ref_moddown_coeff(self._h, out.ctypes.data_as(u64p), xp, C.c_uint32(nlimbs), C.c_uint32(ncoef)))
        return out

    # ---- the hot-path calls ----
    def keyswitch(self, d, evk, galois_elt=0):
        d, dp = _u64(d)
        evk, ep = _u64(evk)
        B, nl = d.shape[0], d.shape[1]
        assert evk.shape == (self.params.dnum, 2, self.nm, self.N)
        out = np.empty((B, 2, nl, self.N), dtype=np.uint64)
        _check(lib().ref_keyswitch(self._h, out.ctypes.data_as(u64p), dp, C.c_uint32(B), C.c_uint32(nl), ep,
                                   C.c_uint32(galois_elt), C.c_uint32(self.params.dnum)))
        return out

    def hrot(self, ct, g, evk):
        ct, cp = _u64(ct)
        evk, ep = _u64(evk)
        B, two, nl, _ = ct.shape
        assert two == 2 and evk.shape == (self.params.dnum, 2, self.nm, self.N)
        out = np.empty_like(ct)
        _check(lib().ref_hrot(self._h, out.ctypes.data_as(u64p), cp, C.c_uint32(B), C.c_uint32(nl), C.c_uint32(g), ep))
        return out

    def hmult_relin(self, ct_a, ct_b, evk):
        ct_a, ap = _u64(ct_a)
        ct_b, bp = _u64(ct_b)
        evk, ep = _u64(evk)
        B, two, nl, _ = ct_a.shape
        assert ct_b.shape == ct_a.shape and two == 2
        out = np.empty_like(ct_a)
        _check(lib().ref_hmult_relin(self._h, out.ctypes.data_as(u64p), ap, bp, C.c_uint32(B), C.c_uint32(nl), ep))
        return out

    def pcmm_bsgs_double_hoisted(self, ct, pt_ext, n1, n2, stride, evk_baby, evk_giant):
        """BSGS matmul with the baby steps kept in the extended basis; pt_ext [n2][n1][nlimbs + K][N]."""
        ct, cp = _u64(ct)
        pt_ext, pp = _u64(pt_ext)
        B, two, nl, _ = ct.shape
        assert pt_ext.shape == (n2, n1, nl + self.np_, self.N)
        assert len(evk_baby) == n1 - 1 and len(evk_giant) == n2 - 1
        keep = [_u64(k) for k in list(evk_baby) + list(evk_giant)]
        PA = u64p * max(1, n1 - 1)
        PG = u64p * max(1, n2 - 1)
        baby = PA(*[k[1] for k in keep[:n1 - 1]])
        giant = PG(*[k[1] for k in keep[n1 - 1:]])
        out = np.empty_like(ct)
        _check(lib().ref_pcmm_bsgs_double_hoisted(self._h, out.ctypes.data_as(u64p), cp, C.c_uint32(B), C.c_uint32(nl),
                                                  pp, C.c_uint32(n1), C.c_uint32(n2), C.c_uint32(stride), baby, giant))
        return out

    def hrot_sum(self, ct, galois_elts, evks):
        """ct + sum_r HRot_{g_r}(ct) with one ModDown for all rotations (hoisted rotate-and-sum)."""
        ct, cp = _u64(ct)
        B, two, nl, _ = ct.shape
        R = len(galois_elts)
        assert two == 2 and len(evks) == R
        keep = [_u64(k) for k in evks]
        PA = u64p * max(1, R)
        keys = PA(*[k[1] for k in keep])
        gs = (C.c_uint32 * max(1, R))(*[int(g) for g in galois_elts])
        out = np.empty_like(ct)
        _check(lib().ref_hrot_sum(self._h, out.ctypes.data_as(u64p), cp, C.c_uint32(B), C.c_uint32(nl), gs, keys,
                                  C.c_uint32(R)))
        return out

    def tensor_acc(self, ct_a, ct_b, d_acc=None):
        """Un-relinearised product [B][3][nl][N], added to d_acc when given (late relinearisation, Sec. 5.2)."""
        ct_a, ap = _u64(ct_a)
        ct_b, bp = _u64(ct_b)
        B, two, nl, _ = ct_a.shape
        assert ct_b.shape == ct_a.shape and two == 2
        out = np.empty((B, 3, nl, self.N), dtype=np.uint64)
        ep = None
        if d_acc is not None:
            d_acc, ep = _u64(d_acc)
            assert d_acc.shape == out.shape
        _check(lib().ref_tensor_acc(self._h, out.ctypes.data_as(u64p), ap, bp, ep, C.c_uint32(B), C.c_uint32(nl)))
        return out

    def relin(self, d, evk):
        d, dp = _u64(d)
        evk, ep = _u64(evk)
        B, three, nl, _ = d.shape
        assert three == 3 and evk.shape == (self.params.dnum, 2, self.nm, self.N)
        out = np.empty((B, 2, nl, self.N), dtype=np.uint64)
        _check(lib().ref_relin(self._h, out.ctypes.data_as(u64p), dp, C.c_uint32(B), C.c_uint32(nl), ep))
        return out

    def pcmm_bsgs(self, ct, pt, n1, n2, stride, evk_baby, evk_giant):
        ct, cp = _u64(ct)
        pt, pp = _u64(pt)
        B, two, nl, _ = ct.shape
        assert pt.shape == (n2, n1, nl, self.N)
        assert len(evk_baby) == n1 - 1 and len(evk_giant) == n2 - 1
        keep = [_u64(k) for k in list(evk_baby) + list(evk_giant)]
        PA = u64p * max(1, n1 - 1)
        PG = u64p * max(1, n2 - 1)
        baby = PA(*[k[1] for k in keep[:n1 - 1]])
        giant = PG(*[k[1] for k in keep[n1 - 1:]])
        out = np.empty_like(ct)
        _check(lib().ref_pcmm_bsgs(self._h, out.ctypes.data_as(u64p), cp, C.c_uint32(B), C.c_uint32(nl), pp,
                                   C.c_uint32(n1), C.c_uint32(n2), C.c_uint32(stride), baby, giant))
        return out

    def rescale(self, ct):
        ct, cp = _u64(ct)
        B, two, nl, _ = ct.shape
        out = np.empty((B, 2, nl - 1, self.N), dtype=np.uint64)
        _check(lib().ref_rescale(self._h, out.ctypes.data_as(u64p), cp, C.c_uint32(B), C.c_uint32(nl)))
        return out

    def pmult(self, ct, pt):
        """ct [B][2][nl][N] times plaintext pt [nl][N], pointwise per limb."""
        B, two, nl, N = ct.shape
        ids = list(range(nl))
        return self.pointwise(ct.reshape(B * 2, nl, N), np.asarray(pt).reshape(1, nl, N), ids, "mul").reshape(ct.shape)

    # ---- keys / encryption (semantic pins) ----
    def gen_evk(self, s, s_from, a_eval, e):
        """evk [dnum][2][nm][N] switching s_from -> s. a_eval [dnum][nm][N] uniform, e [dnum][N] signed."""
        s, sp = _i64(s)
        sf, sfp = _i64(s_from)
        a_eval, ap = _u64(a_eval)
        e, ep = _i64(e)
        d = self.params.dnum
        assert a_eval.shape == (d, self.nm, self.N) and e.shape == (d, self.N)
        evk = np.empty((d, 2, self.nm, self.N), dtype=np.uint64)
        _check(lib().ref_gen_evk(self._h, evk.ctypes.data_as(u64p), sp, sfp, ap, ep))
        return evk

    def encrypt(self, msg, s, a_eval, e, nlimbs):
        msg, mp = _i64(msg)
        s, sp = _i64(s)
        a_eval, ap = _u64(a_eval)
        e, ep = _i64(e)
        assert a_eval.shape == (nlimbs, self.N)
        ct = np.empty((2, nlimbs, self.N), dtype=np.uint64)
        _check(lib().ref_encrypt(self._h, ct.ctypes.data_as(u64p), mp, sp, ap, ep, C.c_uint32(nlimbs)))
        return ct

    def decrypt_rns(self, ct, s):
        ct, cp = _u64(ct)
        s, sp = _i64(s)
        ncomp, nl, _ = ct.shape
        out = np.empty((nl, self.N), dtype=np.uint64)
        _check(lib().ref_decrypt_rns(self._h, out.ctypes.data_as(u64p), cp, sp, C.c_uint32(nl), C.c_uint32(ncomp)))
        return out

    def decrypt_centred(self, ct, s):
        """Coefficients of c0 + c1*s as centred Python integers (list of N ints)."""
        r = self.decrypt_rns(ct, s)
        return crt_centred(r, self.moduli[:r.shape[0]])


# ---------------- exact integer helpers ----------------
def schoolbook(a, b, q):
    a, ap = _u64(a)
    b, bp = _u64(b)
    out = np.empty_like(a)
    _check(lib().ref_negacyclic_schoolbook(out.ctypes.data_as(u64p), ap, bp, C.c_uint32(len(a)), C.c_uint64(q)))
    return out


def negacyclic_signed(a, b):
    a, ap = _i64(a)
    b, bp = _i64(b)
    out = np.empty_like(a)
    _check(lib().ref_negacyclic_signed(out.ctypes.data_as(i64p), ap, bp, C.c_uint32(len(a))))
    return out


def automorph_signed(a, g):
    a, ap = _i64(a)
    out = np.empty_like(a)
    _check(lib().ref_automorph_signed(out.ctypes.data_as(i64p), ap, C.c_uint32(len(a)), C.c_uint32(g)))
    return out


def crt_centred(res, moduli):
    """res: uint64 [nlimbs][n] -> list of n centred Python ints in (-Q/2, Q/2]."""
    Q = 1
    for m in moduli:
        Q *= int(m)
    coef = []
    for m in moduli:
        h = Q // int(m)
        coef.append(h * pow(h % int(m), -1, int(m)))
    out = []
    cols = [r.tolist() for r in res]
    for k in range(res.shape[1]):
        v = 0
        for i in range(len(moduli)):
            v += cols[i][k] * coef[i]
        v %= Q
        if v > Q // 2:
            v -= Q
        out.append(v)
    return out


# ---------------- CKKS encode / decode ----------------
def _slot_exponents(N):
    """Slot i is the evaluation at zeta^(5^i), zeta = exp(i*pi/N)."""
    e = np.empty(N // 2, dtype=np.int64)
    x = 1
    for i in range(N // 2):
        e[i] = x
        x = x * 5 % (2 * N)
    return e


def encode(z, N, scale):
    """Real-coefficient polynomial m with m(zeta^(5^i)) ~ scale * z[i]; returns int64[N] (rounded)."""
    z = np.asarray(z, dtype=np.complex128)
    assert z.shape == (N // 2,)
    e = _slot_exponents(N)
    v = np.zeros(N, dtype=np.complex128)          # v[k] = value at zeta^(2k+1)
    v[(e - 1) // 2] = z
    v[(2 * N - e - 1) // 2] = np.conj(z)          # conjugate points make the coefficients real
    # m_j = zeta^-j / N * sum_k v[k] w^-jk,  w = zeta^2
    j = np.arange(N)
    m = np.fft.fft(v) / N * np.exp(-1j * np.pi * j / N)
    return np.rint(m.real * scale).astype(np.int64)


def decode(coeffs, N, scale):
    """coeffs: N numbers (Python ints allowed, any size) -> complex128[N/2] slot values."""
    c = np.array([float(x) / scale for x in coeffs], dtype=np.float64) if not isinstance(coeffs, np.ndarray) \
        else coeffs.astype(np.float64) / scale
    j = np.arange(N)
    # value at zeta^(2k+1) = sum_j c_j zeta^j w^(jk) = N * ifft(c_j zeta^j)[k]
    v = np.fft.ifft(c * np.exp(1j * np.pi * j / N)) * N
    return v[(_slot_exponents(N) - 1) // 2]


def decode_definition(coeffs, N, scale, slots):
    """O(N) per slot evaluation of the definition, for pinning decode()."""
    e = _slot_exponents(N)
    out = []
    for i in slots:
        x = np.exp(1j * np.pi * int(e[i]) * np.arange(N) / N)
        out.append(np.sum(np.array([float(c) for c in coeffs]) * x) / scale)
    return np.array(out)
