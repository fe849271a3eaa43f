"""Test-side helpers that assemble keys, ciphertexts and plaintexts from seeded arrays via the oracle."""
import numpy as np

from ckks_inputs import gaussian_error, galois_element, ternary_secret, uniform_residues
from oracle import ref


class Keys:
    def __init__(self, params, ctx, seed, hamming_weight=64):
        self.params, self.ctx, self.seed = params, ctx, seed
        self.s = ternary_secret(seed, params.N, min(hamming_weight, params.N // 2))
        self._n = 0

    def _next(self):
        self._n += 1
        return self.seed * 1000003 + self._n

    def evk_for(self, s_from):
        p = self.params
        a = uniform_residues(self._next(), p.moduli, (p.dnum,), p.N)
        e = gaussian_error(self._next(), (p.dnum, p.N))
        return self.ctx.gen_evk(self.s, s_from, a, e)

    def rotation_key(self, g):
        return self.evk_for(ref.automorph_signed(self.s, g))

    def relin_key(self):
        return self.evk_for(ref.negacyclic_signed(self.s, self.s))

    def encrypt_slots(self, z, scale, nlimbs):
        p = self.params
        msg = ref.encode(z, p.N, scale)
        a = uniform_residues(self._next(), p.q[:nlimbs], (), p.N)
        e = gaussian_error(self._next(), (p.N,))
        return self.ctx.encrypt(msg, self.s, a, e, nlimbs)

    def decrypt_slots(self, ct, scale):
        return ref.decode(self.ctx.decrypt_centred(ct, self.s), self.params.N, scale)


def encode_plain_eval(ctx, z, scale, nlimbs):
    """Plaintext polynomial for slot vector z, as eval-domain residues [nlimbs][N]."""
    msg = ref.encode(z, ctx.N, scale)
    ids = list(range(nlimbs))
    return ctx.ntt(ctx.signed_to_rns(msg, ids)[None], ids)[0]


def encode_plain_eval_ext(ctx, z, scale, nlimbs):
    """The same plaintext in the extended basis q_0..q_{nlimbs-1}, p_0..p_{K-1}: [nlimbs + K][N]."""
    msg = ref.encode(z, ctx.N, scale)
    ids = list(range(nlimbs)) + [len(ctx.params.q) + k for k in range(len(ctx.params.p))]
    return ctx.ntt(ctx.signed_to_rns(msg, ids)[None], ids)[0]
