"""Call sequences of the attention workloads, written once against a small adapter so that the oracle and the
C-ABI library are driven by the same sequence of calls (the adapter holds no arithmetic, only marshalling).

Packing (token-major, `hd` slots per token, T = S/hd tokens per ciphertext): slot hd*t + j holds component j of
token t. The r-th unit of a (query block, key block) pair works on the key/value ciphertext rotated left by r
tokens, so it produces the r-th cyclic diagonal of the score block (Sec. 4.3: rotate-multiply-accumulate over
local score slices; the aggregation with V is local).
"""
import numpy as np

from ckks_inputs import galois_element


class RefOps:
    """Adapter over oracle.ref.RefContext (numpy arrays)."""

    def __init__(self, ctx):
        self.c = ctx

    def hmult(self, a, b, relin):
        return self.c.hmult_relin(a, b, relin)

    def hrot(self, a, g, key):
        return self.c.hrot(a, g, key)

    def add(self, a, b):
        return self.c.pointwise(a, b, list(range(a.shape[2])), "add")

    def hrot_add(self, a, add, g, key):
        """add + HRot_g(a): by definition the rotation followed by the addition."""
        return self.add(add, self.c.hrot(a, g, key))

    def tensor_acc(self, a, b, acc):
        return self.c.tensor_acc(a, b, acc)

    def hrot_sum(self, a, gs, keys):
        return self.c.hrot_sum(a, gs, keys)

    def relin(self, d, relin):
        return self.c.relin(d, relin)

    def rescale(self, a):
        return self.c.rescale(a)

    def pmult(self, a, pt):
        return self.c.pmult(a, pt)

    def drop_to(self, a, nl):
        return np.ascontiguousarray(a[:, :, :nl])


class GpuOps:
    """Adapter over the C-ABI binding (torch int64 device tensors)."""

    def __init__(self, mod, ctx, batch, max_limbs):
        self.m, self.c = mod, ctx
        self.ws = ctx.workspace(mod.OP_HROT, batch, max_limbs)

    def _new(self, like, nl=None):
        import torch
        B, two, n, N = like.shape
        return torch.empty((B, two, nl or n, N), dtype=like.dtype, device=like.device)

    def hmult(self, a, b, relin):
        out = self._new(a)
        self.m.ckks_hmult_relin(self.c, out, a, b, a.shape[0], a.shape[2], relin, self.ws)
        return out

    def hrot(self, a, g, key):
        out = self._new(a)
        self.m.ckks_hrot(self.c, out, a, a.shape[0], a.shape[2], g, key, self.ws)
        return out

    def add(self, a, b):
        out = self._new(a)
        self.m.ckks_add(self.c, out, a, b, a.shape[0] * 2, a.shape[2])
        return out

    def hrot_add(self, a, add, g, key):
        out = self._new(a)
        self.m.ckks_hrot_add(self.c, out, a, add, a.shape[0], a.shape[2], g, key, self.ws)
        return out

    def hrot_sum(self, a, gs, keys):
        out = self._new(a)
        B, n = a.shape[0], a.shape[2]
        self.m.ckks_hrot_sum(self.c, out, a, B, n, gs, keys, self.c.workspace(self.m.OP_HROT_SUM, B, n))
        return out

    def tensor_acc(self, a, b, acc):
        """Accumulates in place when acc is given."""
        import torch
        B, _, n, N = a.shape
        out = acc if acc is not None else torch.empty((B, 3, n, N), dtype=a.dtype, device=a.device)
        self.m.ckks_tensor_acc(self.c, out, a, b, acc, B, n)
        return out

    def relin(self, d, relin):
        import torch
        B, _, n, N = d.shape
        out = torch.empty((B, 2, n, N), dtype=d.dtype, device=d.device)
        self.m.ckks_relin(self.c, out, d, B, n, relin, self.ws)
        return out

    def rescale(self, a):
        out = self._new(a, a.shape[2] - 1)
        self.m.ckks_rescale(self.c, out, a, a.shape[0], a.shape[2], self.ws)
        return out

    def pmult(self, a, pt):
        out = self._new(a)
        self.m.ckks_pmult(self.c, out, a, pt, a.shape[0], a.shape[2])
        return out

    def drop_to(self, a, nl):
        return a[:, :, :nl].contiguous()


def score_diagonal(ops, logN, q_ct, k_rot, relin, sum_keys, hd):
    """QK^T unit: HMult+relin, then rotate-and-sum over the hd slots of a token. Slot hd*t of the result holds
    <q_t, k_{t+r}> (scale Delta^2); the other slots hold partial sums."""
    d = ops.hmult(q_ct, k_rot, relin)
    for i in range(hd.bit_length() - 1):
        d = ops.hrot_add(d, d, galois_element(1 << i, logN), sum_keys[i])
    return d


def mask_and_pack(ops, logN, d, mask_pt, rep_keys, hd):
    """Keeps slot hd*t of every token (PMult by a 0/1 mask, then Rescale) and replicates it over the token's hd
    slots by rotations to the right by 1, 2, 4, ...; mask_pt is at one limb fewer than d."""
    m = ops.rescale(ops.pmult(ops.rescale(d), mask_pt))
    for i in range(hd.bit_length() - 1):
        m = ops.hrot_add(m, m, galois_element(-(1 << i), logN), rep_keys[i])
    return m


def av_unit(ops, logN, q_ct, k_rot, v_rot, relin, sum_keys, mask_pt, rep_keys, hd):
    """One unit of A x V on raw scores: diagonal r of the score block, packed, times V rotated by the same r
    tokens. Summing the units over r (and over key blocks) gives rows of (Q K^T) V. v_rot is at two limbs fewer
    than q_ct."""
    a = mask_and_pack(ops, logN, score_diagonal(ops, logN, q_ct, k_rot, relin, sum_keys, hd), mask_pt, rep_keys, hd)
    return ops.hmult(a, v_rot, relin)


def av_unit_late(ops, logN, q_ct, k_rot, v_rot, relin, sum_keys, mask_pt, rep_keys, hd, acc):
    """av_unit with late relinearisation (Sec. 5.2): the product with V stays in three components and is added to
    acc (None for the first unit); one ops.relin after the last unit of the block replaces a key switch per unit."""
    a = mask_and_pack(ops, logN, score_diagonal(ops, logN, q_ct, k_rot, relin, sum_keys, hd), mask_pt, rep_keys, hd)
    return ops.tensor_acc(a, v_rot, acc)


def sum_steps(hd):
    """Steps of a two-level sum over hd = a * b consecutive slots: (1 .. a-1) and (a, 2a, .. (b-1)a)."""
    bits = hd.bit_length() - 1
    a = 1 << (bits - bits // 2)
    return list(range(1, a)), [a * j for j in range(1, hd // a)]


def score_diagonal_hoisted(ops, logN, q_ct, k_rot, relin, inner_keys, outer_keys, hd):
    """The QK^T unit with the rotate-and-sum over the hd slots of a token done as two hoisted sums (the ciphertext
    plus its rotations by 1..a-1, then that plus its rotations by a, 2a, ..): two decompositions and two ModDowns
    instead of log2(hd) key switches. Same slot sums as score_diagonal, other rounding."""
    d = ops.hmult(q_ct, k_rot, relin)
    inner, outer = sum_steps(hd)
    d = ops.hrot_sum(d, [galois_element(k, logN) for k in inner], inner_keys)
    return ops.hrot_sum(d, [galois_element(k, logN) for k in outer], outer_keys)


def av_unit_hoisted(ops, logN, q_ct, k_rot, v_rot, relin, keys, mask_pt, hd, acc):
    """av_unit_late with every slot sum done as two hoisted sums: the score diagonal through score_diagonal_hoisted,
    the replication over a token's slots as the same two sums with right rotations. keys = (inner, outer, inner_right,
    outer_right) lists of rotation keys for sum_steps(hd) and their negatives. Four decompositions and four ModDowns
    replace 2 log2(hd) key switches; the product with V stays in three components (acc, None for the first unit)."""
    inner, outer = sum_steps(hd)
    d = score_diagonal_hoisted(ops, logN, q_ct, k_rot, relin, keys[0], keys[1], hd)
    m = ops.rescale(ops.pmult(ops.rescale(d), mask_pt))
    m = ops.hrot_sum(m, [galois_element(-k, logN) for k in inner], keys[2])
    m = ops.hrot_sum(m, [galois_element(-k, logN) for k in outer], keys[3])
    return ops.tensor_acc(m, v_rot, acc)
