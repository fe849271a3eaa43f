"""GPU parity on seeded random parameter sets: ring degree, number and size of the primes, dnum, level, batch and
Galois elements are drawn from a fixed seed; every call of the library is compared with the oracle, bit for bit."""
import random

import numpy as np
import pytest

from ckks_inputs import galois_element, make_params, uniform_residues
from oracle import ref

pytestmark = pytest.mark.gpu


def _draw(rng):
    logN = rng.choice([12, 12, 13, 16, 16])
    nq = rng.randint(2, 10 if logN < 16 else 6)
    dnum = rng.randint(1, min(nq, 6))
    alpha = -(-nq // dnum)
    K = rng.choice([alpha, max(1, alpha - 1), alpha + 1])
    qbits = rng.choice([45, 50, 50, 55, 60]) if logN == 16 else rng.choice([40, 45, 50, 55, 60])
    pbits = rng.choice([50, 55, 60, 60])
    return logN, nq, qbits, K, pbits, dnum


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_parameter_sets(seed):
    import torch
    import paper_2604_03425_amd as gpu
    from gpu_util import to_dev, to_host
    rng = random.Random(seed)
    ref.set_threads(4)
    for _ in range(5):
        shape = _draw(rng)
        p = make_params(*shape)
        nl, B = rng.randint(1, len(p.q)), rng.randint(1, 3)
        s = rng.randrange(1 << 30)
        g, g2 = (galois_element(rng.randrange(1, p.N // 2), p.logN) for _ in range(2))
        tag = "shape=%s nl=%d B=%d seed=%d g=%d" % (shape, nl, B, s, g)
        rc, gc = ref.RefContext(p), gpu.Context(p)
        ct = uniform_residues(s, p.q[:nl], (B, 2), p.N)
        ct2 = uniform_residues(s + 1, p.q[:nl], (B, 2), p.N)
        evk = uniform_residues(s + 2, p.moduli, (p.dnum, 2), p.N)
        evk2 = uniform_residues(s + 3, p.moduli, (p.dnum, 2), p.N)
        d_ct, d_ct2, d_evk, d_evk2 = to_dev(ct), to_dev(ct2), to_dev(evk), to_dev(evk2)
        ws = gc.workspace(gpu.OP_HROT, B, nl)
        out = torch.empty_like(d_ct)

        def same(got, want, what):
            assert (to_host(got) == want).all(), "%s differs: %s" % (what, tag)
        rot = rc.hrot(ct, g, evk)
        gpu.ckks_hrot(gc, out, d_ct, B, nl, g, d_evk, ws)
        same(out, rot, "hrot")
        gpu.ckks_hrot_add(gc, out, d_ct, d_ct2, B, nl, g, d_evk, ws)
        same(out, rc.pointwise(ct2, rot, list(range(nl)), "add"), "hrot_add")
        gs = [g if b % 2 == 0 else g2 for b in range(B)]
        multi = np.concatenate([rc.hrot(ct[b:b + 1], gs[b], evk if b % 2 == 0 else evk2) for b in range(B)])
        gpu.ckks_hrot_multi(gc, out, d_ct, B, nl, gs, [d_evk if b % 2 == 0 else d_evk2 for b in range(B)], ws)
        same(out, multi, "hrot_multi")
        gpu.ckks_hmult_relin(gc, out, d_ct, d_ct2, B, nl, d_evk, ws)
        same(out, rc.hmult_relin(ct, ct2, evk), "hmult_relin")
        d3 = torch.empty((B, 3, nl, p.N), dtype=torch.int64, device="cuda")
        gpu.ckks_tensor_acc(gc, d3, d_ct, d_ct2, None, B, nl)
        gpu.ckks_tensor_acc(gc, d3, d_ct2, d_ct2, d3, B, nl)
        want3 = rc.tensor_acc(ct2, ct2, rc.tensor_acc(ct, ct2))
        same(d3, want3, "tensor_acc")
        gpu.ckks_relin(gc, out, d3, B, nl, d_evk2, ws)
        same(out, rc.relin(want3, evk2), "relin")
        if p.logN == 16:
            R = rng.randint(0, 4)
            sg = [galois_element(rng.randrange(1, p.N // 2), p.logN) for _ in range(R)]
            sk = [evk if r % 2 == 0 else evk2 for r in range(R)]
            gpu.ckks_hrot_sum(gc, out, d_ct, B, nl, sg, [d_evk if r % 2 == 0 else d_evk2 for r in range(R)],
                              gc.workspace(gpu.OP_HROT_SUM, B, nl))
            same(out, rc.hrot_sum(ct, sg, sk), "hrot_sum R=%d" % R)
        if nl >= 2:
            rs = torch.empty((B, 2, nl - 1, p.N), dtype=torch.int64, device="cuda")
            gpu.ckks_rescale(gc, rs, d_ct, B, nl, gc.workspace(gpu.OP_RESCALE, B, nl))
            same(rs, rc.rescale(ct), "rescale")
        n1, n2 = rng.randint(1, 4), rng.randint(1, 7)
        pt = uniform_residues(s + 5, p.q[:nl], (n2, n1), p.N)
        want = rc.pcmm_bsgs(ct, pt, n1, n2, 1, [evk] * (n1 - 1), [evk2] * (n2 - 1))
        wsp = gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1)
        d_pt = to_dev(pt)
        gpu.ckks_pcmm_bsgs(gc, out, d_ct, B, nl, d_pt, n1, n2, 1, [d_evk] * (n1 - 1), [d_evk2] * (n2 - 1), wsp)
        same(out, want, "pcmm_bsgs")
        gpu.ckks_pcmm_bsgs_hoisted(gc, out, d_ct, B, nl, d_pt, n1, n2, 1, [d_evk] * (n1 - 1), [d_evk2] * (n2 - 1), wsp)
        same(out, want, "pcmm_bsgs_hoisted")
        gc.close()
    ref.set_threads(1)
