"""GPU parity at the shapes of the remaining workloads: BSGS PCMM with 32x24 diagonals, the attention
QK^T unit (HMult+relin followed by log2(64) rotate-and-sum steps), and points of the level/dnum sweep."""
import numpy as np
import pytest

from ckks_inputs import config_params, galois_element, make_params, uniform_residues, uniform_slots, normal_slots
from oracle import ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2604_03425_amd as pkg
    return pkg


def test_pcmm_768_diagonals_small_ring(gpu):
    """FFN-layer packing (x||x||0 per 2048-slot segment, 768x768 weight slice, baby 32 x giant 24) on the
    N=2^12 ring: one token per ciphertext. Bit-exact against the oracle, and the decrypted result is x W."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    from harness import Keys, encode_plain_eval
    p = make_params(12, 4, 40, 2, 50, 2)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    keys = Keys(p, rc, 71)
    dim, n1, n2, nl, B = 768, 32, 24, 4, 2
    S = p.N // 2
    rng = np.random.default_rng(3)
    X = rng.uniform(-1, 1, (B, dim))
    W = rng.normal(0, 0.02, (dim, dim))
    cts = []
    for b in range(B):
        z = np.zeros(S)
        z[:dim] = X[b]
        z[dim:2 * dim] = X[b]
        cts.append(keys.encrypt_slots(z, 2.0**30, nl))
    ct = np.stack(cts)
    pts = np.empty((n2, n1, nl, p.N), dtype=np.uint64)
    jj = np.arange(dim)
    for g in range(n2):
        for b in range(n1):
            dvec = np.zeros(S)
            dvec[jj + g * n1] = W[(jj + g * n1 + b) % dim, jj]
            pts[g, b] = encode_plain_eval(rc, dvec, 2.0**30, nl)
    baby = [keys.rotation_key(galois_element(b, p.logN)) for b in range(1, n1)]
    giant = [keys.rotation_key(galois_element(g * n1, p.logN)) for g in range(1, n2)]
    ref.set_threads(2)
    want = rc.pcmm_bsgs(ct, pts, n1, n2, 1, baby, giant)
    ref.set_threads(1)
    out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_pcmm_bsgs(gc, out, to_dev(ct), B, nl, to_dev(pts), n1, n2, 1, [to_dev(k) for k in baby],
                       [to_dev(k) for k in giant], gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
    got = to_host(out)
    assert_same(got, want, "pcmm 32x24")
    Y = X @ W
    for b in range(B):
        y = keys.decrypt_slots(got[b], 2.0**60).real
        assert np.max(np.abs(y[:dim] - Y[b])) < 2.0**-12     # slots beyond 768 hold partial sums, not results


def test_pcmm_full_ring_small_bsgs(gpu):
    """N=2^16, 24 limbs, dnum=3: PCMM with 3 baby and 2 giant steps, bit-exact."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")
    rc, gc = ref.RefContext(p), gpu.Context(p)
    B, nl, n1, n2 = 2, 24, 3, 2
    ct = uniform_residues(81, p.q, (B, 2), p.N)
    pt = uniform_residues(82, p.q, (n2, n1), p.N)
    baby = [uniform_residues(83 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n1 - 1)]
    giant = [uniform_residues(93 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n2 - 1)]
    ref.set_threads(2)
    want = rc.pcmm_bsgs(ct, pt, n1, n2, 1, baby, giant)
    ref.set_threads(1)
    out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_pcmm_bsgs(gc, out, to_dev(ct), B, nl, to_dev(pt), n1, n2, 1, [to_dev(k) for k in baby],
                       [to_dev(k) for k in giant], gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
    assert_same(to_host(out), want, "pcmm N=2^16")


@pytest.mark.timeout(600)
def test_pcmm_ffn_share_real_shape_against_oracle_digests(gpu):
    """The FFN-layer workload at its real shape: N=2^16, 24 limbs, dnum=3, 32 baby x 24 giant steps, a batch of 8.
    SHA-256 of every output ciphertext equals the digest the oracle wrote (tests/golden/pcmm_ffn_digests.txt, made
    by make_pcmm_ffn_digests.py from the same seeded inputs), for the one-rotation-at-a-time schedule and for the
    hoisted one, which is bit-identical by definition. This is the shape at which the N=2^16 schedule runs whole
    tiles of 24 giant steps (6-giant-step launches of the double-precision inner sums, 3-giant-step integer ones),
    accumulates the giant steps in place, and packs the hoisted baby steps' accumulators into the inner-sum region."""
    import hashlib
    import importlib.util
    import os
    import torch
    from gpu_util import to_dev, to_host
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("_pcmm_ffn_inputs", os.path.join(here, "golden", "make_pcmm_ffn_digests.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    want = {}
    with open(os.path.join(here, "golden", "pcmm_ffn_digests.txt")) as f:
        for line in f:
            if line.startswith("pcmm "):
                _, b, h = line.split()
                want[int(b)] = h
    B, n1, n2, nl = mk.B, mk.N1, mk.N2, 24
    assert sorted(want) == list(range(B))
    p = config_params("keyswitch_micro")
    gc = gpu.Context(p)
    ct, pt, baby, giant = mk.inputs(p)
    d_ct, d_pt = to_dev(ct), to_dev(pt)
    del pt
    d_baby, d_giant = [to_dev(k) for k in baby], [to_dev(k) for k in giant]
    del baby, giant
    ws = gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1)
    for name, fn in (("plain", gpu.ckks_pcmm_bsgs), ("hoisted", gpu.ckks_pcmm_bsgs_hoisted)):
        out = torch.zeros((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
        fn(gc, out, d_ct, B, nl, d_pt, n1, n2, 1, d_baby, d_giant, ws)
        got = to_host(out)
        bad = [b for b in range(B) if hashlib.sha256(np.ascontiguousarray(got[b]).tobytes()).hexdigest() != want[b]]
        assert not bad, "%s schedule: ciphertexts %s differ from the oracle's digests" % (name, bad)
    gc.close()


def test_attention_unit_full_ring(gpu):
    """N=2^16, 20 limbs, dnum=4, 5 special primes: one QK^T unit = HMult+relin, then rotate-and-sum by
    1,2,4,...,32 (six HRot + add steps)."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("attention_qk")
    rc, gc = ref.RefContext(p), gpu.Context(p)
    B, nl = 2, 20
    qa = uniform_residues(91, p.q, (B, 2), p.N)
    kb = uniform_residues(92, p.q, (B, 2), p.N)
    relin = uniform_residues(93, p.moduli, (p.dnum, 2), p.N)
    rot = [uniform_residues(100 + i, p.moduli, (p.dnum, 2), p.N) for i in range(6)]
    ids = list(range(nl))
    ref.set_threads(2)
    want = rc.hmult_relin(qa, kb, relin)
    for i in range(6):
        r = rc.hrot(want, galois_element(1 << i, p.logN), rot[i])
        want = rc.pointwise(want, r, ids, "add")
    ref.set_threads(1)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    acc = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    tmp = torch.empty_like(acc)
    gpu.ckks_hmult_relin(gc, acc, to_dev(qa), to_dev(kb), B, nl, to_dev(relin), ws)
    mods = torch.tensor(np.array(p.q, dtype=np.int64), device="cuda").view(1, 1, nl, 1)
    for i in range(6):
        gpu.ckks_hrot(gc, tmp, acc, B, nl, galois_element(1 << i, p.logN), to_dev(rot[i]), ws)
        s = acc + tmp                      # residues < 2^50: no int64 overflow; test-side modular add
        acc = torch.where(s >= mods, s - mods, s)
    assert_same(to_host(acc), want, "attention unit")
    # the unit with the sum over a token's 64 slots as two hoisted sums (flows.score_diagonal_hoisted)
    from flows import GpuOps, RefOps, score_diagonal_hoisted, sum_steps
    inner, outer = sum_steps(64)
    ik = [uniform_residues(120 + i, p.moduli, (p.dnum, 2), p.N) for i in range(len(inner))]
    ok = [uniform_residues(140 + i, p.moduli, (p.dnum, 2), p.N) for i in range(len(outer))]
    ref.set_threads(4)
    want_h = score_diagonal_hoisted(RefOps(rc), p.logN, qa, kb, relin, ik, ok, 64)
    ref.set_threads(1)
    got_h = score_diagonal_hoisted(GpuOps(gpu, gc, B, nl), p.logN, to_dev(qa), to_dev(kb), to_dev(relin),
                                   [to_dev(k) for k in ik], [to_dev(k) for k in ok], 64)
    assert_same(to_host(got_h), want_h, "attention unit, hoisted sums")


SWEEP = [
    # limbs, dnum  (alpha = K = ceil(limbs/dnum))
    (4, 3),      # ragged: digits 2,2 (beta = 2 < dnum)
    (12, 6),
    (36, 6),
    (36, 1),     # one 36-limb digit, 36 special primes
    (20, 3),     # ragged: 7,7,6
]


@pytest.mark.parametrize("limbs,dnum", SWEEP)
def test_sweep_point_keyswitch(gpu, limbs, dnum):
    import torch
    from gpu_util import to_dev, to_host, assert_same
    K = -(-limbs // dnum)
    p = make_params(16, limbs, 50, K, 60, dnum)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    B = 1
    d = uniform_residues(limbs * 10 + dnum, p.q, (B,), p.N)
    evk = uniform_residues(limbs * 10 + dnum + 1, p.moduli, (p.dnum, 2), p.N)
    want = rc.keyswitch(d, evk)
    out = torch.empty((B, 2, limbs, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_keyswitch(gc, out, to_dev(d), B, limbs, to_dev(evk), 0, dnum, gc.workspace(gpu.OP_KEYSWITCH, B, limbs))
    assert_same(to_host(out), want, "sweep point %d limbs dnum %d" % (limbs, dnum))
    gc.close()


def test_paper_parameter_shape_keyswitch(gpu):
    """The paper's own parameter set as an extra point (Sec. 5.1, Encryption Parameters: N = 2^16, 35 primes in Q and
    4 special primes, 1661 bits in all): here 35 x 42-bit + 4 x 48-bit primes (1662 bits), 9 digits of 4 limbs with the
    last one short (3 limbs). Key switch and HRot at the top level and at 14 limbs (the level left after bootstrapping
    in the paper's schedule), bit-exact."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(16, 35, 42, 4, 48, 9)
    assert p.alpha == 4
    rc, gc = ref.RefContext(p), gpu.Context(p)
    evk = uniform_residues(902, p.moduli, (p.dnum, 2), p.N)
    d_evk = to_dev(evk)
    for nl in (35, 14):
        ct = uniform_residues(900 + nl, p.q[:nl], (1, 2), p.N)
        g = galois_element(321, p.logN)
        out = torch.empty((1, 2, nl, p.N), dtype=torch.int64, device="cuda")
        gpu.ckks_hrot(gc, out, to_dev(ct), 1, nl, g, d_evk, gc.workspace(gpu.OP_HROT, 1, nl))
        assert_same(to_host(out), rc.hrot(ct, g, evk), "paper-shape HRot at %d limbs" % nl)
    gc.close()


@pytest.mark.parametrize("shape,nlimbs,B", [((12, 4, 40, 1, 50, 2), 4, 3), ((12, 5, 50, 2, 60, 2), 3, 2),
                                            ((16, 6, 50, 2, 60, 2), 6, 2), ((16, 3, 60, 1, 60, 1), 3, 1)])
def test_rescale_pmult_add(gpu, shape, nlimbs, B):
    """Rescale (incl. 60-bit main primes on the integer bodies), PMult and Add, bit-exact."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    ct = uniform_residues(71, p.q[:nlimbs], (B, 2), p.N)
    pt = uniform_residues(72, p.q[:nlimbs], (), p.N)
    ids = list(range(nlimbs))
    d_ct = to_dev(ct)
    prod = torch.empty_like(d_ct)
    gpu.ckks_pmult(gc, prod, d_ct, to_dev(pt), B, nlimbs)
    want_prod = rc.pmult(ct, pt)
    assert_same(to_host(prod), want_prod, "pmult")
    s = torch.empty_like(d_ct)
    gpu.ckks_add(gc, s, prod, d_ct, B * 2, nlimbs)
    want_sum = rc.pointwise(want_prod.reshape(B * 2, nlimbs, p.N), ct.reshape(B * 2, nlimbs, p.N), ids, "add").reshape(ct.shape)
    assert_same(to_host(s), want_sum, "add")
    out = torch.empty((B, 2, nlimbs - 1, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_rescale(gc, out, s, B, nlimbs, gc.workspace(gpu.OP_RESCALE, B, nlimbs))
    assert_same(to_host(out), rc.rescale(want_sum), "rescale")
    gc.close()


def test_hoisted_rotations_are_bit_identical(gpu):
    """N=2^16, 24 limbs, dnum=3: three rotations of one batch with shared decomposition equal three HRots."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")
    rc, gc = ref.RefContext(p), gpu.Context(p)
    B, nl = 2, 24
    ct = uniform_residues(301, p.q, (B, 2), p.N)
    gs = [galois_element(k, p.logN) for k in (1, 7, 31000)]
    evks = [uniform_residues(310 + i, p.moduli, (p.dnum, 2), p.N) for i in range(3)]
    out = torch.empty((3, B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hrot_hoisted(gc, out, to_dev(ct), B, nl, gs, [to_dev(k) for k in evks], gc.workspace(gpu.OP_HROT, B, nl))
    got = to_host(out)
    ref.set_threads(2)
    for r in range(3):
        assert_same(got[r], rc.hrot(ct, gs[r], evks[r]), "hoisted rotation %d" % r)
    ref.set_threads(1)
    # a workspace with room for two more accumulator pairs: rotations share passes over the digits, two at a time
    # (one pass of two, one of one); same bits
    need = gpu.ckks_workspace_bytes(gc, gpu.OP_HROT, B, nl, 0)
    one = B * 2 * (nl + len(p.p)) * p.N * 8
    big = torch.empty((need + 2 * one + 8) // 8, dtype=torch.int64, device="cuda")
    out2 = torch.empty_like(out)
    gpu.ckks_hrot_hoisted(gc, out2, to_dev(ct), B, nl, gs, [to_dev(k) for k in evks], big)
    assert torch.equal(out2, out)
    gc.close()


def test_pcmm_hoisted_matches_oracle(gpu):
    """Hoisted baby steps: N=2^16 (shared decomposition) and N=2^12 (falls back to single rotations)."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    for shape, B, nl, n1, n2 in (((16, 6, 50, 2, 60, 3), 2, 6, 4, 2), ((12, 4, 40, 2, 50, 2), 2, 4, 3, 3)):
        p = make_params(*shape)
        rc, gc = ref.RefContext(p), gpu.Context(p)
        ct = uniform_residues(401, p.q, (B, 2), p.N)
        pt = uniform_residues(402, p.q, (n2, n1), p.N)
        baby = [uniform_residues(410 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n1 - 1)]
        giant = [uniform_residues(420 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n2 - 1)]
        ref.set_threads(2)
        want = rc.pcmm_bsgs(ct, pt, n1, n2, 2, baby, giant)
        ref.set_threads(1)
        out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
        gpu.ckks_pcmm_bsgs_hoisted(gc, out, to_dev(ct), B, nl, to_dev(pt), n1, n2, 2, [to_dev(k) for k in baby],
                                   [to_dev(k) for k in giant], gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
        assert_same(to_host(out), want, "hoisted pcmm logN=%d" % shape[0])
        gc.close()


def _av_inputs(p, B, nl, hd, seed):
    """Uniform-residue stand-ins for Q, K (nl limbs), V (nl - 2 limbs), the mask plaintext (nl - 1 limbs) and keys."""
    q_ct = uniform_residues(seed, p.q[:nl], (B, 2), p.N)
    k_ct = uniform_residues(seed + 1, p.q[:nl], (B, 2), p.N)
    v_ct = uniform_residues(seed + 2, p.q[:nl - 2], (B, 2), p.N)
    mask = uniform_residues(seed + 3, p.q[:nl - 1], (), p.N)
    nk = hd.bit_length() - 1
    key = lambda i: uniform_residues(seed + 10 + i, p.moduli, (p.dnum, 2), p.N)
    return q_ct, k_ct, v_ct, mask, key(0), [key(1 + i) for i in range(nk)], [key(20 + i) for i in range(nk)]


@pytest.mark.parametrize("name,nl,B,hd", [("tiny_hrot_k2", 4, 3, 8), ((16, 8, 50, 2, 60, 4), 8, 2, 8)])
def test_attention_av_unit(gpu, name, nl, B, hd):
    """Second attention workload: score diagonal, mask-and-pack (PMult, two Rescales, replication by right
    rotations) and the product with V, as one sequence of C-ABI calls against the same sequence on the oracle."""
    from flows import GpuOps, RefOps, av_unit
    from gpu_util import to_dev, to_host, assert_same
    p = config_params(name) if isinstance(name, str) else make_params(*name)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    q_ct, k_ct, v_ct, mask, relin, sum_keys, rep_keys = _av_inputs(p, B, nl, hd, 300)
    ref.set_threads(4)
    want = av_unit(RefOps(rc), p.logN, q_ct, k_ct, v_ct, relin, sum_keys, mask, rep_keys, hd)
    ref.set_threads(1)
    got = av_unit(GpuOps(gpu, gc, B, nl), p.logN, to_dev(q_ct), to_dev(k_ct), to_dev(v_ct), to_dev(relin),
                  [to_dev(k) for k in sum_keys], to_dev(mask), [to_dev(k) for k in rep_keys], hd)
    assert got.shape == (B, 2, nl - 2, p.N)
    assert_same(to_host(got), want, "attention A x V unit")
    # late relinearisation: two units accumulated in three components (here the same unit twice), one key switch
    from flows import av_unit_late
    rops, gops = RefOps(rc), GpuOps(gpu, gc, B, nl)
    dev = (to_dev(q_ct), to_dev(k_ct), to_dev(v_ct), to_dev(relin), [to_dev(k) for k in sum_keys], to_dev(mask),
           [to_dev(k) for k in rep_keys])
    ref.set_threads(4)
    w = g = None
    for _ in range(2):
        w = av_unit_late(rops, p.logN, q_ct, k_ct, v_ct, relin, sum_keys, mask, rep_keys, hd, w)
        g = av_unit_late(gops, p.logN, *dev, hd, g)
    want_late = rops.relin(w, relin)
    ref.set_threads(1)
    assert_same(to_host(g), w, "A x V units in three components")
    assert_same(to_host(gops.relin(g, dev[3])), want_late, "A x V block relinearised late")
    if p.logN == 16:
        # every slot sum as two hoisted sums (ckks_hrot_sum), products kept in three components
        from flows import av_unit_hoisted, sum_steps
        inner, outer = sum_steps(hd)
        key = lambda i: uniform_residues(700 + i, p.moduli, (p.dnum, 2), p.N)
        hk = ([key(i) for i in range(len(inner))], [key(10 + i) for i in range(len(outer))],
              [key(20 + i) for i in range(len(inner))], [key(30 + i) for i in range(len(outer))])
        dhk = tuple([to_dev(k) for k in ks] for ks in hk)
        ref.set_threads(4)
        wh = av_unit_hoisted(rops, p.logN, q_ct, k_ct, v_ct, relin, hk, mask, hd, None)
        ref.set_threads(1)
        gh = av_unit_hoisted(gops, p.logN, dev[0], dev[1], dev[2], dev[3], dhk, dev[5], hd, None)
        assert_same(to_host(gh), wh, "A x V unit with hoisted sums")


@pytest.mark.parametrize("name,nl,B", [("tiny_hrot", 4, 8), ("keyswitch_micro", 24, 3),
                                       ((16, 2, 50, 1, 60, 2), 2, 67)])   # more than 64: two launch sequences
def test_hrot_multi_matches_single_rotations(gpu, name, nl, B):
    """One Galois element and key per ciphertext in one call = the oracle's HRot of each ciphertext on its own
    (the tiny configuration's "each rotated by a seeded step"; the micro-benchmark's seeded Galois elements)."""
    import torch
    from ckks_inputs import seeded_rotation_steps
    from gpu_util import to_dev, to_host, assert_same
    p = config_params(name) if isinstance(name, str) else make_params(*name)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    ct = uniform_residues(400, p.q[:nl], (B, 2), p.N)
    steps = seeded_rotation_steps(401, B, 1, p.N // 2 - 1)
    gs = [galois_element(k, p.logN) for k in steps]
    nkeys = min(9, max(2, B - 1))             # fewer keys than ciphertexts: pointers repeat
    keys = [uniform_residues(410 + i, p.moduli, (p.dnum, 2), p.N) for i in range(nkeys)]
    kidx = [i % nkeys for i in range(B)]
    ref.set_threads(4)
    want = np.concatenate([rc.hrot(ct[b:b + 1], gs[b], keys[kidx[b]]) for b in range(B)])
    ref.set_threads(1)
    dkeys = [to_dev(k) for k in keys]
    out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hrot_multi(gc, out, to_dev(ct), B, nl, gs, [dkeys[i] for i in kidx], gc.workspace(gpu.OP_HROT, B, nl))
    assert_same(to_host(out), want, "hrot_multi")
    gc.close()


def test_one_context_serves_calls_on_several_streams(gpu):
    """Single-ciphertext rotations and products issued round-robin on four streams (a workspace each, one context)
    while all of them are in flight: every result equals the oracle's. The context holds only constants once it is
    created, so calls on different streams share nothing they write."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(16, 6, 50, 2, 60, 3)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    nl, B = 6, 8
    ct = uniform_residues(900, p.q[:nl], (B, 2), p.N)
    keys = [uniform_residues(910 + i, p.moduli, (p.dnum, 2), p.N) for i in range(2)]
    gs = [galois_element(3 + 5 * b, p.logN) for b in range(B)]
    ref.set_threads(4)
    want_rot = np.concatenate([rc.hrot(ct[b:b + 1], gs[b], keys[b % 2]) for b in range(B)])
    want_mul = np.concatenate([rc.hmult_relin(ct[b:b + 1], ct[(b + 1) % B:(b + 1) % B + 1], keys[b % 2]) for b in range(B)])
    ref.set_threads(1)
    d_ct, dkeys = to_dev(ct), [to_dev(k) for k in keys]
    d_next = torch.roll(d_ct, -1, 0).contiguous()
    out_rot, out_mul = torch.empty_like(d_ct), torch.empty_like(d_ct)
    streams = [torch.cuda.Stream() for _ in range(4)]
    wss = [gc.workspace(gpu.OP_HROT, 1, nl) for _ in range(4)]
    cur = torch.cuda.current_stream()
    for rep in range(2):
        for s_ in streams:
            s_.wait_stream(cur)
        for b in range(B):
            with torch.cuda.stream(streams[b % 4]):
                gpu.ckks_hrot(gc, out_rot[b:b + 1], d_ct[b:b + 1], 1, nl, gs[b], dkeys[b % 2], wss[b % 4])
                gpu.ckks_hmult_relin(gc, out_mul[b:b + 1], d_ct[b:b + 1], d_next[b:b + 1], 1, nl, dkeys[b % 2], wss[b % 4])
        for s_ in streams:
            cur.wait_stream(s_)
        torch.cuda.synchronize()
        assert_same(to_host(out_rot), want_rot, "rotations on four streams, pass %d" % rep)
        assert_same(to_host(out_mul), want_mul, "products on four streams, pass %d" % rep)
        out_rot.zero_()
        out_mul.zero_()
    gc.close()


@pytest.mark.parametrize("shape", [(16, 4, 50, 2, 60, 2), (12, 4, 40, 2, 50, 2), (16, 3, 60, 2, 60, 2),
                                   (16, 4, 52, 2, 60, 2), (12, 4, 51, 2, 52, 2)])
def test_extreme_residues(gpu, shape):
    """Inputs at the ends of the residue range (every residue q-1, and 0 / q-1 alternating), keys and plaintexts at
    m-1: the lazy ranges of the kernels (double-precision sums, 30-bit partial products, Harvey butterflies) are
    argued from these maxima. The primes sit just below 2^bits, so the 52- and 51-bit shapes put the uncorrected
    integer butterflies (primes in [2^50, 2^52)) at the top of their range, as the 60-bit ones do for the Harvey form."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    nl, B = len(p.q), 2
    top = np.array(p.q, dtype=np.uint64)[None, None, :, None] - np.uint64(1)
    ct = np.broadcast_to(top, (B, 2, nl, p.N)).copy()
    ct[1, :, :, ::2] = 0
    mtop = np.array(p.moduli, dtype=np.uint64)[None, None, :, None] - np.uint64(1)
    evk = np.broadcast_to(mtop, (p.dnum, 2, len(p.moduli), p.N)).copy()
    g = galois_element(5, p.logN)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    d_ct, d_evk = to_dev(ct), to_dev(evk)
    out = torch.empty_like(d_ct)
    ref.set_threads(2)
    gpu.ckks_hrot(gc, out, d_ct, B, nl, g, d_evk, ws)
    assert_same(to_host(out), rc.hrot(ct, g, evk), "hrot at the maxima")
    gpu.ckks_hmult_relin(gc, out, d_ct, d_ct.flip(0).contiguous(), B, nl, d_evk, ws)
    assert_same(to_host(out), rc.hmult_relin(ct, ct[::-1].copy(), evk), "hmult at the maxima")
    rs = torch.empty((B, 2, nl - 1, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_rescale(gc, rs, d_ct, B, nl, gc.workspace(gpu.OP_RESCALE, B, nl))
    assert_same(to_host(rs), rc.rescale(ct), "rescale at the maxima")
    n1, n2 = 17, 2     # more baby steps than one fold of the integer inner sums (15)
    pt = np.broadcast_to(top[0], (n2, n1, nl, p.N)).copy()
    keys = [evk] * (n1 - 1 + n2 - 1)
    want = rc.pcmm_bsgs(ct, pt, n1, n2, 1, keys[:n1 - 1], keys[n1 - 1:])
    ref.set_threads(1)
    gpu.ckks_pcmm_bsgs(gc, out, d_ct, B, nl, to_dev(pt), n1, n2, 1, [d_evk] * (n1 - 1), [d_evk] * (n2 - 1),
                       gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
    assert_same(to_host(out), want, "pcmm at the maxima")
    gc.close()


def test_tuning_knobs_do_not_change_results(gpu):
    """Every alternative code path selectable with ckks_tune_set gives the oracle's bits: workgroup mappings, the
    unfused form of the inner product on double-precision moduli (plain block pass, streaming product, separate
    assembly kernel), the base conversions done inside the row passes, integer-only arithmetic, the general
    base-conversion reduction, and the two-stream fork/join of a key switch."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(16, 5, 50, 3, 60, 2)
    rc = ref.RefContext(p)
    B, nl = 3, 5
    ct = uniform_residues(500, p.q, (B, 2), p.N)
    evk = uniform_residues(501, p.moduli, (p.dnum, 2), p.N)
    g = galois_element(77, p.logN)
    ref.set_threads(3)
    want_rot = rc.hrot(ct, g, evk)
    want_mul = rc.hmult_relin(ct, ct[::-1].copy(), evk)
    ref.set_threads(1)
    d_ct, d_evk = to_dev(ct), to_dev(evk)
    d_rev = d_ct.flip(0).contiguous()
    for knobs in ({0: 0}, {0: 1}, {0: 2}, {0: 3}, {0: 4}, {3: 1}, {3: 1, 4: 0}, {4: 0}, {1: 1}, {1: 1, 3: 1}, {5: 1},
                  {5: 1, 4: 0}, {2: 1}, {2: 1, 4: 0}, {2: 1, 5: 1}, {2: 1, 1: 1}, {2: 1, 3: 1}):
        gc = gpu.Context(p)
        for k, v in knobs.items():
            gpu.ckks_tune_set(gc, k, v)
        ws = gc.workspace(gpu.OP_HROT, B, nl)
        out = torch.empty_like(d_ct)
        gpu.ckks_hrot(gc, out, d_ct, B, nl, g, d_evk, ws)
        assert_same(to_host(out), want_rot, "hrot with knobs %s" % knobs)
        gpu.ckks_hmult_relin(gc, out, d_ct, d_rev, B, nl, d_evk, ws)
        assert_same(to_host(out), want_mul, "hmult with knobs %s" % knobs)
        gc.close()


@pytest.mark.parametrize("shape,nl,B", [((12, 4, 40, 2, 50, 2), 4, 3), ((16, 5, 50, 3, 60, 2), 5, 2), ((16, 3, 60, 2, 60, 2), 3, 2)])
def test_hrot_add(gpu, shape, nl, B):
    """ct_add + HRot(ct_in) in one call: with a third ciphertext, with ct_add = ct_in (rotate-and-sum) and, at
    N = 2^16, accumulated into ct_out in place."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    ct = uniform_residues(600, p.q[:nl], (B, 2), p.N)
    other = uniform_residues(601, p.q[:nl], (B, 2), p.N)
    evk = uniform_residues(602, p.moduli, (p.dnum, 2), p.N)
    g = galois_element(321, p.logN)
    ids = list(range(nl))
    ref.set_threads(2)
    rot = rc.hrot(ct, g, evk)
    ref.set_threads(1)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    d_ct, d_other, d_evk = to_dev(ct), to_dev(other), to_dev(evk)
    out = torch.empty_like(d_ct)
    gpu.ckks_hrot_add(gc, out, d_ct, d_other, B, nl, g, d_evk, ws)
    assert_same(to_host(out), rc.pointwise(other, rot, ids, "add"), "hrot_add, third ciphertext")
    gpu.ckks_hrot_add(gc, out, d_ct, d_ct, B, nl, g, d_evk, ws)
    assert_same(to_host(out), rc.pointwise(ct, rot, ids, "add"), "hrot_add, rotate-and-sum")
    if p.logN == 16:
        acc = d_other.clone()
        gpu.ckks_hrot_add(gc, acc, d_ct, acc, B, nl, g, d_evk, ws)
        assert_same(to_host(acc), rc.pointwise(other, rot, ids, "add"), "hrot_add, in place")
    else:
        with pytest.raises(gpu.CkksError):
            gpu.ckks_hrot_add(gc, out, d_ct, out, B, nl, g, d_evk, ws)
    gc.close()


@pytest.mark.parametrize("shape,nl,B", [((12, 4, 40, 2, 50, 2), 4, 3), ((12, 5, 50, 3, 60, 2), 3, 2),
                                        ((16, 5, 50, 3, 60, 2), 5, 2), ((16, 4, 60, 2, 60, 2), 3, 2)])
def test_late_relinearisation(gpu, shape, nl, B):
    """Three-component products accumulated over three pairs (first call without addend, then in place and into
    a second buffer), relinearised once; and relin(tensor(a, b)) against HMult+relin of the library itself."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    pairs = [(uniform_residues(700 + 2 * i, p.q[:nl], (B, 2), p.N), uniform_residues(701 + 2 * i, p.q[:nl], (B, 2), p.N))
             for i in range(3)]
    evk = uniform_residues(710, p.moduli, (p.dnum, 2), p.N)
    ref.set_threads(2)
    want = None
    for a, b in pairs:
        want = rc.tensor_acc(a, b, want)
    want_ct = rc.relin(want, evk)
    ref.set_threads(1)
    d_evk = to_dev(evk)
    dp = [(to_dev(a), to_dev(b)) for a, b in pairs]
    acc = torch.empty((B, 3, nl, p.N), dtype=dp[0][0].dtype, device=dp[0][0].device)
    gpu.ckks_tensor_acc(gc, acc, dp[0][0], dp[0][1], None, B, nl)
    assert_same(to_host(acc), rc.tensor_acc(*pairs[0]), "tensor, no addend")
    gpu.ckks_tensor_acc(gc, acc, dp[1][0], dp[1][1], acc, B, nl)          # in place
    acc2 = torch.empty_like(acc)
    gpu.ckks_tensor_acc(gc, acc2, dp[2][0], dp[2][1], acc, B, nl)         # into another buffer
    assert_same(to_host(acc2), want, "tensor, accumulated")
    ws = gc.workspace(gpu.OP_KEYSWITCH, B, nl)
    out = torch.empty((B, 2, nl, p.N), dtype=acc.dtype, device=acc.device)
    gpu.ckks_relin(gc, out, acc2, B, nl, d_evk, ws)
    assert_same(to_host(out), want_ct, "relin of the sum")
    assert_same(to_host(acc2), want, "relin leaves its input alone")
    # one product: relin(tensor) is HMult+relin
    one = torch.empty_like(acc)
    gpu.ckks_tensor_acc(gc, one, dp[0][0], dp[0][1], None, B, nl)
    gpu.ckks_relin(gc, out, one, B, nl, d_evk, ws)
    ws2 = gc.workspace(gpu.OP_HMULT_RELIN, B, nl)
    hm = torch.empty_like(out)
    gpu.ckks_hmult_relin(gc, hm, dp[0][0], dp[0][1], B, nl, d_evk, ws2)
    assert torch.equal(out, hm)
    # error paths: overlap of output and input, partial overlap of addend and output
    with pytest.raises(gpu.CkksError):
        gpu.ckks_relin(gc, acc2.view(-1)[:out.numel()].view_as(out), acc2, B, nl, d_evk, ws)
    pl, part = nl * p.N, (B - 1) * 3 * nl * p.N
    shifted = acc.view(-1)[pl:pl + part].view(B - 1, 3, nl, p.N)     # one component further on: overlaps acc[:B-1]
    with pytest.raises(gpu.CkksError):
        gpu.ckks_tensor_acc(gc, shifted, dp[0][0][1:], dp[0][1][1:], acc[:B - 1], B - 1, nl)
    gc.close()


@pytest.mark.parametrize("shape,nl,B,n1,n2,stride", [
    ((16, 5, 50, 3, 60, 2), 5, 2, 3, 2, 1),     # double-precision main primes, integer-class special primes
    ((16, 5, 50, 3, 60, 2), 3, 1, 4, 1, 2),     # lower level, no giant step
    ((16, 4, 60, 2, 60, 2), 3, 2, 2, 3, 1),     # integer-class moduli everywhere
    ((16, 4, 45, 2, 50, 2), 4, 1, 1, 3, 1),     # double-precision special primes too; n1 = 1
    ((16, 4, 45, 2, 50, 2), 3, 2, 1, 2, 3),     # n1 = 1 and one giant step: the plain schedule's bits
    ((16, 6, 50, 2, 60, 3), 6, 1, 9, 2, 1),     # three digits, more baby steps than one fold of the inner sums
    ((16, 4, 50, 2, 60, 2), 4, 5, 3, 5, 1),     # five ciphertexts (a short last group of 4); giant steps in tiles of 2
])
def test_pcmm_double_hoisted(gpu, shape, nl, B, n1, n2, stride):
    """Baby and giant steps kept in the extended basis: bit-exact against the oracle's statement of that schedule;
    with n1 = 1 and a single giant rotation also against the plain schedule of the library itself."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    K = len(p.p)
    ct = uniform_residues(800, p.q[:nl], (B, 2), p.N)
    pt = uniform_residues(801, list(p.q[:nl]) + list(p.p), (n2, n1), p.N)
    baby = [uniform_residues(810 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n1 - 1)]
    giant = [uniform_residues(830 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n2 - 1)]
    ref.set_threads(4)
    want = rc.pcmm_bsgs_double_hoisted(ct, pt, n1, n2, stride, baby, giant)
    ref.set_threads(1)
    d_ct, d_pt = to_dev(ct), to_dev(pt)
    d_baby, d_giant = [to_dev(k) for k in baby], [to_dev(k) for k in giant]
    out = torch.empty_like(d_ct)
    ws = gc.workspace(gpu.OP_PCMM_BSGS_DH, B, nl, n1)
    if n2 == 5:
        gpu.ckks_tune_set(gc, 7, 2)      # at most two giant steps' inner sums held at once: three tiles
    gpu.ckks_pcmm_bsgs_double_hoisted(gc, out, d_ct, B, nl, d_pt, n1, n2, stride, d_baby, d_giant, ws)
    assert_same(to_host(out), want, "double-hoisted PCMM")
    if n2 == 5:
        # with another form of the inner product selected the giant steps take the streaming kernels: same bits
        gpu.ckks_tune_set(gc, 3, 1)
        again = torch.empty_like(d_ct)
        gpu.ckks_pcmm_bsgs_double_hoisted(gc, again, d_ct, B, nl, d_pt, n1, n2, stride, d_baby, d_giant, ws)
        assert torch.equal(again, out)
        gpu.ckks_tune_set(gc, 3, 2)
    if n1 == 1 and n2 <= 2:
        plain = torch.empty_like(d_ct)
        gpu.ckks_pcmm_bsgs(gc, plain, d_ct, B, nl, d_pt[:, :, :nl].contiguous(), n1, n2, stride, d_baby, d_giant,
                           gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
        assert torch.equal(out, plain)
    with pytest.raises(gpu.CkksError):     # workspace of the plain schedule is too small here
        small = gc.workspace(gpu.OP_HROT, B, nl)
        gpu.ckks_pcmm_bsgs_double_hoisted(gc, out, d_ct, B, nl, d_pt, n1, n2, stride, d_baby, d_giant, small)
    gc.close()


def test_pcmm_double_hoisted_needs_full_ring(gpu):
    import torch
    from gpu_util import to_dev
    p = make_params(12, 4, 40, 2, 50, 2)
    gc = gpu.Context(p)
    ct = to_dev(uniform_residues(1, p.q, (1, 2), p.N))
    pt = to_dev(uniform_residues(2, p.moduli, (1, 1), p.N))
    ws = gc.workspace(gpu.OP_PCMM_BSGS, 1, 4, 1)
    with pytest.raises(gpu.CkksError):
        gpu.ckks_pcmm_bsgs_double_hoisted(gc, torch.empty_like(ct), ct, 1, 4, pt, 1, 1, 1, [], [], ws)
    gc.close()


def test_pcmm_schedules_under_knobs(gpu):
    """The hoisted and the extended-basis schedule give the oracle's bits under every alternative code path that
    ckks_tune_set selects (integer-only arithmetic, general base-conversion reduction, integer inner sums, workgroup
    mappings, the other forms of the fused inner product, two streams)."""
    import torch
    from gpu_util import to_dev, to_host
    p = make_params(16, 5, 50, 3, 60, 2)
    nl, B, n1, n2 = 5, 3, 5, 3
    rc = ref.RefContext(p)
    ct = uniform_residues(1, p.q[:nl], (B, 2), p.N)
    pte = uniform_residues(2, list(p.q[:nl]) + list(p.p), (n2, n1), p.N)
    pt = np.ascontiguousarray(pte[:, :, :nl])
    bk = [uniform_residues(10 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n1 - 1)]
    gk = [uniform_residues(20 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n2 - 1)]
    ref.set_threads(4)
    want_d = rc.pcmm_bsgs_double_hoisted(ct, pte, n1, n2, 1, bk, gk)
    want_p = rc.pcmm_bsgs(ct, pt, n1, n2, 1, bk, gk)
    ref.set_threads(1)
    d_ct, d_pte, d_pt = to_dev(ct), to_dev(pte), to_dev(pt)
    dbk, dgk = [to_dev(k) for k in bk], [to_dev(k) for k in gk]
    for knobs in [{1: 1}, {5: 1}, {6: 1}, {0: 0}, {0: 2}, {3: 1}, {4: 0}, {2: 1}, {1: 1, 5: 1, 6: 1}]:
        gc = gpu.Context(p)
        for k, v in knobs.items():
            gpu.ckks_tune_set(gc, k, v)
        out = torch.empty_like(d_ct)
        gpu.ckks_pcmm_bsgs_double_hoisted(gc, out, d_ct, B, nl, d_pte, n1, n2, 1, dbk, dgk,
                                          gc.workspace(gpu.OP_PCMM_BSGS_DH, B, nl, n1))
        assert (to_host(out) == want_d).all(), "extended-basis schedule with knobs %s" % knobs
        gpu.ckks_pcmm_bsgs_hoisted(gc, out, d_ct, B, nl, d_pt, n1, n2, 1, dbk, dgk,
                                   gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
        assert (to_host(out) == want_p).all(), "hoisted schedule with knobs %s" % knobs
        gc.close()


@pytest.mark.parametrize("shape,nl,B,steps", [
    ((16, 5, 50, 3, 60, 2), 5, 2, (1, 2, 3)),      # double-precision main primes, integer-class special primes
    ((16, 4, 60, 2, 60, 2), 3, 3, (5,)),           # integer-class everywhere, one rotation
    ((16, 4, 45, 2, 50, 2), 4, 1, ()),             # no rotation: the input comes back
    ((16, 6, 50, 2, 60, 3), 4, 2, (8, 16, 24, 32, 40, 48, 56)),   # lower level, seven rotations (the outer sum of 64)
    ((16, 2, 50, 1, 60, 2), 2, 1, tuple(range(1, 66))),           # 65 rotations: two launches, the second adds on
])
def test_hrot_sum(gpu, shape, nl, B, steps):
    """ct + sum of rotations with one ModDown, bit-exact against the oracle; one rotation also equals the library's
    own rotate-and-add, none returns the input."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = make_params(*shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    ct = uniform_residues(900, p.q[:nl], (B, 2), p.N)
    gs = [galois_element(k, p.logN) for k in steps]
    nkeys = min(len(steps), 7)                 # keys repeat beyond seven rotations
    kpool = [uniform_residues(910 + i, p.moduli, (p.dnum, 2), p.N) for i in range(nkeys)]
    evks = [kpool[i % nkeys] for i in range(len(steps))]
    ref.set_threads(4)
    want = rc.hrot_sum(ct, gs, evks)
    ref.set_threads(1)
    d_pool = [to_dev(k) for k in kpool]
    d_ct, d_evks = to_dev(ct), [d_pool[i % nkeys] for i in range(len(steps))]
    out = torch.empty_like(d_ct)
    ws = gc.workspace(gpu.OP_HROT_SUM, B, nl)
    gpu.ckks_hrot_sum(gc, out, d_ct, B, nl, gs, d_evks, ws)
    assert_same(to_host(out), want, "hrot_sum")
    if len(steps) == 1:
        ra = torch.empty_like(d_ct)
        gpu.ckks_hrot_add(gc, ra, d_ct, d_ct, B, nl, gs[0], d_evks[0], gc.workspace(gpu.OP_HROT, B, nl))
        assert torch.equal(out, ra)
    if not steps:
        assert torch.equal(out, d_ct)
    with pytest.raises(gpu.CkksError):
        gpu.ckks_hrot_sum(gc, d_ct, d_ct, B, nl, gs, d_evks, ws)                    # output overlaps input
    with pytest.raises(gpu.CkksError):
        gpu.ckks_hrot_sum(gc, out, d_ct, B, nl, gs, d_evks, gc.workspace(gpu.OP_HROT, B, nl))   # workspace too small
    gc.close()


def test_hrot_sum_needs_full_ring(gpu):
    import torch
    from gpu_util import to_dev
    p = make_params(12, 4, 40, 2, 50, 2)
    gc = gpu.Context(p)
    ct = to_dev(uniform_residues(1, p.q, (1, 2), p.N))
    with pytest.raises(gpu.CkksError):
        gpu.ckks_hrot_sum(gc, torch.empty_like(ct), ct, 1, 4, [], [], gc.workspace(gpu.OP_HROT, 1, 4))
    gc.close()
