"""GPU parity: every ABI call of the HIP library against the CPU oracle, bit-exact on every residue."""
import numpy as np
import pytest

from ckks_inputs import (config_params, galois_element, make_params, seeded_rotation_steps, uniform_residues)
from oracle import ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2604_03425_amd as pkg
    return pkg


_ctx_cache = {}


def contexts(gpu, params_key, params):
    if params_key not in _ctx_cache:
        _ctx_cache[params_key] = (ref.RefContext(params), gpu.Context(params))
    return _ctx_cache[params_key]


def shape_params(shape):
    return make_params(*shape)


TRANSFORM_SHAPES = [
    # logN nq qbits np pbits dnum
    (10, 2, 40, 1, 50, 1),
    (11, 2, 50, 1, 60, 1),
    (12, 4, 40, 1, 50, 2),
    (13, 2, 50, 2, 60, 1),
    (14, 2, 50, 1, 60, 1),
    (15, 2, 40, 1, 60, 1),
    (16, 3, 50, 2, 60, 1),
    (17, 2, 50, 1, 60, 1),
]


@pytest.mark.parametrize("shape", TRANSFORM_SHAPES)
def test_ntt_intt(gpu, shape):
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    rc, gc = contexts(gpu, shape, p)
    ids = list(range(len(p.moduli)))[::-1]           # reversed: slot -> modulus map is honoured
    npoly = 3
    x = uniform_residues(100 + shape[0], [p.moduli[i] for i in ids], (npoly,), p.N)
    # edge values: zeros and m-1 everywhere in one polynomial
    x[0, 0, :] = 0
    x[1, 1, :] = p.moduli[ids[1]] - 1
    d = to_dev(x)
    gpu.ckks_ntt(gc, d, npoly, ids)
    f = to_host(d)
    assert_same(f, rc.ntt(x, ids), "ntt")
    gpu.ckks_intt(gc, d, npoly, ids)
    assert_same(to_host(d), x, "intt(ntt)")
    d2 = to_dev(x)
    gpu.ckks_intt(gc, d2, npoly, ids)
    assert_same(to_host(d2), rc.intt(x, ids), "intt")


@pytest.mark.parametrize("shape", [(12, 4, 40, 1, 50, 2), (16, 2, 50, 1, 60, 1)])
def test_automorph(gpu, shape):
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    rc, gc = contexts(gpu, shape, p)
    ids = list(range(len(p.moduli)))
    x = uniform_residues(7, p.moduli, (2,), p.N)
    x[0, 0, :5] = 0                                   # zero stays zero under the sign flip
    d = to_dev(x)
    out = torch.empty_like(d)
    for g in (5, galois_element(1234, p.logN), 2 * p.N - 1, 3):
        for ev in (True, False):
            gpu.ckks_automorph(gc, out, d, 2, ids, g, ev)
            assert_same(to_host(out), rc.automorph(x, ids, g, ev), "automorph g=%d eval=%s" % (g, ev))


KS_SHAPES = [
    # (logN nq qbits np pbits dnum), nlimbs, B
    ((12, 4, 40, 1, 50, 2), 4, 3),     # literal tiny config
    ((12, 4, 40, 2, 50, 2), 3, 2),     # lower level, ragged last digit
    ((12, 4, 40, 1, 50, 4), 4, 2),     # alpha = 1
    ((12, 6, 50, 3, 60, 2), 6, 2),
    ((12, 6, 50, 3, 60, 2), 2, 1),     # only one digit present
    ((12, 5, 50, 5, 60, 1), 5, 2),     # dnum = 1
    ((12, 7, 50, 3, 60, 3), 7, 2),     # ragged at the top level: digits 3,3,1
    ((13, 4, 50, 2, 60, 2), 4, 2),     # two-pass transform
    ((12, 8, 60, 8, 60, 1), 8, 2),     # 60-bit sources and targets, 8 terms: the general 128-bit reduction
    ((12, 6, 60, 3, 60, 2), 6, 2),     # 60-bit both sides but only 3 terms: the three-sum reduction still fits
    ((12, 16, 50, 16, 60, 1), 16, 1),  # 16 sources: two chunks of the dot product
    ((12, 40, 45, 40, 55, 1), 40, 1),  # 40 sources: three chunks, the widest instantiation
]


@pytest.mark.parametrize("shape,nlimbs,B", KS_SHAPES)
def test_keyswitch(gpu, shape, nlimbs, B):
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    rc, gc = contexts(gpu, shape, p)
    d = uniform_residues(11, p.q[:nlimbs], (B,), p.N)
    evk = uniform_residues(12, p.moduli, (p.dnum, 2), p.N)
    want = rc.keyswitch(d, evk)
    ws = gc.workspace(gpu.OP_KEYSWITCH, B, nlimbs)
    out = torch.empty((B, 2, nlimbs, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_keyswitch(gc, out, to_dev(d), B, nlimbs, to_dev(evk), 0, p.dnum, ws)
    assert_same(to_host(out), want, "keyswitch")


@pytest.mark.parametrize("shape,nlimbs,B", [((12, 6, 50, 3, 60, 2), 6, 2), ((16, 4, 50, 2, 60, 2), 4, 2)])
def test_keyswitch_general_reduction(gpu, shape, nlimbs, B):
    """Base conversions forced onto the general four-sum / 128-bit reduction where the three-sum form would do."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    rc, gc = ref.RefContext(p), gpu.Context(p)
    gpu.ckks_tune_set(gc, 5, 1)
    d = uniform_residues(13, p.q[:nlimbs], (B,), p.N)
    evk = uniform_residues(14, p.moduli, (p.dnum, 2), p.N)
    want = rc.keyswitch(d, evk)
    out = torch.empty((B, 2, nlimbs, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_keyswitch(gc, out, to_dev(d), B, nlimbs, to_dev(evk), 0, p.dnum, gc.workspace(gpu.OP_KEYSWITCH, B, nlimbs))
    assert_same(to_host(out), want, "keyswitch, general reduction")
    ct = uniform_residues(15, p.q[:nlimbs], (B, 2), p.N)
    out2 = torch.empty((B, 2, nlimbs - 1, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_rescale(gc, out2, to_dev(ct), B, nlimbs, gc.workspace(gpu.OP_RESCALE, B, nlimbs))
    assert_same(to_host(out2), rc.rescale(ct), "rescale, general reduction")
    gc.close()


def test_hrot_tiny_config_batch(gpu):
    """N=2^12, 4x40-bit + 1x50-bit, dnum=2, 8 ciphertexts each rotated by its own seeded step in [1,2047]."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("tiny_hrot")
    rc, gc = contexts(gpu, "tiny_hrot", p)
    B, nl = 8, 4
    ct = uniform_residues(21, p.q, (B, 2), p.N)
    steps = seeded_rotation_steps(22, B, 1, 2047)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    dct = to_dev(ct)
    for i, k in enumerate(steps):
        g = galois_element(k, p.logN)
        evk = uniform_residues(1000 + i, p.moduli, (p.dnum, 2), p.N)
        out = torch.empty((1, 2, nl, p.N), dtype=torch.int64, device="cuda")
        gpu.ckks_hrot(gc, out, dct[i:i + 1].contiguous(), 1, nl, g, to_dev(evk), ws)
        assert_same(to_host(out), rc.hrot(ct[i:i + 1], g, evk), "hrot ct %d step %d" % (i, k))
    # whole batch with one shared step and key
    g = galois_element(steps[0], p.logN)
    evk = uniform_residues(999, p.moduli, (p.dnum, 2), p.N)
    out = torch.empty_like(dct)
    gpu.ckks_hrot(gc, out, dct, B, nl, g, to_dev(evk), ws)
    assert_same(to_host(out), rc.hrot(ct, g, evk), "hrot batch")


def test_hrot_decrypts_to_rotated_slots(gpu):
    """End to end through the GPU: encrypt (oracle), HRot (GPU), decrypt (oracle) = rotated slots, err < 2^-16."""
    import torch
    from gpu_util import to_dev, to_host
    from harness import Keys
    from ckks_inputs import uniform_slots
    p = config_params("tiny_hrot_k2")
    rc, gc = contexts(gpu, "tiny_hrot_k2", p)
    keys = Keys(p, rc, 21)
    z = uniform_slots(8, p.N // 2)
    ct = keys.encrypt_slots(z, 2.0**30, 4)[None]
    k = 77
    g = galois_element(k, p.logN)
    out = torch.empty((1, 2, 4, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hrot(gc, out, to_dev(ct), 1, 4, g, to_dev(keys.rotation_key(g)), gc.workspace(gpu.OP_HROT, 1, 4))
    err = np.max(np.abs(keys.decrypt_slots(to_host(out)[0], 2.0**30) - np.roll(z, -k)))
    assert err < 2.0**-16, err


@pytest.mark.parametrize("shape,nlimbs,B", [((12, 4, 40, 1, 50, 2), 4, 3), ((12, 6, 50, 3, 60, 2), 5, 2)])
def test_hmult_relin(gpu, shape, nlimbs, B):
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    rc, gc = contexts(gpu, shape, p)
    a = uniform_residues(31, p.q[:nlimbs], (B, 2), p.N)
    b = uniform_residues(32, p.q[:nlimbs], (B, 2), p.N)
    evk = uniform_residues(33, p.moduli, (p.dnum, 2), p.N)
    out = torch.empty((B, 2, nlimbs, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hmult_relin(gc, out, to_dev(a), to_dev(b), B, nlimbs, to_dev(evk), gc.workspace(gpu.OP_HMULT_RELIN, B, nlimbs))
    assert_same(to_host(out), rc.hmult_relin(a, b, evk), "hmult_relin")


PCMM_CASES = [
    # n1 n2 stride, shape, tuning knobs
    (3, 2, 1, (12, 4, 40, 2, 50, 2), {}),
    (1, 3, 2, (12, 4, 40, 2, 50, 2), {}),
    (4, 1, 1, (12, 4, 40, 2, 50, 2), {}),
    (9, 2, 1, (12, 4, 40, 2, 50, 2), {}),
    (5, 7, 1, (12, 4, 40, 2, 50, 2), {}),          # 7 giant steps = passes of 6 and 1
    (17, 13, 1, (12, 4, 40, 2, 50, 2), {7: 12}),   # more than 16 terms per sum; passes of 12 and 1
    (5, 7, 1, (12, 4, 40, 2, 50, 2), {6: 1}),      # integer kernel on every limb: passes of 4 and 3
    (3, 5, 1, (12, 4, 60, 2, 60, 2), {}),          # 60-bit primes: integer kernel by necessity
]


@pytest.mark.parametrize("n1,n2,stride,shape,knobs", PCMM_CASES)
def test_pcmm_bsgs(gpu, n1, n2, stride, shape, knobs):
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = shape_params(shape)
    if knobs:
        rc, gc = ref.RefContext(p), gpu.Context(p)
        for k, v in knobs.items():
            gpu.ckks_tune_set(gc, k, v)
    else:
        rc, gc = contexts(gpu, shape, p)
    B, nl = 2, 4
    ct = uniform_residues(41, p.q, (B, 2), p.N)
    pt = uniform_residues(42, p.q, (n2, n1), p.N)
    baby = [uniform_residues(500 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n1 - 1)]
    giant = [uniform_residues(600 + i, p.moduli, (p.dnum, 2), p.N) for i in range(n2 - 1)]
    want = rc.pcmm_bsgs(ct, pt, n1, n2, stride, baby, giant)
    out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    db = [to_dev(k) for k in baby]
    dg = [to_dev(k) for k in giant]
    gpu.ckks_pcmm_bsgs(gc, out, to_dev(ct), B, nl, to_dev(pt), n1, n2, stride, db, dg,
                       gc.workspace(gpu.OP_PCMM_BSGS, B, nl, n1))
    assert_same(to_host(out), want, "pcmm_bsgs")


def test_full_size_hrot_and_hmult_sampled(gpu):
    """N=2^16, 24 limbs, dnum=3, K=8: batch of 64 in one launch sequence (the benchmarked configuration);
    three sampled ciphertexts are recomputed whole by the oracle."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")
    rc, gc = contexts(gpu, "keyswitch_micro", p)
    ref.set_threads(8)
    B, nl = 64, 24
    rng = torch.Generator(device="cuda").manual_seed(5)
    # batch filled on the device (uniform 62-bit values reduced per limb would need modular ops; instead
    # draw below the smallest modulus so every residue is canonical), sampled rows replaced by seeded numpy rows
    lim = int(min(p.q))
    dct = torch.randint(0, lim, (B, 2, nl, p.N), dtype=torch.int64, device="cuda", generator=rng)
    sample = [0, 37, 63]
    rows = uniform_residues(51, p.q, (len(sample), 2), p.N)
    for r, i in enumerate(sample):
        dct[i] = to_dev(rows[r])
    evk = uniform_residues(52, p.moduli, (p.dnum, 2), p.N)
    devk = to_dev(evk)
    g = galois_element(4321, p.logN)
    out = torch.empty_like(dct)
    gpu.ckks_hrot(gc, out, dct, B, nl, g, devk, gc.workspace(gpu.OP_HROT, B, nl))
    got = to_host(out[sample])
    assert_same(got, rc.hrot(rows, g, evk), "hrot full size")
    # HMult+relin on pairs (2i, 2i+1): sample pair (0, 37) and (63, 0) by building them explicitly
    a = dct[[0, 63]].contiguous()
    b = dct[[37, 0]].contiguous()
    out2 = torch.empty_like(a)
    gpu.ckks_hmult_relin(gc, out2, a, b, 2, nl, devk, gc.workspace(gpu.OP_HMULT_RELIN, 2, nl))
    assert_same(to_host(out2), rc.hmult_relin(rows[[0, 2]], rows[[1, 0]], evk), "hmult full size")
    ref.set_threads(1)


def test_full_batch_against_oracle_digests(gpu):
    """The whole micro-benchmark batch (64 rotations with their own elements and keys in one call, 32 products):
    SHA-256 of every output ciphertext equals the digest the oracle wrote (tests/golden/, made by
    make_keyswitch_micro_digests.py from the same seeded inputs)."""
    import hashlib
    import os
    import torch
    from gpu_util import to_dev, to_host
    p = config_params("keyswitch_micro")
    gc = gpu.Context(p)
    B, nl = 64, 24
    want = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "keyswitch_micro_digests.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                parts = line.split()
                want[(parts[0], int(parts[1]))] = parts[-1]
    assert len(want) == B + B // 2
    ct = uniform_residues(0xC0FFEE, p.q, (B, 2), p.N)
    steps = seeded_rotation_steps(7, B, 1, p.N // 2 - 1)
    keys = [to_dev(uniform_residues(1000 + b, p.moduli, (p.dnum, 2), p.N)) for b in range(B)]
    d_ct = to_dev(ct)
    out = torch.empty_like(d_ct)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    gpu.ckks_hrot_multi(gc, out, d_ct, B, nl, [galois_element(k, p.logN) for k in steps], keys, ws)
    got = to_host(out)
    bad = [b for b in range(B) if hashlib.sha256(np.ascontiguousarray(got[b]).tobytes()).hexdigest() != want[("hrot", b)]]
    assert not bad, "rotations differ from the oracle's digests: %s" % bad
    del keys
    relin = to_dev(uniform_residues(999, p.moduli, (p.dnum, 2), p.N))
    prod = torch.empty((B // 2, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hmult_relin(gc, prod, d_ct[0::2].contiguous(), d_ct[1::2].contiguous(), B // 2, nl, relin, ws)
    got = to_host(prod)
    bad = [i for i in range(B // 2)
           if hashlib.sha256(np.ascontiguousarray(got[i]).tobytes()).hexdigest() != want[("hmult", i)]]
    assert not bad, "products differ from the oracle's digests: %s" % bad
    gc.close()


def test_argument_errors(gpu):
    import torch
    from gpu_util import to_dev
    shape = (12, 4, 40, 1, 50, 2)
    p = shape_params(shape)
    rc, gc = contexts(gpu, shape, p)
    x = torch.zeros((1, 2, 4, p.N), dtype=torch.int64, device="cuda")
    evk = torch.zeros((2, 2, 5, p.N), dtype=torch.int64, device="cuda")
    ws = gc.workspace(gpu.OP_HROT, 1, 4)
    out = torch.empty_like(x)
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_hrot(gc, out, x, 1, 4, 4, evk, ws)            # even Galois element
    assert e.value.code == -1
    x5 = torch.zeros((1, 2, 5, p.N), dtype=torch.int64, device="cuda")
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_hrot(gc, torch.empty_like(x5), x5, 1, 5, 5, evk, ws)   # more limbs than the context has
    assert e.value.code == -2
    with pytest.raises(ValueError):
        gpu.ckks_hrot(gc, out, x, 2, 4, 5, evk, ws)            # the binding refuses tensors smaller than the call's shape
    with pytest.raises(ValueError):
        gpu.ckks_hrot(gc, out, x, 1, 4, 5, evk[:1], ws)        # ... and a key with too few digits
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_hrot(gc, out, x, 1, 4, 5, evk, ws[:1024])     # workspace too small
    assert e.value.code == -3
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_hrot(gc, x, x, 1, 4, 5, evk, ws)              # aliasing
    assert e.value.code == -1
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_ntt(gc, x, 2, [0, 1, 2, 9])                   # modulus id out of range
    assert e.value.code == -1
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_keyswitch(gc, out, x[:, 0].contiguous(), 1, 4, evk, 0, 3, ws)   # wrong dnum
    assert e.value.code == -2
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_hrot_multi(gc, out, x, 1, 4, [6], [evk], ws)   # even Galois element in the per-ciphertext list
    assert e.value.code == -1
    with pytest.raises(ValueError):
        gpu.ckks_hrot_multi(gc, out, x, 1, 4, [5, 25], [evk], ws)   # list lengths must equal the batch
    with pytest.raises(gpu.CkksError) as e:
        gpu.ckks_rescale(gc, out, x, 1, 1, ws)                  # nothing to drop
    assert e.value.code == -2
    bad = make_params(12, 2, 40, 1, 50, 1)
    bad.q[0] += 2
    with pytest.raises(gpu.CkksError):
        gpu.Context(bad)


def test_integer_bodies_only_at_full_ring(gpu):
    """The double-precision bodies (primes < 2^50) can be switched off; the integer bodies must give the same bits."""
    import torch
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")
    rc = ref.RefContext(p)
    gc = gpu.Context(p)
    gpu.ckks_tune_set(gc, 1, 1)
    B, nl = 2, 24
    ct = uniform_residues(61, p.q, (B, 2), p.N)
    evk = uniform_residues(62, p.moduli, (p.dnum, 2), p.N)
    g = galois_element(99, p.logN)
    ref.set_threads(2)
    want_rot = rc.hrot(ct, g, evk)
    want_mul = rc.hmult_relin(ct[:1], ct[1:], evk)
    ref.set_threads(1)
    ws = gc.workspace(gpu.OP_HROT, B, nl)
    out = torch.empty((B, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hrot(gc, out, to_dev(ct), B, nl, g, to_dev(evk), ws)
    assert_same(to_host(out), want_rot, "hrot, integer bodies")
    out2 = torch.empty((1, 2, nl, p.N), dtype=torch.int64, device="cuda")
    gpu.ckks_hmult_relin(gc, out2, to_dev(ct[:1]), to_dev(ct[1:]), 1, nl, to_dev(evk), ws)
    assert_same(to_host(out2), want_mul, "hmult, integer bodies")
    x = uniform_residues(63, p.moduli, (2,), p.N)
    ids = list(range(len(p.moduli)))
    d = to_dev(x)
    gpu.ckks_ntt(gc, d, 2, ids)
    assert_same(to_host(d), rc.ntt(x, ids), "ntt, integer bodies")
    gpu.ckks_intt(gc, d, 2, ids)
    assert_same(to_host(d), x, "intt, integer bodies")
    gc.close()
