"""The entry point for callers that cannot allocate (ckks_hrot_noalloc) against ckks_hrot, bit for bit.

Two calls in a row on one context, the second on a smaller input, so that the fixed scratch array is reused with
whatever the first call left in it; then the size check and the refusal while per-kernel timing is on.
"""
import numpy as np
import pytest

from ckks_inputs import config_params, galois_element, uniform_residues

pytestmark = pytest.mark.gpu


def test_hrot_noalloc_matches_hrot_twice_second_smaller():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2604_03425_amd as ck
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")          # N = 2^16, 24 x 50-bit + 8 x 60-bit primes, dnum = 3
    ctx = ck.Context(p, 0)
    assert ck.ckks_noalloc_scratch_bytes() == 128 << 20
    evk = to_dev(uniform_residues(11, p.moduli, (p.dnum, 2), p.N))
    for call, (B, nl, step) in enumerate([(1, 24, 77), (1, 9, 5), (2, 5, 1234)]):
        assert ck.ckks_workspace_bytes(ctx, ck.OP_HROT, B, nl) <= ck.ckks_noalloc_scratch_bytes()
        ct = to_dev(uniform_residues(100 + call, p.q[:nl], (B, 2), p.N))
        g = galois_element(step, p.logN)
        want = torch.empty_like(ct)
        ck.ckks_hrot(ctx, want, ct, B, nl, g, evk, ctx.workspace(ck.OP_HROT, B, nl))
        want_h = to_host(want)
        got = torch.zeros_like(ct)
        before = torch.cuda.memory_allocated()
        ck.ckks_hrot_noalloc(ctx, got, ct, B, nl, g, evk)
        assert torch.cuda.memory_allocated() == before
        assert_same(to_host(got), want_h, "ckks_hrot_noalloc call %d (B=%d, %d limbs)" % (call, B, nl))
    # too large for the fixed array: refused, nothing enqueued
    ct = to_dev(uniform_residues(7, p.q, (2, 2), p.N))
    out = torch.empty_like(ct)
    with pytest.raises(ck.CkksError) as e:
        ck.ckks_hrot_noalloc(ctx, out, ct, 2, 24, galois_element(3, p.logN), evk)
    assert e.value.code == -3 and "scratch" in str(e.value)
    # per-kernel timing creates events: refused while it is on
    ck.ckks_prof_enable(ctx, True)
    with pytest.raises(ck.CkksError):
        ck.ckks_hrot_noalloc(ctx, out[:1], ct[:1], 1, 24, galois_element(3, p.logN), evk)
    ck.ckks_prof_enable(ctx, False)
    ctx.close()


def test_hrot_noalloc_small_ring():
    """The general (other ring degrees) path through the same entry point: the tiny configuration, batch of 8."""
    import torch
    import paper_2604_03425_amd as ck
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("tiny_hrot")
    ctx = ck.Context(p, 0)
    nl = len(p.q)
    evk = to_dev(uniform_residues(21, p.moduli, (p.dnum, 2), p.N))
    for B, step in ((8, 99), (3, 2047)):
        ct = to_dev(uniform_residues(200 + B, p.q, (B, 2), p.N))
        g = galois_element(step, p.logN)
        want = torch.empty_like(ct)
        ck.ckks_hrot(ctx, want, ct, B, nl, g, evk, ctx.workspace(ck.OP_HROT, B, nl))
        got = torch.zeros_like(ct)
        ck.ckks_hrot_noalloc(ctx, got, ct, B, nl, g, evk)
        assert_same(to_host(got), to_host(want), "ckks_hrot_noalloc tiny B=%d" % B)
    ctx.close()


def test_hrot_noalloc_replayed_from_a_hip_graph():
    """What the entry point is for: captured once into a HIP graph (capture forbids allocation), then replayed with
    new inputs in the same buffers. Every replay is checked against an eager ckks_hrot, with eager work and
    synchronisations between the replays."""
    import torch
    import paper_2604_03425_amd as ck
    from gpu_util import to_dev, to_host, assert_same
    p = config_params("keyswitch_micro")
    ctx = ck.Context(p, 0)
    nl, B = 24, 1
    evk = to_dev(uniform_residues(31, p.moduli, (p.dnum, 2), p.N))
    g = galois_element(4242, p.logN)
    static_in = to_dev(uniform_residues(300, p.q, (B, 2), p.N))
    static_out = torch.zeros_like(static_in)
    ws = ctx.workspace(ck.OP_HROT, B, nl)
    ck.ckks_hrot_noalloc(ctx, static_out, static_in, B, nl, g, evk)      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ck.ckks_hrot_noalloc(ctx, static_out, static_in, B, nl, g, evk)
    for trial in range(3):
        fresh = to_dev(uniform_residues(310 + trial, p.q, (B, 2), p.N))
        want = torch.empty_like(fresh)
        ck.ckks_hrot(ctx, want, fresh, B, nl, g, evk, ws)               # eager work between the replays
        torch.cuda.synchronize()
        static_in.copy_(fresh)
        static_out.zero_()
        graph.replay()
        assert_same(to_host(static_out), to_host(want), "graph replay %d" % trial)
    ctx.close()
