"""Helpers for the GPU parity tests: move uint64 numpy arrays to the device and back."""
import numpy as np
import torch


def to_dev(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return torch.from_numpy(a.view(np.int64)).cuda()


def to_host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy().view(np.uint64)


def assert_same(got, want, what=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not (got == want).all():
        bad = np.argwhere(got != want)
        raise AssertionError("%s: %d of %d residues differ; first at %s: got %d want %d" % (
            what, len(bad), got.size, tuple(bad[0]), got[tuple(bad[0])], want[tuple(bad[0])]))
