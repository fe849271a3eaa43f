"""Digest of the library's sources: what a stored counter summary is valid for."""
import hashlib
import os

_HERE = os.path.dirname(os.path.abspath(__file__))


def source_digest():
    """SHA-256 over the kernels, the host code and the public header (file names and contents, sorted)."""
    h = hashlib.sha256()
    files = []
    for d in (os.path.join(_HERE, "csrc"), os.path.join(os.path.dirname(_HERE), "include")):
        files += [os.path.join(d, f) for f in sorted(os.listdir(d))]
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()
