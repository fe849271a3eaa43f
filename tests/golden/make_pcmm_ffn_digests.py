"""Writes tests/golden/pcmm_ffn_digests.txt: SHA-256 of every output ciphertext of the diagonal BSGS
ciphertext-plaintext matmul at the shape of the FFN-layer workload (N = 2^16, 24 limbs of 50 bits, 8 special primes
of 60 bits, dnum = 3, 32 baby steps x 24 giant steps = 768 diagonals, stride 1) on a batch of 8 seeded ciphertexts,
computed by the CPU oracle only (one rotation at a time, no hoisting). Ciphertexts, plaintext diagonals and the 54
rotation keys are seeded uniform residues: parity of integer arithmetic needs no meaningful plaintext. The GPU test
regenerates the same inputs and compares the digests of its own outputs, for the plain and the hoisted schedule.
Takes several minutes on 8 cores and about 20 GiB of memory.

Run from the repository root:  python tests/golden/make_pcmm_ffn_digests.py
"""
import hashlib
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

from ckks_inputs import config_params, uniform_residues  # noqa: E402
from oracle import ref  # noqa: E402

CT_SEED, PT_SEED, BABY_SEED0, GIANT_SEED0, B, N1, N2 = 0xFF17, 0xD1A6, 5000, 6000, 8, 32, 24


def inputs(p):
    """The seeded inputs of the test, shared with tests/test_gpu_configs.py (which imports this function)."""
    ct = uniform_residues(CT_SEED, p.q, (B, 2), p.N)
    pt = uniform_residues(PT_SEED, p.q, (N2, N1), p.N)
    baby = [uniform_residues(BABY_SEED0 + b, p.moduli, (p.dnum, 2), p.N) for b in range(1, N1)]
    giant = [uniform_residues(GIANT_SEED0 + g, p.moduli, (p.dnum, 2), p.N) for g in range(1, N2)]
    return ct, pt, baby, giant


def main():
    p = config_params("keyswitch_micro")
    rc = ref.RefContext(p)
    t0 = time.time()
    ct, pt, baby, giant = inputs(p)
    print("inputs ready after %.0f s" % (time.time() - t0), flush=True)
    ref.set_threads(min(B, os.cpu_count() or 1))
    out = rc.pcmm_bsgs(ct, pt, N1, N2, 1, baby, giant)
    ref.set_threads(1)
    print("oracle done after %.0f s" % (time.time() - t0), flush=True)
    lines = ["# sha256 of the oracle's output ciphertexts [2][24][65536] uint64 (little endian, C order) of "
             "ref_pcmm_bsgs, n1 = %d, n2 = %d, stride 1" % (N1, N2),
             "# inputs: ct = uniform_residues(0x%X, q, (%d, 2)); pt = uniform_residues(0x%X, q, (%d, %d)); baby key b = "
             "uniform_residues(%d + b, q||p, (3, 2)), b = 1..%d; giant key g = uniform_residues(%d + g, ...), g = 1..%d"
             % (CT_SEED, B, PT_SEED, N2, N1, BABY_SEED0, N1 - 1, GIANT_SEED0, N2 - 1)]
    for b in range(B):
        lines.append("pcmm %d %s" % (b, hashlib.sha256(np.ascontiguousarray(out[b]).tobytes()).hexdigest()))
        print(lines[-1], flush=True)
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "pcmm_ffn_digests.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
