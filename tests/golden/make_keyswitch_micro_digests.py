"""Writes tests/golden/keyswitch_micro_digests.txt: SHA-256 of every output ciphertext of the key-switch
micro-benchmark batch (N = 2^16, 24 limbs of 50 bits, 8 special primes of 60 bits, dnum = 3; 64 ciphertexts each
rotated by its own seeded Galois element with its own seeded key, and HMult+relin of the 32 pairs (2i, 2i+1)),
computed by the CPU oracle only. The GPU test regenerates the same seeded inputs and compares the digests of its
own outputs, so every residue of every ciphertext of the full batch is covered. Takes a few minutes.

Run from the repository root:  python tests/golden/make_keyswitch_micro_digests.py
"""
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

from ckks_inputs import config_params, galois_element, seeded_rotation_steps, uniform_residues  # noqa: E402
from oracle import ref  # noqa: E402

CT_SEED, STEP_SEED, KEY_SEED0, RELIN_SEED, B = 0xC0FFEE, 7, 1000, 999, 64


def main():
    p = config_params("keyswitch_micro")
    rc = ref.RefContext(p)
    ct = uniform_residues(CT_SEED, p.q, (B, 2), p.N)
    steps = seeded_rotation_steps(STEP_SEED, B, 1, p.N // 2 - 1)
    lines = ["# sha256 of the oracle's output ciphertexts [2][24][65536] uint64 (little endian, C order)",
             "# inputs: uniform_residues(0x%X, q, (64, 2)); steps seeded_rotation_steps(%d, 64, 1, N/2-1); "
             "key b = uniform_residues(%d + b, q||p, (3, 2)); relin key = uniform_residues(%d, ...)"
             % (CT_SEED, STEP_SEED, KEY_SEED0, RELIN_SEED)]
    for b in range(B):
        key = uniform_residues(KEY_SEED0 + b, p.moduli, (p.dnum, 2), p.N)
        out = rc.hrot(ct[b:b + 1], galois_element(steps[b], p.logN), key)
        lines.append("hrot %d %d %s" % (b, steps[b], hashlib.sha256(np.ascontiguousarray(out[0]).tobytes()).hexdigest()))
        print(lines[-1], flush=True)
    relin = uniform_residues(RELIN_SEED, p.moduli, (p.dnum, 2), p.N)
    ref.set_threads(min(8, os.cpu_count() or 1))
    prod = rc.hmult_relin(np.ascontiguousarray(ct[0::2]), np.ascontiguousarray(ct[1::2]), relin)
    ref.set_threads(1)
    for i in range(B // 2):
        lines.append("hmult %d %s" % (i, hashlib.sha256(np.ascontiguousarray(prod[i]).tobytes()).hexdigest()))
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "keyswitch_micro_digests.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
