"""Shapes of the benchmark / parity workloads (primes by bit-size, digit count, batch)."""
from .params import make_params

# name -> dict(logN, nq, q_bits, np, p_bits, dnum, batch)
CONFIGS = {
    # tiny HRot batch, literal: one 50-bit special prime for two 2-limb digits
    "tiny_hrot": dict(logN=12, nq=4, q_bits=40, np=1, p_bits=50, dnum=2, batch=8),
    # noise-sound variants of the tiny case used for the decrypt checks
    "tiny_hrot_k2": dict(logN=12, nq=4, q_bits=40, np=2, p_bits=50, dnum=2, batch=8),
    "tiny_hrot_d4": dict(logN=12, nq=4, q_bits=40, np=1, p_bits=50, dnum=4, batch=8),
    # key-switch microbenchmark (the headline metric's workload); also the FFN layer's ring
    "keyswitch_micro": dict(logN=16, nq=24, q_bits=50, np=8, p_bits=60, dnum=3, batch=64),
    # attention QK^T ring
    "attention_qk": dict(logN=16, nq=20, q_bits=50, np=5, p_bits=60, dnum=4, batch=32),
}

_cache = {}


def config_params(name):
    if name not in _cache:
        c = CONFIGS[name]
        _cache[name] = make_params(c["logN"], c["nq"], c["q_bits"], c["np"], c["p_bits"], c["dnum"])
    return _cache[name]
