"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds parameter selection (primes, roots of unity) and seeded random
draws only. It contains none of the method's polynomial arithmetic (no NTT, no base
conversion, no key switching): both implementations receive the arrays produced here
as plain inputs.
"""
from .params import CkksParams, find_ntt_primes, find_psi, make_params, is_prime
from .gen import (uniform_residues, ternary_secret, gaussian_error, uniform_slots, normal_slots,
                  seeded_rotation_steps, galois_element)
from .configs import CONFIGS, config_params
