"""CPU oracle (test infrastructure only): see ref_ckks.cpp and ref.py."""
