"""MI355X-native batched RNS-CKKS polynomial arithmetic: thin Python binding over the C-ABI HIP library.

The package only marshals arguments (tensor data pointers, sizes, the current HIP stream) into
libckks_mi355.so. It has no CPU fallback: importing `binding` fails if the library is missing.
"""
from .binding import (Context, CkksError, ckks_ntt, ckks_intt, ckks_automorph, ckks_keyswitch, ckks_hrot,
                      ckks_hmult_relin, ckks_pcmm_bsgs, ckks_hrot_hoisted, ckks_hrot_multi, ckks_hrot_add, ckks_hrot_sum, ckks_hrot_noalloc,
                      ckks_noalloc_scratch_bytes, ckks_tensor_acc, ckks_relin, ckks_pcmm_bsgs_hoisted, ckks_pcmm_bsgs_double_hoisted, ckks_rescale, ckks_pmult, ckks_add, ckks_workspace_bytes, ckks_prof_enable, ckks_tune_set, ckks_prof_reset, ckks_prof_collect, ckks_prof_copy, library_path, exported_symbols,
                      OP_KEYSWITCH, OP_HROT, OP_HMULT_RELIN, OP_PCMM_BSGS, OP_RESCALE, OP_PCMM_BSGS_DH, OP_HROT_SUM)
