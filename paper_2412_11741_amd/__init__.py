"""MI355X-native CSR hot path: Matching Pursuit encode and decode attention on codes.

The product is libcsr_hip.so (C ABI in include/csr.h); this package is its thin binding.
"""
from .binding import (CSR_ERR_DEVICE, CSR_ERR_INVALID_ARG, CSR_ERR_UNSUPPORTED, CSR_ERR_WORKSPACE, CSR_OK, CSR_FLAG_CLOSED_LOOP, STATIC_SCRATCH_BYTES,
                      csr_decode_attn_static, CSR_ENCODE_AUTO, CSR_ENCODE_GRAM, CSR_ENCODE_MFMA, CSR_ENCODE_RESIDENT, CSR_ENCODE_SPLIT, CSR_ENCODE_VALU,
                      CsrError,  # noqa: F401
                      csr_atom_norms2, csr_check_codes, csr_code_bytes, csr_decode_attn, csr_decode_workspace_bytes, csr_encode,
                      csr_encode_workspace_bytes, csr_gram_build, csr_reconstruct, decode_desc, encode_desc, last_error, lib)
