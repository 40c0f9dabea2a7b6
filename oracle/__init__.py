"""CPU oracle of the CSR hot path.  Test infrastructure only; see csr_oracle.c."""
from .csr_oracle import (code_bytes, compression_ratio, decode_attn, equivalent_bits,  # noqa: F401
                         max_threads, mp_encode, mp_encode_heads, reconstruct)
