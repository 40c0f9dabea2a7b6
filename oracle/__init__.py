"""CPU oracle of the CSR hot path.  Test infrastructure only; see csr_oracle.c."""
from .csr_oracle import (code_bytes, compression_ratio, decode_attn, decode_attn_chunked, decode_attn_rope,  # noqa: F401
                         equivalent_bits, max_threads, mp_encode, mp_encode_chunked, mp_encode_heads,
                         reconstruct, rope_rotate)
