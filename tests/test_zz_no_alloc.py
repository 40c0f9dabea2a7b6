"""csr_decode_attn_static - the entry point for callers that cannot allocate - against csr_decode_attn.

Same kernels on the library's static device scratch instead of a caller's workspace: the outputs must be the same
bits, on two calls in a row, the second on a smaller input (the scratch then still holds the first call's partial
results), and a shape beyond the static scratch must be refused with a status, not run.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


def _case(seed, B, Hq, Hkv, T, N, sK, sV):
    d = 128
    g = lambda a: torch.from_numpy(a).cuda()
    q = synth.queries(seed, B, Hq, d, "f16")
    DK = synth.dictionary(seed, "dict_k", Hkv, N, d, "f16")
    DV = synth.dictionary(seed, "dict_v", Hkv, N, d, "f16")
    iK, cK = synth.random_codes(seed, 0, B, Hkv, T, sK, N, "f16", "i16")
    iV, cV = synth.random_codes(seed, 1, B, Hkv, T, sV, N, "f16", "i16")
    host = (q, DK, iK, cK, DV, iV, cV)
    return host, tuple(g(a) for a in host)


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    shapes = [(2, 8, 2, 5000, 4096, 8, 8),     # several chunks, query groups of 4
              (1, 4, 4, 700, 1024, 8, 4)]      # smaller: fewer chunks, fewer atoms, shorter value codes
    for i, (B, Hq, Hkv, T, N, sK, sV) in enumerate(shapes):
        host, dev = _case(900 + i, B, Hq, Hkv, T, N, sK, sV)
        lens = torch.tensor([T] + [max(1, T // 3)] * (B - 1), dtype=torch.int32, device="cuda")
        ref = csr.csr_decode_attn(*dev, seq_lens=lens)
        out = torch.full_like(ref, float("nan"))
        count = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]     # allocations made so far
        before = count()
        got = csr.csr_decode_attn_static(*dev, out=out, seq_lens=lens)
        assert count() == before                                  # nothing came from torch's allocator either
        torch.cuda.synchronize()
        assert got is out and torch.equal(out, ref), f"call {i}: outputs differ"
        want = oracle.decode_attn(*host, seq_lens=lens.cpu().numpy())
        parity.assert_decode_close(out.cpu().numpy(), want, 2e-3, f"static scratch, call {i}")


def test_static_scratch_entry_point_refuses_shapes_beyond_its_scratch():
    B, Hq, Hkv, T, N = 8, 32, 8, 131072, 4096          # needs tens of MB of chunk histograms
    q = torch.zeros(B, Hq, 128, dtype=torch.float16, device="cuda")
    D = torch.zeros(Hkv, N, 128, dtype=torch.float16, device="cuda")
    idx = torch.zeros(B, Hkv, T, 8, dtype=torch.int16, device="cuda")
    coef = torch.zeros(B, Hkv, T, 8, dtype=torch.float16, device="cuda")
    need = csr.csr_decode_workspace_bytes(csr.decode_desc(q, D, idx, coef, idx))
    assert need > csr.STATIC_SCRATCH_BYTES
    with pytest.raises(csr.CsrError, match="static") as err:
        csr.csr_decode_attn_static(q, D, idx, coef, D, idx, coef, out=torch.empty_like(q))
    assert err.value.status == csr.CSR_ERR_WORKSPACE
