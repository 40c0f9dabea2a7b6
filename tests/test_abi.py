"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad descriptors before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2412_11741_amd as csr
from paper_2412_11741_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "csr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(csr_[a-z0-9_]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = csr.lib()
    names = _declared_functions()
    assert names == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.csr_version() == 100


def test_code_bytes_follow_the_papers_accounting():
    # s * s_n * (index bytes + coefficient bytes); fp16 + int16 -> 4 bytes a pair
    import torch
    assert csr.csr_code_bytes(8) == 32 and csr.csr_code_bytes(4, 2) == 32 and csr.csr_code_bytes(16) == 64
    assert csr.csr_code_bytes(8, 1, torch.int32, torch.float32) == 64
    assert csr.lib().csr_code_bytes(0, 1, 1, 1) == 0


def _enc(**kw):
    base = dict(H=2, T=100, d=128, N=256, s=8, x_dtype=B.CSR_F16, dict_dtype=B.CSR_F16,
                coef_dtype=B.CSR_F16, idx_dtype=B.CSR_I16, x_stride_h=0, x_stride_t=0, dict_count=0,
                code_stride_h=0, algo=0, flags=0)
    base.update(kw)
    return B.EncodeDesc(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(H=-1), B.CSR_ERR_INVALID_ARG), (dict(T=-5), B.CSR_ERR_INVALID_ARG),
    (dict(s=0), B.CSR_ERR_INVALID_ARG), (dict(s=33), B.CSR_ERR_INVALID_ARG),
    (dict(N=0), B.CSR_ERR_INVALID_ARG), (dict(N=70000), B.CSR_ERR_INVALID_ARG),
    (dict(x_dtype=7), B.CSR_ERR_INVALID_ARG), (dict(idx_dtype=3), B.CSR_ERR_INVALID_ARG),
    (dict(flags=2), B.CSR_ERR_INVALID_ARG), (dict(flags=5), B.CSR_ERR_INVALID_ARG), (dict(algo=9), B.CSR_ERR_INVALID_ARG),
    (dict(flags=1, N=256, algo=B.CSR_ENCODE_GRAM), B.CSR_ERR_UNSUPPORTED),
    (dict(x_stride_t=100), B.CSR_ERR_INVALID_ARG), (dict(x_stride_t=132), B.CSR_ERR_INVALID_ARG),
    (dict(x_stride_t=256, x_stride_h=128), B.CSR_ERR_INVALID_ARG),
    (dict(d=100), B.CSR_ERR_UNSUPPORTED), (dict(dict_dtype=B.CSR_F32), B.CSR_ERR_UNSUPPORTED),
    (dict(d=16, algo=B.CSR_ENCODE_MFMA), B.CSR_ERR_UNSUPPORTED),
    (dict(s_n=3), B.CSR_ERR_INVALID_ARG), (dict(s_n=16), B.CSR_ERR_INVALID_ARG), (dict(s_n=-1), B.CSR_ERR_INVALID_ARG),
    (dict(s_n=8), B.CSR_ERR_UNSUPPORTED),                              # chunks of 16 dimensions
    (dict(dict_count=-1), B.CSR_ERR_INVALID_ARG), (dict(H=6, dict_count=4), B.CSR_ERR_INVALID_ARG),
    (dict(code_stride_h=-8), B.CSR_ERR_INVALID_ARG), (dict(code_stride_h=792), B.CSR_ERR_INVALID_ARG),   # < T*s = 800
    (dict(T=200, algo=B.CSR_ENCODE_SPLIT), B.CSR_ERR_UNSUPPORTED), (dict(d=32, T=1, algo=B.CSR_ENCODE_SPLIT), B.CSR_ERR_UNSUPPORTED),
    (dict(s_n=4, algo=B.CSR_ENCODE_RESIDENT), B.CSR_ERR_UNSUPPORTED),  # chunks of 32: matrix-core or vector-ALU encoder
    (dict(x_dtype=B.CSR_F32, dict_dtype=B.CSR_F32, algo=B.CSR_ENCODE_MFMA), B.CSR_ERR_UNSUPPORTED),
    (dict(N=512, algo=B.CSR_ENCODE_GRAM), B.CSR_ERR_UNSUPPORTED),      # the Gram matrix has to fit the LDS
    (dict(N=200, algo=B.CSR_ENCODE_GRAM), B.CSR_ERR_UNSUPPORTED), (dict(N=256, d=32, algo=B.CSR_ENCODE_GRAM), B.CSR_ERR_UNSUPPORTED),
    (dict(N=256, x_dtype=B.CSR_F32, dict_dtype=B.CSR_F32, algo=B.CSR_ENCODE_GRAM), B.CSR_ERR_UNSUPPORTED),
])
def test_encode_rejects_bad_descriptors_before_launch(kw, status):
    lib = csr.lib()
    d = _enc(**kw)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    assert lib.csr_encode(ctypes.byref(d), fake, fake, fake, fake, None, 0, None) == status
    assert csr.last_error() != ""
    assert lib.csr_encode_workspace_bytes(ctypes.byref(d)) == ctypes.c_size_t(-1).value


def test_encode_chunk_count_scales_the_workspace_and_zero_means_whole_vectors():
    lib = csr.lib()
    size = lambda **kw: lib.csr_encode_workspace_bytes(ctypes.byref(_enc(algo=B.CSR_ENCODE_MFMA, **kw)))
    assert size(s_n=0) == size(s_n=1) == size() > 0
    assert size(H=64, s_n=2) == size(H=128) and size(H=64, s_n=2) > size(H=64)   # one norm record per dictionary
    assert size(d=64) > 0 and size(d=256, s_n=2) > 0                           # fp16 chunks of 64 / 128: matrix cores
    assert size(H=64, dict_count=8) == size(H=8)                               # shared dictionaries: fewer records
    assert size(s_n=4) > 0 and size(d=32) > 0                                  # ... and of 32 (s_n = 4 of a 128-dim head)
    assert size(H=64, s_n=4) == size(H=256)


def test_encode_kernel_choice_follows_the_vectors_per_dictionary_and_the_dictionary_size():
    lib = csr.lib()
    size = lambda **kw: lib.csr_encode_workspace_bytes(ctypes.byref(_enc(**kw)))
    big = dict(N=4096)      # 1 MB of atoms: beyond the LDS
    # few vectors per dictionary (a decoding step): AUTO is the split encoder, whose scratch holds residuals
    assert size(T=1, **big) == size(T=1, algo=B.CSR_ENCODE_SPLIT, **big) != size(T=1, algo=B.CSR_ENCODE_MFMA, **big)
    assert size(T=128, **big) == size(T=128, algo=B.CSR_ENCODE_SPLIT, **big)
    assert size(T=129, **big) == size(T=129, algo=B.CSR_ENCODE_MFMA, **big) > 0
    # 16 blocks on 2 dictionaries: 8 x 20 = 160 vectors per dictionary, too many for the split encoder
    assert size(H=16, T=20, dict_count=2, **big) == size(H=16, T=20, dict_count=2, algo=B.CSR_ENCODE_MFMA, **big)
    assert size(H=16, T=20, dict_count=2, algo=B.CSR_ENCODE_SPLIT, **big) == ctypes.c_size_t(-1).value
    assert size(H=16, T=20, dict_count=4, **big) == size(H=16, T=20, dict_count=4, algo=B.CSR_ENCODE_SPLIT, **big)
    assert size(T=1, x_dtype=B.CSR_F32, dict_dtype=B.CSR_F32) == 0            # fp32: vector-ALU encoder
    # many vectors on a dictionary that fits the LDS (128 KB): the resident encoder, which needs no scratch
    assert size(T=1000, N=512) == size(T=1000, N=512, algo=B.CSR_ENCODE_RESIDENT) == 0
    assert size(T=1000, N=512, algo=B.CSR_ENCODE_MFMA) > 0
    assert size(T=1000, N=544) == size(T=1000, N=544, algo=B.CSR_ENCODE_MFMA) > 0
    assert size(T=1000, N=544, algo=B.CSR_ENCODE_RESIDENT) == ctypes.c_size_t(-1).value
    assert size(T=1000, N=1024, d=64) == 0 and size(T=1000, N=1056, d=64) > 0  # 64-dimensional atoms: twice as many fit


def test_gram_matrices_in_the_descriptor_select_the_decoding_step_gram_encoder():
    lib = csr.lib()
    G = 0x2000
    size = lambda **kw: lib.csr_encode_workspace_bytes(ctypes.byref(_enc(**kw)))
    bad = ctypes.c_size_t(-1).value
    big = dict(N=4096)
    # scratch: C_1 (N floats per vector) and the slices' norm records; by default whenever gram is given and fits
    want = 2 * 1 * 4096 * 4 + 256
    assert size(T=1, gram=G, **big) == size(T=1, gram=G, algo=B.CSR_ENCODE_GRAM, **big) == want
    assert size(T=16, gram=G, **big) == 2 * 16 * 4096 * 4 + 256
    assert size(T=1, gram=G, **big) != size(T=1, **big)                       # (the split encoder's is another)
    # more than 128 vectors per dictionary: refused when asked for, otherwise the encoder the shape would get anyway
    assert size(T=129, gram=G, algo=B.CSR_ENCODE_GRAM, **big) == bad and "at most 128 vectors" in csr.last_error()
    assert size(T=129, gram=G, **big) == size(T=129, **big)
    assert size(H=8, T=4, dict_count=2, gram=G, **big) == 2 * 16 * 4096 * 4 + 256
    assert size(H=8, T=33, dict_count=2, gram=G, algo=B.CSR_ENCODE_GRAM, **big) == bad
    # other explicit kernels ignore the matrices; without them GRAM is the LDS form with its 256 atoms
    assert size(T=1, gram=G, algo=B.CSR_ENCODE_SPLIT, **big) == size(T=1, algo=B.CSR_ENCODE_SPLIT, **big)
    assert size(T=1, algo=B.CSR_ENCODE_GRAM, **big) == bad
    assert size(T=1, N=16384, gram=G) > 0 and size(T=1, N=16416, gram=G, algo=B.CSR_ENCODE_GRAM) == bad
    assert size(T=1, gram=G, x_dtype=B.CSR_F32, dict_dtype=B.CSR_F32, algo=B.CSR_ENCODE_GRAM) == bad
    assert size(T=1, d=256, s_n=2, gram=G, **big) == 2 * 2 * 4096 * 4 + 256   # a Gram matrix per chunk dictionary
    # the matrices' pointer is checked like the others
    ok = ctypes.c_void_p(0x1000)
    d = _enc(T=1, gram=0x2004, **big)
    ws = ctypes.c_void_p(0x4000)
    assert lib.csr_encode(ctypes.byref(d), ok, ok, ok, ok, ws, 1 << 20, None) == B.CSR_ERR_INVALID_ARG
    assert "gram" in csr.last_error()
    assert lib.csr_encode(ctypes.byref(_enc(T=1, gram=G, **big)), ok, ok, ok, ok, None, 0, None) == B.CSR_ERR_WORKSPACE


def test_gram_build_arguments():
    lib = csr.lib()
    assert lib.csr_gram_bytes(64, 4096) == 64 * 4096 * 4096 * 2 and lib.csr_gram_bytes(0, 4096) == 0
    assert lib.csr_gram_bytes(-1, 4096) == ctypes.c_size_t(-1).value
    p = ctypes.c_void_p(0x1000)
    assert lib.csr_gram_build(p, 2, 100, 128, p, None) == B.CSR_ERR_UNSUPPORTED      # N a multiple of 32
    assert lib.csr_gram_build(p, 2, 256, 32, p, None) == B.CSR_ERR_UNSUPPORTED       # rows of 64 or 128 elements
    assert lib.csr_gram_build(p, 2, 16416, 128, p, None) == B.CSR_ERR_UNSUPPORTED
    assert lib.csr_gram_build(p, 70000, 256, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_gram_build(None, 2, 256, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_gram_build(p, 2, 256, 128, ctypes.c_void_p(0x1008), None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_gram_build(None, 0, 256, 128, None, None) == B.CSR_OK


def test_encode_null_and_misaligned_pointers_and_noop_sizes():
    lib = csr.lib()
    d = _enc()
    ok = ctypes.c_void_p(0x1000)
    assert lib.csr_encode(None, ok, ok, ok, ok, None, 0, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_encode(ctypes.byref(d), None, ok, ok, ok, None, 0, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_encode(ctypes.byref(d), ctypes.c_void_p(0x1004), ok, ok, ok, None, 0, None) == B.CSR_ERR_INVALID_ARG
    # codes: aligned to their element size (a row of a cache of 16-bit codes may start at any even address)
    odd, even = ctypes.c_void_p(0x1001), ctypes.c_void_p(0x1002)
    assert lib.csr_encode(ctypes.byref(d), ok, ok, odd, ok, None, 0, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_encode(ctypes.byref(d), ok, ok, even, even, None, 0, None) == B.CSR_ERR_WORKSPACE   # passed the pointer checks
    d32 = _enc(idx_dtype=B.CSR_I32, coef_dtype=B.CSR_F32)
    assert lib.csr_encode(ctypes.byref(d32), ok, ok, even, ok, None, 0, None) == B.CSR_ERR_INVALID_ARG
    # empty problems are a no-op and touch nothing, even with NULL pointers
    assert lib.csr_encode(ctypes.byref(_enc(T=0)), None, None, None, None, None, 0, None) == B.CSR_OK
    assert lib.csr_encode(ctypes.byref(_enc(H=0)), None, None, None, None, None, 0, None) == B.CSR_OK


def _dec(**kw):
    base = dict(B=2, Hq=8, Hkv=2, T=1000, d=128, N=4096, sK=8, sV=8, scale=0.0, q_dtype=B.CSR_F16,
                dict_dtype=B.CSR_F16, coef_dtype=B.CSR_F16, idx_dtype=B.CSR_I16, out_dtype=B.CSR_F16, flags=0)
    base.update(kw)
    return B.DecodeDesc(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(B=-1), B.CSR_ERR_INVALID_ARG), (dict(T=-1), B.CSR_ERR_INVALID_ARG),
    (dict(Hq=7), B.CSR_ERR_INVALID_ARG), (dict(Hkv=0), B.CSR_ERR_INVALID_ARG),
    (dict(sK=0), B.CSR_ERR_INVALID_ARG), (dict(sV=40), B.CSR_ERR_INVALID_ARG),
    (dict(N=0), B.CSR_ERR_INVALID_ARG), (dict(N=65537), B.CSR_ERR_INVALID_ARG),
    (dict(scale=-1.0), B.CSR_ERR_INVALID_ARG), (dict(scale=float("nan")), B.CSR_ERR_INVALID_ARG),
    (dict(out_dtype=5), B.CSR_ERR_INVALID_ARG), (dict(flags=2), B.CSR_ERR_INVALID_ARG),
    (dict(d=64), B.CSR_ERR_UNSUPPORTED), (dict(Hq=32, Hkv=2), B.CSR_ERR_UNSUPPORTED),
    (dict(N=60000, Hq=2), B.CSR_ERR_UNSUPPORTED),
    (dict(snV=3), B.CSR_ERR_INVALID_ARG), (dict(snK=16), B.CSR_ERR_INVALID_ARG), (dict(snK=-2), B.CSR_ERR_INVALID_ARG),
    (dict(snV=2, q_dtype=B.CSR_F32), B.CSR_ERR_UNSUPPORTED), (dict(snV=2, dict_dtype=B.CSR_F32), B.CSR_ERR_UNSUPPORTED),
    (dict(snK=2, N=4000), B.CSR_ERR_UNSUPPORTED), (dict(snV=8, sV=8), B.CSR_ERR_UNSUPPORTED),
    (dict(snV=8, N=8192, Hq=2), B.CSR_ERR_UNSUPPORTED),   # 8 x 8192 histogram bins of 8 bytes exceed the LDS
    # keys coded before the rotary embedding: the key dictionary has to fit the LDS, paper's storage types only
    (dict(rope_base=10000.0, N=70000, idx_dtype=B.CSR_I16), B.CSR_ERR_INVALID_ARG),
    (dict(rope_base=10000.0, N=512, sK=6), B.CSR_ERR_UNSUPPORTED),
    (dict(rope_base=10000.0, N=512, snK=2, sK=4), B.CSR_ERR_UNSUPPORTED),
    (dict(rope_base=10000.0, N=512, coef_dtype=B.CSR_F32), B.CSR_ERR_UNSUPPORTED),
    (dict(rope_base=10000.0, N=512, idx_dtype=B.CSR_I32), B.CSR_ERR_UNSUPPORTED),
    (dict(rope_base=1.0, N=512), B.CSR_ERR_INVALID_ARG), (dict(rope_base=-3.0, N=512), B.CSR_ERR_INVALID_ARG),
    (dict(rope_base=float("inf"), N=512), B.CSR_ERR_INVALID_ARG),
    (dict(rope_base=10000.0, N=512, rope_layout=2), B.CSR_ERR_INVALID_ARG),
    (dict(rope_base=10000.0, N=512, rope_pos0=-1), B.CSR_ERR_INVALID_ARG),
    (dict(rope_layout=1), B.CSR_ERR_INVALID_ARG), (dict(rope_pos0=5), B.CSR_ERR_INVALID_ARG),   # set without rope_base
])
def test_decode_rejects_bad_descriptors_before_launch(kw, status):
    lib = csr.lib()
    d = _dec(**kw)
    p = ctypes.c_void_p(0x1000)
    assert lib.csr_decode_attn(ctypes.byref(d), p, p, p, p, p, p, p, None, p, p, 1 << 40, None) == status
    assert lib.csr_decode_workspace_bytes(ctypes.byref(d)) == ctypes.c_size_t(-1).value


def test_decode_workspace_is_required_and_checked():
    lib = csr.lib()
    d = _dec()
    need = lib.csr_decode_workspace_bytes(ctypes.byref(d))
    assert 0 < need < 1 << 32
    p = ctypes.c_void_p(0x1000)
    assert lib.csr_decode_attn(ctypes.byref(d), p, p, p, p, p, p, p, None, p, None, 0, None) == B.CSR_ERR_WORKSPACE
    assert lib.csr_decode_attn(ctypes.byref(d), p, p, p, p, p, p, p, None, p, p, need - 1, None) == B.CSR_ERR_WORKSPACE
    assert lib.csr_decode_attn(ctypes.byref(d), p, p, p, p, p, p, p, None, p, ctypes.c_void_p(0x1010), need, None) == B.CSR_ERR_WORKSPACE
    assert lib.csr_decode_attn(ctypes.byref(d), None, p, p, p, p, p, p, None, p, p, need, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_decode_attn(ctypes.byref(_dec(B=0)), None, None, None, None, None, None, None, None, None, None, 0, None) == B.CSR_OK


def test_decode_accepts_rotary_descriptors_within_the_resident_limit():
    lib = csr.lib()
    for kw in (dict(N=512), dict(N=256, Hq=2, Hkv=2, sK=4), dict(N=128, snV=2, sV=4, rope_layout=1, rope_pos0=1 << 30),
               dict(N=768), dict(N=4096, Hq=4, Hkv=1), dict(N=8192, sK=16, sV=16)):   # beyond the LDS: gathered rows
        need = lib.csr_decode_workspace_bytes(ctypes.byref(_dec(rope_base=10000.0, **kw)))
        assert 0 < need < 1 << 32, kw


def test_decode_accepts_one_long_sequence_up_to_the_token_limit():
    # few (sequence, head) pairs and a long context: the token axis is cut into the most chunks the plan allows
    lib = csr.lib()
    for kw in (dict(B=1, Hq=1, Hkv=1, T=1 << 20), dict(B=1, Hq=8, Hkv=8, T=300000),
               dict(B=1, Hq=2, Hkv=2, T=40000, N=256, rope_base=10000.0)):
        need = lib.csr_decode_workspace_bytes(ctypes.byref(_dec(**kw)))
        assert 0 < need < 1 << 34, kw
    # the rotary kernel keeps a score per round in registers: its chunks hold fewer tokens (the header states the limits)
    none = ctypes.c_size_t(-1).value
    rope = lambda **kw: lib.csr_decode_workspace_bytes(ctypes.byref(_dec(N=256, rope_base=1e4, **kw)))
    assert rope(B=1, Hq=1, Hkv=1, T=1 << 20) != none and rope(Hq=2, Hkv=2, T=1 << 20) != none
    assert rope(Hq=8, Hkv=2, T=1 << 19) != none and rope(Hq=8, Hkv=2, T=(1 << 19) + 1) == none
    # four query heads per KV head and workgroup keep 8 rounds of 1024 tokens per chunk, 128 chunks: the whole 2^20
    assert lib.csr_decode_workspace_bytes(ctypes.byref(_dec(B=1, Hq=4, Hkv=1, T=1 << 20))) != none


def test_decode_workspace_grows_with_the_chunk_count_and_zero_means_one_chunk():
    lib = csr.lib()
    size = lambda **kw: lib.csr_decode_workspace_bytes(ctypes.byref(_dec(**kw)))
    assert size(snK=0, snV=0) == size(snK=1, snV=1) == size()
    assert size(sV=4, snV=2) > size(sV=4)   # two histograms' worth of bins per query head
    assert size(sK=4, snK=2) > size(sK=4)   # twice the score table


def test_reconstruct_rejects_bad_descriptors():
    lib = csr.lib()
    base = dict(H=2, T=10, d=128, N=256, s=8, s_n=1, dict_dtype=B.CSR_F16, coef_dtype=B.CSR_F16, idx_dtype=B.CSR_I16,
                out_dtype=B.CSR_F16, dict_count=0, code_stride_h=0, out_stride_h=0, out_stride_t=0, flags=0)
    p = ctypes.c_void_p(0x1000)
    for kw in (dict(s=0), dict(s=33), dict(d=100), dict(d=2048), dict(s_n=3), dict(dict_count=3), dict(N=0),
               dict(N=70000), dict(code_stride_h=79), dict(out_stride_t=120), dict(out_stride_t=132), dict(flags=1),
               dict(out_dtype=7)):
        d = B.ReconstructDesc(**{**base, **kw})
        assert lib.csr_reconstruct(ctypes.byref(d), p, p, p, p, None) == B.CSR_ERR_INVALID_ARG, kw
    assert lib.csr_reconstruct(ctypes.byref(B.ReconstructDesc(**{**base, "T": 0})), None, None, None, None, None) == B.CSR_OK
    assert lib.csr_reconstruct(ctypes.byref(B.ReconstructDesc(**base)), None, p, p, p, None) == B.CSR_ERR_INVALID_ARG


def test_atom_norms2_rejects_bad_arguments():
    lib = csr.lib()
    p = ctypes.c_void_p(0x1000)
    assert lib.csr_atom_norms2(p, 7, 10, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_atom_norms2(p, B.CSR_F16, -1, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_atom_norms2(p, B.CSR_F16, 10, 0, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_atom_norms2(p, B.CSR_F16, 10, 70000, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_atom_norms2(None, B.CSR_F16, 10, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert lib.csr_atom_norms2(ctypes.c_void_p(0x1002), B.CSR_F32, 10, 128, p, None) == B.CSR_ERR_INVALID_ARG
    assert b"misaligned" in lib.csr_last_error()
    assert lib.csr_atom_norms2(None, B.CSR_F16, 0, 128, None, None) == B.CSR_OK


def test_binding_refuses_cpu_tensors():
    import torch
    X = torch.zeros(1, 4, 128, dtype=torch.float16)
    D = torch.zeros(1, 32, 128, dtype=torch.float16)
    with pytest.raises(ValueError, match="GPU tensor"):
        csr.csr_encode(X, D, 4)


def test_the_header_is_plain_c99():
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    prog = '#include "csr.h"\nint main(void) { csr_encode_desc e; csr_decode_desc d; csr_reconstruct_desc r; (void)e; (void)d; (void)r; return 0; }\n'
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I",
                        os.path.join(root, "include"), "-x", "c", "-"], input=prog, text=True, capture_output=True)
    assert r.returncode == 0, r.stderr
