"""GPU parity: csr_decode_attn with keys coded before the rotary embedding (rope_base set) against the oracle,
which rebuilds every key by Eq.12, rotates it to its position and runs plain attention in float64."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

# Relative L2 error per (sequence, query head).  On top of the position-free path's budget (fp32 accumulation,
# fp16 output rounding ~3e-4) the scores carry the rounding of the turned-back query to fp16: a relative 2^-11 per
# component with random signs, i.e. about 2^-11 / sqrt(3) * |q~| |K~| / sqrt(d) ~ 1e-4 of a score of order one,
# and the fp32 rotation recurrence (a few hundred steps, ~1e-6).
TOL = 2e-3


def _case(seed, B, Hq, Hkv, T, N, sK, sV, snV=1):
    d = 128
    q = synth.queries(seed, B, Hq, d, "f16")
    DK = synth.dictionary(seed, "dict_k", Hkv, N, d, "f16")
    idxK, coefK = synth.random_codes(seed, 0, B, Hkv, T, sK, N, "f16", "i16")
    if snV == 1:
        DV = synth.dictionary(seed, "dict_v", Hkv, N, d, "f16")
        idxV, coefV = synth.random_codes(seed, 1, B, Hkv, T, sV, N, "f16", "i16")
    else:
        DV = synth.dictionary(seed, "dict_v", Hkv * snV, N, d // snV, "f16").reshape(Hkv, snV, N, d // snV)
        idxV, coefV = synth.random_codes(seed, 1, B, Hkv, T, snV * sV, N, "f16", "i16")
        idxV = np.ascontiguousarray(idxV.reshape(B, Hkv, T, snV, sV))
        coefV = np.ascontiguousarray(coefV.reshape(B, Hkv, T, snV, sV))
    return q, DK, idxK, coefK, DV, idxV, coefV


def _run(args, base, layout, pos0, seq_lens=None, scale=0.0):
    g = lambda a: torch.from_numpy(a).cuda()  # noqa: E731
    sl = None if seq_lens is None else torch.from_numpy(np.asarray(seq_lens, dtype=np.int32)).cuda()
    out = csr.csr_decode_attn(*[g(a) for a in args], scale=scale, seq_lens=sl, rope_base=base, rope_layout=layout,
                              rope_pos0=pos0)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _check(out, ref, what):
    rel, mx = parity.assert_decode_close(out, ref, TOL, what)
    print(f"[rope decode parity] {what} max rel L2 {rel.max():.2e}, max element error / peak {mx:.2e}", flush=True)


@pytest.mark.parametrize("B,Hq,Hkv,T,N,sK,sV,snV,layout,pos0", [
    (2, 4, 4, 1500, 768, 8, 8, 1, 0, 0),        # 16384 + 8192 atoms over 32 heads (the appendix's largest setting): 768 per head
    (1, 8, 2, 2100, 4096, 8, 8, 1, 0, 11),      # the benchmark's dictionaries, query groups of 4, rotate-half pairs
    (2, 2, 2, 1025, 4096, 16, 4, 1, 1, 5000),   # interleaved pairs, two blocks of 8 key pairs
    (1, 2, 1, 700, 1024, 4, 8, 2, 1, 3),        # groups of 2, 4 key pairs per token, values in two chunks
    (1, 3, 3, 3000, 8192, 16, 16, 1, 0, 100000),  # the long-context dictionaries, far positions
])
def test_rotary_keys_with_dictionaries_beyond_the_lds(B, Hq, Hkv, T, N, sK, sV, snV, layout, pos0):
    # larger key dictionaries than the LDS holds: the same arithmetic on rows gathered from device memory
    args = _case(77, B, Hq, Hkv, T, N, sK, sV, snV)
    lens = np.full(B, T, dtype=np.int32)
    lens[-1] = max(1, T - 333)
    out = _run(args, 10000.0, layout, pos0, seq_lens=lens)
    ref = oracle.decode_attn_rope(*args, 10000.0, layout, pos0, seq_lens=lens)
    _check(out, ref, f"gathered rows: B{B} Hq{Hq} Hkv{Hkv} T{T} N{N} sK{sK} sV{sV} snV{snV} layout{layout} pos0 {pos0}")


@pytest.mark.parametrize("B,Hq,Hkv,T,N,sK,sV,snV,layout,pos0", [
    (2, 4, 4, 3000, 512, 8, 8, 1, 0, 0),        # MHA, the largest resident dictionary, three rounds of 1024
    (2, 8, 2, 1500, 256, 8, 4, 1, 1, 17),       # query groups of 4 = two slices of 2, interleaved pairs
    (1, 2, 2, 40000, 256, 8, 8, 1, 0, 100000),  # several chunks, many rounds, positions past 10^5
    (3, 3, 3, 700, 384, 4, 8, 1, 0, 5),         # 4 key pairs per token (8-byte code loads)
    (1, 2, 1, 1, 128, 12, 3, 1, 1, 0),          # a single token; three blocks of 4 key pairs; odd value pairs
    (2, 4, 2, 1025, 512, 16, 8, 1, 0, 0),       # two blocks of 8 key pairs, one token past a round
    (1, 4, 4, 2100, 256, 8, 4, 2, 0, 3),        # the experiments' cache: keys whole s = 8, values s = 4 in 2 chunks
    (70, 2, 1, 130, 256, 8, 8, 1, 1, 1000),     # many short sequences, a ragged wave
])
def test_rotary_keys_shapes(B, Hq, Hkv, T, N, sK, sV, snV, layout, pos0):
    args = _case(30, B, Hq, Hkv, T, N, sK, sV, snV)
    out = _run(args, 10000.0, layout, pos0)
    ref = oracle.decode_attn_rope(*args, 10000.0, layout, pos0)
    _check(out, ref, f"B{B} Hq{Hq} Hkv{Hkv} T{T} N{N} s{sK}/{sV} snV{snV} layout{layout} pos0 {pos0}")


def test_rotary_keys_sequence_lengths_base_and_scale():
    B, T = 5, 2600
    args = _case(31, B, 4, 2, T, 256, 8, 8)
    lens = np.array([T, 0, 1, 1024, 2047], dtype=np.int32)
    out = _run(args, 500000.0, 0, 64, seq_lens=lens, scale=0.05)
    ref = oracle.decode_attn_rope(*args, 500000.0, 0, 64, scale=0.05, seq_lens=lens)
    assert np.all(out[1] == 0)
    _check(out, ref, "seq_lens, base 5e5, scale 0.05")


def test_rotation_matters_and_single_position_equals_plain_path():
    # one cached token at position 0 is not rotated at all: both paths must agree to the bit
    args = _case(32, 3, 4, 2, 1, 256, 8, 8)
    g = lambda a: torch.from_numpy(a).cuda()  # noqa: E731
    plain = csr.csr_decode_attn(*[g(a) for a in args]).cpu().numpy()
    roped = _run(args, 10000.0, 0, 0)
    np.testing.assert_array_equal(plain, roped)
    # with a real context the rotation changes the result (so the test above cannot pass by ignoring it)
    args = _case(32, 1, 2, 2, 500, 256, 8, 8)
    plain = csr.csr_decode_attn(*[g(a) for a in args]).cpu().numpy().astype(np.float64)
    roped = _run(args, 10000.0, 0, 0).astype(np.float64)
    assert np.abs(plain - roped).max() > 1e-2


def test_keys_encoded_before_rotation_end_to_end():
    # keys drawn, encoded on the GPU as they are (before any rotation), then attended with rotation: close to
    # dense attention over the rotated keys themselves, as far as s = 8 atoms can carry a key
    B, H, T, N, s = 1, 2, 1500, 512, 8
    DK = synth.dictionary(33, "dict_k", H, N, 128, "f16")
    DV = synth.dictionary(33, "dict_v", H, N, 128, "f16")
    XK = synth.vectors(33, "keys", H, T, 128, "f16")
    XV = synth.vectors(33, "values", H, T, 128, "f16")
    q = synth.queries(33, B, H, 128, "f16")
    g = lambda a: torch.from_numpy(a).cuda()  # noqa: E731
    iK, cK = csr.csr_encode(g(XK), g(DK), s)
    iV, cV = csr.csr_encode(g(XV), g(DV), s)
    out = csr.csr_decode_attn(g(q), g(DK), iK[None], cK[None], g(DV), iV[None], cV[None], rope_base=10000.0)
    torch.cuda.synchronize()
    codes = [a.cpu().numpy()[None] for a in (iK, cK, iV, cV)]
    ref = oracle.decode_attn_rope(q, DK, codes[0], codes[1], DV, codes[2], codes[3], 10000.0)
    _check(out.cpu().numpy(), ref, "end to end")
    # dense attention on the rotated uncompressed keys
    dense = np.zeros((B, H, 128))
    for h in range(H):
        K = oracle.rope_rotate(XK[h].astype(np.float64), np.arange(T), 10000.0, 0)
        sc = (K @ q[0, h].astype(np.float64)) / np.sqrt(128.0)
        p = np.exp(sc - sc.max())
        dense[0, h] = (p / p.sum()) @ XV[h].astype(np.float64)
    assert np.linalg.norm(ref - dense) < np.linalg.norm(dense)  # loose: sanity only


@pytest.mark.parametrize("shape,picks", [("rope_mha_32heads", [(0, 0), (3, 31), (2, 17)]),
                                         ("rope_gqa_8x4heads", [(0, 0), (7, 7), (4, 3)])])
def test_bench_shapes_full_launch_sampled(shape, picks):
    """The whole configuration bench.py times in one call (random codes drawn on the GPU, keys whole with s = 8,
    values in two chunks with s = 4, 32768 tokens at positions from 1000 on); the oracle recomputes the sampled
    (sequence, KV head) pairs from the bits copied back."""
    import bench
    sh = next(x for x in bench.ROPE_SHAPES if x["name"] == shape)
    B, Hq, Hkv, T, N, sK, sV, snV = (sh[k] for k in ("B", "Hq", "Hkv", "T", "N", "sK", "sV", "snV"))
    G, d = Hq // Hkv, 128
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(21)
    unit = lambda *s_: (lambda a: (a / a.norm(dim=-1, keepdim=True)).half())(torch.randn(*s_, device=dev, generator=gen))
    ri = lambda *s_: torch.randint(0, N, s_, device=dev, generator=gen, dtype=torch.int32).to(torch.int16)
    rc = lambda *s_: (torch.randn(*s_, device=dev, generator=gen) * 3).half()
    q, DK, DV = torch.randn(B, Hq, d, device=dev, generator=gen).half(), unit(Hkv, N, d), unit(Hkv, snV, N, d // snV)
    iK, cK, iV, cV = ri(B, Hkv, T, sK), rc(B, Hkv, T, sK), ri(B, Hkv, T, snV, sV), rc(B, Hkv, T, snV, sV)
    out = csr.csr_decode_attn(q, DK, iK, cK, DV, iV, cV, rope_base=10000.0, rope_pos0=1000)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    h_ = lambda t: t.cpu().numpy()
    for b, h in picks:
        print(f"[rope full launch] {shape} sequence {b} KV head {h}", flush=True)
        ref = oracle.decode_attn_rope(h_(q[b:b + 1, h * G:(h + 1) * G]), h_(DK[h:h + 1]), h_(iK[b:b + 1, h:h + 1]),
                                      h_(cK[b:b + 1, h:h + 1]), h_(DV[h:h + 1]), h_(iV[b:b + 1, h:h + 1]),
                                      h_(cV[b:b + 1, h:h + 1]), 10000.0, 0, 1000)
        _check(h_(out[b:b + 1, h * G:(h + 1) * G]), ref, f"{shape} full launch, sequence {b} KV head {h}")
