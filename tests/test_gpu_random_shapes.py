"""GPU parity on seeded random shapes: every encoder that takes the shape, shared dictionaries, chunks, in-place
codes - against the oracle's plain Matching Pursuit per chunk - and the decode call on the resulting codes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

ALGOS = {"valu": csr.CSR_ENCODE_VALU, "mfma": csr.CSR_ENCODE_MFMA, "split": csr.CSR_ENCODE_SPLIT,
         "resident": csr.CSR_ENCODE_RESIDENT, "gram": csr.CSR_ENCODE_GRAM,
         "gram step": csr.CSR_ENCODE_GRAM}   # with the Gram matrices prepared in device memory


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    sn = int(rng.choice([1, 1, 2]))
    dc = int(rng.choice([64, 128]))
    d = dc * sn
    N = 32 * int(rng.integers(1, 40))
    dicts = int(rng.integers(1, 5))
    reps = int(rng.integers(1, 4))
    T = int(rng.choice([1, 2, 7, 33, 70, 300]))
    s = int(rng.integers(1, 10))
    return dict(sn=sn, dc=dc, d=d, N=N, dicts=dicts, H=dicts * reps, T=T, s=s, pad=int(rng.integers(0, 3)))


def _supported(c, algo):
    M = c["H"] // c["dicts"] * c["T"]
    if algo == "split":
        return M <= 128
    if algo == "resident":
        return c["N"] * c["dc"] * 2 <= 128 * 1024
    if algo == "gram":
        return c["N"] <= 256
    if algo == "gram step":
        return M <= 128
    return True


@pytest.mark.parametrize("seed", range(24))
def test_encoders_on_random_shapes(seed):
    c = _draw(seed)
    H, T, N, d, dc, sn, s, dicts = (c[k] for k in ("H", "T", "N", "d", "dc", "sn", "s", "dicts"))
    D = synth.dictionary(200 + seed, "dict_k", dicts * sn, N, dc, "f16").reshape(dicts, sn, N, dc)
    X = synth.vectors(200 + seed, "keys", H, T, d, "f16", outliers=4)
    Dg = torch.from_numpy(D if sn > 1 else D[:, 0]).cuda()
    Xg = torch.from_numpy(X).cuda()
    T_max = T + c["pad"]
    D_blocks = np.stack([D[h % dicts] for h in range(H)])
    results = {}
    for name, algo in ALGOS.items():
        if not _supported(c, name):
            continue
        shape = (H, T_max, sn, s) if sn > 1 else (H, T_max, s)
        ci = torch.full(shape, -1, dtype=torch.int16, device="cuda")
        cc = torch.full(shape, 9.0, dtype=torch.float16, device="cuda")
        rn = torch.empty((H, T, sn) if sn > 1 else (H, T), dtype=torch.float32, device="cuda")
        extra = dict(gram=csr.csr_gram_build(Dg)) if name == "gram step" else {}
        csr.csr_encode(Xg, Dg, s, algo=algo, idx=ci[:, c["pad"]:], coef=cc[:, c["pad"]:], res_norm2=rn, **extra)
        torch.cuda.synchronize()
        assert (ci[:, :c["pad"]] == -1).all() and (cc[:, :c["pad"]] == 9.0).all(), name
        idx = ci[:, c["pad"]:].cpu().numpy().reshape(H, T, sn, s)
        coef = cc[:, c["pad"]:].cpu().numpy().reshape(H, T, sn, s)
        results[name] = idx
        for h in range(H):
            for ch in range(sn):
                Xc = np.ascontiguousarray(X[h][:, ch * dc:(ch + 1) * dc])
                io, co, diag = oracle.mp_encode(Xc, D_blocks[h, ch], s, diagnostics=True)
                rep = parity.check_encode(Xc, D_blocks[h, ch], idx[h][:, ch], coef[h][:, ch], io,
                                          co.astype(np.float16).astype(np.float64), diag, 1e-3, coef_storage="f16",
                                          coef_o_exact=co)
                assert rep.ok, (name, c, h, ch, rep.summary(), rep.failures[:3])
        assert torch.isfinite(rn).all() and (rn >= 0).all(), name
    assert results, c


@pytest.mark.parametrize("seed", range(8))
def test_decode_on_random_shapes_with_chunks(seed):
    rng = np.random.default_rng(3000 + seed)
    B, Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 4]))
    T = int(rng.choice([1, 5, 100, 1025, 3000]))
    N = 128 * int(rng.integers(1, 9))
    snK, snV = int(rng.choice([1, 2])), int(rng.choice([1, 2, 4]))
    sK, sV = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    d = 128
    q = synth.queries(300 + seed, B, Hkv * G, d, "f16")
    DK = synth.dictionary(300 + seed, "dict_k", Hkv * snK, N, d // snK, "f16").reshape(Hkv, snK, N, d // snK)
    DV = synth.dictionary(300 + seed, "dict_v", Hkv * snV, N, d // snV, "f16").reshape(Hkv, snV, N, d // snV)
    iK, cK = synth.random_codes(300 + seed, 0, B, Hkv, T, snK * sK, N, "f16", "i16")
    iV, cV = synth.random_codes(300 + seed, 1, B, Hkv, T, snV * sV, N, "f16", "i16")
    r = lambda a, sn, s: np.ascontiguousarray(a.reshape(B, Hkv, T, sn, s))
    iK, cK, iV, cV = r(iK, snK, sK), r(cK, snK, sK), r(iV, snV, sV), r(cV, snV, sV)
    lens = rng.integers(0, T + 1, size=B).astype(np.int32)
    lens[0] = T
    g = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    sq = lambda D, i, c, sn: (D, i, c) if sn > 1 else (D[:, 0], i[:, :, :, 0], c[:, :, :, 0])
    aK, aV = sq(DK, iK, cK, snK), sq(DV, iV, cV, snV)
    out = csr.csr_decode_attn(g(q), g(aK[0]), g(aK[1]), g(aK[2]), g(aV[0]), g(aV[1]), g(aV[2]),
                              seq_lens=torch.from_numpy(lens).cuda())
    torch.cuda.synchronize()
    u = lambda i: i.view(np.uint16).astype(np.int64)
    ref = oracle.decode_attn_chunked(q, DK, u(iK), cK, DV, u(iV), cV, seq_lens=lens)
    out = out.cpu().numpy()
    for b in range(B):
        if lens[b] == 0:
            assert np.all(out[b] == 0)
    parity.assert_decode_close(out[lens > 0], ref[lens > 0], 2e-3, f"seed {seed}")


@pytest.mark.parametrize("seed", range(12))
def test_rotary_key_decode_on_random_shapes(seed):
    rng = np.random.default_rng(4000 + seed)
    B, Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 3, 4, 8]))
    T = int(rng.choice([1, 7, 100, 513, 1025, 2100, 9000]))
    sK, snV, sV = int(rng.choice([4, 8, 12, 16])), int(rng.choice([1, 2])), int(rng.integers(1, 9))
    N = int(rng.choice([128, 256, 384, 512] if snV > 1 else [64, 200, 256, 384, 512]))  # chunked values: multiples of 128
    layout, pos0 = int(rng.integers(0, 2)), int(rng.choice([0, 1, 4096, 123457]))
    base = float(rng.choice([10000.0, 500000.0]))
    d = 128
    q = synth.queries(400 + seed, B, Hkv * G, d, "f16")
    DK = synth.dictionary(400 + seed, "dict_k", Hkv, N, d, "f16")
    DV = synth.dictionary(400 + seed, "dict_v", Hkv * snV, N, d // snV, "f16").reshape(Hkv, snV, N, d // snV)
    iK, cK = synth.random_codes(400 + seed, 0, B, Hkv, T, sK, N, "f16", "i16")
    iV, cV = synth.random_codes(400 + seed, 1, B, Hkv, T, snV * sV, N, "f16", "i16")
    iV, cV = (np.ascontiguousarray(a.reshape(B, Hkv, T, snV, sV)) for a in (iV, cV))
    lens = rng.integers(0, T + 1, size=B).astype(np.int32)
    lens[0] = T
    g = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    aV = (DV, iV, cV) if snV > 1 else (DV[:, 0], iV[:, :, :, 0], cV[:, :, :, 0])
    print(f"[rotary random] seed {seed}: B{B} Hkv{Hkv} G{G} T{T} N{N} sK{sK} snV{snV} sV{sV} layout{layout} pos0 {pos0}", flush=True)
    out = csr.csr_decode_attn(g(q), g(DK), g(iK), g(cK), g(aV[0]), g(aV[1]), g(aV[2]), seq_lens=torch.from_numpy(lens).cuda(),
                              rope_base=base, rope_layout=layout, rope_pos0=pos0)
    torch.cuda.synchronize()
    ref = oracle.decode_attn_rope(q, DK, iK, cK, aV[0], aV[1], aV[2], base, layout, pos0, seq_lens=lens)
    out = out.cpu().numpy()
    for b in range(B):
        if lens[b] == 0:
            assert np.all(out[b] == 0)
    parity.assert_decode_close(out[lens > 0], ref[lens > 0], 2e-3, f"seed {seed}")


@pytest.mark.parametrize("seed", range(10))
def test_whole_vector_decode_on_random_large_shapes(seed):
    # Batches, KV heads, query groups, context lengths (up to 66000 tokens), dictionary sizes, pairs per code, storage
    # types and ragged lengths drawn at random: between them the cases reach every launch shape of the streaming
    # kernel and every form of the D_V product.  Codes are drawn on the GPU; the oracle recomputes sampled
    # (sequence, KV head) pairs from the bits copied back.
    rng = np.random.default_rng(7000 + seed)
    G = int(rng.choice([1, 1, 2, 4, 4, 8]))
    Hkv = int(rng.choice([1, 2, 4, 8, 8, 16]))
    B = int(rng.choice([1, 2, 4, 8, 8, 16, 33]))
    s = int(rng.choice([8, 8, 16, 4, 3, 12]))
    N = int(rng.choice([128, 256, 1024, 4096, 4096, 2048, 8192 if G == 1 else 4096, 96, 4000]))
    T = int(rng.choice([40000, 66000, 33000, 20000])) if rng.random() < 0.4 else int(rng.choice([1, 17, 1024, 1025, 5000, 9000, 16385]))
    while B * Hkv * T * s > 1.0e8:
        B = max(1, B // 2)
        if B == 1:
            break
    f32 = rng.random() < 0.15
    cdt, idt = (torch.float32, torch.int32) if f32 else (torch.float16, torch.int16)
    odt = torch.float32 if rng.random() < 0.5 else torch.float16
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7000 + seed)
    d = 128
    unit = lambda *sh: (lambda a: (a / a.norm(dim=-1, keepdim=True)).to(cdt))(torch.randn(*sh, device=dev, generator=gen))
    idx = lambda: torch.randint(0, N, (B, Hkv, T, s), device=dev, generator=gen, dtype=torch.int32).to(idt)
    coef = lambda: (torch.randn(B, Hkv, T, s, device=dev, generator=gen) * 3).to(cdt)
    q, DK, DV = torch.randn(B, Hkv * G, d, device=dev, generator=gen).to(cdt), unit(Hkv, N, d), unit(Hkv, N, d)
    ik, ck, iv, cv = idx(), coef(), idx(), coef()
    lens = None
    if rng.random() < 0.6:
        lens = rng.integers(0, T + 1, size=B).astype(np.int32)
        lens[rng.integers(0, B)] = T
    what = f"B {B} Hkv {Hkv} G {G} T {T} N {N} s {s} {'f32' if f32 else 'f16'} codes, {'f32' if odt == torch.float32 else 'f16'} out"
    print("[random decode]", what, flush=True)
    out = csr.csr_decode_attn(q, DK, ik, ck, DV, iv, cv, seq_lens=None if lens is None else torch.from_numpy(lens).to(dev),
                              out_dtype=odt)
    torch.cuda.synchronize()
    h_ = lambda t: t.float().cpu().numpy() if t.dtype == torch.float16 else t.cpu().numpy()
    picks = {(int(rng.integers(0, B)), int(rng.integers(0, Hkv))) for _ in range(3)} | {(0, 0), (B - 1, Hkv - 1)}
    for b, h in sorted(picks):
        ref = oracle.decode_attn(h_(q[b:b + 1, h * G:(h + 1) * G]), h_(DK[h:h + 1]), ik[b:b + 1, h:h + 1].cpu().numpy(),
                                 h_(ck[b:b + 1, h:h + 1]), h_(DV[h:h + 1]), iv[b:b + 1, h:h + 1].cpu().numpy(),
                                 h_(cv[b:b + 1, h:h + 1]), seq_lens=None if lens is None else lens[b:b + 1])
        parity.assert_decode_close(h_(out[b:b + 1, h * G:(h + 1) * G]), ref, 1e-3 if odt == torch.float32 else 2e-3,
                                   f"{what}, sequence {b} KV head {h}")
