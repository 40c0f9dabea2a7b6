"""ctypes front end of the CPU oracle (oracle/csr_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  Every array is
converted to float64 / int32 before the call; fp16 and fp32 inputs upcast
exactly, so the oracle sees the same input bits the GPU saw.

Functions and the passages they follow:
  mp_encode        Matching Pursuit, Eq.2-4, s iterations ("Sparse representation",
                   "KV Decomposition and Sparse Storage"); optionally with Eq.4 subtracting the coefficient as
                   it is stored (fp16, "Analysis for CSR")
  mp_encode_chunked
                   Matching Pursuit of every chunk of a vector on that chunk's dictionary (the s_n of
                   Section "NeuralDict": a head vector of d_h values is cut into s_n pieces of
                   d_h / s_n, each represented on a dictionary of atoms of that length)
  reconstruct      X~ = D r, Eq.12
  decode_attn      softmax attention of one query per sequence over K~, V~
                   ("De-Sparse to restore", last paragraph)
  decode_attn_chunked
                   the same with every head vector split into s_n chunks of d/s_n dimensions, each
                   chunk with its own dictionary and codes (the s_n of Section "NeuralDict" /
                   "Analysis for CSR": the value cache of the experiments uses s = 4, s_n = 2)
  equivalent_bits, compression_ratio, code_bytes
                   storage accounting of "Analysis for CSR"
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.csr_oracle_max_threads.restype = ctypes.c_int
        lib.csr_oracle_mp_encode.restype = ctypes.c_int
        lib.csr_oracle_mp_encode.argtypes = [p, p, i64, i32, i32, i32, p, p, p, p, p, i32, i32]
        lib.csr_oracle_reconstruct.restype = ctypes.c_int
        lib.csr_oracle_reconstruct.argtypes = [p, p, p, i64, i32, i32, i32, p]
        lib.csr_oracle_decode_attn.restype = ctypes.c_int
        lib.csr_oracle_decode_attn.argtypes = [p, p, p, p, p, p, p, i32, i32, i32, i64, i32, i32,
                                               i32, i32, ctypes.c_double, p, p, i32]
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().csr_oracle_max_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _i32(a):
    a = np.asarray(a)
    if a.dtype == np.int16:          # 16-bit indices are stored unsigned
        a = a.view(np.uint16)
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def mp_encode(X, D, s, nthreads=0, diagnostics=False, closed_loop=None):
    """Matching Pursuit of X[T, d] against atoms D[N, d] for s iterations.

    Returns (idx int32 [T, s], coef float64 [T, s]) and, with diagnostics=True, a
    third dict with best_abs / second_abs [T, s] (|correlation| of the picked atom
    and of the runner-up) and res_norm2 [T, s+1] (squared residual norms).
    closed_loop: None - Eq.4 subtracts the unrounded coefficient (the default reading); "f16" / "f32" - the
    coefficient is rounded to that storage type first, and the rounded value is both returned and subtracted.
    """
    cl = {None: 0, "f16": 1, "f32": 2}[closed_loop]
    X, D = _f64(X), _f64(D)
    assert X.ndim == 2 and D.ndim == 2 and X.shape[1] == D.shape[1]
    T, d = X.shape
    N = D.shape[0]
    idx = np.zeros((T, s), dtype=np.int32)
    coef = np.zeros((T, s), dtype=np.float64)
    best = second = rn = None
    if diagnostics:
        best = np.zeros((T, s))
        second = np.zeros((T, s))
        rn = np.zeros((T, s + 1))
    rc = _load().csr_oracle_mp_encode(_ptr(X), _ptr(D), T, d, N, s, _ptr(idx), _ptr(coef),
                                      _ptr(best), _ptr(second), _ptr(rn), nthreads, cl)
    if rc != 0:
        raise RuntimeError(f"csr_oracle_mp_encode failed: {rc}")
    if diagnostics:
        return idx, coef, {"best_abs": best, "second_abs": second, "res_norm2": rn}
    return idx, coef


def mp_encode_heads(X, D, s, nthreads=0, diagnostics=False):
    """mp_encode applied per dictionary: X[H, T, d], D[H, N, d]."""
    outs = [mp_encode(X[h], D[h], s, nthreads, diagnostics) for h in range(len(X))]
    idx = np.stack([o[0] for o in outs])
    coef = np.stack([o[1] for o in outs])
    if diagnostics:
        diag = {k: np.stack([o[2][k] for o in outs]) for k in outs[0][2]}
        return idx, coef, diag
    return idx, coef


def mp_encode_chunked(X, D, s, nthreads=0):
    """Chunked Matching Pursuit: X [T, d], D [s_n, N, d / s_n] -> idx int32, coef float64 [T, s_n, s].

    Chunk c of a vector is its dimensions c d/s_n .. (c+1) d/s_n - 1; it is encoded by mp_encode as a vector
    of its own against D[c], with atom numbers local to that dictionary.  Reading taken: the chunks are
    independent problems (each has its own residual and its own s iterations).
    """
    X, D = np.asarray(X), np.asarray(D)
    sn, N, dc = D.shape
    assert X.ndim == 2 and X.shape[1] == sn * dc
    outs = [mp_encode(X[:, c * dc:(c + 1) * dc], D[c], s, nthreads) for c in range(sn)]
    return np.stack([o[0] for o in outs], axis=1), np.stack([o[1] for o in outs], axis=1)


def reconstruct(idx, coef, D):
    """Eq.12 for one dictionary: idx/coef [T, s], D [N, d] -> X~ [T, d] (float64)."""
    idx, coef, D = _i32(idx), _f64(coef), _f64(D)
    T, s = idx.shape
    N, d = D.shape
    out = np.zeros((T, d))
    rc = _load().csr_oracle_reconstruct(_ptr(idx), _ptr(coef), _ptr(D), T, d, N, s, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"csr_oracle_reconstruct failed: {rc}")
    return out


def decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, scale=None, seq_lens=None, nthreads=0):
    """Attention of q[B, Hq, d] over codes [B, Hkv, T, s*]; dictionaries [Hkv, N, d].

    scale defaults to 1/sqrt(d).  Returns out [B, Hq, d] float64.
    """
    q, DK, DV = _f64(q), _f64(DK), _f64(DV)
    idxK, idxV, coefK, coefV = _i32(idxK), _i32(idxV), _f64(coefK), _f64(coefV)
    B, Hq, d = q.shape
    Hkv, N, _ = DK.shape
    T, sK = idxK.shape[2], idxK.shape[3]
    sV = idxV.shape[3]
    assert DV.shape == DK.shape and idxK.shape[:2] == (B, Hkv) and idxV.shape[:3] == (B, Hkv, T)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    sl = None if seq_lens is None else np.ascontiguousarray(seq_lens, dtype=np.int32)
    out = np.zeros((B, Hq, d))
    rc = _load().csr_oracle_decode_attn(_ptr(q), _ptr(DK), _ptr(idxK), _ptr(coefK), _ptr(DV),
                                        _ptr(idxV), _ptr(coefV), B, Hq, Hkv, T, d, N, sK, sV,
                                        float(scale), _ptr(sl), _ptr(out), nthreads)
    if rc != 0:
        raise RuntimeError(f"csr_oracle_decode_attn failed: {rc}")
    return out


def decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV, scale=None, seq_lens=None):
    """Attention over a cache whose head vectors are stored as s_n chunks (Section "NeuralDict": the vector is cut
    into s_n pieces of d/s_n dimensions, every piece sparsely represented on its own).

    q [B, Hq, d]; DK [Hkv, snK, N, d/snK], idxK/coefK [B, Hkv, T, snK, sK]; likewise for V with snV, sV.
    K~_t is the concatenation over chunks of D_c r_{t,c} (Eq.12 per chunk), then plain softmax attention,
    written out in numpy float64.  Reading taken: every chunk has its own dictionary (a caller who shares one
    passes it s_n times).  Returns out [B, Hq, d] float64.
    """
    q = _f64(q)
    B, Hq, d = q.shape
    Hkv = DK.shape[0]
    G = Hq // Hkv
    T = idxK.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((B, Hq, d))

    def dense(D, idx, coef, b, h, L):
        sn = D.shape[1]
        return np.concatenate([reconstruct(idx[b, h, :L, c], coef[b, h, :L, c], D[h, c]) for c in range(sn)], axis=1)

    for b in range(B):
        L = T if seq_lens is None else int(seq_lens[b])
        if L <= 0:
            continue
        for h in range(Hkv):
            Kt, Vt = dense(DK, idxK, coefK, b, h, L), dense(DV, idxV, coefV, b, h, L)
            for g in range(G):
                sc = scale * (Kt @ q[b, h * G + g])
                p = np.exp(sc - sc.max())
                out[b, h * G + g] = (p / p.sum()) @ Vt
    return out


def rope_rotate(X, positions, base, layout=0):
    """Rotary position embedding of the rows of X [T, d] at integer positions [T] (float64).

    Section "Position embedding makes nonstationary Keys" has the keys sparsely represented BEFORE the position
    embedding, so attention must rotate the rebuilt keys.  The paper does not restate the embedding; this is the
    public rotary definition: dimension pair k = 0 .. d/2-1 is turned by the angle p * base^(-2k/d) at position p.
    layout 0 pairs dimension k with k + d/2, layout 1 pairs 2k with 2k + 1.
    """
    X = _f64(X)
    T, d = X.shape
    hd = d // 2
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(hd, dtype=np.float64) / d)
    ang = np.asarray(positions, dtype=np.float64).reshape(T, 1) * theta.reshape(1, hd)
    co, si = np.cos(ang), np.sin(ang)
    if layout == 0:
        a, b = X[:, :hd], X[:, hd:]
    else:
        a, b = X[:, 0::2], X[:, 1::2]
    ra, rb = a * co - b * si, b * co + a * si
    out = np.empty_like(X)
    if layout == 0:
        out[:, :hd], out[:, hd:] = ra, rb
    else:
        out[:, 0::2], out[:, 1::2] = ra, rb
    return out


def decode_attn_rope(q, DK, idxK, coefK, DV, idxV, coefV, rope_base, layout=0, pos0=0, scale=None, seq_lens=None):
    """Attention over a cache whose keys were coded before the rotary embedding.

    q [B, Hq, d] is the query as attention receives it (already rotated at its own position).  Cache token t of
    every sequence sits at position pos0 + t: its key is rebuilt by Eq.12, K~_t = D_K r_t, rotated there, and
    then plain softmax attention runs, written out in numpy float64.  Values carry no position (whole or
    chunked codes: DV [Hkv, N, d] with idxV [B, Hkv, T, sV], or DV [Hkv, snV, N, d/snV] with idxV
    [B, Hkv, T, snV, sV]); keys are whole vectors, DK [Hkv, N, d], idxK [B, Hkv, T, sK].
    Returns out [B, Hq, d] float64.
    """
    q = _f64(q)
    B, Hq, d = q.shape
    Hkv = DK.shape[0]
    G = Hq // Hkv
    T = idxK.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((B, Hq, d))
    for b in range(B):
        L = T if seq_lens is None else int(seq_lens[b])
        if L <= 0:
            continue
        pos = pos0 + np.arange(L)
        for h in range(Hkv):
            Kt = rope_rotate(reconstruct(idxK[b, h, :L], coefK[b, h, :L], DK[h]), pos, rope_base, layout)
            if DV.ndim == 4:
                Vt = np.concatenate([reconstruct(idxV[b, h, :L, c], coefV[b, h, :L, c], DV[h, c])
                                     for c in range(DV.shape[1])], axis=1)
            else:
                Vt = reconstruct(idxV[b, h, :L], coefV[b, h, :L], DV[h])
            for g in range(G):
                sc = scale * (Kt @ q[b, h * G + g])
                p = np.exp(sc - sc.max())
                out[b, h * G + g] = (p / p.sum()) @ Vt
    return out


# --- storage accounting, "Analysis for CSR" ---------------------------------------------------

def code_bytes(s, s_n=1, idx_bytes=2, coef_bytes=2):
    """Bytes stored per head vector: s*s_n coefficients and as many indices."""
    return s * s_n * (idx_bytes + coef_bytes)


def compression_ratio(d_h, s, s_n=1):
    """fp16 vector bits over code bits: 16 d_h / (16 s s_n + 16 s s_n)."""
    return (16.0 * d_h) / (16.0 * s * s_n + 16.0 * s * s_n)


def equivalent_bits(d_h, s, s_n=1):
    """Bits per channel of the equivalent quantiser: 16 / compression ratio."""
    return 16.0 / compression_ratio(d_h, s, s_n)
