"""Seeded synthetic inputs shaped like the paper's Llama-class KV workloads.

This module only draws random tensors; none of the method's arithmetic (no
correlation, no arg-max, no attention) lives here, so both the GPU tests and the
CPU oracle can be fed from it.  The tensors stand in for real KV caches and
trained dictionaries, of which only shapes and types are kept:

  dictionary   iid N(0,1) entries, every atom scaled to unit L2 norm (the unit-norm
               atoms of Section "Sparse representation"), then cast to the storage type
  keys         iid N(0,1) with a fixed per-head set of outlier channels multiplied by 10
  values       iid N(0,1)
  queries      iid N(0,1)

Sub-streams are keyed by (seed, tensor kind, head...) so a subset of a big
workload can be regenerated without drawing the rest.
"""
from dataclasses import dataclass

import numpy as np

_KINDS = {"dict_k": 1, "dict_v": 2, "keys": 3, "values": 4, "queries": 5, "outliers": 6,
          "codes_idx": 7, "codes_coef": 8, "misc": 9}


@dataclass(frozen=True)
class Workload:
    """One of the five benchmark configurations (single transformer layer unless noted)."""
    name: str
    hkv: int            # KV heads
    hq: int             # query heads
    d: int              # head dimension
    n_atoms: int        # atoms per dictionary
    tokens: int         # cached tokens per head and sequence
    s: int              # matching-pursuit iterations
    batch: int          # decode batch (sequences)
    key_outliers: int   # outlier channels in the keys
    dtype: str          # "f32" or "f16" for vectors / dictionary / coefficients
    itype: str          # "i32" or "i16" index storage
    layers: int = 1


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 128, 1024, 4096, 8, 1, 4, "f32", "i32"),
    "llama7b_layer": Workload("llama7b_layer", 32, 32, 128, 4096, 4096, 8, 1, 8, "f16", "i16"),
    "long_context": Workload("long_context", 32, 32, 128, 8192, 32768, 16, 4, 8, "f16", "i16"),
    "gqa_llama3_8b": Workload("gqa_llama3_8b", 8, 32, 128, 4096, 131072, 8, 8, 8, "f16", "i16"),
    "prefill_stress": Workload("prefill_stress", 8, 32, 128, 4096, 8192, 8, 16, 8, "f16", "i16",
                               layers=32),
}

NP_DTYPE = {"f32": np.float32, "f16": np.float16}
NP_ITYPE = {"i32": np.int32, "i16": np.int16}


def stream(seed, kind, *ids):
    """Independent generator for (seed, kind, ids...)."""
    ss = np.random.SeedSequence([int(seed), _KINDS[kind], *[int(i) for i in ids]])
    return np.random.Generator(np.random.Philox(ss))


def dictionary(seed, kind, heads, n_atoms, d, dtype="f16", head0=0):
    """[heads][n_atoms][d] unit-norm Gaussian atoms; kind is "dict_k" or "dict_v"."""
    out = np.empty((heads, n_atoms, d), dtype=NP_DTYPE[dtype])
    for h in range(heads):
        a = stream(seed, kind, head0 + h).standard_normal((n_atoms, d), dtype=np.float32)
        a /= np.sqrt((a.astype(np.float64) ** 2).sum(axis=1, keepdims=True)).astype(np.float32)
        out[h] = a.astype(NP_DTYPE[dtype])
    return out


def outlier_channels(seed, kind, head, d, count):
    """The fixed outlier channel ids of one head: first `count` of a seeded permutation."""
    return stream(seed, "outliers", _KINDS[kind], head).permutation(d)[:count]


def vectors(seed, kind, heads, tokens, d, dtype="f16", outliers=0, head0=0, token0=0):
    """[heads][tokens][d] N(0,1) vectors; `outliers` channels per head are scaled by 10.

    kind is "keys" or "values".  token0 lets a caller regenerate a token range of a
    larger tensor only if it draws whole heads; sub-ranges are taken by slicing.
    """
    out = np.empty((heads, tokens, d), dtype=NP_DTYPE[dtype])
    for h in range(heads):
        x = stream(seed, kind, head0 + h, token0).standard_normal((tokens, d), dtype=np.float32)
        if outliers:
            x[:, outlier_channels(seed, kind, head0 + h, d, outliers)] *= 10.0
        out[h] = x.astype(NP_DTYPE[dtype])
    return out


def queries(seed, batch, hq, d, dtype="f16"):
    x = stream(seed, "queries").standard_normal((batch, hq, d), dtype=np.float32)
    return x.astype(NP_DTYPE[dtype])


def random_codes(seed, tag, batch, hkv, tokens, s, n_atoms, dtype="f16", itype="i16"):
    """Random but code-like (index, coefficient) streams [batch][hkv][tokens][s].

    Indices are uniform over the atoms; coefficient magnitudes decay with the pair
    position like matching-pursuit output does, with random signs.  Used where decode
    is exercised on its own at sizes the encoder oracle cannot produce quickly.
    """
    g = stream(seed, "codes_idx", tag)
    idx = g.integers(0, n_atoms, size=(batch, hkv, tokens, s), dtype=np.int64)
    g = stream(seed, "codes_coef", tag)
    mag = 3.0 * (0.85 ** np.arange(s, dtype=np.float32))
    coef = g.standard_normal((batch, hkv, tokens, s), dtype=np.float32) * 0.25 + 1.0
    coef *= mag * g.choice(np.float32([-1.0, 1.0]), size=coef.shape)
    if itype == "i16":
        idx_out = idx.astype(np.uint16).view(np.int16)
    else:
        idx_out = idx.astype(np.int32)
    return idx_out, coef.astype(NP_DTYPE[dtype])
