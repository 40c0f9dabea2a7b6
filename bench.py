"""Benchmark of the CSR hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, inputs resident in HBM:
  1. Matching Pursuit encode of one layer's keys and values (csr_encode, 64 dictionaries x 4096
     vectors at the Llama-7B-shaped workload), producing (index, coefficient) codes;
  2. decode attention of one query token per head on those codes (csr_decode_attn).
Prints ONE JSON line.  `value` is encoded KV vectors per second over the whole step; the decode
rate (context tokens per second) and both rooflines are reported beside it, together with the CPU
oracle timed on this machine's host cores on a bounded sample.  `decode_rooflines` adds the decode
call alone at the long-context and GQA shapes (random codes drawn on the GPU, cache-cold), where
the code streams rather than the dictionaries dominate the traffic.  `chunked_step` is the same step in the
storage layout of the paper's experiments ("CSR-8": keys whole with s = 8, values in s_n = 2 chunks of 64
dimensions with s = 4 each), which runs the 64-dimensional variants of the encoder and the chunk-aware decode.
`decode_step` is one decoding step: the new token's codes appended in place, then attention over the cache
(`decode_step_gqa`: the same at the grouped-query shape, 8 sequences on shared dictionaries; `decode_step_batch64`:
the benchmark layer serving 64 sequences).
`rope_decode` is csr_decode_attn on keys coded before the rotary embedding (rope_base set), at the dictionary sizes
of the paper's own experiments (256 atoms per KV head), where the key dictionary stays in LDS; `paper_sized_step` is
the chunked step with those dictionaries and that decode.

All kernels run on PyTorch's current stream, and the HIP events that time them (torch.cuda.Event)
are recorded on that same stream.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b_layer] [--algo auto]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16 matrix peak
PEAK_VALU_F32_TFLOPS = 157.3    # MI355X fp32 vector peak
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E peak
# HBM bytes per dispatch of the dominant kernel (fetched + written), RECORDED from earlier rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs (each scaled by what the counter reads for a 1 GiB copy): hardware counters cannot be
# read from inside this process, so `traffic` in the JSON line is not a measurement of this run; `traffic_source`
# names the summary under profiles/ that holds the commands and the raw counts.
PMC_TRAFFIC_BYTES = {("llama7b_layer", "mfma"): (719.4e6 + 131.0e6, "profiles/encode_mfma_kernel_llama7b_layer.txt")}
# The same for one csr_decode_attn call (its launches added up), per workload.
PMC_DECODE_TRAFFIC_BYTES = {
    "llama7b_layer": (79.0e6 + 3.2e6, "profiles/decode_kernels_llama7b_layer.txt"),
    "long_context": (689.5e6 + 16.8e6, "profiles/decode_kernels_long_context_gqa.txt"),
    "gqa_llama3_8b": (598.5e6 + 42.0e6, "profiles/decode_kernels_long_context_gqa.txt")}


def recorded_traffic(table, key):
    """{"traffic": bytes or None, "traffic_source": file or None}: counter traffic recorded under profiles/."""
    t = table.get(key)
    return {"traffic": t[0] if t else None, "traffic_source": (t[1] + " (recorded rocprofv3 --pmc run, not this run)") if t else None}


def mfma_only_rate():
    """What the matrix cores of this GPU sustain with nothing else running (paper_2412_11741_amd/mfma_rate.bin, built
    from csrc/probe/mfma_rate.hip): {"mfma_only_tflops_random": .., "mfma_only_tflops_smooth": ..}, or None if the
    probe is not built.  Run as a child process before this process touches the GPU; left out under a profiler
    (whose preloaded library has initialised the GPU already, and whose kernel statistics it would only clutter)."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2412_11741_amd", "mfma_rate.bin")
    if not os.path.exists(exe):
        return None
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return None
    try:
        out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
        return json.loads(out.stdout.strip().splitlines()[-1]) if out.returncode == 0 else None
    except Exception:
        return None


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def timed_ms(fn, reps, warmup=2):
    """Median and list of HIP-event times (ms) of `reps` calls of fn on the current stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a_, b_ in ev:
        a_.record(); fn(); b_.record()
    torch.cuda.synchronize()
    ms = [a_.elapsed_time(b_) for a_, b_ in ev]
    return median(ms), ms


def decode_only(csr, w, dev):
    """csr_decode_attn alone on workload `w`: uniformly random atom indices, N(0, 3) coefficients, unit-norm
    Gaussian dictionaries, all drawn on the GPU with a fixed seed.  Distinct input copies are rotated
    so that more than 1 GB is touched between reuses (the Infinity Cache holds 256 MB)."""
    import torch
    B, Hkv, Hq, T, N, d, s = w.batch, w.hkv, w.hq, w.tokens, w.n_atoms, w.d, w.s
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def unit(*shape):
        a = torch.randn(*shape, device=dev, generator=gen)
        return (a / a.norm(dim=-1, keepdim=True)).half()

    def make():
        idx = lambda: torch.randint(0, N, (B, Hkv, T, s), device=dev, generator=gen, dtype=torch.int32).to(torch.int16)
        coef = lambda: (torch.randn(B, Hkv, T, s, device=dev, generator=gen) * 3).half()
        return dict(q=torch.randn(B, Hq, d, device=dev, generator=gen).half(), DK=unit(Hkv, N, d), ik=idx(),
                    ck=coef(), DV=unit(Hkv, N, d), iv=idx(), cv=coef(),
                    out=torch.empty(B, Hq, d, device=dev, dtype=torch.float16))

    nbytes = B * Hkv * T * 2 * s * 4 + Hkv * 2 * N * d * 2 + B * Hq * d * 4
    copies = max(2, min(16, int(1.2e9 // nbytes) + 1))
    sets = [make() for _ in range(copies)]
    desc = csr.decode_desc(sets[0]["q"], sets[0]["DK"], sets[0]["ik"], sets[0]["ck"], sets[0]["iv"])
    ws = torch.empty(max(csr.csr_decode_workspace_bytes(desc), 256), dtype=torch.uint8, device=dev)

    def run(S):
        csr.csr_decode_attn(S["q"], S["DK"], S["ik"], S["ck"], S["DV"], S["iv"], S["cv"], out=S["out"], workspace=ws)

    for S in sets:
        run(S)
    torch.cuda.synchronize()
    reps = max(2 * copies, 10)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for r in range(reps):
        ev[r][0].record()
        run(sets[r % copies])
        ev[r][1].record()
    torch.cuda.synchronize()
    ms = median([a.elapsed_time(b) for a, b in ev])
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"workload": w.name, "kernel": "csr_decode_attn (4 launches), cache-cold", "bound": "hbm",
            "achieved": round(gbs, 2), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 5),
            **recorded_traffic(PMC_DECODE_TRAFFIC_BYTES, w.name), "bytes_per_call": nbytes, "median_call_ms": round(ms, 5),
            "decode_ctx_tokens_per_s": round(B * T / (ms * 1e-3), 1), "copies_rotated": copies,
            "config": {"kv_heads": Hkv, "query_heads": Hq, "atoms": N, "tokens_per_head": T, "s": s, "decode_batch": B}}


def encode_only(csr, w, dev, reps):
    """csr_encode alone at workload `w`'s full shape, one launch per layer: every (sequence, KV head) block of keys
    and of values in one call on the heads' shared dictionaries (2 Hkv dictionaries, block h on dictionary
    h % (2 Hkv)).  Vectors N(0,1) with the keys' outlier channels x 10, unit-norm Gaussian atoms, drawn on the GPU
    with a fixed seed.  A workload of several layers is streamed layer by layer through the same buffers (the
    encoder's time does not depend on the values), and the time is that of all its layers."""
    import torch
    B, Hkv, T, N, d, s = w.batch, w.hkv, w.tokens, w.n_atoms, w.d, w.s
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    dicts, H = 2 * Hkv, 2 * Hkv * B
    D = torch.randn(dicts, N, d, device=dev, generator=gen)
    D = (D / D.norm(dim=-1, keepdim=True)).half()
    X = torch.empty(H, T, d, device=dev, dtype=torch.float16)
    for h in range(H):
        x = torch.randn(T, d, device=dev, generator=gen)
        if h % dicts < Hkv:
            x[:, :w.key_outliers] *= 10
        X[h] = x.half()
    idx = torch.empty((H, T, s), dtype=torch.int16, device=dev)
    coef = torch.empty((H, T, s), dtype=torch.float16, device=dev)
    need = csr.csr_encode_workspace_bytes(csr.encode_desc(X, D, s, torch.float16, torch.int16))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)

    def run():
        for _ in range(w.layers):
            csr.csr_encode(X, D, s, idx=idx, coef=coef, workspace=ws)

    ms, all_ms = timed_ms(run, reps, warmup=1)
    n_vec = H * T * w.layers
    flop = 2.0 * d * N * s * n_vec
    tf = flop / (ms * 1e-3) / 1e12
    return {"workload": w.name, "kernel": "csr_encode (mfma)", "bound": "mfma", "achieved": round(tf, 2),
            "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_MFMA_F16_TFLOPS, 5), "traffic": None,
            "vectors": n_vec, "launches": w.layers, "vectors_per_launch": H * T, "flop_per_vector": 2.0 * d * N * s,
            "median_ms": round(ms, 3), "all_ms": [round(m, 3) for m in all_ms],
            "encode_vectors_per_s": round(n_vec / (ms * 1e-3), 1),
            "config": {"kv_heads": Hkv, "atoms": N, "tokens_per_head": T, "s": s, "sequences": B, "layers": w.layers,
                       "dictionaries_per_launch": dicts, "blocks_per_launch": H}}


def chunked_step(csr, synth, w, dev, steps, n_atoms=None, rope_base=0.0):
    """Encode + decode of one layer in the experiments' "CSR-8" layout: keys whole (s = 8), values in two chunks of
    d/2 dimensions (s = 4 each, one dictionary of N atoms per chunk).  Same vectors as the main workload.
    n_atoms overrides the workload's dictionary size (256: the paper's own budget per head, which csr_encode serves
    with its LDS-resident kernel); rope_base > 0 attends with the keys taken as coded before the rotary embedding."""
    import numpy as np
    import torch
    B, Hkv, Hq, T, N, d = w.batch, w.hkv, w.hq, w.tokens, n_atoms or w.n_atoms, w.d
    sK, sV, sn = 8, 4, 2
    g = lambda a: torch.from_numpy(a).to(dev)
    XK = g(np.concatenate([synth.vectors(0, "keys", Hkv, T, d, "f16", outliers=w.key_outliers, token0=b) for b in range(B)]))
    XV = g(np.concatenate([synth.vectors(0, "values", Hkv, T, d, "f16", token0=b) for b in range(B)]))
    DK = g(synth.dictionary(0, "dict_k", Hkv, N, d, "f16"))
    DV = g(synth.dictionary(0, "dict_v", Hkv * sn, N, d // sn, "f16").reshape(Hkv, sn, N, d // sn))
    q = g(synth.queries(0, B, Hq, d, "f16"))
    DKe, DVe = DK.repeat(B, 1, 1), DV.repeat(B, 1, 1, 1)
    iK = torch.empty((B * Hkv, T, sK), dtype=torch.int16, device=dev)
    cK = torch.empty((B * Hkv, T, sK), dtype=torch.float16, device=dev)
    iV = torch.empty((B * Hkv, T, sn, sV), dtype=torch.int16, device=dev)
    cV = torch.empty((B * Hkv, T, sn, sV), dtype=torch.float16, device=dev)
    out = torch.empty((B, Hq, d), dtype=torch.float16, device=dev)
    wsK = torch.empty(max(csr.csr_encode_workspace_bytes(csr.encode_desc(XK, DKe, sK, torch.float16, torch.int16)), 256),
                      dtype=torch.uint8, device=dev)
    wsV = torch.empty(max(csr.csr_encode_workspace_bytes(csr.encode_desc(XV, DVe, sV, torch.float16, torch.int16)), 256),
                      dtype=torch.uint8, device=dev)
    v5 = lambda t, s_: t.view(B, Hkv, T, sn, s_)
    v4 = lambda t, s_: t.view(B, Hkv, T, s_)
    ddesc = csr.decode_desc(q, DK, v4(iK, sK), v4(cK, sK), v5(iV, sV), rope_base=rope_base)
    wsD = torch.empty(max(csr.csr_decode_workspace_bytes(ddesc), 256), dtype=torch.uint8, device=dev)

    def enc_k(): csr.csr_encode(XK, DKe, sK, idx=iK, coef=cK, workspace=wsK)
    def enc_v(): csr.csr_encode(XV, DVe, sV, idx=iV, coef=cV, workspace=wsV)
    def dec(): csr.csr_decode_attn(q, DK, v4(iK, sK), v4(cK, sK), DV, v5(iV, sV), v5(cV, sV), out=out, workspace=wsD,
                                   rope_base=rope_base)

    for _ in range(2):
        enc_k(); enc_v(); dec()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        ev[i][0].record(); enc_k(); ev[i][1].record(); enc_v(); ev[i][2].record(); dec(); ev[i][3].record()
    torch.cuda.synchronize()
    k_ms, v_ms, d_ms = (median([e[j].elapsed_time(e[j + 1]) for e in ev]) for j in range(3))
    nv = B * Hkv * T
    tf = lambda flop, ms: round(flop / (ms * 1e-3) / 1e12, 2)
    v_flop = 2.0 * (d // sn) * N * sV * sn * nv
    dec_bytes = nv * (sK + sn * sV) * 4 + Hkv * 2 * N * d * 2 + B * Hq * d * 4
    resident = N * d * 2 <= 128 * 1024   # csr_encode's choice for dictionaries that fit the LDS
    k_flop = 2.0 * d * N * sK * nv
    return {"layout": "K s=8 s_n=1, V s=4 s_n=2 (chunks of %d)" % (d // sn), "atoms": N, "rope_base": rope_base,
            "vectors_per_step": 2 * nv,
            "value": round(2 * nv / ((k_ms + v_ms + d_ms) * 1e-3), 1), "unit": "vectors/s",
            "encode_k_ms": round(k_ms, 4), "encode_v_ms": round(v_ms, 4), "decode_ms_warm": round(d_ms, 5),
            "encode_k_tflops": tf(k_flop, k_ms),
            "roofline_encode_v": {"kernel": "csr_encode (%s, 64-dimensional chunks)" % ("resident" if resident else "mfma"),
                                  "bound": "mfma",
                                  "achieved": tf(v_flop, v_ms), "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                                  "frac": round(tf(v_flop, v_ms) / PEAK_MFMA_F16_TFLOPS, 5)},
            "decode_bytes_per_call": dec_bytes,
            "decode_gbs_warm": round(dec_bytes / (d_ms * 1e-3) / 1e9, 1)}


# Shapes of the rotary-key decode: the paper's dictionary budget (8192 atoms over 32 heads, 2048 over 8 KV heads:
# 256 per KV head) and cache layout (keys whole with s = 8, values in 2 chunks with s = 4), 32768 cached tokens.
ROPE_SHAPES = [
    {"name": "rope_mha_32heads", "B": 4, "Hq": 32, "Hkv": 32, "T": 32768, "N": 256, "sK": 8, "sV": 4, "snV": 2},
    {"name": "rope_gqa_8x4heads", "B": 8, "Hq": 32, "Hkv": 8, "T": 32768, "N": 256, "sK": 8, "sV": 4, "snV": 2},
    # the benchmark layer's own dictionaries (4096 atoms: beyond the LDS, key rows gathered from device memory)
    {"name": "rope_llama7b_layer_n4096", "B": 1, "Hq": 32, "Hkv": 32, "T": 4096, "N": 4096, "sK": 8, "sV": 8, "snV": 1},
]


def rope_decode(csr, dev, steps):
    """csr_decode_attn with rope_base = 10000 on ROPE_SHAPES (random codes drawn on the GPU), next to the
    position-free call on the same tensors.  The rotary path is bound by the vector ALU: its arithmetic per
    (sequence, KV head, token) is the rebuild of the key (2 s d flop), its rotation (6 flop per frequency pair)
    and one dot product per query head of the group (2 d flop each), priced against the fp32 vector peak."""
    import torch
    d = 128
    out = []
    for sh in ROPE_SHAPES:
        B, Hq, Hkv, T, N, sK, sV, snV = (sh[k] for k in ("B", "Hq", "Hkv", "T", "N", "sK", "sV", "snV"))
        gen = torch.Generator(device=dev)
        gen.manual_seed(2)

        def unit(*shape):
            a = torch.randn(*shape, device=dev, generator=gen)
            return (a / a.norm(dim=-1, keepdim=True)).half()

        ri = lambda *shape: torch.randint(0, N, shape, device=dev, generator=gen, dtype=torch.int32).to(torch.int16)
        rc = lambda *shape: (torch.randn(*shape, device=dev, generator=gen) * 3).half()
        q, DK = torch.randn(B, Hq, d, device=dev, generator=gen).half(), unit(Hkv, N, d)
        DV = unit(Hkv, snV, N, d // snV) if snV > 1 else unit(Hkv, N, d)
        iK, cK = ri(B, Hkv, T, sK), rc(B, Hkv, T, sK)
        iV, cV = (ri(B, Hkv, T, snV, sV), rc(B, Hkv, T, snV, sV)) if snV > 1 else (ri(B, Hkv, T, sV), rc(B, Hkv, T, sV))
        o = torch.empty(B, Hq, d, device=dev, dtype=torch.float16)
        times = {}
        for base in (10000.0, 0.0):
            desc = csr.decode_desc(q, DK, iK, cK, iV, rope_base=base)
            ws = torch.empty(max(csr.csr_decode_workspace_bytes(desc), 256), dtype=torch.uint8, device=dev)
            run = lambda: csr.csr_decode_attn(q, DK, iK, cK, DV, iV, cV, out=o, workspace=ws, rope_base=base)
            for _ in range(2):
                run()
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for a_, b_ in ev:
                a_.record(); run(); b_.record()
            torch.cuda.synchronize()
            times[base] = median([a_.elapsed_time(b_) for a_, b_ in ev])
        ms = times[10000.0]
        G = Hq // Hkv
        flop = B * Hkv * T * (2 * sK * d + 6 * (d // 2) + 2 * d * G)
        tf = flop / (ms * 1e-3) / 1e12
        code_bytes = B * Hkv * T * (sK + snV * sV) * 4
        out.append({"workload": sh["name"], "kernel": "csr_decode_attn, rope_base = 10000 (3 launches)" +
                    ("" if N * d * 2 <= 128 * 1024 else ", key rows gathered from device memory"), "bound": "alu",
                    "achieved": round(tf, 2), "peak": PEAK_VALU_F32_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf / PEAK_VALU_F32_TFLOPS, 5), "flop_per_call": flop, "median_call_ms": round(ms, 5),
                    # the dot products of this kernel are packed fp16 (v_dot2_f32_f16: two multiply-adds per lane and
                    # issue), whose own rate is twice the fp32 vector peak the line above is priced against
                    "peak_packed_fp16_dot": 2 * PEAK_VALU_F32_TFLOPS,
                    "frac_of_packed_fp16_dot_peak": round(tf / (2 * PEAK_VALU_F32_TFLOPS), 5),
                    "key_tokens_per_s": round(B * Hkv * T / (ms * 1e-3), 1),
                    "decode_ctx_tokens_per_s": round(B * T / (ms * 1e-3), 1),
                    "code_gbs": round(code_bytes / (ms * 1e-3) / 1e9, 1),
                    "dense_fp16_cache_gbs_equivalent": round(B * Hkv * T * 2 * d * 2 / (ms * 1e-3) / 1e9, 1),
                    "position_free_call_ms": round(times[0.0], 5),
                    "config": {"kv_heads": Hkv, "query_heads": Hq, "atoms": N, "tokens_per_head": T, "sK": sK, "sV": sV,
                               "snV": snV, "decode_batch": B}})
        del q, DK, DV, iK, cK, iV, cV, o, ws
    return out


def small_dict_encoders(csr, dev, steps):
    """The two encoders for dictionaries that fit the LDS - CSR_ENCODE_RESIDENT (what AUTO picks) and
    CSR_ENCODE_GRAM (the Gram-matrix update of the correlations) - on 64 dictionaries x 4096 vectors of 128
    dimensions (the benchmark layer's vector count), unit-norm Gaussian atoms and N(0,1) vectors drawn on the GPU."""
    import torch
    H, T, d = 64, 4096, 128
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    X = torch.randn(H, T, d, device=dev, generator=gen).half()
    out = []
    for N in (32, 128, 256):
        D = torch.randn(H, N, d, device=dev, generator=gen)
        D = (D / D.norm(dim=-1, keepdim=True)).half()
        for name, algo in (("resident", csr.CSR_ENCODE_RESIDENT), ("gram", csr.CSR_ENCODE_GRAM)):
            row = {"atoms": N, "encoder": name}
            for s in (1, 8):
                idx = torch.empty((H, T, s), dtype=torch.int16, device=dev)
                coef = torch.empty((H, T, s), dtype=torch.float16, device=dev)
                for _ in range(2):
                    csr.csr_encode(X, D, s, algo=algo, idx=idx, coef=coef)
                torch.cuda.synchronize()
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
                for a_, b_ in ev:
                    a_.record(); csr.csr_encode(X, D, s, algo=algo, idx=idx, coef=coef); b_.record()
                torch.cuda.synchronize()
                row["ms_s%d" % s] = round(median([a_.elapsed_time(b_) for a_, b_ in ev]), 4)
            out.append(row)
    return out


def decode_step(csr, synth, w, dev, steps):
    """One decoding step at the workload's shape: the new token's key and value of every (sequence, KV head) are
    encoded straight into the next row of the code cache (csr_encode picks its few-vectors kernel), then
    csr_decode_attn runs over the grown cache.  The cache holds random codes (the step's cost does not depend on
    their values); T - 1 tokens are cached, the step appends token T - 1."""
    import numpy as np
    import torch
    B, Hkv, Hq, T, N, d, s = w.batch, w.hkv, w.hq, w.tokens, w.n_atoms, w.d, w.s
    g = lambda a: torch.from_numpy(a).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    DK, DV = g(synth.dictionary(0, "dict_k", Hkv, N, d, "f16")), g(synth.dictionary(0, "dict_v", Hkv, N, d, "f16"))
    q = g(synth.queries(0, B, Hq, d, "f16"))
    XK = g(synth.vectors(1, "keys", B * Hkv, 1, d, "f16", outliers=w.key_outliers))
    XV = g(synth.vectors(1, "values", B * Hkv, 1, d, "f16"))
    ri = lambda: torch.randint(0, N, (B * Hkv, T, s), device=dev, generator=gen, dtype=torch.int32).to(torch.int16)
    rc = lambda: (torch.randn(B * Hkv, T, s, device=dev, generator=gen) * 3).half()
    # one cache tensor, keys' blocks first: with one sequence, block j of the stacked tensor uses dictionary j, so
    # a single csr_encode call appends the keys' and the values' codes
    icache = torch.cat([ri(), ri()])
    ccache = torch.cat([rc(), rc()])
    nkv = B * Hkv
    iK, cK, iV, cV = icache[:nkv], ccache[:nkv], icache[nkv:], ccache[nkv:]
    XKV, DKV = torch.cat([XK, XV]), torch.cat([DK, DV])
    out = torch.empty((B, Hq, d), dtype=torch.float16, device=dev)
    lens = torch.full((B,), T, dtype=torch.int32, device=dev)
    row = lambda t: t[:, T - 1:T]
    ews = csr.csr_encode_workspace_bytes(csr.encode_desc(XKV, DKV, s, torch.float16, torch.int16, code_stride_h=T * s))
    wsE = torch.empty(max(ews, 2 * B * Hkv * N * 4 + (1 << 20), 256), dtype=torch.uint8, device=dev)   # either encoder's
    v = lambda t: t.view(B, Hkv, T, s)
    wsD = torch.empty(max(csr.csr_decode_workspace_bytes(csr.decode_desc(q, DK, v(iK), v(cK), v(iV))), 256),
                      dtype=torch.uint8, device=dev)

    # G = D D^T per dictionary, prepared once like the dictionaries themselves (not part of a step): with it the
    # append sweeps every dictionary once instead of s times
    GKV = csr.csr_gram_build(DKV)
    GK, GV = GKV[:Hkv], GKV[Hkv:]
    use_gram = [True]

    def append():
        gk = dict(gram=GKV) if use_gram[0] else {}
        if B == 1:
            csr.csr_encode(XKV, DKV, s, idx=row(icache), coef=row(ccache), workspace=wsE, **gk)
        else:
            csr.csr_encode(XK, DK, s, idx=row(iK), coef=row(cK), workspace=wsE, **(dict(gram=GK) if use_gram[0] else {}))
            csr.csr_encode(XV, DV, s, idx=row(iV), coef=row(cV), workspace=wsE, **(dict(gram=GV) if use_gram[0] else {}))

    def attend():
        csr.csr_decode_attn(q, DK, v(iK), v(cK), DV, v(iV), v(cV), seq_lens=lens, out=out, workspace=wsD)

    def timed():
        for _ in range(2):
            append(); attend()
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for i in range(steps):
            ev[i][0].record(); append(); ev[i][1].record(); attend(); ev[i][2].record()
        torch.cuda.synchronize()
        return [median([e[j].elapsed_time(e[j + 1]) for e in ev]) for j in range(2)]

    use_gram[0] = False
    split_ms, _ = timed()
    split_row = (row(icache).clone(), row(ccache).clone())
    use_gram[0] = True
    a_ms, d_ms = timed()
    same_codes = bool(torch.equal(row(icache), split_row[0]))
    # the same step recorded once in a HIP graph and replayed: the launches lose their gaps
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            append(); attend()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a_, b_ in gev:
        a_.record(); graph.replay(); b_.record()
    torch.cuda.synchronize()
    g_ms = median([a_.elapsed_time(b_) for a_, b_ in gev])
    dict_bytes = 2 * Hkv * N * d * 2
    sweep_bytes = dict_bytes * s              # without G every iteration reads every dictionary once
    nvec = 2 * B * Hkv
    gram_bytes = dict_bytes + nvec * ((s - 1) * 2 * N + 2 * 4 * N)   # one sweep, a row of G per later iteration, C_1 out and in
    return {"append_vectors": nvec, "append_ms": round(a_ms, 4), "attend_ms_warm": round(d_ms, 5),
            "step_ms": round(a_ms + d_ms, 4), "step_ms_graph": round(g_ms, 4),
            "tokens_per_s": round(B / (min(g_ms, a_ms + d_ms) * 1e-3), 1),
            "workload": w.name, "decode_batch": B,
            "append_ms_without_gram": round(split_ms, 4), "same_atoms_as_without_gram": same_codes,
            "gram_matrices_mb": round(GKV.numel() * 2 / 1e6, 1),
            "roofline_append": {"kernel": "csr_encode with the dictionaries' Gram matrices (sweep + iterate, 2 launches)",
                                "bound": "hbm", "achieved": round(gram_bytes / (a_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "frac": round(gram_bytes / (a_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 5),
                                "bytes_per_step": gram_bytes,
                                "note": "one sweep of every dictionary, then s - 1 rows of G per vector: the iterations "
                                        "are a chain of dependent loads, one workgroup per vector"},
            "roofline_append_without_gram": {"kernel": "csr_encode (split), s + 1 launches per call", "bound": "hbm",
                                "achieved": round(sweep_bytes / (split_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "frac": round(sweep_bytes / (split_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 5),
                                "bytes_per_step": sweep_bytes,
                                "note": "s sweeps over all dictionaries; re-reads may be served by the Infinity Cache"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_layer")
    ap.add_argument("--algo", default="auto", choices=["auto", "valu", "mfma"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-decode", action="store_true",
                    help="skip the decode-only lines at the long-context and GQA shapes")
    ap.add_argument("--no-chunked", action="store_true",
                    help="skip the step in the chunked (s_n = 2 values) storage layout")
    ap.add_argument("--no-decode-step", action="store_true",
                    help="skip the decoding step (append one token's codes, then attend)")
    ap.add_argument("--no-extra-encode", action="store_true",
                    help="skip the encode-only lines at the long-context, GQA and prefill-stress shapes")
    ap.add_argument("--only-extra-encode", action="store_true",
                    help="run only the encode-only lines (for profiling them apart from the main workload)")
    ap.add_argument("--only-extra-decode", action="store_true",
                    help="run only the decode-only lines (for profiling them apart from the main workload)")
    ap.add_argument("--only-chunked", action="store_true", help="run only the chunked-layout step (for profiling)")
    ap.add_argument("--only-decode-step", action="store_true", help="run only the decoding step (for profiling)")
    ap.add_argument("--only-small-dict", action="store_true",
                    help="time the LDS-resident and the Gram-update encoder on small dictionaries (for profiling)")
    ap.add_argument("--no-rope", action="store_true", help="skip the rotary-key decode shapes")
    ap.add_argument("--only-rope", action="store_true", help="run only the rotary-key decode shapes (for profiling)")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="do not run the stand-alone matrix-core rate probe (a child process) first")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only copy 1 GiB device-to-device five times and exit: run under rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE, it shows what those counters read for a known amount of traffic")
    ap.add_argument("--cold-copies", type=int, default=16,
                    help="distinct input copies rotated through for the cache-cold decode figure")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU kernel path; run it with --gpus 1 "
              "(there is no sharded or multi-rank mode to measure)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.copy_calibration:
        torch.cuda.set_device(0)
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "copy_calibration_bytes_written": 1 << 30, "copies": 5}))
        return

    probe = None if args.no_mfma_probe else mfma_only_rate()

    import paper_2412_11741_amd as csr
    from paper_2412_11741_amd import synth

    if args.only_extra_decode:
        torch.cuda.set_device(0)
        print(json.dumps({"decode_rooflines": [decode_only(csr, synth.WORKLOADS[n], torch.device("cuda:0"))
                                               for n in ("long_context", "gqa_llama3_8b")]}))
        return

    if args.only_extra_encode:
        torch.cuda.set_device(0)
        print(json.dumps({"encode_rooflines": [encode_only(csr, synth.WORKLOADS[n], torch.device("cuda:0"), 3)
                                               for n in ("long_context", "gqa_llama3_8b", "prefill_stress")]}))
        return

    if args.only_small_dict:
        torch.cuda.set_device(0)
        print(json.dumps({"small_dict_encoders": small_dict_encoders(csr, torch.device("cuda:0"), args.steps)}))
        return

    if args.only_rope:
        torch.cuda.set_device(0)
        print(json.dumps({"rope_decode": rope_decode(csr, torch.device("cuda:0"), args.steps)}))
        return

    if args.only_chunked or args.only_decode_step:
        torch.cuda.set_device(0)
        w = synth.WORKLOADS[args.workload]
        leg = chunked_step if args.only_chunked else decode_step
        res = {"chunked_step" if args.only_chunked else "decode_step": leg(csr, synth, w, torch.device("cuda:0"), args.steps)}
        if args.only_decode_step:
            res["decode_step_gqa"] = decode_step(csr, synth, synth.WORKLOADS["gqa_llama3_8b"], torch.device("cuda:0"), args.steps)
            import dataclasses
            res["decode_step_batch64"] = decode_step(csr, synth, dataclasses.replace(w, name=w.name + " x 64 sequences", batch=64),
                                                     torch.device("cuda:0"), args.steps)
        if args.only_chunked and not args.no_rope:
            res["paper_sized_step"] = chunked_step(csr, synth, w, torch.device("cuda:0"), args.steps, n_atoms=256,
                                                   rope_base=10000.0)
        print(json.dumps(res))
        return

    w = synth.WORKLOADS[args.workload]
    if w.layers != 1:
        print("bench.py: only single-layer workloads are benchmark lines", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    algo = {"auto": csr.CSR_ENCODE_AUTO, "valu": csr.CSR_ENCODE_VALU, "mfma": csr.CSR_ENCODE_MFMA}[args.algo]
    tdt = torch.float16 if w.dtype == "f16" else torch.float32
    tit = torch.int16 if w.itype == "i16" else torch.int32

    # ---- synthetic inputs (host-generated, then resident on the GPU) ---------------------------
    B, Hkv, Hq, T, N, d, s = w.batch, w.hkv, w.hq, w.tokens, w.n_atoms, w.d, w.s
    DK = synth.dictionary(0, "dict_k", Hkv, N, d, w.dtype)
    DV = synth.dictionary(0, "dict_v", Hkv, N, d, w.dtype)
    q_h = synth.queries(0, B, Hq, d, w.dtype)
    # vectors of sequence b, KV head h live at row b*Hkv + h; keys first, then values
    XK = np.concatenate([synth.vectors(0, "keys", Hkv, T, d, w.dtype, outliers=w.key_outliers, token0=b)
                         for b in range(B)])
    XV = np.concatenate([synth.vectors(0, "values", Hkv, T, d, w.dtype, token0=b) for b in range(B)])
    X_h = np.concatenate([XK, XV])
    D_h = np.concatenate([np.tile(DK, (B, 1, 1)), np.tile(DV, (B, 1, 1))])
    X, D = torch.from_numpy(X_h).to(dev), torch.from_numpy(D_h).to(dev)
    DKg, DVg, q = torch.from_numpy(DK).to(dev), torch.from_numpy(DV).to(dev), torch.from_numpy(q_h).to(dev)
    H = X.shape[0]
    n_vec = H * T
    idx = torch.empty((H, T, s), dtype=tit, device=dev)
    coef = torch.empty((H, T, s), dtype=tdt, device=dev)
    out = torch.empty((B, Hq, d), dtype=tdt, device=dev)
    edesc = csr.encode_desc(X, D, s, tdt, tit, algo)
    ews = csr.csr_encode_workspace_bytes(edesc)
    enc_ws = torch.empty(max(ews, 256), dtype=torch.uint8, device=dev)
    nkv = B * Hkv
    idxK, coefK = idx[:nkv].view(B, Hkv, T, s), coef[:nkv].view(B, Hkv, T, s)
    idxV, coefV = idx[nkv:].view(B, Hkv, T, s), coef[nkv:].view(B, Hkv, T, s)
    ddesc = csr.decode_desc(q, DKg, idxK, coefK, idxV)
    dec_ws = torch.empty(max(csr.csr_decode_workspace_bytes(ddesc), 256), dtype=torch.uint8, device=dev)

    def encode():
        csr.csr_encode(X, D, s, tdt, tit, algo, idx=idx, coef=coef, workspace=enc_ws if ews else None)

    def decode(qq=q, dk=DKg, dv=DVg, ik=idxK, ck=coefK, iv=idxV, cv=coefV, o=out):
        csr.csr_decode_attn(qq, dk, ik, ck, dv, iv, cv, out=o, workspace=dec_ws)

    for _ in range(args.warmup):
        encode(); decode()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` passes ---------------------------------------------------
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        encode()
        ev[i][1].record()
        decode()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    enc_ms = median([e[0].elapsed_time(e[1]) for e in ev])
    dec_ms = median([e[1].elapsed_time(e[2]) for e in ev])

    # ---- cache-cold decode: rotate distinct copies so nothing is served from the Infinity Cache --
    code_b = csr.csr_code_bytes(s, 1, tit, tdt)
    dict_b = 2 if w.dtype == "f16" else 4
    dec_bytes = B * Hkv * T * 2 * code_b + Hkv * 2 * N * d * dict_b + B * Hq * d * 2 * dict_b
    copies = max(1, args.cold_copies)
    while copies > 1 and copies * dec_bytes > 24e9:
        copies //= 2
    sets = []
    for c in range(copies):
        sets.append(dict(qq=q.clone(), dk=DKg.clone(), dv=DVg.clone(), ik=idxK.clone(), ck=coefK.clone(),
                         iv=idxV.clone(), cv=coefV.clone(), o=torch.empty_like(out)))
    for c in range(copies):
        decode(**sets[c])
    torch.cuda.synchronize()
    reps = max(copies, 2 * copies if dec_bytes * copies < 4e9 else copies)
    cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for r in range(reps):
        cev[r][0].record()
        decode(**sets[r % copies])
        cev[r][1].record()
    torch.cuda.synchronize()
    dec_cold_ms = median([a.elapsed_time(b) for a, b in cev])
    del sets

    enc_flop = 2.0 * d * N * s * n_vec
    enc_tflops = enc_flop / (enc_ms * 1e-3) / 1e12
    uses_mfma = args.algo != "valu" and ews > 0
    roofline = {"kernel": "csr_encode (%s)" % ("mfma" if uses_mfma else "valu"),
                "bound": "mfma", "achieved": round(enc_tflops, 3), "peak": PEAK_MFMA_F16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(enc_tflops / PEAK_MFMA_F16_TFLOPS, 5),
                **recorded_traffic(PMC_TRAFFIC_BYTES, (w.name, "mfma" if uses_mfma else "valu")),
                "algorithmic_bytes": n_vec * (d * dict_b + code_b) + H * N * d * dict_b,
                "flop_per_vector": 2.0 * d * N * s, "median_launch_ms": round(enc_ms, 4),
                "avg_launch_ms": round(sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps, 4)}
    if probe:
        # the chip is power-limited under matrix-core load: a loop of nothing but this MFMA on random operands runs
        # well below the nominal peak, and that rate is what a kernel feeding the matrix cores real data can approach
        roofline["mfma_only_sustained"] = probe
        roofline["frac_of_mfma_only_encoder_like"] = round(enc_tflops / probe["mfma_only_tflops_encoder_like"], 5)
    dec_gbs = dec_bytes / (dec_cold_ms * 1e-3) / 1e9
    roofline_decode = {"kernel": "csr_decode_attn (4 launches), cache-cold", "bound": "hbm",
                       "achieved": round(dec_gbs, 2), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": round(dec_gbs / PEAK_HBM_GBS, 5), **recorded_traffic(PMC_DECODE_TRAFFIC_BYTES, w.name),
                       "bytes_per_call": dec_bytes, "median_call_ms": round(dec_cold_ms, 5),
                       "warm_call_ms": round(dec_ms, 5), "copies_rotated": copies}

    result = {
        "metric": "MP-encoded KV vectors/sec over the whole step (encode K+V, then decode attention on the codes)",
        "value": round(n_vec / (ms_step * 1e-3), 1), "unit": "vectors/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16" if uses_mfma else "f32", "data": "synthetic",
        "config": {"workload": w.name,
                   "workload_note": "the configuration the metric is quoted on (BASELINE.json configs[1]); the larger "
                                    "single-GPU shapes are in encode_rooflines and decode_rooflines",
                   "kv_heads": Hkv, "query_heads": Hq, "head_dim": d, "atoms": N,
                   "tokens_per_head": T, "s": s, "decode_batch": B, "vectors_per_step": n_vec,
                   "storage": f"{w.dtype}+{w.itype}", "encode_algo": args.algo},
        "encode_vectors_per_s": round(n_vec / (enc_ms * 1e-3), 1), "encode_ms": round(enc_ms, 4),
        "decode_ctx_tokens_per_s": round(B * T / (dec_cold_ms * 1e-3), 1),
        "decode_ctx_tokens_per_s_warm": round(B * T / (dec_ms * 1e-3), 1),
        "decode_ms_cold": round(dec_cold_ms, 5), "decode_ms_warm": round(dec_ms, 5),
        "roofline": roofline, "roofline_decode": roofline_decode,
    }

    # ---- Eq.12 on the step's codes: rebuild all keys and values densely (not part of the step) ---------------
    rec_out = torch.empty((H, T, d), dtype=tdt, device=dev)
    for _ in range(2):
        csr.csr_reconstruct(D, idx, coef, out=rec_out)
    rev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a_, b_ in rev:
        a_.record(); csr.csr_reconstruct(D, idx, coef, out=rec_out); b_.record()
    torch.cuda.synchronize()
    rec_ms = median([a_.elapsed_time(b_) for a_, b_ in rev])
    rec_bytes = n_vec * (code_b + d * dict_b)
    result["reconstruct"] = {"kernel": "csr_reconstruct", "bound": "hbm", "ms": round(rec_ms, 5),
                             "achieved": round(rec_bytes / (rec_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                             "unit": "GB/s", "frac": round(rec_bytes / (rec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 5),
                             "bytes_per_call": rec_bytes,
                             "note": "the s atom rows per vector (8x the output at s = 8) are gathers from L2: the "
                                     "address path of the CUs (64 B per clock each), not HBM, bounds this call"}
    del rec_out

    # ---- decode alone at the shapes where the code streams dominate (random codes, cache-cold) --------
    if not args.no_extra_decode:
        result["decode_rooflines"] = [decode_only(csr, synth.WORKLOADS[n], dev)
                                      for n in ("long_context", "gqa_llama3_8b")]

    # ---- encode alone at the full shapes of the larger configurations (one launch per layer) ------------------
    if not args.no_extra_encode and uses_mfma:
        torch.cuda.empty_cache()
        result["encode_rooflines"] = [encode_only(csr, synth.WORKLOADS[n], dev, 3)
                                      for n in ("long_context", "gqa_llama3_8b", "prefill_stress")]
        torch.cuda.empty_cache()

    # ---- the same layer in the chunked storage layout of the paper's experiments --------------------------
    if not args.no_chunked and w.dtype == "f16" and d == 128:
        result["chunked_step"] = chunked_step(csr, synth, w, dev, args.steps)
        # the same layer with the paper's own dictionary budget (256 atoms per head) and keys coded before the
        # rotary embedding: the LDS-resident encoder and the rotary-key decode together
        if not args.no_rope:
            result["paper_sized_step"] = chunked_step(csr, synth, w, dev, args.steps, n_atoms=256, rope_base=10000.0)

    # ---- one decoding step: append the new token's codes in place, attend over the grown cache ------------
    if not args.no_decode_step and w.dtype == "f16":
        result["decode_step"] = decode_step(csr, synth, w, dev, args.steps)
        if not args.no_extra_decode:
            # a batch of sequences on shared dictionaries: 8 new keys and 8 new values per dictionary and step
            result["decode_step_gqa"] = decode_step(csr, synth, synth.WORKLOADS["gqa_llama3_8b"], dev, args.steps)
            # the benchmark layer serving 64 sequences: 64 new keys and 64 new values per dictionary and step
            import dataclasses
            result["decode_step_batch64"] = decode_step(csr, synth, dataclasses.replace(w, name=w.name + " x 64 sequences", batch=64),
                                                        dev, args.steps)

    # ---- decode attention on keys coded before the rotary embedding, paper-sized dictionaries -------------
    if not args.no_rope:
        result["rope_decode"] = rope_decode(csr, dev, args.steps)

    # ---- CPU oracle on a bounded sample of the same workload ---------------------------------------
    if not args.no_cpu_baseline:
        import oracle
        per_dict = max(1, 131072 // H)   # ~10-15 s of oracle work on 16 host threads
        t1 = time.perf_counter()
        for h in range(H):
            oracle.mp_encode(X_h[h, :per_dict], D_h[h], s)
        cpu_enc = time.perf_counter() - t1
        ik_h, ck_h = idxK.cpu().numpy(), coefK.cpu().numpy()
        iv_h, cv_h = idxV.cpu().numpy(), coefV.cpu().numpy()
        t1 = time.perf_counter()
        oracle.decode_attn(q_h[:1], DK, ik_h[:1], ck_h[:1], DV, iv_h[:1], cv_h[:1])
        cpu_dec = time.perf_counter() - t1
        result["cpu_baseline"] = {
            "value": round(H * per_dict / cpu_enc, 1), "unit": "vectors/s", "cores": oracle.max_threads(),
            "kind": "oracle",
            "sample": f"encode: first {per_dict} vectors of each of the {H} dictionaries "
                      f"({H * per_dict} vectors, {cpu_enc:.1f} s); decode: sequence 0, all {Hq} heads "
                      f"({T} tokens, {cpu_dec:.2f} s)",
            "decode_ctx_tokens_per_s": round(T / cpu_dec, 1)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
