"""Comparison rules between a candidate encoder / decoder output and the CPU oracle.

Encode (per vector, walking the iterations in order):
  * same atom index as the oracle  -> the coefficient must agree within coef_tol * |c|, or within
    the absolute floor below if that is larger;
  * different index -> accepted only if, at that step, the oracle's best and runner-up
    |correlation| differ by at most tie_rel * best, or by at most the absolute floor (a tie: either
    atom is a correct greedy pick).
  Absolute floor: 2^-23 |x| (one fp32 ulp of the input's norm).  The candidate accumulates in fp32:
  its residual carries an absolute error of that order whatever the residual has shrunk to, so on a
  vector that is (nearly) a combination of a few atoms neither a correlation difference nor a
  coefficient below that floor can be resolved, while the fp64 oracle still resolves them.  With
  fp16 coefficient storage one storage ulp of the value is allowed on top (fp16 subnormals are
  spaced 6e-8 apart: a one-ulp flip there exceeds any relative tolerance).
    From there on the two paths legitimately differ, so the remaining steps of that vector are
    checked for greedy validity instead: each pick must reach the largest |R . d_n| of the residual
    built (in float64) from the candidate's own earlier picks, within tie_rel, and its coefficient
    must be that projection within coef_tol.
Decode: relative L2 error per (sequence, query head).
"""
from dataclasses import dataclass, field

import numpy as np

TIE_REL = 1e-6
FP32_ULP = 2.0 ** -23


@dataclass
class EncodeReport:
    vectors: int = 0
    steps: int = 0
    exact_steps: int = 0
    tie_vectors: int = 0          # vectors whose path left the oracle's at an accepted tie (either clause)
    floor_ties: int = 0           # ... of which only the absolute-floor clause (not the relative one) accepted
    floor_coefs: int = 0          # coefficients outside coef_tol * |c| that only the absolute floor accepted
    failures: list = field(default_factory=list)
    max_coef_err: float = 0.0

    @property
    def ok(self):
        return not self.failures

    def summary(self):
        return (f"{self.vectors} vectors, {self.exact_steps}/{self.steps} steps index-identical, "
                f"{self.tie_vectors} vectors diverged at an accepted tie ({self.floor_ties} by the absolute floor only), "
                f"{self.floor_coefs} coefficients accepted by the absolute floor only, "
                f"{len(self.failures)} failures, max rel coef err {self.max_coef_err:.3e}")


def _as_index(a):
    a = np.asarray(a)
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    return a.astype(np.int64)


def check_encode(X, D, idx_c, coef_c, idx_o, coef_o, diag, coef_tol, tie_rel=TIE_REL, max_report=10,
                 coef_storage="f32", coef_o_exact=None):
    """X [T, d], D [N, d] (the exact input bits, any float dtype); candidate and oracle codes [T, s];
    diag = the oracle's diagnostics dict for these vectors.  coef_o may be rounded to the storage type (it is what
    the candidate's stored values are compared with); coef_o_exact, the oracle's unrounded coefficients, is then
    what the residual of a vector that diverged at a tie is rebuilt from."""
    X = np.asarray(X, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    idx_c, idx_o = _as_index(idx_c), _as_index(idx_o)
    coef_c = np.asarray(coef_c, dtype=np.float64)
    coef_o = np.asarray(coef_o, dtype=np.float64)
    coef_rebuild = coef_o if coef_o_exact is None else np.asarray(coef_o_exact, dtype=np.float64)
    T, s = idx_o.shape
    rep = EncodeReport(vectors=T, steps=T * s)
    xnorm = np.linalg.norm(X, axis=1)
    same = idx_c == idx_o
    # number of leading steps that agree, per vector
    lead = np.where(same.all(axis=1), s, np.argmin(same, axis=1))
    rep.exact_steps = int(same.sum())
    abs_floor = FP32_ULP * xnorm                       # per vector
    ulp = np.zeros_like(coef_o)
    if coef_storage == "f16":
        ulp = np.spacing(np.abs(coef_o).astype(np.float16)).astype(np.float64)
    # error measured against the larger of |c| and (floor + storage ulp) / coef_tol: `rel <= coef_tol` then
    # reads |err| <= max(coef_tol |c|, floor + ulp)
    denom = np.maximum(np.abs(coef_o), (abs_floor[:, None] + ulp) / coef_tol)
    rel = np.abs(coef_c - coef_o) / np.where(denom > 0, denom, 1.0)
    # the same error against |c| alone: where it exceeds coef_tol although `rel` does not, the floor decided
    plain = np.abs(coef_c - coef_o) > coef_tol * np.abs(coef_o)
    for t in range(T):
        L = int(lead[t])
        if L:
            e = float(rel[t, :L].max())
            rep.floor_coefs += int(np.count_nonzero(plain[t, :L] & (rel[t, :L] <= coef_tol)))
            rep.max_coef_err = max(rep.max_coef_err, e)
            if e > coef_tol and len(rep.failures) < max_report:
                g = int(np.argmax(rel[t, :L]))
                rep.failures.append(f"vector {t} step {g}: coef {coef_c[t, g]!r} vs oracle {coef_o[t, g]!r}")
        if L == s:
            continue
        best, second = diag["best_abs"][t, L], diag["second_abs"][t, L]
        if best - second > max(tie_rel * best, abs_floor[t]):
            if len(rep.failures) < max_report:
                rep.failures.append(f"vector {t} step {L}: index {idx_c[t, L]} vs oracle {idx_o[t, L]} "
                                    f"(best {best!r}, runner-up {second!r}: not a tie)")
            continue
        rep.tie_vectors += 1
        if best - second > tie_rel * best:
            rep.floor_ties += 1
        # greedy validity of the candidate's own path from step L on
        R = X[t].copy()
        for g in range(L):
            R -= coef_rebuild[t, g] * D[idx_o[t, g]]
        for g in range(L, s):
            C = D @ R
            a = np.abs(C)
            n = int(idx_c[t, g])
            if a[n] < a.max() - max(tie_rel * a.max(), abs_floor[t]) - 1e-300:
                if len(rep.failures) < max_report:
                    rep.failures.append(f"vector {t} step {g} (after tie at {L}): index {n} is not a greedy pick")
                break
            u16 = float(np.spacing(np.float16(abs(C[n])))) if coef_storage == "f16" else 0.0
            e = abs(coef_c[t, g] - C[n]) / max(abs(C[n]), (abs_floor[t] + u16) / coef_tol, 1e-300)
            rep.max_coef_err = max(rep.max_coef_err, float(e))
            if e > coef_tol:
                if len(rep.failures) < max_report:
                    rep.failures.append(f"vector {t} step {g} (after tie at {L}): coef {coef_c[t, g]!r} vs {C[n]!r}")
                break
            R -= C[n] * D[n]
    return rep


def decode_errors(out_c, out_o):
    """Relative L2 error per (b, hq), and the largest absolute error of any element relative to the largest
    |element| of its own (b, hq) output vector (0 where that vector is all zero)."""
    out_c = np.asarray(out_c, dtype=np.float64)
    out_o = np.asarray(out_o, dtype=np.float64)
    if not out_o.size:
        return np.zeros(out_o.shape[:-1]), 0.0
    num = np.linalg.norm(out_c - out_o, axis=-1)
    den = np.linalg.norm(out_o, axis=-1)
    rel = np.where(den > 0, num / np.where(den > 0, den, 1.0), num)
    peak = np.abs(out_o).max(axis=-1)
    worst = np.abs(out_c - out_o).max(axis=-1)
    mx = np.where(peak > 0, worst / np.where(peak > 0, peak, 1.0), worst)
    return rel, float(mx.max())


def assert_decode_close(out_c, out_o, tol, what=""):
    """Both rules of the decode comparison: relative L2 error per (sequence, query head) and every element's
    absolute error against the largest |element| of its output vector, each at most tol."""
    rel, mx = decode_errors(out_c, out_o)
    assert np.all(np.isfinite(np.asarray(out_c, dtype=np.float64))), what + ": non-finite output"
    assert rel.size == 0 or rel.max() <= tol, f"{what}: relative L2 error {rel.max():.3e} above {tol:.1e}"
    assert mx <= tol, f"{what}: largest element error {mx:.3e} of the vector's peak, above {tol:.1e}"
    return rel, mx
