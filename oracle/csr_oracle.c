/*
 * CPU oracle for the CSR sparse-representation hot path (arXiv 2412.11741).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  Only the test suite, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product path never does.
 * It shares no code, header, table or helper with the HIP implementation.
 *
 * What is here, and the passage of the paper each function follows:
 *
 *   csr_oracle_mp_encode     Matching Pursuit, Section "Sparse representation",
 *                            Eq.2 (coefficient), Eq.3 (atom index), Eq.4
 *                            (residual update), run for exactly s iterations
 *                            (Section "KV Decomposition and Sparse Storage").
 *   csr_oracle_reconstruct   De-sparse X~ = D r, Eq.12 (Section "De-Sparse to
 *                            restore").
 *   csr_oracle_decode_attn   Attention of one query token per sequence over the
 *                            reconstructed K~ / V~ (Eq.12 followed by ordinary
 *                            softmax attention, as the last paragraph of
 *                            "De-Sparse to restore" prescribes).
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - Eq.2 prints the coefficient as a supremum of absolute values, yet Eq.4
 *     subtracts c_g * d_{i_g}.  Only the SIGNED projection c_g = R_g . d_{i_g}
 *     makes Eq.4 shrink the residual, so that is what is computed.
 *   - The residual starts as the vector itself and exactly s iterations run;
 *     pairs are emitted in iteration order.
 *   - The same atom may be picked again later; the code is a list of s pairs
 *     and D r means the sum of c_g * d_{i_g} over the list.
 *   - Ties in Eq.3 go to the lowest atom index.  An all-zero correlation gives
 *     index 0, coefficient 0.
 *   - No division by |d|^2: atoms are taken as unit norm as Section "Sparse
 *     representation" states; the dictionary bits are used as given.
 *   - Eq.4 uses the unrounded coefficient; rounding to the storage type is the
 *     caller's business (done on the returned doubles).  That is the default
 *     ("open loop").  Section "Analysis for CSR" stores the coefficients as
 *     fp16, and Eq.4 does not say which value it subtracts; the other reading
 *     ("closed loop") is offered as an option: the coefficient is rounded to
 *     its storage type first, the ROUNDED value is what is stored and what
 *     Eq.4 subtracts, so that the residual the iterations work on is exactly
 *     the error of the code as it is stored.
 *   - Attention scale is a parameter (the paper never writes the formula); no
 *     mask, no position embedding (Section "KV cache in attention" sets the
 *     position embedding aside).
 *   - A sequence with zero cached tokens yields an all-zero output row.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force best atom, orthonormal
 * dictionaries reducing to top-|s| selection, the energy identity, exact
 * reconstruction at s = d, textbook softmax attention special cases.
 *
 * All arrays are row-major doubles / int32; a dictionary is atom-major
 * D[n][k], n < N, k < d.  Threads (OpenMP) split independent vectors or
 * (batch, head) pairs only; no arithmetic is reordered by threading.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int csr_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * x rounded to the nearest fp16 value (IEEE binary16: 10 fraction bits, exponents -14 .. 15, subnormals with a
 * spacing of 2^-24, ties to even, overflow to infinity), returned as a double.  Written from the format's
 * definition: the spacing of fp16 values around x is 2^(e - 10) with e = floor(log2 |x|), at least -14.
 */
static double round_to_half(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(fabs(x), &e);        /* |x| = f 2^e, f in [0.5, 1)  =>  floor(log2 |x|) = e - 1 */
    int e2 = e - 1;
    if (e2 < -14) e2 = -14;
    const double q = ldexp(1.0, e2 - 10);
    const double r = nearbyint(x / q) * q;   /* default rounding mode: to nearest, ties to even */
    if (fabs(r) > 65504.0) return x > 0 ? INFINITY : -INFINITY;
    return r;
}

/*
 * Matching Pursuit for T vectors against one dictionary.
 *   X          [T][d]   input vectors
 *   D          [N][d]   atoms (rows)
 *   idx        [T][s]   out: atom picked at iteration g (Eq.3)
 *   coef       [T][s]   out: signed projection at iteration g (Eq.2, signed reading)
 *   best_abs   [T][s]   out (may be NULL): |C| of the picked atom
 *   second_abs [T][s]   out (may be NULL): largest |C| among all other atoms
 *   res_norm2  [T][s+1] out (may be NULL): |R_g|^2 before iteration g = 1..s, then after the last
 *   closed_loop  0: Eq.4 subtracts the unrounded coefficient, which is also what is returned;
 *                1 / 2: the coefficient is rounded to fp16 / fp32 first; the rounded value is returned
 *                and subtracted (see the readings above)
 * Returns 0, or -1 on bad sizes / allocation failure.
 */
int csr_oracle_mp_encode(const double *X, const double *D, int64_t T, int d, int N, int s,
                         int32_t *idx, double *coef, double *best_abs, double *second_abs,
                         double *res_norm2, int nthreads, int closed_loop)
{
    if (T < 0 || d <= 0 || N <= 0 || s < 0 || closed_loop < 0 || closed_loop > 2) return -1;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *R = (double *)malloc(sizeof(double) * (size_t)d);
        double *C = (double *)malloc(sizeof(double) * (size_t)N);
        if (!R || !C) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            fail = 1;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 8)
#endif
            for (int64_t t = 0; t < T; ++t) {
                /* R_1 = x */
                for (int k = 0; k < d; ++k) R[k] = X[t * d + k];
                for (int g = 0; g < s; ++g) {
                    if (res_norm2) {
                        double e = 0.0;
                        for (int k = 0; k < d; ++k) e += R[k] * R[k];
                        res_norm2[t * (s + 1) + g] = e;
                    }
                    /* correlations of the residual with every atom */
                    for (int n = 0; n < N; ++n) {
                        const double *dn = D + (size_t)n * d;
                        double acc = 0.0;
                        for (int k = 0; k < d; ++k) acc += R[k] * dn[k];
                        C[n] = acc;
                    }
                    /* Eq.3: first atom of largest |C| */
                    int best = 0;
                    double babs = fabs(C[0]);
                    for (int n = 1; n < N; ++n) {
                        double a = fabs(C[n]);
                        if (a > babs) { babs = a; best = n; }
                    }
                    if (second_abs) {
                        double sabs = 0.0;
                        for (int n = 0; n < N; ++n) {
                            if (n == best) continue;
                            double a = fabs(C[n]);
                            if (a > sabs) sabs = a;
                        }
                        second_abs[t * s + g] = sabs;
                    }
                    if (best_abs) best_abs[t * s + g] = babs;
                    /* Eq.2 read as the signed projection */
                    double c = C[best];
                    if (closed_loop == 1) c = round_to_half(c);
                    else if (closed_loop == 2) c = (double)(float)c;
                    idx[t * s + g] = best;
                    coef[t * s + g] = c;
                    /* Eq.4 */
                    const double *db = D + (size_t)best * d;
                    for (int k = 0; k < d; ++k) R[k] -= c * db[k];
                }
                if (res_norm2) {
                    double e = 0.0;
                    for (int k = 0; k < d; ++k) e += R[k] * R[k];
                    res_norm2[t * (s + 1) + s] = e;
                }
            }
        }
        free(R);
        free(C);
    }
    return fail ? -1 : 0;
}

/*
 * Eq.12: Xt[t] = sum_g coef[t][g] * D[idx[t][g]].  Repeated indices add up.
 * Returns 0, or -2 if an index is outside [0, N).
 */
int csr_oracle_reconstruct(const int32_t *idx, const double *coef, const double *D, int64_t T,
                           int d, int N, int s, double *Xt)
{
    for (int64_t t = 0; t < T; ++t) {
        double *o = Xt + t * d;
        for (int k = 0; k < d; ++k) o[k] = 0.0;
        for (int g = 0; g < s; ++g) {
            int32_t n = idx[t * s + g];
            if (n < 0 || n >= N) return -2;
            double c = coef[t * s + g];
            const double *dn = D + (size_t)n * d;
            for (int k = 0; k < d; ++k) o[k] += c * dn[k];
        }
    }
    return 0;
}

/*
 * Decode attention on reconstructed keys and values.
 *   q      [B][Hq][d]           one query token per sequence and query head
 *   DK,DV  [Hkv][N][d]          key / value dictionaries, shared by the batch
 *   idxK   [B][Hkv][T][sK], coefK likewise; idxV/coefV with sV
 *   seq_lens [B] or NULL        number of valid cached tokens (<= T); NULL = T
 *   out    [B][Hq][d]
 * Query head hq reads KV head hq / (Hq / Hkv).
 * For each (b, hq): K~ = D_K r_K, V~ = D_V r_V (Eq.12); score_t = scale * q . K~_t;
 * p = softmax(score); out = sum_t p_t V~_t.
 */
int csr_oracle_decode_attn(const double *q, const double *DK, const int32_t *idxK,
                           const double *coefK, const double *DV, const int32_t *idxV,
                           const double *coefV, int B, int Hq, int Hkv, int64_t T, int d, int N,
                           int sK, int sV, double scale, const int32_t *seq_lens, double *out,
                           int nthreads)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || T < 0 || d <= 0 || N <= 0) return -1;
    const int G = Hq / Hkv;
    int fail = 0;
    const int64_t pairs = (int64_t)B * Hkv;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int64_t bh = 0; bh < pairs; ++bh) {
        const int b = (int)(bh / Hkv), h = (int)(bh % Hkv);
        int64_t L = seq_lens ? seq_lens[b] : T;
        if (L < 0 || L > T) { fail = 1; continue; }
        double *Kt = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * d);
        double *Vt = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * d);
        double *sc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        if (!Kt || !Vt || !sc) { fail = 1; free(Kt); free(Vt); free(sc); continue; }
        const size_t cK = ((size_t)b * Hkv + h) * (size_t)T * sK;
        const size_t cV = ((size_t)b * Hkv + h) * (size_t)T * sV;
        int rc = csr_oracle_reconstruct(idxK + cK, coefK + cK, DK + (size_t)h * N * d, L, d, N, sK, Kt);
        if (rc == 0)
            rc = csr_oracle_reconstruct(idxV + cV, coefV + cV, DV + (size_t)h * N * d, L, d, N, sV, Vt);
        if (rc != 0) { fail = 2; free(Kt); free(Vt); free(sc); continue; }
        for (int g = 0; g < G; ++g) {
            const int hq = h * G + g;
            const double *qv = q + ((size_t)b * Hq + hq) * d;
            double *o = out + ((size_t)b * Hq + hq) * d;
            for (int k = 0; k < d; ++k) o[k] = 0.0;
            if (L == 0) continue;
            double m = -INFINITY;
            for (int64_t t = 0; t < L; ++t) {
                double acc = 0.0;
                for (int k = 0; k < d; ++k) acc += qv[k] * Kt[t * d + k];
                sc[t] = scale * acc;
                if (sc[t] > m) m = sc[t];
            }
            double l = 0.0;
            for (int64_t t = 0; t < L; ++t) { sc[t] = exp(sc[t] - m); l += sc[t]; }
            for (int64_t t = 0; t < L; ++t) {
                double p = sc[t] / l;
                for (int k = 0; k < d; ++k) o[k] += p * Vt[t * d + k];
            }
        }
        free(Kt); free(Vt); free(sc);
    }
    return fail ? -fail : 0;
}
