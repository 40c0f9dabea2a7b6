/*
 * The C ABI used from plain C, without Python or PyTorch: Matching Pursuit encode of a few vectors, Eq.12
 * reconstruction of the codes, decode attention over them.  Checks status codes and two facts that need no
 * oracle: a vector that is a multiple of an atom is coded as that atom with that coefficient, and attention over
 * a single cached token returns that token's (reconstructed) value whatever the query is.
 * Built by the package's build step (hipcc as the C compiler driver for the host), run by the GPU tests.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "csr.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_CSR(x) do { csr_status s_ = (x); if (s_ != CSR_OK) { printf("csr status %d at line %d: %s\n", (int)s_, __LINE__, csr_last_error()); return 3; } } while (0)

/* fp32 -> fp16 bits, round to nearest even (normal range is all this program needs) */
static unsigned short to_half(float f)
{
    unsigned int x;
    memcpy(&x, &f, 4);
    unsigned int sign = (x >> 16) & 0x8000u, exp = (x >> 23) & 0xffu, man = x & 0x7fffffu;
    if (exp == 0) return (unsigned short)sign;
    int e = (int)exp - 127 + 15;
    if (e <= 0) return (unsigned short)sign;
    if (e >= 31) return (unsigned short)(sign | 0x7c00u);
    unsigned int h = (unsigned int)(e << 10) | (man >> 13);
    unsigned int rem = man & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;
    return (unsigned short)(sign | h);
}
static float from_half(unsigned short h)
{
    unsigned int sign = (unsigned int)(h & 0x8000u) << 16, exp = (h >> 10) & 0x1fu, man = h & 0x3ffu, x;
    if (exp == 0) {
        if (man == 0) x = sign;
        else { int e = -1; do { ++e; man <<= 1; } while (!(man & 0x400u)); x = sign | (unsigned int)(127 - 15 - e) << 23 | (man & 0x3ffu) << 13; }
    } else x = sign | (exp - 15 + 127) << 23 | man << 13;
    float f;
    memcpy(&f, &x, 4);
    return f;
}

int main(void)
{
    enum { H = 2, T = 4, D = 128, N = 256, S = 4 };  /* T * S * 2 bytes: the second block of codes stays 16-byte aligned */
    printf("csr_version %d\n", csr_version());
    unsigned short *hD = (unsigned short *)malloc(sizeof(unsigned short) * H * N * D);
    unsigned short *hX = (unsigned short *)calloc(H * T * D, sizeof(unsigned short));
    unsigned int seed = 12345u;
    for (int h = 0; h < H; ++h)
        for (int n = 0; n < N; ++n) {
            float row[D], ss = 0.0f;
            for (int k = 0; k < D; ++k) { seed = seed * 1664525u + 1013904223u; row[k] = (float)(seed >> 8) / 8388608.0f - 1.0f; ss += row[k] * row[k]; }
            for (int k = 0; k < D; ++k) hD[((size_t)h * N + n) * D + k] = to_half(row[k] / sqrtf(ss));
        }
    /* vector (h, t) = (t + 1.5) times atom 10 h + 7 t + 3 */
    for (int h = 0; h < H; ++h)
        for (int t = 0; t < T; ++t)
            for (int k = 0; k < D; ++k)
                hX[((size_t)h * T + t) * D + k] = to_half((t + 1.5f) * from_half(hD[((size_t)h * N + 10 * h + 7 * t + 3) * D + k]));

    void *dD, *dX, *dIdx, *dCoef, *dRec, *dQ, *dOut, *dWs = NULL;
    CHECK_HIP(hipMalloc(&dD, sizeof(unsigned short) * H * N * D));
    CHECK_HIP(hipMalloc(&dX, sizeof(unsigned short) * H * T * D));
    CHECK_HIP(hipMalloc(&dIdx, 2 * H * T * S));
    CHECK_HIP(hipMalloc(&dCoef, 2 * H * T * S));
    CHECK_HIP(hipMalloc(&dRec, 2 * H * T * D));
    CHECK_HIP(hipMalloc(&dQ, 2 * H * D));
    CHECK_HIP(hipMalloc(&dOut, 2 * H * D));
    CHECK_HIP(hipMemcpy(dD, hD, sizeof(unsigned short) * H * N * D, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dX, hX, sizeof(unsigned short) * H * T * D, hipMemcpyHostToDevice));

    csr_encode_desc e;
    memset(&e, 0, sizeof e);
    e.H = H; e.T = T; e.d = D; e.N = N; e.s = S; e.x_dtype = CSR_F16; e.dict_dtype = CSR_F16; e.coef_dtype = CSR_F16;
    e.idx_dtype = CSR_I16; e.algo = CSR_ENCODE_AUTO;
    size_t need = csr_encode_workspace_bytes(&e);
    if (need == (size_t)-1) { printf("bad encode descriptor: %s\n", csr_last_error()); return 4; }
    if (need) CHECK_HIP(hipMalloc(&dWs, need));
    CHECK_CSR(csr_encode(&e, dX, dD, dIdx, dCoef, dWs, need, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    unsigned short hIdx[H * T * S], hCoef[H * T * S];
    CHECK_HIP(hipMemcpy(hIdx, dIdx, sizeof hIdx, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hCoef, dCoef, sizeof hCoef, hipMemcpyDeviceToHost));
    for (int h = 0; h < H; ++h)
        for (int t = 0; t < T; ++t) {
            int i0 = hIdx[(h * T + t) * S];
            float c0 = from_half(hCoef[(h * T + t) * S]);
            if (i0 != 10 * h + 7 * t + 3 || fabsf(c0 - (t + 1.5f)) > 4e-3f * (t + 1.5f)) {
                printf("encode: vector (%d, %d) gave atom %d coefficient %g\n", h, t, i0, c0);
                return 5;
            }
        }

    csr_reconstruct_desc r;
    memset(&r, 0, sizeof r);
    r.H = H; r.T = T; r.d = D; r.N = N; r.s = S; r.dict_dtype = CSR_F16; r.coef_dtype = CSR_F16; r.idx_dtype = CSR_I16;
    r.out_dtype = CSR_F16;
    CHECK_CSR(csr_reconstruct(&r, dD, dIdx, dCoef, dRec, NULL));

    /* decode: the two blocks are the key and the value cache of one head; one cached token */
    csr_decode_desc q;
    memset(&q, 0, sizeof q);
    q.B = 1; q.Hq = 1; q.Hkv = 1; q.T = T; q.d = D; q.N = N; q.sK = S; q.sV = S; q.q_dtype = CSR_F16; q.dict_dtype = CSR_F16;
    q.coef_dtype = CSR_F16; q.idx_dtype = CSR_I16; q.out_dtype = CSR_F16;
    size_t dneed = csr_decode_workspace_bytes(&q);
    if (dneed == (size_t)-1) { printf("bad decode descriptor: %s\n", csr_last_error()); return 6; }
    void *dWs2, *dLens;
    CHECK_HIP(hipMalloc(&dWs2, dneed ? dneed : 256));
    CHECK_HIP(hipMalloc(&dLens, 4));
    int one = 1;
    CHECK_HIP(hipMemcpy(dLens, &one, 4, hipMemcpyHostToDevice));
    unsigned short hQ[D];
    for (int k = 0; k < D; ++k) hQ[k] = to_half((float)(k % 7) - 3.0f);
    CHECK_HIP(hipMemcpy(dQ, hQ, sizeof hQ, hipMemcpyHostToDevice));
    const char *idxV = (const char *)dIdx + 2 * T * S, *coefV = (const char *)dCoef + 2 * T * S;
    CHECK_CSR(csr_decode_attn(&q, dQ, dD, dIdx, dCoef, (const char *)dD + 2 * N * D, idxV, coefV, (const int32_t *)dLens, dOut,
                              dWs2, dneed, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    unsigned short hOut[D], hRec[H * T * D];
    CHECK_HIP(hipMemcpy(hOut, dOut, sizeof hOut, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hRec, dRec, sizeof hRec, hipMemcpyDeviceToHost));
    double err = 0.0, ref = 0.0;
    for (int k = 0; k < D; ++k) {
        const double a = from_half(hOut[k]), b = from_half(hRec[(1 * T + 0) * D + k]);   /* value block, token 0 */
        err += (a - b) * (a - b);
        ref += b * b;
    }
    if (!(ref > 0.0) || sqrt(err / ref) > 2e-3) { printf("decode: one cached token, relative error %g\n", sqrt(err / ref)); return 7; }

    /* the entry point that allocates nothing (its scratch is a static device array of the library): same bits */
    {
        unsigned short hOutS[D];
        CHECK_HIP(hipMemset(dOut, 0, 2 * D));
        CHECK_CSR(csr_decode_attn_static(&q, dQ, dD, dIdx, dCoef, (const char *)dD + 2 * N * D, idxV, coefV,
                                         (const int32_t *)dLens, dOut, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hOutS, dOut, sizeof hOutS, hipMemcpyDeviceToHost));
        if (memcmp(hOut, hOutS, sizeof hOut) != 0) { printf("csr_decode_attn_static differs from csr_decode_attn\n"); return 14; }
    }
    /* the encoder's indices all lie inside the dictionary; with a dictionary one atom shorter, those equal to N - 1 do not */
    {
        long long *dBad, hBad[2];
        int top = 0;
        CHECK_HIP(hipMalloc((void **)&dBad, 16));
        CHECK_CSR(csr_check_codes(dIdx, CSR_I16, (int64_t)H * T * S, N, (int64_t *)dBad, NULL));
        CHECK_CSR(csr_check_codes(dIdx, CSR_I16, (int64_t)H * T * S, N - 1, (int64_t *)(dBad + 1), NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hBad, dBad, sizeof hBad, hipMemcpyDeviceToHost));
        for (int i = 0; i < H * T * S; ++i) top += hIdx[i] == N - 1;
        if (hBad[0] != 0 || hBad[1] != top) { printf("csr_check_codes counted %lld and %lld (expected 0 and %d)\n", hBad[0], hBad[1], top); return 15; }
        CHECK_HIP(hipFree(dBad));
    }

    /* the same attention with the keys taken as coded before the rotary embedding: with a single cached token the
     * soft-max weight is 1 whatever the rotation, so the output is again that token's value */
    q.rope_base = 10000.0f; q.rope_layout = 0; q.rope_pos0 = 5;
    if (csr_decode_workspace_bytes(&q) > (dneed ? dneed : 256)) { printf("rotary decode wants a larger workspace\n"); return 9; }
    CHECK_HIP(hipMemset(dOut, 0, 2 * D));
    CHECK_CSR(csr_decode_attn(&q, dQ, dD, dIdx, dCoef, (const char *)dD + 2 * N * D, idxV, coefV, (const int32_t *)dLens, dOut,
                              dWs2, dneed ? dneed : 256, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    unsigned short hOut2[D];
    CHECK_HIP(hipMemcpy(hOut2, dOut, sizeof hOut2, hipMemcpyDeviceToHost));
    if (memcmp(hOut, hOut2, sizeof hOut) != 0) { printf("rotary decode of one cached token differs from the plain one\n"); return 10; }

    /* the Gram-update encoder is a different kernel for the same codes */
    e.algo = CSR_ENCODE_GRAM;
    CHECK_HIP(hipMemset(dIdx, 0xff, sizeof hIdx));
    CHECK_CSR(csr_encode(&e, dX, dD, dIdx, dCoef, NULL, 0, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    unsigned short hIdx2[H * T * S];
    CHECK_HIP(hipMemcpy(hIdx2, dIdx, sizeof hIdx2, hipMemcpyDeviceToHost));
    if (memcmp(hIdx, hIdx2, sizeof hIdx) != 0) { printf("the Gram encoder picked other atoms\n"); return 11; }
    e.algo = CSR_ENCODE_AUTO;

    /* and so is the one that takes the dictionaries' Gram matrices from device memory (T vectors per dictionary) */
    {
        void *dG = NULL, *dWs2 = NULL;
        size_t gbytes = csr_gram_bytes(H, N);
        CHECK_HIP(hipMalloc(&dG, gbytes));
        CHECK_CSR(csr_gram_build(dD, H, N, D, dG, NULL));
        e.gram = dG;
        size_t need2 = csr_encode_workspace_bytes(&e);
        if (need2 == (size_t)-1 || need2 == 0) { printf("bad descriptor with gram: %s\n", csr_last_error()); return 12; }
        CHECK_HIP(hipMalloc(&dWs2, need2));
        CHECK_HIP(hipMemset(dIdx, 0xff, sizeof hIdx));
        CHECK_CSR(csr_encode(&e, dX, dD, dIdx, dCoef, dWs2, need2, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hIdx2, dIdx, sizeof hIdx2, hipMemcpyDeviceToHost));
        if (memcmp(hIdx, hIdx2, sizeof hIdx) != 0) { printf("the Gram-step encoder picked other atoms\n"); return 13; }
        e.gram = NULL;
        CHECK_HIP(hipFree(dG));
        CHECK_HIP(hipFree(dWs2));
    }

    /* an invalid request comes back as a status with a message, not as a crash */
    e.s = 0;
    if (csr_encode(&e, dX, dD, dIdx, dCoef, dWs, need, NULL) != CSR_ERR_INVALID_ARG || csr_last_error()[0] == 0) return 8;
    printf("c abi smoke ok: encode (three kernels), reconstruct, decode (workspace, static scratch, rotary keys; rel err %.2e), code check\n", sqrt(err / ref));
    return 0;
}
