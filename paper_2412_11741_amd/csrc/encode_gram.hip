// Matching Pursuit encoder with the Gram-matrix residual update, for dictionaries of at most 256 atoms (gfx950).
//
// Eq.2-4 of Section "Sparse representation".  All correlations C_g[n] = R_g . d_n obey
//     C_{g+1}[n] = (R_g - c_g d_i) . d_n = C_g[n] - c_g G[i][n],        G = D D^T,
// so after one matrix-core sweep C_1 = D x every further iteration is an N-long multiply-add per vector instead
// of another sweep over the dictionary.  A workgroup builds the Gram matrix of its dictionary once with the matrix
// cores and keeps it in LDS in fp16 (N x N x 2 bytes <= 128 KB).  The rounding of G makes the recursion a SCREEN,
// exactly like the fp16 sweeps of the other encoders: |C_g[n] - R_g . d_n| <= delta_g with
//     delta_1 = gamma |x| dmax,    delta_{g+1} = delta_g + |c_g| dmax^2 (2^-12 + gamma) + 2^-22 rmax dmax
// (gamma bounds the fp32 accumulation of a dot product of exact fp16 products; |G| <= dmax^2; rmax is the largest
// residual norm so far).  The decision is
// taken exactly: every vector keeps its residual R in fp32 registers, gathers the rows of the screen's best AND
// second-best atom, and computes both R . d in fp32 - the coefficient of Eq.3 needs the winner's anyway.  When the
// second is within 2 delta of the first, the exact values decide (lowest index on ties); when even the third is,
// all atoms inside the band are evaluated exactly (rare).  Eq.4 then updates R with the unrounded coefficient.
//
// Mapping.  v_mfma_f32_16x16x32_f16: a wave works on 16 vectors at a time, 4 lanes per vector.  Lane
// (col = lane % 16, q = lane / 16) holds 8 dimensions of every 32-dimension slice of vector col's residual and the
// correlations of atoms 16 t + 4 q + e (t < N / 16, e < 4): the matrix-core result layout, so C_1 needs no
// shuffling.  A row of G is stored so that these atoms are contiguous for each q (position q N/4 + 4 t + e), with
// the row's 16-byte pieces XOR-swizzled by the row number: the 16 vectors of a wave read 16 different rows at once.
#include <atomic>

#include "csr_internal.h"
#include "encode_common.h"

namespace csr {
namespace {

using namespace enc;

constexpr int kWaves = 8;                    // two per SIMD, 256 registers each; one workgroup per CU (G fills the LDS)
constexpr int kThreads = 64 * kWaves;
constexpr int kBlocksPerWave = 4;            // 16-vector blocks a wave works through, one after the other
constexpr int kTokPerWG = kWaves * kBlocksPerWave * 16;  // 512
constexpr int kMaxAtoms = 256;
constexpr int kMaxTiles = kMaxAtoms / 16;

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// sum over the 4 lanes of a vector (lanes col, col + 16, col + 32, col + 48)
__device__ __forceinline__ float sum4(float v)
{
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// (a1 >= a2 >= a3) merged with the same triple of lane ^ m: the three largest of the six
__device__ __forceinline__ void merge3(uint32_t &a1, uint32_t &a2, uint32_t &a3, int m)
{
    const uint32_t b1 = (uint32_t)__shfl_xor((int)a1, m, 64), b2 = (uint32_t)__shfl_xor((int)a2, m, 64),
                   b3 = (uint32_t)__shfl_xor((int)a3, m, 64);
    const uint32_t m1 = umax(a1, b1);
    const uint32_t lo1 = umin(a1, b1);  // the smaller of the two leaders
    const uint32_t m2 = umax(lo1, umax(a2, b2));
    // third: the second largest of {lo1, a2, b2} or the largest of {a3, b3}
    a3 = umax(umed3(lo1, a2, b2), umax(a3, b3));
    a1 = m1;
    a2 = m2;
}

template <int DC>
__global__ __launch_bounds__(kThreads) void encode_gram_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, int64_t T, int64_t M, int32_t N, int32_t s, int32_t sn, int64_t x_stride_h, int64_t x_stride_t,
    int32_t dict_count, int64_t code_stride_h, int32_t tiles_per_h, int32_t idx16, int32_t coef16,
    float *__restrict__ res_norm2)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    constexpr int kF = DC / 32;  // matrix-core steps per product; a lane holds 8 dimensions of each

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, q = lane >> 4;
    // work is dealt per dictionary: dct = dictionary * sn + chunk owns the vectors of all blocks that use it
    // (block h uses dictionary h % dict_count), numbered m = (h / dict_count) * T + t, in tiles of 512
    const int dct = blockIdx.x / tiles_per_h;
    const int tile_wg = blockIdx.x - dct * tiles_per_h;
    const int dict = dct / sn, ch = dct - dict * sn;
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    const int ntile = N >> 4;            // 16-atom tiles
    const int row_bytes = N * 2;         // a row of G in LDS
    const int pieces = N >> 3;           // its 16-byte pieces (a multiple of 4)
    const int qpieces = pieces >> 2;     // pieces per lane quarter
    float *red = reinterpret_cast<float *>(lds + (size_t)N * row_bytes);

    // this lane's fragment of atom row n: dimensions 32 f + 8 q .. + 7
    auto atom_frag = [&](int n, int f) { return *reinterpret_cast<const half8 *>(Dh + (int64_t)n * DC + 32 * f + 8 * q); };
    // XOR term of row i's piece positions: i modulo the largest power of two that divides the piece count (N = 96
    // has 12 pieces: modulo 4), so that a swizzled position stays inside the row
    int swz_mask = 1;
    while (swz_mask * 2 <= pieces && pieces % (swz_mask * 2) == 0) swz_mask *= 2;
    swz_mask -= 1;

    // ---- G = D D^T in fp16, row i at lds + i * row_bytes, element (i, n = 16 t + 4 qq + e) at position
    //      qq * N/4 + 4 t + e; and the largest squared atom norm (the diagonal) -------------------------------
    float dmax2 = 0.0f;
    for (int rb = wave; rb < ntile; rb += kWaves) {
        const int i = 16 * rb + col;
        half8 bfr[kF];
#pragma unroll
        for (int f = 0; f < kF; ++f) bfr[f] = atom_frag(i, f);
        const int sw = i & swz_mask;
        for (int t = 0; t < ntile; ++t) {
            floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int f = 0; f < kF; ++f) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(atom_frag(16 * t + col, f), bfr[f], acc, 0, 0, 0);
            // acc[e] = G[n = 16 t + 4 q + e][i]
            if (16 * t + 4 * q <= i && i < 16 * t + 4 * q + 4) dmax2 = fmaxf(dmax2, acc[i - (16 * t + 4 * q)]);
            const __half2 p0 = __floats2half2_rn(acc[0], acc[1]), p1 = __floats2half2_rn(acc[2], acc[3]);
            const int pos = q * (N >> 2) + 4 * t;  // in halfs
            const int piece = (pos >> 3) ^ sw;
            uint2 w;
            w.x = *reinterpret_cast<const uint32_t *>(&p0);
            w.y = *reinterpret_cast<const uint32_t *>(&p1);
            *reinterpret_cast<uint2 *>(lds + (size_t)i * row_bytes + (piece << 4) + ((pos & 7) << 1)) = w;
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dmax2 = fmaxf(dmax2, __shfl_xor(dmax2, m, 64));
    if (lane == 0) red[wave] = dmax2;
    __syncthreads();  // the only barrier: from here on the waves do not meet again
    dmax2 = red[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) dmax2 = fmaxf(dmax2, red[w]);
    const float dmax = sqrtf(dmax2);
    const float g_eps = dmax2 * (2.44140625e-4f + kGammaAcc);  // |G16 - G| <= g_eps

    for (int bi = 0; bi < kBlocksPerWave; ++bi) {
        const int64_t m0 = (int64_t)tile_wg * kTokPerWG + (wave * kBlocksPerWave + bi) * 16;
        if (m0 >= M) break;  // wave-uniform
        const int64_t m = m0 + col;
        const bool valid = m < M;
        const int64_t mc = valid ? m : M - 1;  // tail lanes recompute the last vector, never store
        const int rep = (int)(mc / T);
        const int64_t tok = mc - rep * T;     // position in its block
        const int h = rep * dict_count + dict;

        // ---- the vector: matrix-core operand, fp32 residual, norm ----------------------------------
        half8 xb[kF];
        float R[kF][8];
        float r2 = 0.0f;
        {
            const __half *xr = X + (int64_t)h * x_stride_h + tok * x_stride_t + ch * DC + 8 * q;
#pragma unroll
            for (int f = 0; f < kF; ++f) {
                xb[f] = *reinterpret_cast<const half8 *>(xr + 32 * f);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    R[f][e] = (float)xb[f][e];
                    r2 = fmaf(R[f][e], R[f][e], r2);
                }
            }
            r2 = sum4(r2);
        }
        const float xnorm = sqrtf(r2);

        // ---- C_1 = D x on the matrix cores -------------------------------------------------------------
        float C[kMaxTiles][4];
#pragma unroll
        for (int t = 0; t < kMaxTiles; ++t) {
            floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
            if (t < ntile) {
#pragma unroll
                for (int f = 0; f < kF; ++f) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(atom_frag(16 * t + col, f), xb[f], acc, 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) C[t][e] = acc[e];
        }
        float delta = kGammaAcc * xnorm * dmax;
        float rmax = xnorm;  // largest residual norm so far

        for (int g = 0; g < s; ++g) {
            // ---- screen: the three largest |C| of the vector, atom number in the low 8 bits -------------
            uint32_t k1 = 0u, k2 = 0u, k3 = 0u;
#pragma unroll
            for (int t = 0; t < kMaxTiles; ++t) {
                if (t < ntile) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // larger code = lower atom number; the lane's 4 q is subtracted from the winners below
                        const uint32_t key = (__float_as_uint(C[t][e]) & 0x7fffff00u) | (uint32_t)(255 - 16 * t - e);
                        k3 = umed3(k2, k3, key);   // (k1 >= k2 >= k3 stays sorted)
                        k2 = umed3(k1, k2, key);
                        k1 = umax(k1, key);
                    }
                }
            }
            k1 -= 4u * q; k2 -= 4u * q; k3 -= 4u * q;
            merge3(k1, k2, k3, 16);
            merge3(k1, k2, k3, 32);
            const int n1 = 255 - (int)(k1 & 255u), n2 = 255 - (int)(k2 & 255u);
            const float A1 = __uint_as_float(k1 & 0x7fffff00u), A2 = __uint_as_float(k2 & 0x7fffff00u),
                        A3 = __uint_as_float(k3 & 0x7fffff00u);
            // values were cut to 15 mantissa bits: two atoms are told apart only beyond 2 delta + 2^-14 of the larger
            const float thr = A1 * (1.0f - 6.1035156e-5f) - 2.0f * delta;
            const bool zero = !(r2 > 0.0f);

            // ---- exact: R . d for the first two, always -----------------------------------------------------
            half8 d1[kF], d2[kF];
            const int n2c = n2 < N ? n2 : n1;  // (fewer than two atoms tracked cannot happen: N >= 32)
#pragma unroll
            for (int f = 0; f < kF; ++f) { d1[f] = atom_frag(n1, f); d2[f] = atom_frag(n2c, f); }
            float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
            for (int f = 0; f < kF; ++f) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    c1 = fmaf(R[f][e], (float)d1[f][e], c1);
                    c2 = fmaf(R[f][e], (float)d2[f][e], c2);
                }
            }
            c1 = sum4(c1);
            c2 = sum4(c2);
            int best_n = n1;
            float best_c = c1;
            bool second = false;
            if (A2 >= thr && n2c != n1) {
                const float a1 = fabsf(c1), a2 = fabsf(c2);
                if (a2 > a1 || (a2 == a1 && n2c < n1)) { best_n = n2c; best_c = c2; second = true; }
            }
            // ---- rare: a third atom inside the band: every atom inside it is evaluated -----------------
            if (__ballot(A3 >= thr && !zero)) {
                const bool mine = A3 >= thr && !zero;
                float ba = mine ? fabsf(best_c) : 0.0f;
                for (int n = 0; n < N; ++n) {
                    // the lane that holds C[n] says whether n lies inside its vector's band
                    const int t = n >> 4, qq = (n >> 2) & 3, e = n & 3;
                    float cv = 0.0f;
#pragma unroll
                    for (int tt = 0; tt < kMaxTiles; ++tt)
                        if (tt == t) cv = e == 0 ? C[tt][0] : e == 1 ? C[tt][1] : e == 2 ? C[tt][2] : C[tt][3];
                    const int src = col + 16 * qq;
                    const float cvn = __shfl(cv, src, 64);
                    const bool hit = mine && fabsf(cvn) >= thr && n != n1 && n != n2c;
                    if (__ballot(hit)) {
                        float cx = 0.0f;
#pragma unroll
                        for (int f = 0; f < kF; ++f) {
                            const half8 dn = atom_frag(n, f);
#pragma unroll
                            for (int ee = 0; ee < 8; ++ee) cx = fmaf(R[f][ee], (float)dn[ee], cx);
                        }
                        cx = sum4(cx);
                        const float ax = fabsf(cx);
                        if (hit && (ax > ba || (ax == ba && n < best_n))) { ba = ax; best_n = n; best_c = cx; }
                    }
                }
            }
            if (zero) { best_n = 0; best_c = 0.0f; }

            // ---- update: Eq.4 on the residual (unrounded c), the recursion on the correlations ------------
            {
                const bool need_row = best_n != n1 && !(second && best_n == n2c);  // chosen in the rare path
                float r2n = 0.0f;
#pragma unroll
                for (int f = 0; f < kF; ++f) {
                    half8 dsel = second ? d2[f] : d1[f];
                    if (__ballot(need_row)) {
                        const half8 dn = atom_frag(best_n, f);
                        if (need_row) dsel = dn;
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        R[f][e] = fmaf(-best_c, (float)dsel[e], R[f][e]);
                        r2n = fmaf(R[f][e], R[f][e], r2n);
                    }
                }
                r2 = sum4(r2n);
            }
            {
                const unsigned char *grow = lds + (size_t)best_n * row_bytes;
                const int sw = best_n & swz_mask;
                const float mc_ = -best_c;
#pragma unroll
                for (int p = 0; p < kMaxTiles / 2; ++p) {  // piece p of this quarter: tiles 2 p, 2 p + 1
                    if (p < qpieces) {
                        const half8 gv = *reinterpret_cast<const half8 *>(grow + (((q * qpieces + p) ^ sw) << 4));
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            C[2 * p][e] = fmaf(mc_, (float)gv[e], C[2 * p][e]);
                            C[2 * p + 1][e] = fmaf(mc_, (float)gv[4 + e], C[2 * p + 1][e]);
                        }
                    }
                }
            }
            rmax = fmaxf(rmax, sqrtf(r2));  // (atoms longer than sqrt 2 can make a residual grow)
            delta += fabsf(best_c) * g_eps + 2.4e-7f * rmax * dmax;

            if (valid && q == 0) {
                const int64_t o = (int64_t)h * code_stride_h + (tok * sn + ch) * s + g;
                if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n;
                else reinterpret_cast<int32_t *>(idx_out)[o] = best_n;
                if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(best_c);
                else reinterpret_cast<float *>(coef_out)[o] = best_c;
            }
        }
        if (res_norm2 && valid && q == 0) res_norm2[((int64_t)h * T + tok) * sn + ch] = r2;
    }
}

}  // namespace

bool encode_gram_supported(const EncodeArgs &a)
{
    return a.f16 && (a.d == 128 || a.d == 64) && a.N >= 32 && a.N % 32 == 0 && a.N <= kMaxAtoms;
}

template <int DC>
static hipError_t launch_gram_t(const EncodeArgs &a)
{
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;  // vectors per dictionary
    const int64_t tiles = (M + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.dict_count * a.sn;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    const int lds_bytes = a.N * a.N * 2 + kWaves * 4 + 64;
    static std::atomic<bool> attr_set[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(encode_gram_kernel<DC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxAtoms * kMaxAtoms * 2 + kWaves * 4 + 64);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(encode_gram_kernel<DC>, dim3((unsigned)groups), dim3(kThreads), lds_bytes, a.stream,
                       (const __half *)a.X, (const __half *)a.D, a.idx, a.coef, a.T, M, a.N, a.s, a.sn, a.x_stride_h,
                       a.x_stride_t, a.dict_count, a.code_stride_h, (int32_t)tiles, (int32_t)a.idx16, (int32_t)a.coef16,
                       a.res_norm2);
    return hipGetLastError();
}

hipError_t launch_encode_gram(const EncodeArgs &a)
{
    return a.d == 64 ? launch_gram_t<64>(a) : launch_gram_t<128>(a);
}

}  // namespace csr
