// Matrix-core Matching Pursuit encoder for fp16 vectors and dictionaries, d = 128 (gfx950).
//
// What is computed is exactly Eq.2-4 of the paper's Section "Sparse representation": every
// iteration picks the atom of largest |R . d_n| (lowest n on ties), takes the signed projection as
// coefficient and subtracts it.  The decision and the coefficient are made in fp32 on the exact fp32
// residual, as in the vector-ALU encoder; the matrix cores only SCREEN the N atoms:
//
//   screen   c^[n] = hi . d_n with hi = fp16(R), one v_mfma_f32_32x32x16_f16 sweep over the
//            dictionary.  |c^[n] - R . d_n| <= |lo| |d_n| + accumulation error, lo = R - hi, so the
//            atom of largest true |correlation| lies within `delta` of the largest screened value.
//            The epilogue keeps, per lane, the three largest GROUP maxima of the sweep (a group =
//            the 16 atoms one lane holds of one 32x32 output tile), with the tile number packed into
//            the low mantissa bits so one integer max/med3/min chain tracks value and position.
//   select   the (at most three) groups within delta of the best are re-scored exactly: fp32 dot
//            products of the fp32 residual with the fp16 atoms, 16 atoms per group, the two lanes
//            that share a token each doing half of the 128 dimensions.  The exact arg-max (lowest
//            index on ties) and its signed projection are the iteration's pair.
//   update   R -= c d (fp32), new hi / lo split, new delta.
//   overflow if more groups than tracked could matter (degenerate dictionaries, denormal-scale
//            inputs, residuals beyond fp16 range) the token is flagged and re-encoded afterwards by
//            an exact fp32 kernel, one workgroup per flagged token.  On Gaussian-like data this is
//            of the order of 1e-4 of the vectors.
//
// Orientation: atoms are the M rows of the MFMA (A operand = dictionary tile from LDS), tokens the
// N columns (B operand = residual, held in registers for the whole sweep).  Each lane therefore owns
// one token column and 16 atom rows per tile, and the running maxima never leave its registers.
// A wave owns 2 x 32 tokens so that every A fragment read from LDS feeds two MFMAs.
#include "csr_internal.h"

namespace csr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = 128;
constexpr int kBlocks = 2;                            // 32-token blocks per wave
constexpr int kWavesPerWG = 4;
constexpr int kTokPerWave = 32 * kBlocks;             // 64
constexpr int kTokPerWG = kWavesPerWG * kTokPerWave;  // 256
constexpr int kStageAtoms = 64;   // atoms staged in LDS per pipeline step (two 32-row tiles)
constexpr int kRowPitch = 272;    // bytes per atom row in LDS: 256 + 16 pad -> conflict-free b128 reads
constexpr int kStageBytes = kStageAtoms * kRowPitch;
constexpr float kGammaAcc = 7.7e-6f;  // fp32 accumulation error of a 128-term MFMA dot, relative to |hi||d|
constexpr float kHalfSafe = 6.0e4f;   // residual norms above this may not convert to fp16
constexpr int kFallbackGrid = 1024;

__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c)
{
    return max(min(a, b), min(max(a, b), c));
}

__device__ __forceinline__ void unpack8(const uint4 &raw, float (&f)[8])
{
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = __half22float2(h2[j]);
        f[2 * j] = v.x;
        f[2 * j + 1] = v.y;
    }
}

// Partial dot product over this lane's half of the dimensions: k = 16 j + 8 hf + e.
__device__ __forceinline__ float half_dot(const __half *__restrict__ row, int hf, const float (&R)[8][8])
{
    float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(row + 16 * j + 8 * hf);
        float f[8];
        unpack8(raw, f);
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            a0 = fmaf(R[j][e], f[e], a0);
            a1 = fmaf(R[j][e + 1], f[e + 1], a1);
        }
    }
    return a0 + a1;
}

// dmax[h] = max over atoms of |d_n|_2: the screening bound scales with it.
__global__ __launch_bounds__(256) void dict_norm_kernel(const __half *__restrict__ Dict, float *__restrict__ dmax, int32_t N)
{
    __shared__ float red[4];
    const int h = blockIdx.x, tid = threadIdx.x;
    const __half *Dh = Dict + (int64_t)h * N * kD;
    const int sub = tid & 15;
    float best = 0.0f;
    for (int n = tid >> 4; n < N; n += 16) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)n * kD + sub * 8);
        float f[8];
        unpack8(raw, f);
        float ss = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(f[e], f[e], ss);
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
        best = fmaxf(best, ss);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) best = fmaxf(best, __shfl_xor(best, m, 64));
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) dmax[h] = sqrtf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])));
}

__global__ __launch_bounds__(256) void encode_mfma_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, const float *__restrict__ dmax_arr, unsigned long long *__restrict__ flags,
    int64_t T, int32_t N, int32_t s, int64_t x_stride_h, int64_t x_stride_t, int32_t tiles_per_h,
    int32_t n_groups, int32_t idx16, int32_t coef16, uint32_t code_mask)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStageBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31, hf = lane >> 5;

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of work so
    // that workgroups sharing a dictionary share an L2.
    int work = blockIdx.x;
    if ((n_groups & 7) == 0) work = (blockIdx.x & 7) * (n_groups >> 3) + (blockIdx.x >> 3);
    const int h = work / tiles_per_h;
    const int tile_wg = work - h * tiles_per_h;
    const __half *Dh = Dict + (int64_t)h * N * kD;
    const float dmax = dmax_arr[h];
    const int ntiles = N >> 5;
    const int nstages = N / kStageAtoms;
    // relative slack of a packed value: its low mantissa bits were replaced by the tile code
    const float pack_q = (float)(code_mask + 1) * 1.1920929e-7f;

    // ---- load the vectors: R (fp32) and its fp16 image as MFMA B fragments ---------------------
    float R[kBlocks][8][8];
    half8 hi[kBlocks][8];
    bool valid[kBlocks];
    int64_t tok[kBlocks];
    float delta[kBlocks], rn2[kBlocks];
#pragma unroll
    for (int bi = 0; bi < kBlocks; ++bi) {
        tok[bi] = (int64_t)tile_wg * kTokPerWG + wave * kTokPerWave + bi * 32 + col;
        valid[bi] = tok[bi] < T;
        const int64_t tc = valid[bi] ? tok[bi] : T - 1;
        const __half *xr = X + (int64_t)h * x_stride_h + tc * x_stride_t;
        float r2 = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(xr + 16 * j + 8 * hf);
            hi[bi][j] = *reinterpret_cast<const half8 *>(&raw);
            unpack8(raw, R[bi][j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) r2 = fmaf(R[bi][j][e], R[bi][j][e], r2);
        }
        r2 += __shfl_xor(r2, 32, 64);
        rn2[bi] = r2;
        delta[bi] = 2.0f * dmax * kGammaAcc * sqrtf(r2);  // lo = 0: the input is fp16 already
    }

    unsigned long long flag_acc = 0ull;  // wave-uniform: bit (32 bi + col) = token needs the exact kernel

    for (int g = 0; g < s; ++g) {
        // ---- screen: one MFMA sweep over the dictionary ------------------------------------
        uint32_t u1[kBlocks], u2[kBlocks], u3[kBlocks];
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) u1[bi] = u2[bi] = u3[bi] = 0u;

        // stage 0 -> LDS buffer 0 (the previous sweep's last barrier freed both buffers)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i;
            const int row = q >> 4, ch = q & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(Dh + (int64_t)row * kD + ch * 8);
            *reinterpret_cast<uint4 *>(lds + row * kRowPitch + ch * 16) = v;
        }
        __syncthreads();

        for (int st = 0; st < nstages; ++st) {
            const unsigned char *buf = lds + (st & 1) * kStageBytes;
            unsigned char *nbuf = lds + ((st + 1) & 1) * kStageBytes;
            uint4 pre[4];
            const bool more = st + 1 < nstages;
            if (more) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int q = tid + 256 * i;
                    const int row = q >> 4, ch = q & 15;
                    pre[i] = *reinterpret_cast<const uint4 *>(Dh + ((int64_t)(st + 1) * kStageAtoms + row) * kD + ch * 8);
                }
            }
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                floatx16 acc[kBlocks];
#pragma unroll
                for (int bi = 0; bi < kBlocks; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[bi][r] = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const half8 a = *reinterpret_cast<const half8 *>(buf + (rt * 32 + col) * kRowPitch + (2 * j + hf) * 16);
#pragma unroll
                    for (int bi = 0; bi < kBlocks; ++bi)
                        acc[bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, hi[bi][j], acc[bi], 0, 0, 0);
                }
                const uint32_t code = (uint32_t)(ntiles - 1 - (st * 2 + rt));  // earlier tile = larger code
#pragma unroll
                for (int bi = 0; bi < kBlocks; ++bi) {
                    float m = fmaxf(fmaxf(fabsf(acc[bi][0]), fabsf(acc[bi][1])), fabsf(acc[bi][2]));
#pragma unroll
                    for (int r = 3; r < 15; r += 2) m = fmaxf(fmaxf(m, fabsf(acc[bi][r])), fabsf(acc[bi][r + 1]));
                    m = fmaxf(m, fabsf(acc[bi][15]));
                    const uint32_t u = (__float_as_uint(m) & ~code_mask) | code;
                    const uint32_t n3 = max(u3[bi], min(u2[bi], u));
                    const uint32_t n2 = umed3(u1[bi], u2[bi], u);
                    u1[bi] = max(u1[bi], u);
                    u2[bi] = n2;
                    u3[bi] = n3;
                }
            }
            if (more) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int q = tid + 256 * i;
                    const int row = q >> 4, ch = q & 15;
                    *reinterpret_cast<uint4 *>(nbuf + row * kRowPitch + ch * 16) = pre[i];
                }
            }
            __syncthreads();
        }

        // ---- select + update, one 32-token block at a time ----------------------------------
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
            const uint32_t p1 = __shfl_xor(u1[bi], 32, 64), p2 = __shfl_xor(u2[bi], 32, 64),
                           p3 = __shfl_xor(u3[bi], 32, 64);
            // L = triple of lane-half 0, Hh = triple of lane-half 1: both lanes of a pair see the same
            const uint32_t L1 = hf ? p1 : u1[bi], L2 = hf ? p2 : u2[bi], L3 = hf ? p3 : u3[bi];
            const uint32_t H1 = hf ? u1[bi] : p1, H2 = hf ? u2[bi] : p2, H3 = hf ? u3[bi] : p3;
            uint32_t tv[3];
            int to[3];
            {
                uint32_t a1 = L1, a2 = L2, a3 = L3, b1 = H1, b2 = H2, b3 = H3;
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const bool x = a1 >= b1;
                    tv[r] = x ? a1 : b1;
                    to[r] = x ? 0 : 1;
                    if (x) { a1 = a2; a2 = a3; a3 = 0u; }
                    else { b1 = b2; b2 = b3; b3 = 0u; }
                }
            }
            const float A = __uint_as_float(tv[0] & ~code_mask);
            const float thr = (A - delta[bi]) * (1.0f - 2.0f * pack_q);
            const bool zero = rn2[bi] == 0.0f;
            auto cand = [&](uint32_t u) { return __uint_as_float(u & ~code_mask) >= thr; };
            const int ncand = (int)cand(L1) + (int)cand(L2) + (int)cand(L3) + (int)cand(H1) + (int)cand(H2) + (int)cand(H3);
            bool overflow = cand(L3) || cand(H3) || ncand > 3 || !(rn2[bi] < kHalfSafe * kHalfSafe);
            overflow = overflow && !zero && valid[bi];

            float best_a = -1.0f, best_c = 0.0f;
            int best_n = 0;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const bool need = (r == 0) || cand(tv[r]);
                if (r > 0 && __ballot(need) == 0ull) continue;
                const int tile = ntiles - 1 - (int)(tv[r] & code_mask);
                const int base = tile * 32 + 4 * to[r];
#pragma unroll 2
                for (int k = 0; k < 16; ++k) {
                    const int n = base + 8 * (k >> 2) + (k & 3);
                    float c = half_dot(Dh + (int64_t)n * kD, hf, R[bi]);
                    c += __shfl_xor(c, 32, 64);
                    const float a = fabsf(c);
                    if (need && (a > best_a || (a == best_a && n < best_n))) { best_a = a; best_c = c; best_n = n; }
                }
            }
            if (zero) { best_c = 0.0f; best_n = 0; }

            // Eq.4 on the fp32 residual, then the new fp16 image and screening bound
            {
                const __half *row = Dh + (int64_t)best_n * kD;
                float lo2 = 0.0f, r2 = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(row + 16 * j + 8 * hf);
                    float f[8];
                    unpack8(raw, f);
                    half8 hv;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float v = fmaf(-best_c, f[e], R[bi][j][e]);
                        R[bi][j][e] = v;
                        const _Float16 hh = (_Float16)v;
                        hv[e] = hh;
                        const float l = v - (float)hh;
                        lo2 = fmaf(l, l, lo2);
                        r2 = fmaf(v, v, r2);
                    }
                    hi[bi][j] = hv;
                }
                lo2 += __shfl_xor(lo2, 32, 64);
                r2 += __shfl_xor(r2, 32, 64);
                rn2[bi] = r2;
                delta[bi] = 2.0f * dmax * (sqrtf(lo2) + kGammaAcc * sqrtf(r2));
            }
            if (valid[bi] && hf == 0) {
                const int64_t o = ((int64_t)h * T + tok[bi]) * s + g;
                if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n;
                else reinterpret_cast<int32_t *>(idx_out)[o] = best_n;
                if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(best_c);
                else reinterpret_cast<float *>(coef_out)[o] = best_c;
            }
            const unsigned long long bal = __ballot(overflow && hf == 0);  // bits 0..31 = this block's tokens
            flag_acc |= (bal & 0xffffffffull) << (32 * bi);
        }
    }
    // every wave writes its word, flagged or not: the flag array needs no clearing beforehand
    if (lane == 0) flags[((int64_t)h * tiles_per_h + tile_wg) * kWavesPerWG + wave] = flag_acc;
}

// Exact fp32 Matching Pursuit for the flagged tokens, one workgroup per token: 256 threads split
// the atoms, the residual sits in LDS.  Overwrites the codes the screening kernel left for them.
__global__ __launch_bounds__(256) void encode_exact_token_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, const unsigned long long *__restrict__ flags, int64_t T, int32_t N,
    int32_t s, int64_t x_stride_h, int64_t x_stride_t, int32_t tiles_per_h, int64_t n_words,
    int32_t idx16, int32_t coef16)
{
    __shared__ __attribute__((aligned(16))) float R_s[kD];
    __shared__ float w_a[4], w_c[4];
    __shared__ int w_n[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    for (int64_t w = blockIdx.x; w < n_words; w += gridDim.x) {
        unsigned long long word = flags[w];  // same for every thread of the workgroup
        while (word) {
            const int b = __ffsll((long long)word) - 1;
            word &= word - 1;
            const int64_t wg = w / kWavesPerWG;
            const int wv = (int)(w - wg * kWavesPerWG);
            const int h = (int)(wg / tiles_per_h);
            const int64_t t = (wg - (int64_t)h * tiles_per_h) * kTokPerWG + wv * kTokPerWave + b;
            if (t >= T) continue;
            const __half *Dh = Dict + (int64_t)h * N * kD;
            __syncthreads();
            if (tid < kD) R_s[tid] = __half2float(X[(int64_t)h * x_stride_h + t * x_stride_t + tid]);
            __syncthreads();
            for (int g = 0; g < s; ++g) {
                float ba = -1.0f, bc = 0.0f;
                int bn = 0;
                for (int n = tid; n < N; n += 256) {
                    const __half *row = Dh + (int64_t)n * kD;
                    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
                    for (int c8 = 0; c8 < 16; ++c8) {
                        const uint4 raw = *reinterpret_cast<const uint4 *>(row + c8 * 8);
                        float f[8];
                        unpack8(raw, f);
                        const float4 r0 = *reinterpret_cast<const float4 *>(&R_s[c8 * 8]);
                        const float4 r1 = *reinterpret_cast<const float4 *>(&R_s[c8 * 8 + 4]);
                        a0 = fmaf(r0.x, f[0], a0); a1 = fmaf(r0.y, f[1], a1);
                        a2 = fmaf(r0.z, f[2], a2); a3 = fmaf(r0.w, f[3], a3);
                        a0 = fmaf(r1.x, f[4], a0); a1 = fmaf(r1.y, f[5], a1);
                        a2 = fmaf(r1.z, f[6], a2); a3 = fmaf(r1.w, f[7], a3);
                    }
                    const float c = (a0 + a1) + (a2 + a3);
                    const float a = fabsf(c);
                    if (a > ba) { ba = a; bc = c; bn = n; }
                }
                // lowest index among equal magnitudes, across the wave then across the 4 waves
#pragma unroll
                for (int m = 32; m >= 1; m >>= 1) {
                    const float oa = __shfl_xor(ba, m, 64), oc = __shfl_xor(bc, m, 64);
                    const int on = __shfl_xor(bn, m, 64);
                    if (oa > ba || (oa == ba && on < bn)) { ba = oa; bc = oc; bn = on; }
                }
                if (lane == 0) { w_a[wave] = ba; w_c[wave] = bc; w_n[wave] = bn; }
                __syncthreads();
                ba = w_a[0]; bc = w_c[0]; bn = w_n[0];
#pragma unroll
                for (int k = 1; k < 4; ++k) {
                    if (w_a[k] > ba || (w_a[k] == ba && w_n[k] < bn)) { ba = w_a[k]; bc = w_c[k]; bn = w_n[k]; }
                }
                if (tid < kD) R_s[tid] = fmaf(-bc, __half2float(Dh[(int64_t)bn * kD + tid]), R_s[tid]);
                if (tid == 0) {
                    const int64_t o = ((int64_t)h * T + t) * s + g;
                    if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)bn;
                    else reinterpret_cast<int32_t *>(idx_out)[o] = bn;
                    if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(bc);
                    else reinterpret_cast<float *>(coef_out)[o] = bc;
                }
                __syncthreads();
            }
        }
    }
}

size_t r256(size_t v) { return (v + 255) & ~size_t(255); }

}  // namespace

bool encode_mfma_supported(const EncodeArgs &a)
{
    return a.f16 && a.d == kD && a.N >= 128 && a.N % kStageAtoms == 0 && a.N <= 65536;
}

size_t encode_mfma_workspace_bytes(int32_t H, int64_t T, int32_t N, int32_t s)
{
    (void)N; (void)s;
    const int64_t tiles = (T + kTokPerWG - 1) / kTokPerWG;
    return r256((size_t)H * sizeof(float)) + r256((size_t)H * tiles * kWavesPerWG * sizeof(unsigned long long));
}

hipError_t launch_encode_mfma(const EncodeArgs &a)
{
    const int64_t tiles = (a.T + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.H;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    char *ws = static_cast<char *>(a.workspace);
    float *dmax = reinterpret_cast<float *>(ws);
    unsigned long long *flags = reinterpret_cast<unsigned long long *>(ws + r256((size_t)a.H * sizeof(float)));
    const int ntiles = a.N / 32;
    int bits = 0;
    while ((1 << bits) < ntiles) ++bits;
    const uint32_t code_mask = (1u << bits) - 1u;

    hipLaunchKernelGGL(dict_norm_kernel, dim3((unsigned)a.H), dim3(256), 0, a.stream, (const __half *)a.D, dmax, a.N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(encode_mfma_kernel, dim3((unsigned)groups), dim3(256), 0, a.stream, (const __half *)a.X,
                       (const __half *)a.D, a.idx, a.coef, dmax, flags, a.T, a.N, a.s, a.x_stride_h, a.x_stride_t,
                       (int32_t)tiles, (int32_t)groups, (int32_t)a.idx16, (int32_t)a.coef16, code_mask);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t n_words = groups * kWavesPerWG;
    const unsigned fb_grid = (unsigned)(n_words < kFallbackGrid ? n_words : kFallbackGrid);
    hipLaunchKernelGGL(encode_exact_token_kernel, dim3(fb_grid), dim3(256), 0, a.stream, (const __half *)a.X,
                       (const __half *)a.D, a.idx, a.coef, flags, a.T, a.N, a.s, a.x_stride_h, a.x_stride_t,
                       (int32_t)tiles, n_words, (int32_t)a.idx16, (int32_t)a.coef16);
    return hipGetLastError();
}

}  // namespace csr
