// Matrix-core Matching Pursuit encoder for fp16 vectors and dictionaries, d = 128 (gfx950).
//
// What is computed is exactly Eq.2-4 of the paper's Section "Sparse representation": every
// iteration picks the atom of largest |R . d_n| (lowest n on ties), takes the signed projection as
// coefficient and subtracts it.  The decision and the coefficient are made at fp32 precision on the
// full-precision residual, as in the vector-ALU encoder; the matrix cores only SCREEN the N atoms:
//
//   residual R is held per lane as an unevaluated sum hi + lo of two fp16 values (hi = fp16(R),
//            lo = fp16(R - hi)): hi + lo reproduces the fp32 value to within half an fp32 ulp, hi
//            is directly the MFMA operand, and the pair takes half the registers of an fp32 copy.
//            Every vector is first multiplied by a power of two that brings its largest |x_k| into
//            [2^11, 2^12): Matching Pursuit commutes exactly with such a scaling (the coefficient is
//            scaled back on store), nothing can leave the fp16 range (|R_k| <= |R| <= |x| < 2^15.5)
//            and lo never lands in the fp16 subnormals.
//   screen   c^[n] = hi . d_n, one v_mfma_f32_32x32x16_f16 sweep over the dictionary.
//            |c^[n] - R . d_n| <= |lo| |d_n| + accumulation error, so the atom of largest true
//            |correlation| lies within `delta` of the largest screened value.  The epilogue keeps,
//            per lane, the three largest GROUP maxima of the sweep (a group = the 16 atoms one lane
//            holds of one 32x32 output tile), with the tile number packed into the low mantissa bits
//            so that one integer max/med3/min chain tracks value and position together.
//   select   the (at most three) groups within delta of the best are re-scored exactly: products of
//            fp16 pairs are exact in fp32 (v_dot2_f32_f16), hi and lo parts summed separately, the
//            two lanes that share a token each doing half of the 128 dimensions.  The exact arg-max
//            (lowest index on ties) and its signed projection are the iteration's pair.
//   update   R -= c d in fp32 (Eq.4), new hi / lo split, new delta.
//   overflow if more groups than tracked could matter (degenerate dictionaries, atoms far from unit
//            norm) the token is flagged and re-encoded afterwards by an exact fp32 kernel, one
//            workgroup per flagged token.  On Gaussian-like data that is about 1e-3 of the vectors.
//
// Orientation: atoms are the M rows of the MFMA (A operand = dictionary tile from LDS), tokens the
// N columns (B operand = hi, held in registers for the whole sweep).  Each lane therefore owns one
// token column and 16 atom rows per tile, and the running maxima never leave its registers.
// A wave owns 2 x 32 tokens so that every A fragment read from LDS feeds two MFMAs.  Dictionary
// stages go from global memory straight into LDS (global_load_lds_dwordx4), XOR-swizzled so that the
// 16-byte fragment reads are bank-conflict free.  Two 4-wave workgroups share a CU (two waves per
// SIMD), so one workgroup's select/update phase overlaps the other's MFMA sweep.
#include <cstdio>
#include <cstdlib>

#include "csr_internal.h"
#ifndef CSR_DBG
#define CSR_DBG 0
#endif

namespace csr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = 128;
constexpr int kBlocks = 2;                            // 32-token blocks per wave
constexpr int kWavesPerWG = 4;
constexpr int kThreads = 64 * kWavesPerWG;            // 256
constexpr int kTokPerWave = 32 * kBlocks;             // 64
constexpr int kTokPerWG = kWavesPerWG * kTokPerWave;  // 256
constexpr int kStageAtoms = 64;                       // atoms per LDS stage (two 32-row tiles)
constexpr int kStageBytes = kStageAtoms * kD * 2;     // 16 KiB, rows unpadded, chunks XOR-swizzled
constexpr int kNormSlices = 8;                        // workgroups per dictionary in the norm pre-pass
constexpr float kGammaAcc = 7.7e-6f;  // fp32 accumulation error of a 128-term MFMA dot, relative to |hi||d|
constexpr float kNormSafe = 6.0e4f;   // a residual norm beyond this could leave the fp16 range
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

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// One dictionary stage (64 atoms x 256 B) from global memory into an LDS buffer, no registers in
// between.  Each wave instruction fills 1 KiB = 4 rows; lane l lands at byte 16 l of that KiB, i.e.
// row l/16, chunk position l%16, and fetches source chunk position ^ (row & 7).
__device__ __forceinline__ void issue_stage(const __half *__restrict__ Dh, int stage, unsigned char *buf,
                                            int wave, int lane)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int blk = i * kWavesPerWG + wave;            // which KiB of the stage
        const int row = blk * 4 + (lane >> 4);
        const int ch = (lane & 15) ^ (row & 7);
        const __half *src = Dh + ((int64_t)stage * kStageAtoms + row) * kD + ch * 8;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)(buf + blk * 1024), 16, 0, 0);
    }
}

// Exact partial correlation over this lane's half of the dimensions (k = 16 j + 8 hf + e) of the
// residual hi + lo with one atom row.
__device__ __forceinline__ float half_dot(const __half *__restrict__ row, int hf, const half8 (&hi)[8],
                                          const half8 (&lo)[8])
{
    float a0 = 0.0f, a1 = 0.0f, b0 = 0.0f, b1 = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(row + 16 * j + 8 * hf);
        const half8 dv = *reinterpret_cast<const half8 *>(&raw);
        const half2v d0 = __builtin_shufflevector(dv, dv, 0, 1), d1 = __builtin_shufflevector(dv, dv, 2, 3),
                     d2 = __builtin_shufflevector(dv, dv, 4, 5), d3 = __builtin_shufflevector(dv, dv, 6, 7);
        const half8 h = hi[j], l = lo[j];
        a0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(h, h, 0, 1), d0, a0, false);
        a1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(h, h, 2, 3), d1, a1, false);
        a0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(h, h, 4, 5), d2, a0, false);
        a1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(h, h, 6, 7), d3, a1, false);
        b0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(l, l, 0, 1), d0, b0, false);
        b1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(l, l, 2, 3), d1, b1, false);
        b0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(l, l, 4, 5), d2, b0, false);
        b1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(l, l, 6, 7), d3, b1, false);
    }
    return (a0 + a1) + (b0 + b1);
}

// dnorm[h][slice] = max over the slice's atoms of |d_n|_2: the screening bound scales with it.
__global__ __launch_bounds__(256) void dict_norm_kernel(const __half *__restrict__ Dict, float *__restrict__ dnorm, int32_t N)
{
    __shared__ float red[4];
    const int h = blockIdx.x, sl = blockIdx.y, tid = threadIdx.x;
    const __half *Dh = Dict + (int64_t)h * N * kD;
    const int sub = tid & 15;
    float best = 0.0f;
    for (int n = sl * 16 + (tid >> 4); n < N; n += 16 * kNormSlices) {
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
    if (tid == 0) dnorm[h * kNormSlices + sl] = sqrtf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])));
}

__global__ __launch_bounds__(kThreads, 2) void encode_mfma_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, const float *__restrict__ dnorm, unsigned long long *__restrict__ flags,
    int64_t T, int32_t N, int32_t s, int64_t x_stride_h, int64_t x_stride_t, int32_t tiles_per_h,
    int32_t n_groups, int32_t idx16, int32_t coef16, uint32_t code_mask, int32_t stagger_cus)
{
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * kStageBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hf = lane >> 5;
#if CSR_DBG == 3
    const unsigned long long dbg_t0 = __builtin_readcyclecounter();
#endif

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of work so
    // that workgroups sharing a dictionary share an L2.
    int work = blockIdx.x;
    if ((n_groups & 7) == 0) work = (blockIdx.x & 7) * (n_groups >> 3) + (blockIdx.x >> 3);
    const int h = work / tiles_per_h;
    const int tile_wg = work - h * tiles_per_h;
    const __half *Dh = Dict + (int64_t)h * N * kD;
    const int ntiles = N >> 5;
    const int nstages = N / kStageAtoms;

    issue_stage(Dh, 0, lds, wave, lane);  // in flight while the vectors are loaded

    // Two workgroups share a CU.  Started together they would sweep together and select together;
    // holding back every second wave of workgroups by about half an iteration makes one's select
    // phase (vector ALU, gathers) fall into the other's sweep (matrix cores).
    bool hold = false;
    if (stagger_cus > 0) hold = (blockIdx.x / stagger_cus) & 1;
    else if (stagger_cus == -2) hold = (blockIdx.x >> 3) & 1;
    else if (stagger_cus == -3) hold = ((blockIdx.x >> 3) / 32) & 1;
    if (hold) {
        for (int i = 0; i < nstages; ++i) __builtin_amdgcn_s_sleep(32);
    }

    float dmax = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormSlices; ++i) dmax = fmaxf(dmax, dnorm[h * kNormSlices + i]);
    // relative slack of a packed value: its low mantissa bits were replaced by the tile code
    const float pack_q = (float)(code_mask + 1) * 1.1920929e-7f;

    // ---- load the vectors, scale by a power of two, split into hi + lo ---------------------------
    half8 hi[kBlocks][8], lo[kBlocks][8];
    bool valid[kBlocks];
    int64_t tok[kBlocks];
    int sexp[kBlocks];
    float delta[kBlocks], rn2[kBlocks];
#pragma unroll
    for (int bi = 0; bi < kBlocks; ++bi) {
        tok[bi] = (int64_t)tile_wg * kTokPerWG + wave * kTokPerWave + bi * 32 + col;
        valid[bi] = tok[bi] < T;
        const int64_t tc = valid[bi] ? tok[bi] : T - 1;
        const __half *xr = X + (int64_t)h * x_stride_h + tc * x_stride_t;
        float xv[8][8];
        float amax = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(xr + 16 * j + 8 * hf);
            unpack8(raw, xv[j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xv[j][e]));
        }
        amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
        int ex = 0;
        if (amax > 0.0f && amax < INFINITY) {
            (void)frexpf(amax, &ex);  // amax = f 2^ex, f in [0.5, 1)
            ex = 12 - ex;             // brings amax into [2^11, 2^12)
        }
        sexp[bi] = ex;
        float r2 = 0.0f, lo2 = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            half8 hv, lv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = ldexpf(xv[j][e], ex);
                const _Float16 hh = (_Float16)v;
                const float l = v - (float)hh;
                hv[e] = hh;
                lv[e] = (_Float16)l;
                r2 = fmaf(v, v, r2);
                lo2 = fmaf(l, l, lo2);
            }
            hi[bi][j] = hv;
            lo[bi][j] = lv;
        }
        r2 += __shfl_xor(r2, 32, 64);
        lo2 += __shfl_xor(lo2, 32, 64);
        rn2[bi] = r2;
        delta[bi] = 2.0f * dmax * (sqrtf(lo2) + kGammaAcc * sqrtf(r2));
    }

    unsigned long long flag_acc = 0ull;  // wave-uniform: bit (32 bi + col) = token needs the exact kernel

    for (int g = 0; g < s; ++g) {
        // ---- screen: one MFMA sweep over the dictionary ------------------------------------
        uint32_t u1[kBlocks], u2[kBlocks], u3[kBlocks];
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) u1[bi] = u2[bi] = u3[bi] = 0u;

        wait_vmem();
        __syncthreads();  // stage 0 is in buffer 0

#if CSR_DBG == 2
        for (int st = 0; st < 1; ++st) {
#else
        for (int st = 0; st < nstages; ++st) {
#endif
            const unsigned char *buf = lds + (st & 1) * kStageBytes;
            if (st + 1 < nstages) issue_stage(Dh, st + 1, lds + ((st + 1) & 1) * kStageBytes, wave, lane);
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                floatx16 acc[kBlocks];
#pragma unroll
                for (int bi = 0; bi < kBlocks; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[bi][r] = 0.0f;
                const unsigned char *rowp = buf + (rt * 32 + col) * (kD * 2);
                half8 a[8];  // all fragments of the row tile requested before the first MFMA waits
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    a[j] = *reinterpret_cast<const half8 *>(rowp + (((2 * j + hf) ^ (col & 7)) << 4));
#pragma unroll
                for (int j = 0; j < 8; ++j) {
#pragma unroll
                    for (int bi = 0; bi < kBlocks; ++bi)
                        acc[bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], hi[bi][j], acc[bi], 0, 0, 0);
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
            wait_vmem();
            __syncthreads();
        }
        // both buffers are free now: fetch stage 0 for the next sweep behind the select phase
        if (g + 1 < s) issue_stage(Dh, 0, lds, wave, lane);

        // ---- select + update, one 32-token block at a time ----------------------------------
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
            const uint32_t p1 = __shfl_xor(u1[bi], 32, 64), p2 = __shfl_xor(u2[bi], 32, 64),
                           p3 = __shfl_xor(u3[bi], 32, 64);
            // L = triple of lane-half 0, Hh = triple of lane-half 1: both lanes of a pair see the same
            const uint32_t L1 = hf ? p1 : u1[bi], L2 = hf ? p2 : u2[bi], L3 = hf ? p3 : u3[bi];
            const uint32_t H1 = hf ? u1[bi] : p1, H2 = hf ? u2[bi] : p2, H3 = hf ? u3[bi] : p3;
            // merged top three with the owning half (ties: half 0 first)
            uint32_t tv0, tv1, tv2;
            int to0, to1, to2;
            {
                uint32_t a1 = L1, a2 = L2, a3 = L3, b1 = H1, b2 = H2, b3 = H3;
                bool x = a1 >= b1;
                tv0 = x ? a1 : b1; to0 = x ? 0 : 1;
                if (x) { a1 = a2; a2 = a3; } else { b1 = b2; b2 = b3; }
                x = a1 >= b1;
                tv1 = x ? a1 : b1; to1 = x ? 0 : 1;
                if (x) { a1 = a2; } else { b1 = b2; }
                x = a1 >= b1;
                tv2 = x ? a1 : b1; to2 = x ? 0 : 1;
                (void)a3; (void)b3;
            }
            const float A = __uint_as_float(tv0 & ~code_mask);
            const float thr = (A - delta[bi]) * (1.0f - 2.0f * pack_q);
            const bool zero = rn2[bi] == 0.0f;
            auto cand = [&](uint32_t u) { return __uint_as_float(u & ~code_mask) >= thr; };
            const int ncand = (int)cand(L1) + (int)cand(L2) + (int)cand(L3) + (int)cand(H1) + (int)cand(H2) + (int)cand(H3);
            bool overflow = cand(L3) || cand(H3) || ncand > 3 || !(rn2[bi] < kNormSafe * kNormSafe);
            overflow = overflow && !zero && valid[bi];

            float best_a = -1.0f, best_c = 0.0f;
            int best_n = 0;
            auto rescore = [&](uint32_t tv, int to, bool need) {
                const int tile = ntiles - 1 - (int)(tv & code_mask);
                const int base = tile * 32 + 4 * to;
#pragma unroll 4
                for (int k = 0; k < 16; ++k) {
                    const int n = base + 8 * (k >> 2) + (k & 3);
                    float c = half_dot(Dh + (int64_t)n * kD, hf, hi[bi], lo[bi]);
                    c += __shfl_xor(c, 32, 64);
                    const float a = fabsf(c);
                    if (need && (a > best_a || (a == best_a && n < best_n))) { best_a = a; best_c = c; best_n = n; }
                }
            };
#if CSR_DBG == 1
            best_n = (ntiles - 1 - (int)(tv0 & code_mask)) * 32 + 4 * to0; best_c = 1e-3f;
#else
            rescore(tv0, to0, true);
#endif
#if CSR_DBG != 1
            {
                const bool need1 = cand(tv1);
                if (__ballot(need1) != 0ull) rescore(tv1, to1, need1);
                const bool need2 = cand(tv2);
                if (__ballot(need2) != 0ull) rescore(tv2, to2, need2);
            }
#endif
            if (zero) { best_c = 0.0f; best_n = 0; }

            // Eq.4 on the full-precision residual, then the new hi / lo split and screening bound
            {
                const __half *row = Dh + (int64_t)best_n * kD;
                float lo2 = 0.0f, r2 = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(row + 16 * j + 8 * hf);
                    float f[8];
                    unpack8(raw, f);
                    half8 hv, lv;
                    const half8 ho = hi[bi][j], lo_o = lo[bi][j];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float r = (float)ho[e] + (float)lo_o[e];  // exact: 22 significant bits
                        const float v = fmaf(-best_c, f[e], r);
                        const _Float16 hh = (_Float16)v;
                        const float l = v - (float)hh;
                        hv[e] = hh;
                        lv[e] = (_Float16)l;
                        lo2 = fmaf(l, l, lo2);
                        r2 = fmaf(v, v, r2);
                    }
                    hi[bi][j] = hv;
                    lo[bi][j] = lv;
                }
                lo2 += __shfl_xor(lo2, 32, 64);
                r2 += __shfl_xor(r2, 32, 64);
                rn2[bi] = r2;
                delta[bi] = 2.0f * dmax * (sqrtf(lo2) + kGammaAcc * sqrtf(r2));
            }
            if (valid[bi] && hf == 0) {
                const int64_t o = ((int64_t)h * T + tok[bi]) * s + g;
                const float c_out = ldexpf(best_c, -sexp[bi]);
                if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n;
                else reinterpret_cast<int32_t *>(idx_out)[o] = best_n;
                if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(c_out);
                else reinterpret_cast<float *>(coef_out)[o] = c_out;
            }
            const unsigned long long bal = __ballot(overflow && hf == 0);  // bits 0..31 = this block's tokens
            flag_acc |= (bal & 0xffffffffull) << (32 * bi);
        }
    }
    // every wave writes its word, flagged or not: the flag array needs no clearing beforehand
#if CSR_DBG == 3
    if (tid == 0) {
        unsigned long long *rec = flags + (int64_t)blockIdx.x * kWavesPerWG;
        rec[0] = dbg_t0;
        rec[1] = __builtin_readcyclecounter();
        rec[2] = __builtin_amdgcn_s_getreg(0xF804);
        rec[3] = __builtin_amdgcn_s_getreg(0xF814);
    }
    (void)flag_acc;
#else
    if (lane == 0) flags[((int64_t)h * tiles_per_h + tile_wg) * kWavesPerWG + wave] = flag_acc;
#endif
}

// Exact fp32 Matching Pursuit for the flagged tokens, one workgroup per token.  16 lanes share an
// atom row (coalesced 256 B), each holding its 8 residual values in registers; the residual lives
// in LDS between iterations.  Overwrites the codes the screening kernel left for these tokens.
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
    const int sub = tid & 15, grp = tid >> 4;

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
                float rv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) rv[e] = R_s[sub * 8 + e];
                float ba = -1.0f, bc = 0.0f;
                int bn = 0;
                for (int n = grp; n < N; n += 16) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)n * kD + sub * 8);
                    float f[8];
                    unpack8(raw, f);
                    float c0 = 0.0f, c1 = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; e += 2) { c0 = fmaf(rv[e], f[e], c0); c1 = fmaf(rv[e + 1], f[e + 1], c1); }
                    float c = c0 + c1;
#pragma unroll
                    for (int m = 8; m >= 1; m >>= 1) c += __shfl_xor(c, m, 64);
                    const float a = fabsf(c);
                    if (a > ba) { ba = a; bc = c; bn = n; }  // ascending n: the lowest index is kept on ties
                }
                // lowest index among equal magnitudes, across the wave then across the 4 waves
#pragma unroll
                for (int m = 32; m >= 16; m >>= 1) {
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
    return r256((size_t)H * kNormSlices * sizeof(float)) +
           r256((size_t)H * tiles * kWavesPerWG * sizeof(unsigned long long));
}

hipError_t launch_encode_mfma(const EncodeArgs &a)
{
    const int64_t tiles = (a.T + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.H;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    char *ws = static_cast<char *>(a.workspace);
    float *dnorm = reinterpret_cast<float *>(ws);
    unsigned long long *flags =
        reinterpret_cast<unsigned long long *>(ws + r256((size_t)a.H * kNormSlices * sizeof(float)));
    const int ntiles = a.N / 32;
    int bits = 0;
    while ((1 << bits) < ntiles) ++bits;
    const uint32_t code_mask = (1u << bits) - 1u;

    static int n_cus = -1;  // CU count of the current device, asked once
    if (n_cus < 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) v = 0;
        n_cus = v;
    }
    int32_t stagger = (getenv("CSR_NO_STAGGER") || groups <= n_cus) ? 0 : n_cus;
    if (getenv("CSR_STAGGER_MODE")) stagger = -atoi(getenv("CSR_STAGGER_MODE"));

    if (getenv("CSR_DBG_OCC")) {
        int nb = -1;
        hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, encode_mfma_kernel, kThreads, 0);
        fprintf(stderr, "[csr] occupancy: %d workgroups/CU (err %d), CUs %d\n", nb, (int)oe, n_cus);
    }
    hipLaunchKernelGGL(dict_norm_kernel, dim3((unsigned)a.H, kNormSlices), dim3(256), 0, a.stream,
                       (const __half *)a.D, dnorm, a.N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(encode_mfma_kernel, dim3((unsigned)groups), dim3(kThreads), 0, a.stream, (const __half *)a.X,
                       (const __half *)a.D, a.idx, a.coef, dnorm, flags, a.T, a.N, a.s, a.x_stride_h, a.x_stride_t,
                       (int32_t)tiles, (int32_t)groups, (int32_t)a.idx16, (int32_t)a.coef16, code_mask, stagger);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (getenv("CSR_DBG_SKIP_FB")) return hipSuccess;
    const int64_t n_words = groups * kWavesPerWG;
    const unsigned fb_grid = (unsigned)(n_words < kFallbackGrid ? n_words : kFallbackGrid);
    hipLaunchKernelGGL(encode_exact_token_kernel, dim3(fb_grid), dim3(256), 0, a.stream, (const __half *)a.X,
                       (const __half *)a.D, a.idx, a.coef, flags, a.T, a.N, a.s, a.x_stride_h, a.x_stride_t,
                       (int32_t)tiles, n_words, (int32_t)a.idx16, (int32_t)a.coef16);
    return hipGetLastError();
}

}  // namespace csr
