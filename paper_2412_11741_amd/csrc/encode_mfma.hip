// Matrix-core Matching Pursuit encoder for fp16 vectors and dictionaries of 128, 64 or 32 dimensions (gfx950):
// whole head vectors, or the chunks of the paper's Section "NeuralDict" (s_n = 2 or 4 at a head dimension of 128),
// each chunk a vector of its own on its own dictionary.  The description below gives the numbers for 128 dimensions.
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
//            and lo stays clear of the fp16 subnormals.
//   screen   c^[n] = hi . d_n, one v_mfma_f32_32x32x16_f16 sweep over the dictionary.
//            |c^[n] - R . d_n| <= |lo| |d_n| + accumulation error =: delta / 2, so the atom of
//            largest true |correlation| lies within delta of the largest screened value.  The
//            epilogue keeps, per lane, the four largest GROUP maxima of the sweep (a group = the 16
//            atoms one lane holds of one 32x32 output tile), with the tile number packed into the
//            low mantissa bits so that one integer max/med3 chain tracks value and position.
//            The 16 screened magnitudes of the lane's best group so far are carried along as fp16
//            (eight packed registers, rewritten under the lanes' execution mask whenever a group
//            becomes the new best), so that after the sweep the best group's values are at hand.
//   select   if the best group's largest kept value leads the other 15 by more than delta (plus the
//            fp16 rounding of the kept values) and no other tracked group comes within delta of
//            it, that atom is the iteration's pick (about 97 % of the steps on Gaussian-like
//            data): no memory access at all.  Otherwise the wave resolves the token
//            together: the residual
//            goes through LDS to all 64 lanes, which evaluate hi . d + lo . d (products of fp16
//            pairs are exact in fp32) for every atom of every candidate group and take the largest,
//            lowest index on ties.  Should even the fourth tracked group of a lane be a candidate
//            (about 1e-5 of the steps), untracked groups could matter too, and the wave evaluates
//            all N atoms that way.
//   update   c = (hi + lo) . d exactly, R -= c d in fp32 (Eq.4), new hi / lo split, new delta.
//
// Orientation: atoms are the M rows of the MFMA (A operand = dictionary tile from LDS), tokens the
// N columns (B operand = hi, held in registers for the whole sweep).  Each lane therefore owns one
// token column and 16 atom rows per tile, and the running maxima never leave its registers.  The
// contraction index is permuted so that lane half 0 holds dimensions 0..63 and half 1 holds 64..127
// (any order is valid as long as both operands use it): vector and atom rows are then read as 128
// contiguous bytes per lane.  A wave owns 2 x 32 tokens so that every A fragment read from LDS feeds
// two MFMAs.  Dictionary stages (64 atoms, 16 KiB) go from global memory straight into LDS
// (global_load_lds_dwordx4) through a ring of three buffers, fetched two stages ahead, 16-byte
// chunks XOR-swizzled by the row number so that 16 consecutive rows read at the same logical chunk
// cover all LDS banks.  Two waves per SIMD either way: two 4-wave workgroups
// share a CU, so one workgroup's select / update phase (vector ALU, gathers) overlaps the other's
// sweep (matrix cores), or - for launches large enough - one 8-wave workgroup has the CU, whose 512
// vectors share every dictionary stage (half the stage traffic per MFMA).
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "csr_internal.h"
#include "encode_common.h"

namespace csr {
namespace {

using namespace enc;

constexpr int kBlocks = 2;                            // 32-token blocks per wave
constexpr int kTokPerWave = 32 * kBlocks;             // 64
// Waves per workgroup W: 8 (512 vectors, one workgroup per CU) for launches that fill the chip that way - twice
// the vectors share a dictionary stage, so half the stage traffic per MFMA, 3 % faster although the eight waves
// then select and update at the same time - and 4 (256 vectors, two workgroups per CU) for smaller ones.
constexpr int kStageBytes = 16384;                    // one LDS stage: rows unpadded, 16-byte pieces XOR-swizzled
constexpr int kRing = 3;                              // stage buffers; stage st lives in buffer st % 3
template <int W> constexpr int stage_loads() { return kStageBytes / (16 * 64 * W); }  // load instructions per lane and stage
// Shapes that follow from the vector length DC (128, 64 or 32)
template <int DC> struct Shape {
    static constexpr int kRowBytes = DC * 2;
    static constexpr int kFrags = DC / 16;                       // 8-element MFMA operand fragments per lane
    static constexpr int kStageAtoms = kStageBytes / kRowBytes;  // 64 | 128 | 256
    static constexpr int kStageTiles = kStageAtoms / 32;         // 32-atom tiles per stage: 2 | 4 | 8
    static constexpr int kPieces = kRowBytes / 16;               // 16-byte pieces per row: 16 | 8 | 4
    static constexpr int kRowsPerKiB = 1024 / kRowBytes;         // rows one wave-wide load instruction fills: 4 | 8 | 16
    // XOR term of a row's piece positions.  A 256-byte row spans all 64 banks, so 16 consecutive rows must
    // differ; two 128-byte rows span them, so 16 consecutive rows need 8 different terms, one per row pair;
    // four 64-byte rows span them: 4 terms, one per group of four rows.
    static __device__ __forceinline__ int swz(int row)
    {
        return DC == 128 ? (row & 15) : DC == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
    }
};
constexpr int kScratchPerWave = 1024;                 // LDS a wave uses to share one token's state
constexpr int kScratchOff = kRing * kStageBytes;
template <int W> constexpr int lds_bytes() { return kScratchOff + W * kScratchPerWave; }  // 52 KiB (W = 4) | 56 KiB
constexpr int kTrack = 4;                             // group maxima tracked per lane and sweep
constexpr int kNormSlices = 8;                        // workgroups per dictionary in the norm pre-pass







// One dictionary stage (64 atoms x 256 B) from global memory into an LDS buffer, no registers in
// between.  Each wave instruction fills 1 KiB = 4 rows; lane l lands at byte 16 l of that KiB, i.e.
// row l/16, piece position l%16, and fetches source piece position ^ swz(row).  A wave's
// instructions are 16 rows apart (32 rows of 128 B), so that XOR term is the same for all of them and the
// source is (uniform stage base + 4 KiB steps) + one per-lane offset, `lane_off` = stage_lane_offset().
// Rows past the dictionary's end are not fetched; the sweep never reads those tiles.
template <int DC>
__device__ __forceinline__ uint32_t stage_lane_offset(int wave, int lane)
{
    using S = Shape<DC>;
    const int row0 = wave * S::kRowsPerKiB + lane / S::kPieces;
    return (uint32_t)(row0 * S::kRowBytes + (((lane % S::kPieces) ^ S::swz(row0)) << 4));
}

template <int DC, int W>
__device__ __forceinline__ void issue_stage(const __half *__restrict__ Dh, int stage, int32_t N, unsigned char *buf,
                                            int wave, int lane, uint32_t lane_off)
{
    using S = Shape<DC>;
    const unsigned char *sbase = reinterpret_cast<const unsigned char *>(Dh) + (int64_t)stage * kStageBytes;
    const int rows_left = N - stage * S::kStageAtoms - (wave * S::kRowsPerKiB + lane / S::kPieces);  // > 0 for the rows that exist
#pragma unroll
    for (int i = 0; i < stage_loads<W>(); ++i) {
        if (W * S::kRowsPerKiB * i < rows_left)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(sbase + i * (W * 1024) + lane_off),
                (__attribute__((address_space(3))) void *)(buf + (i * W + wave) * 1024), 16, 0, 0);
    }
}

// dnorm[h][slice] = max over the slice's atoms of |d_n|_2: the screening bound scales with it.
template <int DC>
__global__ __launch_bounds__(256) void dict_norm_kernel(const __half *__restrict__ Dict, float *__restrict__ dnorm, int32_t N)
{
    __shared__ float red[4];
    constexpr int kLanes = DC / 8;        // lanes per atom, 8 dimensions each
    constexpr int kAtoms = 256 / kLanes;  // atoms per pass of the workgroup
    const int h = blockIdx.x, sl = blockIdx.y, tid = threadIdx.x;
    const __half *Dh = Dict + (int64_t)h * N * DC;
    const int sub = tid % kLanes;
    float best = 0.0f;
    for (int n = sl * kAtoms + tid / kLanes; n < N; n += kAtoms * kNormSlices) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)n * DC + sub * 8);
        float f[8];
        unpack8(raw, f);
        float ss = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(f[e], f[e], ss);
#pragma unroll
        for (int m = kLanes / 2; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
        best = fmaxf(best, ss);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) best = fmaxf(best, __shfl_xor(best, m, 64));
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) dnorm[h * kNormSlices + sl] = sqrtf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])));
}

// The whole wave resolves ONE token whose pick the fast path could not decide.  `scr` holds that
// token's state, written by its two owner lanes:
//   [0, 256)    hi, dimensions in order        [256, 512)  lo
//   [512, 544)  tracked group values, lane half 0 then half 1
//   [544, 552)  threshold bits, overflow flag
// Lane (a = lane / 4, q = lane % 4) evaluates atom a of a 16-atom group over a quarter of the dimensions.
// Returns the arg-max of |hi . d + lo . d| (lowest index on ties) over the candidate groups, or over
// all atoms when the overflow flag is set.
template <int DC>
__device__ __forceinline__ int resolve_token(const __half *__restrict__ Dh, int32_t N, int ntiles, uint32_t code_mask,
                                             const unsigned char *scr, int lane)
{
    constexpr int kQ = DC / 32;  // 8-element pieces of a quarter vector
    const int a = lane >> 2, q = lane & 3;
    half8 th[kQ], tl[kQ];
#pragma unroll
    for (int j = 0; j < kQ; ++j) {
        th[j] = *reinterpret_cast<const half8 *>(scr + q * (DC / 2) + j * 16);
        tl[j] = *reinterpret_cast<const half8 *>(scr + 256 + q * (DC / 2) + j * 16);
    }
    const uint2 tf = *reinterpret_cast<const uint2 *>(scr + 544);
    const uint32_t thr_bits = __builtin_amdgcn_readfirstlane(tf.x);
    const bool ovf = __builtin_amdgcn_readfirstlane(tf.y) != 0;

    float ba = -1.0f;
    int bn = 0;
    // `batch` atoms at a time: all their rows are requested before the first product waits
    auto eval = [&](const int (&n)[2], int batch) {
        uint4 raw[2][kQ];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            if (b < batch) {
                const __half *row = Dh + (int64_t)n[b] * DC + q * (DC / 4);
#pragma unroll
                for (int j = 0; j < kQ; ++j) raw[b][j] = *reinterpret_cast<const uint4 *>(row + 8 * j);
            }
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            if (b < batch) {
                float s0 = 0.0f, s1 = 0.0f, l0 = 0.0f, l1 = 0.0f;
#pragma unroll
                for (int j = 0; j < kQ; ++j) {
                    const half8 dv = *reinterpret_cast<const half8 *>(&raw[b][j]);
                    dot8(th[j], dv, s0, s1);
                    dot8(tl[j], dv, l0, l1);
                }
                float c = (s0 + s1) + (l0 + l1);
                c += __shfl_xor(c, 1, 64);
                c += __shfl_xor(c, 2, 64);
                const float ab = fabsf(c);
                if (ab > ba || (ab == ba && n[b] < bn)) { ba = ab; bn = n[b]; }
            }
        }
    };
    if (!ovf) {
#pragma unroll 1
        for (int e = 0; e < 2 * kTrack; ++e) {
            const uint32_t u = __builtin_amdgcn_readfirstlane(*reinterpret_cast<const uint32_t *>(scr + 512 + 4 * e));
            if (u < thr_bits) continue;
            const int tile = ntiles - 1 - (int)(u & code_mask);
            const int n[2] = {tile * 32 + 4 * (e / kTrack) + 8 * (a >> 2) + (a & 3), 0};
            eval(n, 1);
        }
    } else {
        int n0 = 0;
#pragma unroll 1
        for (; n0 < N; n0 += 32) {
            const int n[2] = {n0 + a, n0 + 16 + a};
            eval(n, 2);
        }
    }
#pragma unroll
    for (int m = 4; m <= 32; m <<= 1) {
        const float oa = __shfl_xor(ba, m, 64);
        const int on = __shfl_xor(bn, m, 64);
        if (oa > ba || (oa == ba && on < bn)) { ba = oa; bn = on; }
    }
    return __builtin_amdgcn_readfirstlane(bn);
}

template <int DC, int W>
__global__ __launch_bounds__(64 * W, 8 / W) void encode_mfma_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, const float *__restrict__ dnorm, int64_t T, int64_t M, int32_t N, int32_t s, int32_t sn,
    int64_t x_stride_h, int64_t x_stride_t, int32_t dict_count, int64_t code_stride_h, int32_t tiles_per_h,
    int32_t n_groups, int32_t idx16, int32_t coef_mode, uint32_t code_mask,
    float *__restrict__ res_norm2)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    using S = Shape<DC>;
    constexpr int kFrags = S::kFrags, kStageTiles = S::kStageTiles, kStageAtoms = S::kStageAtoms;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hf = lane >> 5;
    unsigned char *scr = lds + kScratchOff + wave * kScratchPerWave;

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of work so
    // that workgroups sharing a dictionary share an L2.
    // (The n_groups % 8 workgroups at the end keep their own numbers.)
    int work = blockIdx.x;
    if ((int)blockIdx.x < (n_groups & ~7)) work = (blockIdx.x & 7) * (n_groups >> 3) + (blockIdx.x >> 3);
    // Work is dealt per dictionary, not per vector block: dct = dictionary * sn + chunk owns the vectors of all
    // blocks that use it (block h uses dictionary h % dict_count), numbered m = (h / dict_count) * T + t, in tiles
    // of 256.  Blocks with few vectors that share a dictionary - a batch of sequences in a decoding step - then
    // fill tiles together instead of taking a nearly empty one each.
    const int dct = work / tiles_per_h;
    const int tile_wg = work - dct * tiles_per_h;
    const int dict = dct / sn, ch = dct - dict * sn;
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    const int ntiles = N >> 5;
    const int nstages = (N + kStageAtoms - 1) / kStageAtoms;
    const int nstages_full = N / kStageAtoms;

    const uint32_t lane_off = stage_lane_offset<DC>(wave, lane);
    issue_stage<DC, W>(Dh, 0, N, lds, wave, lane, lane_off);  // in flight while the vectors are loaded
    if (nstages > 1) issue_stage<DC, W>(Dh, 1, N, lds + kStageBytes, wave, lane, lane_off);
    // LDS byte offset, inside a 32-row tile, of this lane's A fragment j (row = col, piece kFrags hf + j)
    uint32_t frag_off[kFrags];
#pragma unroll
    for (int j = 0; j < kFrags; ++j)
        frag_off[j] = (uint32_t)(col * S::kRowBytes + (((hf * kFrags + j) ^ S::swz(col)) << 4));

    float dmax = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormSlices; ++i) dmax = fmaxf(dmax, dnorm[dct * kNormSlices + i]);
    // ~code_mask in a vector register, so that packing value and tile code is one instruction with
    // the code as its only scalar operand
    uint32_t keep_mask;
    asm volatile("v_mov_b32 %0, %1" : "=v"(keep_mask) : "s"(~code_mask));
    // relative slack of a packed value: its low mantissa bits were replaced by the tile code
    const float pack_q = (float)(code_mask + 1) * 1.1920929e-7f;

    // ---- load the vectors, scale by a power of two, split into hi + lo ---------------------------
    half8 hi[kBlocks][kFrags], lo[kBlocks][kFrags];
    bool valid[kBlocks];
    int hblk[kBlocks];    // the vector's block and its position in the block
    int64_t tpos[kBlocks];
    int sexp[kBlocks];
    float delta[kBlocks], rn2[kBlocks];
#pragma unroll
    for (int bi = 0; bi < kBlocks; ++bi) {
        const int64_t m = (int64_t)tile_wg * (W * kTokPerWave) + wave * kTokPerWave + bi * 32 + col;
        valid[bi] = m < M;
        const int64_t mc = valid[bi] ? m : M - 1;  // tail lanes recompute the last vector, never store
        const int rep_b = (int)(mc / T);
        tpos[bi] = mc - rep_b * T;
        hblk[bi] = rep_b * dict_count + dict;
        const __half *xr = X + (int64_t)hblk[bi] * x_stride_h + tpos[bi] * x_stride_t + ch * DC + hf * (DC / 2);
        float xv[kFrags][8];
        float amax = 0.0f;
#pragma unroll
        for (int j = 0; j < kFrags; ++j) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(xr + 8 * j);
            unpack8(raw, xv[j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xv[j][e]));
        }
        amax = fmaxf(amax, xchg32f(amax, hf));
        int ex = 0;
        if (amax > 0.0f && amax < INFINITY) {
            (void)frexpf(amax, &ex);  // amax = f 2^ex, f in [0.5, 1)
            ex = 12 - ex;             // brings amax into [2^11, 2^12)
        }
        sexp[bi] = ex;
        float r2 = 0.0f, lo2 = 0.0f;
#pragma unroll
        for (int j = 0; j < kFrags; ++j) {
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
        r2 += xchg32f(r2, hf);
        lo2 += xchg32f(lo2, hf);
        rn2[bi] = r2;
        delta[bi] = screen_delta(dmax, lo2, r2);
    }

    for (int g = 0; g < s; ++g) {
        // ---- screen: one MFMA sweep over the dictionary ------------------------------------
        uint32_t u[kBlocks][kTrack];
        uint32_t keep[kBlocks][8];
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
#pragma unroll
            for (int k = 0; k < kTrack; ++k) u[bi][k] = 0u;
#pragma unroll
            for (int r = 0; r < 8; ++r) keep[bi][r] = 0u;
        }

        // stages 0 and 1 were requested before (at kernel start or behind the previous select phase)
        wait_vmem();
        __syncthreads();  // stages 0 and 1 are in buffers 0 and 1

        // one stage: fetch the one after next into the free buffer, sweep this one's tiles, then wait
        // for the next one (the most recent request may stay in flight) and meet the other waves
        auto do_stage = [&](int st, auto buf_c) {
            constexpr int kBuf = decltype(buf_c)::value;
            const bool more = st + 2 < nstages;
            if (more) issue_stage<DC, W>(Dh, st + 2, N, lds + ((kBuf + 2) % kRing) * kStageBytes, wave, lane, lane_off);
            const int tiles_here = min(kStageTiles, ntiles - st * kStageTiles);
#pragma unroll
            for (int rt = 0; rt < kStageTiles; ++rt) {
                if (rt < tiles_here) {
                    floatx16 acc[kBlocks];
#pragma unroll
                    for (int bi = 0; bi < kBlocks; ++bi)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[bi][r] = 0.0f;
                    half8 a[kFrags];  // all fragments of the row tile requested before the first MFMA waits
#pragma unroll
                    for (int j = 0; j < kFrags; ++j)
                        a[j] = *reinterpret_cast<const half8 *>(lds + kBuf * kStageBytes + rt * 32 * S::kRowBytes + frag_off[j]);
#pragma unroll
                    for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                        for (int bi = 0; bi < kBlocks; ++bi)
                            acc[bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], hi[bi][j], acc[bi], 0, 0, 0);
                    }
                    const uint32_t code = (uint32_t)(ntiles - 1 - (st * kStageTiles + rt));  // earlier tile = larger code
#pragma unroll
                    for (int bi = 0; bi < kBlocks; ++bi) {
                        float m = 0.0f;  // eight v_max3_f32 with |.| operand modifiers
#pragma unroll
                        for (int r = 0; r < 16; r += 2) m = fmaxf(fmaxf(m, fabsf(acc[bi][r])), fabsf(acc[bi][r + 1]));
                        const uint32_t v = (__float_as_uint(m) & keep_mask) | code;  // one v_and_or_b32
                        const bool new_best = v > u[bi][0];
                        // keep the magnitudes (fp16, rounded toward zero) of the lane's best group so far.  A branch,
                        // not a select: the eight conversions then run out of line, only in the tiles in which some
                        // lane has a new best group, and only on those lanes
                        if (__builtin_expect(new_best, 0)) {
#pragma unroll
                            for (int r = 0; r < 8; ++r) {
                                const auto pk = __builtin_amdgcn_cvt_pkrtz(fabsf(acc[bi][2 * r]), fabsf(acc[bi][2 * r + 1]));
                                keep[bi][r] = *reinterpret_cast<const uint32_t *>(&pk);
                            }
                        }
                        const uint32_t n3 = umed3(u[bi][2], u[bi][3], v);
                        const uint32_t n2 = umed3(u[bi][1], u[bi][2], v);
                        const uint32_t n1 = umed3(u[bi][0], u[bi][1], v);
                        u[bi][0] = max(u[bi][0], v);
                        u[bi][1] = n1;
                        u[bi][2] = n2;
                        u[bi][3] = n3;
                    }
                }
            }
            // Only a complete stage takes the full count of load instructions: behind the fetch of a partial last
            // stage, "all but the newest ones" could still leave loads of the next stage to be swept in flight.
            if (st + 2 < nstages_full) wait_vmem_but<stage_loads<W>()>(); else wait_vmem();
            __syncthreads();
        };
        for (int st = 0; st < nstages; st += kRing) {
            do_stage(st, std::integral_constant<int, 0>{});
            if (st + 1 < nstages) do_stage(st + 1, std::integral_constant<int, 1>{});
            if (st + 2 < nstages) do_stage(st + 2, std::integral_constant<int, 2>{});
        }
        // all buffers are free now: fetch stages 0 and 1 for the next sweep behind the select phase
        if (g + 1 < s) {
            issue_stage<DC, W>(Dh, 0, N, lds, wave, lane, lane_off);
            if (nstages > 1) issue_stage<DC, W>(Dh, 1, N, lds + kStageBytes, wave, lane, lane_off);
        }

        // ---- select: the iteration's atom for every token, one 32-token block at a time -------
        int best_n[kBlocks];
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
            uint32_t pu[kTrack];
#pragma unroll
            for (int k = 0; k < kTrack; ++k) pu[k] = xchg32(u[bi][k], hf);
            // best group of the token: own or the partner lane's (equal values: lane half 0 first)
            const bool own_best = hf == 0 ? u[bi][0] >= pu[0] : u[bi][0] > pu[0];
            const uint32_t best_u = own_best ? u[bi][0] : pu[0];
            const int best_half = own_best ? hf : 1 - hf;
            const float A = __uint_as_float(best_u & ~code_mask);
            const float thr = (A - delta[bi]) * (1.0f - 2.0f * pack_q);
            const uint32_t thr_bits = thr > 0.0f ? (__float_as_uint(thr) & ~code_mask) : 0u;
            const bool zero = !(rn2[bi] > 0.0f);
            int ncand = 0;
#pragma unroll
            for (int k = 0; k < kTrack; ++k) ncand += (int)(u[bi][k] >= thr_bits) + (int)(pu[k] >= thr_bits);
            const bool overflow = u[bi][kTrack - 1] >= thr_bits || pu[kTrack - 1] >= thr_bits;

            // this lane's best group as kept during the sweep: largest value, its position, runner-up
            float ba = -1.0f, sa = -1.0f;
            int bk = 0;
            {
                const uint32_t(&w)[8] = keep[bi];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float2 f = __half22float2(*reinterpret_cast<const __half2 *>(&w[r]));
                    if (f.x > ba) { sa = ba; ba = f.x; bk = 2 * r; } else sa = fmaxf(sa, f.x);
                    if (f.y > ba) { sa = ba; ba = f.y; bk = 2 * r + 1; } else sa = fmaxf(sa, f.y);
                }
            }
            // kept values were rounded toward zero to 11 bits: two of them are told apart only
            // beyond delta + 2^-10 of the larger
            const bool close_own = !(sa < ba - delta[bi] - ba * 9.765625e-4f);
            const uint32_t mine = (uint32_t)bk | (close_own ? 16u : 0u);
            const uint32_t theirs = xchg32(mine, hf);
            const uint32_t pick = own_best ? mine : theirs;
            const int kk = (int)(pick & 15u);
            const int tile0 = ntiles - 1 - (int)(best_u & code_mask);
            best_n[bi] = tile0 * 32 + 4 * best_half + 8 * (kk >> 2) + (kk & 3);
            const bool unsure = !zero && (ncand > 1 || overflow || (pick & 16u) != 0u);

            // the undecided tokens, one at a time, by the whole wave (both lanes of a pair agree on `unsure`)
            uint32_t todo = (uint32_t)__ballot(unsure);
            while (todo) {
                const int t = __ffs((int)todo) - 1;
                todo &= todo - 1;
                if (col == t) {
#pragma unroll
                    for (int j = 0; j < kFrags; ++j) {
                        *reinterpret_cast<half8 *>(scr + hf * DC + j * 16) = hi[bi][j];
                        *reinterpret_cast<half8 *>(scr + 256 + hf * DC + j * 16) = lo[bi][j];
                    }
                    *reinterpret_cast<uint4 *>(scr + 512 + hf * 16) = make_uint4(u[bi][0], u[bi][1], u[bi][2], u[bi][3]);
                    if (hf == 0) *reinterpret_cast<uint2 *>(scr + 544) = make_uint2(thr_bits, overflow ? 1u : 0u);
                }
                wave_lds_fence();
                const int n_res = resolve_token<DC>(Dh, N, ntiles, code_mask, scr, lane);
                wave_lds_fence();
                if (col == t) best_n[bi] = n_res;
            }
            if (zero) best_n[bi] = 0;
        }

        // ---- update: c = (hi + lo) . d exactly, Eq.4 on the full-precision residual, new split ----
        uint4 raw[kBlocks][kFrags];  // both blocks' atom rows are requested before either is used
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
            const __half *row = Dh + (int64_t)best_n[bi] * DC + hf * (DC / 2);
#pragma unroll
            for (int j = 0; j < kFrags; ++j) raw[bi][j] = *reinterpret_cast<const uint4 *>(row + 8 * j);
        }
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi) {
            float s0 = 0.0f, s1 = 0.0f, l0 = 0.0f, l1 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                const half8 dv = *reinterpret_cast<const half8 *>(&raw[bi][j]);
                dot8(hi[bi][j], dv, s0, s1);
                dot8(lo[bi][j], dv, l0, l1);
            }
            float best_c = (s0 + s1) + (l0 + l1);
            best_c += xchg32f(best_c, hf);
            if (!(rn2[bi] > 0.0f)) best_c = 0.0f;
            // closed loop: what Eq.4 subtracts is the coefficient as it will be stored (rounded in the input's scale)
            if (coef_rounds_in_loop(coef_mode)) best_c = ldexpf(__half2float(__float2half_rn(ldexpf(best_c, -sexp[bi]))), sexp[bi]);
            float v[kFrags][8];
            float r2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                float f[8];
                unpack8(raw[bi][j], f);
                const half8 ho = hi[bi][j], lo_o = lo[bi][j];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float r = (float)ho[e] + (float)lo_o[e];  // exact: 22 significant bits
                    v[j][e] = fmaf(-best_c, f[e], r);
                    r2 = fmaf(v[j][e], v[j][e], r2);
                }
            }
            r2 += xchg32f(r2, hf);
            const int sexp_used = sexp[bi];
            // A residual that has shrunk a lot (a vector that is nearly a multiple of an atom) is
            // scaled up again before the split, or lo would sink into the fp16 subnormals; one that
            // has grown (atoms of norm above sqrt(2) make Eq.4 expand it) is scaled down before hi
            // could leave the fp16 range.
            const bool rescale = (r2 < 65536.0f && r2 > 0.0f) || (r2 >= 1073741824.0f && r2 < INFINITY);
            if (__ballot(rescale) != 0ull) {
                int e2 = 0;
                (void)frexpf(r2, &e2);                        // |R| in [2^((e2-1)/2), 2^(e2/2))
                const int k = rescale ? 14 - (e2 + 1) / 2 : 0;  // brings |R| into [2^12.5, 2^14.5)
                const float sc = ldexpf(1.0f, k);
#pragma unroll
                for (int j = 0; j < kFrags; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[j][e] *= sc;
                r2 *= sc * sc;
                sexp[bi] += k;
            }
            float lo2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                half8 hv, lv;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const _Float16 hh = (_Float16)v[j][e];
                    const float l = v[j][e] - (float)hh;
                    hv[e] = hh;
                    lv[e] = (_Float16)l;
                    lo2 = fmaf(l, l, lo2);
                }
                hi[bi][j] = hv;
                lo[bi][j] = lv;
            }
            lo2 += xchg32f(lo2, hf);
            rn2[bi] = r2;
            delta[bi] = screen_delta(dmax, lo2, r2);
            if (valid[bi]) {
                const int64_t o = (int64_t)hblk[bi] * code_stride_h + (tpos[bi] * sn + ch) * s + g;
                if (hf == 0) {
                    if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n[bi];
                    else reinterpret_cast<int32_t *>(idx_out)[o] = best_n[bi];
                } else {
                    const float c_out = ldexpf(best_c, -sexp_used);
                    if (coef_is_f16(coef_mode)) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(c_out);
                    else reinterpret_cast<float *>(coef_out)[o] = c_out;
                }
            }
        }
    }
    if (res_norm2) {  // |R_{s+1}|^2, back in the input's scale
#pragma unroll
        for (int bi = 0; bi < kBlocks; ++bi)
            if (valid[bi] && hf == 0)
                res_norm2[((int64_t)hblk[bi] * T + tpos[bi]) * sn + ch] = ldexpf(rn2[bi], -2 * sexp[bi]);
    }
}

size_t r256(size_t v) { return (v + 255) & ~size_t(255); }

}  // namespace

bool encode_mfma_supported(const EncodeArgs &a)
{
    return a.f16 && (a.d == 128 || a.d == 64 || a.d == 32) && a.N >= 32 && a.N % 32 == 0 && a.N <= 65536;
}

size_t encode_mfma_workspace_bytes(int32_t H, int64_t T, int32_t N, int32_t s)
{
    (void)T; (void)N; (void)s;
    return r256((size_t)H * kNormSlices * sizeof(float));
}

template <int DC, int W>
hipError_t launch_encode_mfma_w(const EncodeArgs &a)
{
    constexpr int kTokPerWG = W * kTokPerWave;
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;  // vectors per dictionary
    const int64_t tiles = (M + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.dict_count * a.sn;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    float *dnorm = reinterpret_cast<float *>(a.workspace);
    const int ntiles = a.N / 32;
    int bits = 0;
    while ((1 << bits) < ntiles) ++bits;
    const uint32_t code_mask = (1u << bits) - 1u;

    // per device, once: the kernel's LDS need is above the default limit
    static std::atomic<bool> attr_set[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(encode_mfma_kernel<DC, W>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes<W>());
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(dict_norm_kernel<DC>, dim3((unsigned)(a.dict_count * a.sn), kNormSlices), dim3(256), 0, a.stream,
                       (const __half *)a.D, dnorm, a.N);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((encode_mfma_kernel<DC, W>), dim3((unsigned)groups), dim3(64 * W), lds_bytes<W>(), a.stream,
                       (const __half *)a.X, (const __half *)a.D, a.idx, a.coef, dnorm, a.T, M, a.N, a.s, a.sn, a.x_stride_h,
                       a.x_stride_t, a.dict_count, a.code_stride_h, (int32_t)tiles, (int32_t)groups, (int32_t)a.idx16,
                       (a.coef16 ? kCoefF16 : 0) | (a.closed_loop ? kCoefClosed : 0), code_mask,
                       a.res_norm2);
    return hipGetLastError();
}

template <int DC>
hipError_t launch_encode_mfma_t(const EncodeArgs &a)
{
    static std::atomic<int> n_cus[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (n_cus[dev].load(std::memory_order_acquire) == 0) {
        int v = 0;
        e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        n_cus[dev].store(v > 0 ? v : 1, std::memory_order_release);
    }
    const int cus = n_cus[dev].load(std::memory_order_relaxed);
    // 512-vector workgroups (one per CU) once there is one for every CU
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;
    const int64_t groups8 = (M + 8 * kTokPerWave - 1) / (8 * kTokPerWave) * a.dict_count * a.sn;
    if (groups8 >= (int64_t)cus) return launch_encode_mfma_w<DC, 8>(a);
    return launch_encode_mfma_w<DC, 4>(a);
}

hipError_t launch_encode_mfma(const EncodeArgs &a)
{
    return a.d == 32 ? launch_encode_mfma_t<32>(a) : a.d == 64 ? launch_encode_mfma_t<64>(a) : launch_encode_mfma_t<128>(a);
}

}  // namespace csr
