// Matching Pursuit encoder for SMALL dictionaries (gfx950): the whole dictionary of a head - up to 128 KB of fp16
// atoms, e.g. the 256 or 512 atoms per head of the paper's own experiments - stays in LDS for the life of a
// workgroup, and every wave works through its vectors on its own, without a single barrier after the load.
//
// Eq.2-4 of Section "Sparse representation", s iterations per vector.  The method is the large-dictionary encoder's
// (screen all atoms with one fp16 matrix-core sweep of hi, the fp16 rounding of the residual R = hi + lo; decide
// exactly wherever the screened values are closer than the bound delta = 2 dmax (|lo| + gamma |hi|); update in
// fp32), but with so few atoms the sweep is short and that encoder's shape is bound by its chain of dependent
// steps per iteration - staged dictionary loads with barriers, candidate atoms and the chosen atom fetched from
// global memory.  Here:
//
//   sweep    v_mfma_f32_32x32x16_f16, atoms as rows (fragments read from LDS), 32 vectors as columns; per lane the
//            four largest group maxima with the tile number packed into the low mantissa bits, and the 16
//            magnitudes (fp16) of the lane's best group, rewritten under a branch when that group changes.
//   select   decided from the kept values when the leader is ahead by more than delta (about 97 % of the steps);
//            else the wave evaluates hi . d + lo . d (exact products, fp32 sums) for every atom of every candidate
//            group - or for all atoms if even a lane's fourth tracked group is a candidate - out of LDS.
//   update   c = R . d in fp32 with the atom row from LDS, R - c d (Eq.4, unrounded c), new hi, new delta.  The
//            residual itself is kept in fp32 registers here (a wave owns 32 vectors at a time, so there is room):
//            with so short a sweep the conversions of a two-halves residual would be the largest cost.
//
// Every vector is first multiplied by a power of two that brings its largest element into [2^11, 2^12)
// (Matching Pursuit commutes with it; lo stays clear of the fp16 subnormals).  The largest atom norm, which scales
// delta, is computed while the dictionary is loaded.
#include <atomic>

#include "csr_internal.h"
#include "encode_common.h"

namespace csr {
namespace {

using namespace enc;

constexpr int kWaves = 8;                    // two per SIMD; one workgroup per CU (the dictionary fills the LDS)
constexpr int kThreads = 64 * kWaves;
constexpr int kBlocksPerWave = 2;            // 32-vector blocks a wave works through, one after the other
constexpr int kTokPerWG = kWaves * kBlocksPerWave * 32;  // 512
constexpr int kMaxDictBytes = 128 * 1024;
constexpr int kScratchPerWave = 1024;        // LDS a wave uses to share one vector's state
constexpr int kTrack = 4;                    // group maxima tracked per lane and sweep






// XOR term of a row's 16-byte piece positions, so that 16 consecutive rows read at one logical piece cover all
// banks: a 256-byte row spans the 64 banks (16 different terms), two 128-byte rows span them (8, one per pair).
template <int DC> __device__ __forceinline__ int swz(int row) { return DC == 128 ? (row & 15) : ((row >> 1) & 7); }

// byte offset in the LDS copy of the dictionary of piece `piece` (8 dimensions) of atom `row`
template <int DC> __device__ __forceinline__ uint32_t piece_at(int row, int piece)
{
    return (uint32_t)(row * (DC * 2) + ((piece ^ swz<DC>(row)) << 4));
}

// The whole wave resolves ONE vector whose pick the kept values could not decide.  `scr` holds that vector's
// state, written by its two owner lanes:
//   [0, 256)    hi, dimensions in order        [256, 512)  lo
//   [512, 544)  tracked group values, lane half 0 then half 1
//   [544, 552)  threshold bits, overflow flag
// Lane (a = lane / 4, q = lane % 4) evaluates atom a of a 16-atom group over a quarter of the dimensions.
// Returns the arg-max of |hi . d + lo . d| (lowest index on ties) over the candidate groups, or over all atoms
// when the overflow flag is set.
template <int DC>
__device__ __forceinline__ int resolve_vector(const unsigned char *dict, int32_t N, int ntiles, uint32_t code_mask,
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
    auto eval = [&](int n) {
        float s0 = 0.0f, s1 = 0.0f, l0 = 0.0f, l1 = 0.0f;
#pragma unroll
        for (int j = 0; j < kQ; ++j) {
            const half8 dv = *reinterpret_cast<const half8 *>(dict + piece_at<DC>(n, q * kQ + j));
            dot8(th[j], dv, s0, s1);
            dot8(tl[j], dv, l0, l1);
        }
        float c = (s0 + s1) + (l0 + l1);
        c += __shfl_xor(c, 1, 64);
        c += __shfl_xor(c, 2, 64);
        const float ab = fabsf(c);
        if (ab > ba || (ab == ba && n < bn)) { ba = ab; bn = n; }
    };
    if (!ovf) {
#pragma unroll 1
        for (int e = 0; e < 2 * kTrack; ++e) {
            const uint32_t u = __builtin_amdgcn_readfirstlane(*reinterpret_cast<const uint32_t *>(scr + 512 + 4 * e));
            if (u < thr_bits) continue;
            const int tile = ntiles - 1 - (int)(u & code_mask);
            eval(tile * 32 + 4 * (e / kTrack) + 8 * (a >> 2) + (a & 3));
        }
    } else {
#pragma unroll 1
        for (int n0 = 0; n0 < N; n0 += 16) eval(n0 + a);
    }
#pragma unroll
    for (int m = 4; m <= 32; m <<= 1) {
        const float oa = __shfl_xor(ba, m, 64);
        const int on = __shfl_xor(bn, m, 64);
        if (oa > ba || (oa == ba && on < bn)) { ba = oa; bn = on; }
    }
    return __builtin_amdgcn_readfirstlane(bn);
}

// OCC: waves per SIMD the register budget is set for.  64-dimensional vectors need few enough registers for 4, so
// that two workgroups share a CU when their dictionaries both fit its LDS (measured 12 - 14 % faster; with one
// workgroup per CU the tighter budget only costs spills).
template <int DC, int OCC>
__global__ __launch_bounds__(kThreads, OCC) void encode_resident_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, int64_t T, int64_t M, int32_t N, int32_t s, int32_t sn, int64_t x_stride_h, int64_t x_stride_t,
    int32_t dict_count, int64_t code_stride_h, int32_t tiles_per_h, int32_t idx16, int32_t coef_mode, uint32_t code_mask,
    float *__restrict__ res_norm2)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    constexpr int kFrags = DC / 16;       // 8-element operand fragments per lane
    constexpr int kRowBytes = DC * 2;
    constexpr int kPieces = kRowBytes / 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hf = lane >> 5;
    // work is dealt per dictionary: dct = dictionary * sn + chunk owns the vectors of all blocks that use it
    // (block h uses dictionary h % dict_count), numbered m = (h / dict_count) * T + t, in tiles of 512
    const int dct = blockIdx.x / tiles_per_h;
    const int tile_wg = blockIdx.x - dct * tiles_per_h;
    const int dict = dct / sn, ch = dct - dict * sn;
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    const int ntiles = N >> 5;
    const int dict_bytes = N * kRowBytes;
    unsigned char *scr = lds + dict_bytes + wave * kScratchPerWave;
    float *red = reinterpret_cast<float *>(lds + dict_bytes + kWaves * kScratchPerWave);

    // ---- the dictionary, once: piece `pos` of row `row` goes to position pos ^ swz(row); its largest atom norm ---
    float dmax;
    {
        const int total = N * kPieces;
        const uint4 *src = reinterpret_cast<const uint4 *>(Dh);
        float best = 0.0f;
        for (int base = 0; base < total; base += kThreads) {  // kThreads is a multiple of kPieces: a row's pieces
            const int e = base + tid;                         // sit in kPieces consecutive lanes
            float ss = 0.0f;
            if (e < total) {
                const int row = e / kPieces, pos = e - row * kPieces;
                const uint4 raw = src[e];
                *reinterpret_cast<uint4 *>(lds + row * kRowBytes + ((pos ^ swz<DC>(row)) << 4)) = raw;
                float f[8];
                unpack8(raw, f);
#pragma unroll
                for (int k = 0; k < 8; ++k) ss = fmaf(f[k], f[k], ss);
            }
#pragma unroll
            for (int m = kPieces / 2; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
            best = fmaxf(best, ss);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) best = fmaxf(best, __shfl_xor(best, m, 64));
        if (lane == 0) red[wave] = best;
        __syncthreads();  // the only barrier: from here on the waves do not meet again
        float v = red[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) v = fmaxf(v, red[w]);
        dmax = sqrtf(v);
    }

    // LDS byte offset, inside a 32-row tile, of this lane's operand fragment j (row = col, piece kFrags hf + j)
    uint32_t frag_off[kFrags];
#pragma unroll
    for (int j = 0; j < kFrags; ++j) frag_off[j] = piece_at<DC>(col, hf * kFrags + j);
    // ~code_mask in a vector register: packing value and tile code is then one instruction
    uint32_t keep_mask;
    asm volatile("v_mov_b32 %0, %1" : "=v"(keep_mask) : "s"(~code_mask));
    // relative slack of a packed value: its low mantissa bits were replaced by the tile code
    const float pack_q = (float)(code_mask + 1) * 1.1920929e-7f;

    for (int bi = 0; bi < kBlocksPerWave; ++bi) {
        const int64_t m = (int64_t)tile_wg * kTokPerWG + (wave * kBlocksPerWave + bi) * 32 + col;
        if ((int64_t)tile_wg * kTokPerWG + (wave * kBlocksPerWave + bi) * 32 >= M) break;  // wave-uniform
        const bool valid = m < M;
        const int64_t mc = valid ? m : M - 1;  // tail lanes recompute the last vector, never store
        const int rep = (int)(mc / T);
        const int64_t tok = mc - rep * T;     // position in its block
        const int h = rep * dict_count + dict;

        // ---- load the vector, scale by a power of two, split into hi + lo -------------------------
        half8 hi[kFrags];          // fp16 rounding of the residual: the MFMA operand
        float R[kFrags][8];        // the residual, fp32
        int sexp = 0;
        float rn2, delta;
        {
            const __half *xr = X + (int64_t)h * x_stride_h + tok * x_stride_t + ch * DC + hf * (DC / 2);
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
            if (amax > 0.0f && amax < INFINITY) {
                int ex;
                (void)frexpf(amax, &ex);  // amax = f 2^ex, f in [0.5, 1)
                sexp = 12 - ex;           // brings amax into [2^11, 2^12)
            }
            float r2 = 0.0f, lo2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = ldexpf(xv[j][e], sexp);
                    const _Float16 hh = (_Float16)v;
                    const float l = v - (float)hh;
                    hi[j][e] = hh;
                    R[j][e] = v;
                    r2 = fmaf(v, v, r2);
                    lo2 = fmaf(l, l, lo2);
                }
            }
            rn2 = r2 + xchg32f(r2, hf);
            lo2 += xchg32f(lo2, hf);
            delta = screen_delta(dmax, lo2, rn2);
        }

        for (int g = 0; g < s; ++g) {
            // ---- screen: one MFMA sweep over the dictionary in LDS ---------------------------------
            uint32_t u[kTrack];
            uint32_t keep[8];
#pragma unroll
            for (int k = 0; k < kTrack; ++k) u[k] = 0u;
#pragma unroll
            for (int r = 0; r < 8; ++r) keep[r] = 0u;
            for (int t = 0; t < ntiles; ++t) {
                half8 a[kFrags];
#pragma unroll
                for (int j = 0; j < kFrags; ++j)
                    a[j] = *reinterpret_cast<const half8 *>(lds + t * 32 * kRowBytes + frag_off[j]);
                floatx16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
                for (int j = 0; j < kFrags; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], hi[j], acc, 0, 0, 0);
                const uint32_t code = (uint32_t)(ntiles - 1 - t);  // earlier tile = larger code
                float mx = 0.0f;  // eight v_max3_f32 with |.| operand modifiers
#pragma unroll
                for (int r = 0; r < 16; r += 2) mx = fmaxf(fmaxf(mx, fabsf(acc[r])), fabsf(acc[r + 1]));
                const uint32_t v = (__float_as_uint(mx) & keep_mask) | code;
                // the magnitudes (fp16, rounded toward zero) of the lane's best group so far, under a branch
                if (__builtin_expect(v > u[0], 0)) {
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const auto pk = __builtin_amdgcn_cvt_pkrtz(fabsf(acc[2 * r]), fabsf(acc[2 * r + 1]));
                        keep[r] = *reinterpret_cast<const uint32_t *>(&pk);
                    }
                }
                const uint32_t n3 = umed3(u[2], u[3], v);
                const uint32_t n2 = umed3(u[1], u[2], v);
                const uint32_t n1 = umed3(u[0], u[1], v);
                u[0] = max(u[0], v);
                u[1] = n1;
                u[2] = n2;
                u[3] = n3;
            }

            // ---- select: the iteration's atom for every vector of the block -------------------------
            int best_n;
            {
                uint32_t pu[kTrack];
#pragma unroll
                for (int k = 0; k < kTrack; ++k) pu[k] = xchg32(u[k], hf);
                // best group of the vector: own or the partner lane's (equal values: lane half 0 first)
                const bool own_best = hf == 0 ? u[0] >= pu[0] : u[0] > pu[0];
                const uint32_t best_u = own_best ? u[0] : pu[0];
                const int best_half = own_best ? hf : 1 - hf;
                const float A = __uint_as_float(best_u & ~code_mask);
                const float thr = (A - delta) * (1.0f - 2.0f * pack_q);
                const uint32_t thr_bits = thr > 0.0f ? (__float_as_uint(thr) & ~code_mask) : 0u;
                const bool zero = !(rn2 > 0.0f);
                int ncand = 0;
#pragma unroll
                for (int k = 0; k < kTrack; ++k) ncand += (int)(u[k] >= thr_bits) + (int)(pu[k] >= thr_bits);
                const bool overflow = u[kTrack - 1] >= thr_bits || pu[kTrack - 1] >= thr_bits;

                // this lane's best group as kept during the sweep: largest value, its position, runner-up
                float ba = -1.0f, sa = -1.0f;
                int bk = 0;
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float2 f = __half22float2(*reinterpret_cast<const __half2 *>(&keep[r]));
                    if (f.x > ba) { sa = ba; ba = f.x; bk = 2 * r; } else sa = fmaxf(sa, f.x);
                    if (f.y > ba) { sa = ba; ba = f.y; bk = 2 * r + 1; } else sa = fmaxf(sa, f.y);
                }
                // kept values were rounded toward zero to 11 bits: two of them are told apart only beyond
                // delta + 2^-10 of the larger
                const bool close_own = !(sa < ba - delta - ba * 9.765625e-4f);
                const uint32_t mine = (uint32_t)bk | (close_own ? 16u : 0u);
                const uint32_t theirs = xchg32(mine, hf);
                const uint32_t pick = own_best ? mine : theirs;
                const int kk = (int)(pick & 15u);
                const int tile0 = ntiles - 1 - (int)(best_u & code_mask);
                best_n = tile0 * 32 + 4 * best_half + 8 * (kk >> 2) + (kk & 3);
                const bool unsure = !zero && (ncand > 1 || overflow || (pick & 16u) != 0u);

                // the undecided vectors, one at a time, by the whole wave (both lanes of a pair agree on `unsure`)
                uint32_t todo = (uint32_t)__ballot(unsure);
                while (todo) {
                    const int t = __ffs((int)todo) - 1;
                    todo &= todo - 1;
                    if (col == t) {
#pragma unroll
                        for (int j = 0; j < kFrags; ++j) {
                            half8 lo;
#pragma unroll
                            for (int e = 0; e < 8; ++e) lo[e] = (_Float16)(R[j][e] - (float)hi[j][e]);
                            *reinterpret_cast<half8 *>(scr + hf * DC + j * 16) = hi[j];
                            *reinterpret_cast<half8 *>(scr + 256 + hf * DC + j * 16) = lo;
                        }
                        *reinterpret_cast<uint4 *>(scr + 512 + hf * 16) = make_uint4(u[0], u[1], u[2], u[3]);
                        if (hf == 0) *reinterpret_cast<uint2 *>(scr + 544) = make_uint2(thr_bits, overflow ? 1u : 0u);
                    }
                    wave_lds_fence();
                    const int n_res = resolve_vector<DC>(lds, N, ntiles, code_mask, scr, lane);
                    wave_lds_fence();
                    if (col == t) best_n = n_res;
                }
                if (zero) best_n = 0;
            }

            // ---- update: c = R . d in fp32, Eq.4, new hi ----------------------------------------------
            half8 dv[kFrags];
#pragma unroll
            for (int j = 0; j < kFrags; ++j) dv[j] = *reinterpret_cast<const half8 *>(lds + piece_at<DC>(best_n, hf * kFrags + j));
            float c0 = 0.0f, c1 = 0.0f, c2 = 0.0f, c3 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                c0 = fmaf(R[j][0], (float)dv[j][0], c0); c1 = fmaf(R[j][1], (float)dv[j][1], c1);
                c2 = fmaf(R[j][2], (float)dv[j][2], c2); c3 = fmaf(R[j][3], (float)dv[j][3], c3);
                c0 = fmaf(R[j][4], (float)dv[j][4], c0); c1 = fmaf(R[j][5], (float)dv[j][5], c1);
                c2 = fmaf(R[j][6], (float)dv[j][6], c2); c3 = fmaf(R[j][7], (float)dv[j][7], c3);
            }
            float best_c = (c0 + c1) + (c2 + c3);
            best_c += xchg32f(best_c, hf);
            if (!(rn2 > 0.0f)) best_c = 0.0f;
            // closed loop: what Eq.4 subtracts is the coefficient as it will be stored (rounded in the input's scale)
            if (coef_rounds_in_loop(coef_mode)) best_c = ldexpf(__half2float(__float2half_rn(ldexpf(best_c, -sexp))), sexp);
            float r2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    R[j][e] = fmaf(-best_c, (float)dv[j][e], R[j][e]);
                    r2 = fmaf(R[j][e], R[j][e], r2);
                }
            }
            r2 += xchg32f(r2, hf);
            const int sexp_used = sexp;
            // A residual that has shrunk a lot (a vector that is nearly a multiple of an atom) is scaled up again
            // before the split, or lo would sink into the fp16 subnormals; one that has grown (atoms of norm above
            // sqrt(2) make Eq.4 expand it) is scaled down before hi could leave the fp16 range.
            if ((r2 < 65536.0f && r2 > 0.0f) || (r2 >= 1073741824.0f && r2 < INFINITY)) {
                int e2 = 0;
                (void)frexpf(r2, &e2);             // |R| in [2^((e2-1)/2), 2^(e2/2))
                const int k = 14 - (e2 + 1) / 2;   // brings |R| into [2^12.5, 2^14.5)
                const float sc = ldexpf(1.0f, k);
#pragma unroll
                for (int j = 0; j < kFrags; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) R[j][e] *= sc;
                r2 *= sc * sc;
                sexp += k;
            }
            float lo2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const _Float16 hh = (_Float16)R[j][e];
                    const float l = R[j][e] - (float)hh;
                    hi[j][e] = hh;
                    lo2 = fmaf(l, l, lo2);
                }
            }
            lo2 += xchg32f(lo2, hf);
            rn2 = r2;
            delta = screen_delta(dmax, lo2, r2);
            if (valid) {
                const int64_t o = (int64_t)h * code_stride_h + (tok * sn + ch) * s + g;
                if (hf == 0) {
                    if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n;
                    else reinterpret_cast<int32_t *>(idx_out)[o] = best_n;
                } else {
                    const float c_out = ldexpf(best_c, -sexp_used);
                    if (coef_is_f16(coef_mode)) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(c_out);
                    else reinterpret_cast<float *>(coef_out)[o] = c_out;
                }
            }
        }
        if (res_norm2 && valid && hf == 0) res_norm2[((int64_t)h * T + tok) * sn + ch] = ldexpf(rn2, -2 * sexp);
    }
}

}  // namespace

bool encode_resident_supported(const EncodeArgs &a)
{
    return a.f16 && (a.d == 128 || a.d == 64) && a.N >= 32 && a.N % 32 == 0 &&
           (int64_t)a.N * a.d * 2 <= kMaxDictBytes;
}

template <int DC, int OCC>
static hipError_t launch_resident_t(const EncodeArgs &a)
{
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;  // vectors per dictionary
    const int64_t tiles = (M + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.dict_count * a.sn;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    const int lds_bytes = a.N * DC * 2 + kWaves * kScratchPerWave + 64;
    const int ntiles = a.N / 32;
    int bits = 0;
    while ((1 << bits) < ntiles) ++bits;
    const uint32_t code_mask = (1u << bits) - 1u;
    // per device, once: the dictionary needs more LDS than the default limit
    static std::atomic<bool> attr_set[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(encode_resident_kernel<DC, OCC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDictBytes + kWaves * kScratchPerWave + 64);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((encode_resident_kernel<DC, OCC>), dim3((unsigned)groups), dim3(kThreads), lds_bytes, a.stream,
                       (const __half *)a.X, (const __half *)a.D, a.idx, a.coef, a.T, M, a.N, a.s, a.sn, a.x_stride_h,
                       a.x_stride_t, a.dict_count, a.code_stride_h, (int32_t)tiles, (int32_t)a.idx16,
                       (a.coef16 ? kCoefF16 : 0) | (a.closed_loop ? kCoefClosed : 0), code_mask, a.res_norm2);
    return hipGetLastError();
}

hipError_t launch_encode_resident(const EncodeArgs &a)
{
    if (a.d == 128) return launch_resident_t<128, 2>(a);
    // two workgroups per CU when two dictionaries (and the waves' scratch) fit the 160 KB of LDS
    const size_t lds = (size_t)a.N * 64 * 2 + kWaves * kScratchPerWave + 64;
    return 2 * lds <= 160 * 1024 ? launch_resident_t<64, 4>(a) : launch_resident_t<64, 3>(a);
}

}  // namespace csr
