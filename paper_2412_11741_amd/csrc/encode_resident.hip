// Matching Pursuit encoder for SMALL dictionaries (gfx950): the whole dictionary of a head - up to 128 KB of fp16
// atoms, e.g. the 256 or 512 atoms per head of the paper's own experiments - stays in LDS for the life of a
// workgroup, and every wave works through its vectors on its own, without a single barrier after the load.
//
// Eq.2-4 of Section "Sparse representation", s iterations per vector.  With so few atoms the correlation sweep is
// cheap and what bounds the large-dictionary encoder's shape here is its chain of dependent steps per iteration
// (screen, decide within a bound, resolve the undecided against global memory, gather the atom, update).  So this
// kernel pays twice the matrix-core work for a sweep that needs no bound and no resolve:
//
//   sweep    c[n] = hi . d_n + lo . d_n for all atoms, two v_mfma_f32_32x32x16_f16 per operand fragment (residual
//            R = hi + lo as two fp16, 22 significant bits; products of fp16 pairs are exact, accumulation fp32):
//            the correlations have the precision of an fp32 dot product.  Atoms are the MFMA's rows (fragments
//            read from LDS), 32 vectors its columns; a lane sees 16 atoms of one vector per tile and keeps the
//            largest |c| it has seen and - under a branch taken only when that changes - the tile number and the
//            tile's 16 values.
//   select   the largest of the kept 16 (first on ties), merged with the vector's other lane: lowest atom on ties.
//   update   the atom row comes from LDS; R - c d in fp32 (Eq.4, unrounded c), new hi / lo split.
//
// Every vector is first multiplied by a power of two that brings its largest element into [2^11, 2^12), as in the
// large-dictionary encoder (Matching Pursuit commutes with it; lo stays clear of the fp16 subnormals).
#include <atomic>

#include "csr_internal.h"

namespace csr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWaves = 8;                    // two per SIMD; one workgroup per CU (the dictionary fills the LDS)
constexpr int kThreads = 64 * kWaves;
constexpr int kBlocksPerWave = 2;            // 32-vector blocks a wave works through, one after the other
constexpr int kTokPerWG = kWaves * kBlocksPerWave * 32;  // 512
constexpr int kMaxDictBytes = 128 * 1024;

__device__ __forceinline__ uint32_t xchg32(uint32_t v, int hf)
{
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return hf ? r[0] : r[1];
}
__device__ __forceinline__ float xchg32f(float v, int hf) { return __uint_as_float(xchg32(__float_as_uint(v), hf)); }

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

// XOR term of a row's 16-byte piece positions, so that 16 consecutive rows read at one logical piece cover all
// banks: a 256-byte row spans the 64 banks (16 different terms), two 128-byte rows span them (8, one per pair).
template <int DC> __device__ __forceinline__ int swz(int row) { return DC == 128 ? (row & 15) : ((row >> 1) & 7); }

template <int DC>
__global__ __launch_bounds__(kThreads) void encode_resident_kernel(
    const __half *__restrict__ X, const __half *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, int64_t T, int64_t M, int32_t N, int32_t s, int32_t sn, int64_t x_stride_h, int64_t x_stride_t,
    int32_t dict_count, int64_t code_stride_h, int32_t tiles_per_h, int32_t idx16, int32_t coef16,
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

    // ---- the dictionary, once: piece `pos` of row `row` goes to position pos ^ swz(row) ---------------
    {
        const int total = N * kPieces;
        const uint4 *src = reinterpret_cast<const uint4 *>(Dh);
        for (int e = tid; e < total; e += kThreads) {
            const int row = e / kPieces, pos = e - row * kPieces;
            *reinterpret_cast<uint4 *>(lds + row * kRowBytes + ((pos ^ swz<DC>(row)) << 4)) = src[e];
        }
    }
    __syncthreads();  // the only barrier: from here on the waves do not meet again

    // LDS byte offset, inside a 32-row tile, of this lane's operand fragment j (row = col, piece kFrags hf + j)
    uint32_t frag_off[kFrags];
#pragma unroll
    for (int j = 0; j < kFrags; ++j) frag_off[j] = (uint32_t)(col * kRowBytes + (((hf * kFrags + j) ^ swz<DC>(col)) << 4));

    for (int bi = 0; bi < kBlocksPerWave; ++bi) {
        const int64_t m = (int64_t)tile_wg * kTokPerWG + (wave * kBlocksPerWave + bi) * 32 + col;
        if ((int64_t)tile_wg * kTokPerWG + (wave * kBlocksPerWave + bi) * 32 >= M) break;  // wave-uniform
        const bool valid = m < M;
        const int64_t mc = valid ? m : M - 1;  // tail lanes recompute the last vector, never store
        const int rep = (int)(mc / T);
        const int64_t tok = mc - rep * T;     // position in its block
        const int h = rep * dict_count + dict;

        // ---- load the vector, scale by a power of two, split into hi + lo -------------------------
        half8 hi[kFrags], lo[kFrags];
        int sexp = 0;
        float rn2;
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
            float r2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = ldexpf(xv[j][e], sexp);
                    const _Float16 hh = (_Float16)v;
                    hi[j][e] = hh;
                    lo[j][e] = (_Float16)(v - (float)hh);
                    r2 = fmaf(v, v, r2);
                }
            }
            rn2 = r2 + xchg32f(r2, hf);
        }

        for (int g = 0; g < s; ++g) {
            // ---- sweep: exact correlations, the lane's best group kept -------------------------------
            float best = -1.0f;
            int best_tile = 0;
            float keep[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) keep[r] = 0.0f;
            for (int t = 0; t < ntiles; ++t) {
                half8 a[kFrags];
#pragma unroll
                for (int j = 0; j < kFrags; ++j)
                    a[j] = *reinterpret_cast<const half8 *>(lds + t * 32 * kRowBytes + frag_off[j]);
                floatx16 acc_h, acc_l;  // two chains, so that consecutive MFMAs do not wait for each other
#pragma unroll
                for (int r = 0; r < 16; ++r) { acc_h[r] = 0.0f; acc_l[r] = 0.0f; }
#pragma unroll
                for (int j = 0; j < kFrags; ++j) {
                    acc_h = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], hi[j], acc_h, 0, 0, 0);
                    acc_l = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], lo[j], acc_l, 0, 0, 0);
                }
                float c[16];
                float m = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) c[r] = acc_h[r] + acc_l[r];
#pragma unroll
                for (int r = 0; r < 16; r += 2) m = fmaxf(fmaxf(m, fabsf(c[r])), fabsf(c[r + 1]));
                if (__builtin_expect(m > best, 0)) {  // strict: the earliest tile wins ties
                    best = m;
                    best_tile = t;
#pragma unroll
                    for (int r = 0; r < 16; ++r) keep[r] = c[r];
                }
            }

            // ---- select: this lane's candidate, then the vector's other lane ---------------------------
            // accumulator r of lane half hf is atom 8 (r / 4) + (r % 4) + 4 hf of the tile: ascending in r
            float ba = -1.0f, bc = 0.0f;
            int bk = 0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float ab = fabsf(keep[r]);
                if (ab > ba) { ba = ab; bk = r; bc = keep[r]; }
            }
            int bn = best_tile * 32 + 8 * (bk >> 2) + (bk & 3) + 4 * hf;
            {
                const float oa = xchg32f(ba, hf), oc = xchg32f(bc, hf);
                const int on = (int)xchg32((uint32_t)bn, hf);
                if (oa > ba || (oa == ba && on < bn)) { ba = oa; bn = on; bc = oc; }
            }
            if (!(rn2 > 0.0f)) { bn = 0; bc = 0.0f; }  // zero residual: (0, 0)

            // ---- update: Eq.4 on the full-precision residual, new split ---------------------------------
            float v[kFrags][8];
            float r2 = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                const uint4 raw = *reinterpret_cast<const uint4 *>(lds + bn * kRowBytes + (((hf * kFrags + j) ^ swz<DC>(bn)) << 4));
                float f[8];
                unpack8(raw, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float r = (float)hi[j][e] + (float)lo[j][e];  // exact: 22 significant bits
                    v[j][e] = fmaf(-bc, f[e], r);
                    r2 = fmaf(v[j][e], v[j][e], r2);
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
                    for (int e = 0; e < 8; ++e) v[j][e] *= sc;
                r2 *= sc * sc;
                sexp += k;
            }
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const _Float16 hh = (_Float16)v[j][e];
                    hi[j][e] = hh;
                    lo[j][e] = (_Float16)(v[j][e] - (float)hh);
                }
            }
            rn2 = r2;
            if (valid) {
                const int64_t o = (int64_t)h * code_stride_h + (tok * sn + ch) * s + g;
                if (hf == 0) {
                    if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)bn;
                    else reinterpret_cast<int32_t *>(idx_out)[o] = bn;
                } else {
                    const float c_out = ldexpf(bc, -sexp_used);
                    if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(c_out);
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

template <int DC>
static hipError_t launch_resident_t(const EncodeArgs &a)
{
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;  // vectors per dictionary
    const int64_t tiles = (M + kTokPerWG - 1) / kTokPerWG;
    const int64_t groups = tiles * a.dict_count * a.sn;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    const int lds_bytes = a.N * DC * 2;
    // per device, once: the dictionary needs more LDS than the default limit
    static std::atomic<bool> attr_set[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(encode_resident_kernel<DC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDictBytes);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(encode_resident_kernel<DC>, dim3((unsigned)groups), dim3(kThreads), lds_bytes, a.stream,
                       (const __half *)a.X, (const __half *)a.D, a.idx, a.coef, a.T, M, a.N, a.s, a.sn, a.x_stride_h,
                       a.x_stride_t, a.dict_count, a.code_stride_h, (int32_t)tiles, (int32_t)a.idx16, (int32_t)a.coef16,
                       a.res_norm2);
    return hipGetLastError();
}

hipError_t launch_encode_resident(const EncodeArgs &a)
{
    return a.d == 64 ? launch_resident_t<64>(a) : launch_resident_t<128>(a);
}

}  // namespace csr
