// Matching Pursuit encoder for FEW vectors per dictionary (gfx950): the tokens generated in one decoding step,
// which Section "KV Decomposition and Sparse Storage" encodes like the prompt's (Eq.2-4, s iterations).
//
// With a handful of vectors per dictionary the work is a matrix-vector product per iteration: every iteration
// must read the whole dictionary (1 MB at N = 4096) for a few dot products per atom, and one workgroup per
// dictionary - the shape of the prefill encoder - leaves most of the chip idle while a single CU streams it
// (0.7 ms for 64 dictionaries, whatever the vector count).  Here the ATOMS of every dictionary are split over
// k workgroups, so that all CUs stream dictionary slices at once, and the iteration's arg-max over the slices
// is taken by the next launch: one launch per iteration plus one that stores the last pair, s + 1 in all, no
// spinning between workgroups.
//
//   launch g, workgroup (slice sl, dictionary): for each block of 32 vectors of that dictionary
//     g > 0   the slices' candidates of iteration g - 1 give its pick (largest |c|, lowest atom on ties),
//             R_g = R_{g-1} - c d (Eq.4, fp32, residual kept in scratch); every slice's workgroup does this
//             with identical arithmetic, slice 0 stores R_g and the pair (i, c) of iteration g - 1
//     g = 0   R_0 = x, scaled by the power of two that brings its largest element into [2^11, 2^12)
//     g < s   R_g is split into hi + lo (two fp16, 22 significant bits); c[n] = hi . d_n + lo . d_n on the
//             matrix cores (v_mfma_f32_32x32x16_f16, atoms as rows straight from global memory, vectors as
//             columns in registers; products of fp16 pairs are exact, accumulation is fp32), so the decision
//             has the precision of the prefill encoder's exact resolve step; the slice's best (|c|, n, c) per
//             vector goes to scratch.
// Scratch per vector: two residuals (ping-pong: a launch reads one and writes the other), two scale exponents,
// 2 k candidates.
#include <cmath>

#include "csr_internal.h"
#include "encode_common.h"

namespace csr {
namespace {

using namespace enc;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxVectors = 128;  // per dictionary; beyond that the prefill encoder's shape is the better one
constexpr int kMaxSlices = 16;
constexpr int kTargetGroups = 512;  // workgroups per launch aimed at (two per CU)




struct SplitParams {
    const __half *X;
    const __half *Dict;
    void *idx_out;
    void *coef_out;
    float *Rbuf;       // [2][V][DC]
    int32_t *sexp;     // [2][V]
    float4 *cand;      // [2][V][k]
    int64_t V;         // vectors in all
    int64_t T;
    int64_t x_stride_h, x_stride_t, code_stride_h;
    int32_t N, s, sn, dict_count, M, k, g, idx16, coef16;   // coef16: kCoefF16 | kCoefClosed
    float *res_norm2;  // optional [H][T][sn]
};

// Lane (col, hf): column col of the MFMA's B operand = vector m0 + col of the block; it holds dimensions
// hf DC/2 .. hf DC/2 + DC/2 - 1 (the contraction index is permuted the same way in both operands), as
// kFrags pieces of 8.
template <int DC>
__global__ __launch_bounds__(kThreads, 2) void encode_split_kernel(const SplitParams p)
{
    constexpr int kFrags = DC / 16;
    __shared__ float4 red[kWaves][32];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, hf = lane >> 5;
    const int sl = blockIdx.x, dct = blockIdx.y;  // dct = dictionary * sn + chunk
    const int dict = dct / p.sn, ch = dct - dict * p.sn;
    const __half *Dh = p.Dict + (int64_t)dct * p.N * DC;
    const int tiles = p.N >> 5;
    const int per_slice = (tiles + p.k - 1) / p.k;
    const int t_begin = sl * per_slice, t_end = min(tiles, t_begin + per_slice);
    const int g = p.g;

    // This wave's first tiles of the slice are requested before anything else and stay in registers for all
    // blocks of vectors: their fetch overlaps the dependent chain below (candidates -> atom row -> residual),
    // which does not need them.  (The last launch sweeps nothing.)
    constexpr int kPrefetch = 256 / DC;  // tiles: 2 of 128 dimensions, 4 of 64 (64 registers either way)
    auto load_tile = [&](int tile, uint4 (&a)[kFrags]) {
        const __half *row = Dh + ((int64_t)tile * 32 + col) * DC + hf * (DC / 2);
#pragma unroll
        for (int j = 0; j < kFrags; ++j) a[j] = *reinterpret_cast<const uint4 *>(row + 8 * j);
    };
    uint4 pre[kPrefetch][kFrags];
    if (g < p.s) {
#pragma unroll
        for (int q = 0; q < kPrefetch; ++q)
            if (t_begin + wave + q * kWaves < t_end) load_tile(t_begin + wave + q * kWaves, pre[q]);
    }

    for (int m0 = 0; m0 < p.M; m0 += 32) {
        // vector m of this dictionary: block h = (m / T) dict_count + dict, its token m % T
        const bool valid = m0 + col < p.M;
        const int m = valid ? m0 + col : p.M - 1;
        const int rep = (int)(m / p.T);
        const int64_t t = m - rep * p.T;
        const int64_t h = (int64_t)rep * p.dict_count + dict;
        const int64_t vid = (h * p.T + t) * p.sn + ch;

        float R[kFrags][8];
        int sexp_cur = 0;
        if (g == 0) {
            const __half *xr = p.X + h * p.x_stride_h + t * p.x_stride_t + ch * DC + hf * (DC / 2);
            float amax = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                const uint4 raw = *reinterpret_cast<const uint4 *>(xr + 8 * j);
                unpack8(raw, R[j]);
#pragma unroll
                for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(R[j][e]));
            }
            amax = fmaxf(amax, xchg32f(amax, hf));
            if (amax > 0.0f && amax < INFINITY) {
                int ex;
                (void)frexpf(amax, &ex);  // amax = f 2^ex, f in [0.5, 1)
                sexp_cur = 12 - ex;       // brings amax into [2^11, 2^12): hi and lo stay normal fp16 numbers
            }
#pragma unroll
            for (int j = 0; j < kFrags; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) R[j][e] = ldexpf(R[j][e], sexp_cur);
        } else {
            const int prev = (g - 1) & 1;
            // the pick of iteration g - 1: slices ascend, so a strict comparison keeps the lowest atom on ties
            const float4 *cd = p.cand + ((int64_t)prev * p.V + vid) * p.k;
            float ba = -1.0f, bc = 0.0f;
            int bi = 0;
            for (int j = 0; j < p.k; ++j) {
                const float4 c4 = cd[j];
                if (c4.x > ba) { ba = c4.x; bi = __float_as_int(c4.y); bc = c4.z; }
            }
            const float *Rp = p.Rbuf + ((int64_t)prev * p.V + vid) * DC + hf * (DC / 2);
            const __half *row = Dh + (int64_t)bi * DC + hf * (DC / 2);
            const int sexp_prev = p.sexp[(int64_t)prev * p.V + vid];
            // closed loop: what Eq.4 subtracts is the coefficient as it will be stored (rounded in the input's scale)
            if (coef_rounds_in_loop(p.coef16)) bc = ldexpf(__half2float(__float2half_rn(ldexpf(bc, -sexp_prev))), sexp_prev);
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                const float4 r0 = *reinterpret_cast<const float4 *>(Rp + 8 * j);
                const float4 r1 = *reinterpret_cast<const float4 *>(Rp + 8 * j + 4);
                const uint4 raw = *reinterpret_cast<const uint4 *>(row + 8 * j);
                float d[8];
                unpack8(raw, d);
                const float r[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) R[j][e] = fmaf(-bc, d[e], r[e]);  // Eq.4 with the unrounded coefficient
            }
            if (sl == 0 && valid) {
                const int64_t o = h * p.code_stride_h + (t * p.sn + ch) * p.s + (g - 1);
                if (hf == 0) {
                    if (p.idx16) reinterpret_cast<uint16_t *>(p.idx_out)[o] = (uint16_t)bi;
                    else reinterpret_cast<int32_t *>(p.idx_out)[o] = bi;
                } else {
                    const float c_out = ldexpf(bc, -sexp_prev);
                    if (coef_is_f16(p.coef16)) reinterpret_cast<__half *>(p.coef_out)[o] = __float2half_rn(c_out);
                    else reinterpret_cast<float *>(p.coef_out)[o] = c_out;
                }
            }
            sexp_cur = sexp_prev;
        }
        float r2 = 0.0f;
#pragma unroll
        for (int j = 0; j < kFrags; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) r2 = fmaf(R[j][e], R[j][e], r2);
        r2 += xchg32f(r2, hf);
        if (g == p.s) {  // the last launch only stores the last pair and what is left (uniform over the grid)
            if (p.res_norm2 && sl == 0 && valid && hf == 0) p.res_norm2[vid] = ldexpf(r2, -2 * sexp_cur);
            continue;
        }
        // A residual that has shrunk a lot (a vector that is nearly a multiple of an atom) is scaled up again
        // before the split, or lo would sink into the fp16 subnormals; one that has grown (atoms of norm above
        // sqrt(2) make Eq.4 expand it) is scaled down before hi could leave the fp16 range.
        if (g > 0 && ((r2 < 65536.0f && r2 > 0.0f) || (r2 >= 1073741824.0f && r2 < INFINITY))) {
            int e2 = 0;
            (void)frexpf(r2, &e2);                // |R| in [2^((e2-1)/2), 2^(e2/2))
            const int k2 = 14 - (e2 + 1) / 2;     // brings |R| into [2^12.5, 2^14.5)
            const float sc = ldexpf(1.0f, k2);
#pragma unroll
            for (int j = 0; j < kFrags; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) R[j][e] *= sc;
            sexp_cur += k2;
        }
        if (sl == 0 && valid) {
            float *Rw = p.Rbuf + ((int64_t)(g & 1) * p.V + vid) * DC + hf * (DC / 2);
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                *reinterpret_cast<float4 *>(Rw + 8 * j) = make_float4(R[j][0], R[j][1], R[j][2], R[j][3]);
                *reinterpret_cast<float4 *>(Rw + 8 * j + 4) = make_float4(R[j][4], R[j][5], R[j][6], R[j][7]);
            }
            if (hf == 0) p.sexp[(int64_t)(g & 1) * p.V + vid] = sexp_cur;
        }
        half8 hi[kFrags], lo[kFrags];
#pragma unroll
        for (int j = 0; j < kFrags; ++j) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const _Float16 hh = (_Float16)R[j][e];
                hi[j][e] = hh;
                lo[j][e] = (_Float16)(R[j][e] - (float)hh);
            }
        }

        // ---- this wave's tiles of the slice: c[n] = hi . d_n + lo . d_n ---------------------------
        float ba = -1.0f, bc = 0.0f;
        int bi = 0;
        auto sweep_tile = [&](int tile, const uint4 (&a)[kFrags]) {
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int j = 0; j < kFrags; ++j) {
                const half8 av = *reinterpret_cast<const half8 *>(&a[j]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, hi[j], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, lo[j], acc, 0, 0, 0);
            }
            // accumulator r of lane half hf is atom 8 (r / 4) + (r % 4) + 4 hf of the tile: ascending in r
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float ab = fabsf(acc[r]);
                if (ab > ba) { ba = ab; bi = tile * 32 + 8 * (r >> 2) + (r & 3) + 4 * hf; bc = acc[r]; }
            }
        };
#pragma unroll
        for (int q = 0; q < kPrefetch; ++q)
            if (t_begin + wave + q * kWaves < t_end) sweep_tile(t_begin + wave + q * kWaves, pre[q]);
        // tiles beyond the prefetched ones
        for (int tile = t_begin + wave + kPrefetch * kWaves; tile < t_end; tile += kWaves) {
            uint4 a_cur[kFrags];
            load_tile(tile, a_cur);
            sweep_tile(tile, a_cur);
        }
        // the two lanes of a vector, then the waves
        take_better(ba, bi, bc, xchg32f(ba, hf), (int)xchg32((uint32_t)bi, hf), xchg32f(bc, hf));
        if (hf == 0) red[wave][col] = make_float4(ba, __int_as_float(bi), bc, 0.0f);
        __syncthreads();
        if (wave == 0 && hf == 0) {
#pragma unroll
            for (int w = 1; w < kWaves; ++w) {
                const float4 o = red[w][col];
                take_better(ba, bi, bc, o.x, __float_as_int(o.y), o.z);
            }
            if (valid) p.cand[((int64_t)(g & 1) * p.V + vid) * p.k + sl] = make_float4(ba, __int_as_float(bi), bc, 0.0f);
        }
        __syncthreads();  // `red` is reused by the next block of vectors
    }
}

size_t r256(size_t v) { return (v + 255) & ~size_t(255); }

struct SplitPlan {
    int32_t k, M;
    int64_t V;
    size_t off_R, off_sexp, off_cand, total;
};

SplitPlan plan_split(const EncodeArgs &a)
{
    SplitPlan pl{};
    const int n_dicts = a.dict_count * a.sn;
    pl.M = (int32_t)((int64_t)(a.H / a.dict_count) * a.T);
    pl.V = (int64_t)a.H * a.T * a.sn;
    const int tiles = a.N / 32;
    int k = kTargetGroups / (n_dicts > 0 ? n_dicts : 1);
    if (k > tiles / kWaves) k = tiles / kWaves;  // at least one tile per wave
    if (k > kMaxSlices) k = kMaxSlices;
    if (k < 1) k = 1;
    pl.k = k;
    size_t off = 0;
    pl.off_R = off;    off += r256((size_t)2 * pl.V * a.d * sizeof(float));
    pl.off_sexp = off; off += r256((size_t)2 * pl.V * sizeof(int32_t));
    pl.off_cand = off; off += r256((size_t)2 * pl.V * k * sizeof(float4));
    pl.total = off;
    return pl;
}

}  // namespace

bool encode_split_supported(const EncodeArgs &a)
{
    if (!(a.f16 && (a.d == 128 || a.d == 64) && a.N >= 32 && a.N % 32 == 0 && a.N <= (1 << 24))) return false;
    if (a.dict_count < 1 || a.H % a.dict_count != 0) return false;
    if ((int64_t)a.dict_count * a.sn > 65535) return false;  // grid.y
    return (int64_t)(a.H / a.dict_count) * a.T <= kMaxVectors;
}

size_t encode_split_workspace_bytes(const EncodeArgs &a) { return plan_split(a).total; }

hipError_t launch_encode_split(const EncodeArgs &a)
{
    const SplitPlan pl = plan_split(a);
    char *ws = static_cast<char *>(a.workspace);
    SplitParams p{};
    p.X = (const __half *)a.X; p.Dict = (const __half *)a.D; p.idx_out = a.idx; p.coef_out = a.coef;
    p.Rbuf = reinterpret_cast<float *>(ws + pl.off_R);
    p.sexp = reinterpret_cast<int32_t *>(ws + pl.off_sexp);
    p.cand = reinterpret_cast<float4 *>(ws + pl.off_cand);
    p.V = pl.V; p.T = a.T; p.x_stride_h = a.x_stride_h; p.x_stride_t = a.x_stride_t; p.code_stride_h = a.code_stride_h;
    p.N = a.N; p.s = a.s; p.sn = a.sn; p.dict_count = a.dict_count; p.M = pl.M; p.k = pl.k;
    p.idx16 = a.idx16; p.coef16 = (a.coef16 ? kCoefF16 : 0) | (a.closed_loop ? kCoefClosed : 0); p.res_norm2 = a.res_norm2;
    const dim3 grid((unsigned)pl.k, (unsigned)(a.dict_count * a.sn));
    for (int g = 0; g <= a.s; ++g) {
        p.g = g;
        if (a.d == 64) hipLaunchKernelGGL(encode_split_kernel<64>, grid, dim3(kThreads), 0, a.stream, p);
        else hipLaunchKernelGGL(encode_split_kernel<128>, grid, dim3(kThreads), 0, a.stream, p);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace csr
