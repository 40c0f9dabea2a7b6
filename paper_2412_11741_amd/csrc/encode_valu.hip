// fp32 vector-ALU Matching Pursuit encoder (Eq.2-4 of the paper's Section "Sparse
// representation").  The general, any-shape kernel: every correlation is an fp32 dot product,
// the residual lives in registers, no matrix cores.
//
// Mapping.  A workgroup owns 64 consecutive vectors of one dictionary; lane l of every wave owns
// vector l and keeps its whole residual R (d fp32 registers).  The W waves of the workgroup split
// the atom range [0, N) into W contiguous slices.  Because all lanes of a wave look at the SAME
// atom at the same time, the atom row is wave-uniform: it is fetched through the scalar cache and
// fed to v_fma as a scalar operand - no LDS, no vector-memory traffic in the hot loop.
// Per iteration each wave leaves (|c|, index, c) of its slice's best atom per vector in LDS, every
// wave then takes the same cross-slice decision (lowest index wins ties because slices ascend and
// comparisons are strict), and every wave applies Eq.4 to its own copy of R with identical
// arithmetic, so the copies never diverge.
#include "csr_internal.h"

namespace csr {
namespace {

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }

template <typename T> struct Vec16;  // a 16-byte chunk of T
template <> struct Vec16<float> { static constexpr int n = 4; float v[4]; };
template <> struct Vec16<__half> { static constexpr int n = 8; __half v[8]; };

template <int D_, typename TE, int W>
__global__ __launch_bounds__(64 * W) void encode_valu_kernel(
    const TE *__restrict__ X, const TE *__restrict__ Dict, void *__restrict__ idx_out,
    void *__restrict__ coef_out, int64_t T, int64_t M, int32_t N, int32_t s, int64_t x_stride_h,
    int64_t x_stride_t, int32_t tiles_per_h, int32_t sn, int32_t dict_count, int64_t code_stride_h, int32_t idx16,
    int32_t coef_mode, float *__restrict__ res_norm2)
{
    __shared__ float s_abs[2][W][64];
    __shared__ float s_c[2][W][64];
    __shared__ int s_i[2][W][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Work is dealt per dictionary: dct = dictionary * sn + chunk owns the vectors (chunks of D_ dimensions) of all
    // blocks that use it (block h uses dictionary h % dict_count), numbered m = (h / dict_count) * T + t, 64 a tile
    const int dct = blockIdx.x / tiles_per_h;
    const int tile = blockIdx.x - dct * tiles_per_h;
    const int dict = dct / sn, ch = dct - dict * sn;
    const int64_t m = (int64_t)tile * 64 + lane;
    const bool valid = m < M;
    const int64_t mc = valid ? m : M - 1;  // tail lanes recompute the last vector, never store
    const int rep = (int)(mc / T);
    const int64_t t = mc - rep * T;
    const int h = rep * dict_count + dict;

    constexpr int VN = Vec16<TE>::n;
    float R[D_];
    {
        const TE *xr = X + (int64_t)h * x_stride_h + t * x_stride_t + ch * D_;
#pragma unroll
        for (int k = 0; k < D_; k += VN) {
            Vec16<TE> v = *reinterpret_cast<const Vec16<TE> *>(xr + k);
#pragma unroll
            for (int j = 0; j < VN; ++j) R[k + j] = to_f32(v.v[j]);
        }
    }

    const int slice = (N + W - 1) / W;
    const int n0 = wave * slice;
    const int n1 = min(N, n0 + slice);
    const TE *Dh = Dict + (int64_t)dct * N * D_;

    for (int g = 0; g < s; ++g) {
        float best = -1.0f, bc = 0.0f;
        int bi = n0 < N ? n0 : 0;
        for (int n = n0; n < n1; ++n) {
            const TE *__restrict__ row = Dh + (int64_t)n * D_;  // wave-uniform address
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int k = 0; k < D_; k += 4) {
                a0 = fmaf(R[k + 0], to_f32(row[k + 0]), a0);
                a1 = fmaf(R[k + 1], to_f32(row[k + 1]), a1);
                a2 = fmaf(R[k + 2], to_f32(row[k + 2]), a2);
                a3 = fmaf(R[k + 3], to_f32(row[k + 3]), a3);
            }
            const float c = (a0 + a1) + (a2 + a3);
            const float a = fabsf(c);
            if (a > best) { best = a; bi = n; bc = c; }
        }
        const int buf = g & 1;
        s_abs[buf][wave][lane] = best;
        s_c[buf][wave][lane] = bc;
        s_i[buf][wave][lane] = bi;
        __syncthreads();
        float wb = -1.0f, wc = 0.0f;
        int wi = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float a = s_abs[buf][w][lane];
            if (a > wb) { wb = a; wc = s_c[buf][w][lane]; wi = s_i[buf][w][lane]; }
        }
        // Eq.4 with the unrounded coefficient (or, closed loop, with the coefficient as it is stored); per-lane
        // gather of the chosen atom.
        if (coef_rounds_in_loop(coef_mode)) wc = __half2float(__float2half_rn(wc));
        {
            const TE *row = Dh + (int64_t)wi * D_;
#pragma unroll
            for (int k = 0; k < D_; k += VN) {
                Vec16<TE> v = *reinterpret_cast<const Vec16<TE> *>(row + k);
#pragma unroll
                for (int j = 0; j < VN; ++j) R[k + j] = fmaf(-wc, to_f32(v.v[j]), R[k + j]);
            }
        }
        if (wave == 0 && valid) {
            const int64_t o = (int64_t)h * code_stride_h + (t * sn + ch) * s + g;
            if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)wi;
            else reinterpret_cast<int32_t *>(idx_out)[o] = wi;
            if (coef_is_f16(coef_mode)) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(wc);
            else reinterpret_cast<float *>(coef_out)[o] = wc;
        }
        // The LDS buffers alternate, so one barrier per iteration is enough: a wave can only
        // overwrite buffer `buf` two iterations later, after passing the next barrier.
    }
    if (res_norm2 && wave == 0 && valid) {
        float r2 = 0.0f;
#pragma unroll
        for (int k = 0; k < D_; ++k) r2 = fmaf(R[k], R[k], r2);
        res_norm2[((int64_t)h * T + t) * sn + ch] = r2;
    }
}

template <int D_, typename TE>
hipError_t launch_valu_t(const EncodeArgs &a)
{
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;  // vectors per dictionary
    const int64_t tiles = (M + 63) / 64;
    // More waves per workgroup when there are few vectors, so that a small job still spreads
    // over the chip; fewer (less redundant residual work) when there are many.
    const int64_t groups = tiles * a.dict_count * a.sn;
    const dim3 grid((unsigned)groups);
#define CSR_LAUNCH_VALU(W)                                                                      \
    hipLaunchKernelGGL((encode_valu_kernel<D_, TE, W>), grid, dim3(64 * W), 0, a.stream,         \
                       (const TE *)a.X, (const TE *)a.D, a.idx, a.coef, a.T, M, a.N, a.s,       \
                       a.x_stride_h, a.x_stride_t, (int32_t)tiles, a.sn, a.dict_count, a.code_stride_h, \
                       (int32_t)a.idx16, (a.coef16 ? kCoefF16 : 0) | (a.closed_loop ? kCoefClosed : 0), a.res_norm2)
    // (8 waves = 2 per SIMD leaves each lane the 128+ registers its residual needs.)
    if (groups >= 1024) CSR_LAUNCH_VALU(4);
    else CSR_LAUNCH_VALU(8);
#undef CSR_LAUNCH_VALU
    return hipGetLastError();
}

}  // namespace

hipError_t launch_encode_valu(const EncodeArgs &a)
{
    if (a.f16) {
        switch (a.d) {
            case 32: return launch_valu_t<32, __half>(a);
            case 64: return launch_valu_t<64, __half>(a);
            case 128: return launch_valu_t<128, __half>(a);
        }
    } else {
        switch (a.d) {
            case 32: return launch_valu_t<32, float>(a);
            case 64: return launch_valu_t<64, float>(a);
            case 128: return launch_valu_t<128, float>(a);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace csr
