// De-sparse restore, Eq.12 of the paper's Section "De-Sparse to restore": X~ = D r, i.e. every coded vector
// is rebuilt as the sum of its s coefficient-weighted atoms (per chunk with chunked codes).  This is the step the
// paper puts in front of ordinary attention; the code-domain decode kernel never needs it, but callers that must
// touch the dense vectors (a position embedding applied to rebuilt keys, inspection, a loss on X - X~) do.
//
// Bound: HBM writes (2 d bytes per vector in fp16 against 4 s bytes of code read); the atom rows come from L2.
// Lane (vector, chunk, 8-dimension piece): all lanes of a vector's chunk read the same s pairs (one broadcast
// load each) and gather 16 bytes of each of the s atom rows, so a chunk's rows are fetched as whole lines.
#include "csr_internal.h"

namespace csr {
namespace {

template <typename T> __device__ __forceinline__ void load8f(const T *p, float (&f)[8]);
template <> __device__ __forceinline__ void load8f<__half>(const __half *p, float (&f)[8])
{
    const uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = __half22float2(h2[j]);
        f[2 * j] = v.x;
        f[2 * j + 1] = v.y;
    }
}
template <> __device__ __forceinline__ void load8f<float>(const float *p, float (&f)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
__device__ __forceinline__ void store8f(__half *p, const float (&f)[8])
{
    uint4 raw;
    __half2 *h2 = reinterpret_cast<__half2 *>(&raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) h2[j] = __floats2half2_rn(f[2 * j], f[2 * j + 1]);
    *reinterpret_cast<uint4 *>(p) = raw;
}
__device__ __forceinline__ void store8f(float *p, const float (&f)[8])
{
    *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}
__device__ __forceinline__ int load_idx(const uint16_t *p) { return *p; }
__device__ __forceinline__ int load_idx(const int32_t *p) { return *p; }
__device__ __forceinline__ float load_coef(const __half *p) { return __half2float(*p); }
__device__ __forceinline__ float load_coef(const float *p) { return *p; }

// Workgroups are dealt to the 8 XCDs round-robin, and each XCD has an L2 of its own (4 MB).  Numbered plainly, the
// workgroups in flight span several dictionaries and every L2 would have to hold all of them; give each XCD a
// contiguous eighth of the elements instead, so that at any time it gathers from one or two dictionaries.
__device__ __forceinline__ int64_t xcd_contiguous_block()
{
    const unsigned b = blockIdx.x, per = gridDim.x >> 3;
    return b < per * 8u ? (int64_t)(b & 7u) * per + (b >> 3) : (int64_t)b;
}

struct Where {
    int64_t h, t, code;
    int ch, pc;
};
// element e = (vector h * T + t, piece): its block, token, chunk, piece inside the chunk, first pair of its code
__device__ __forceinline__ Where locate(int64_t e, int pieces, int ppc, int64_t T, int sn, int s, int64_t code_stride_h)
{
    Where w;
    const int piece = (int)(e % pieces);
    const int64_t v = e / pieces;
    w.h = v / T;
    w.t = v - w.h * T;
    w.ch = piece / ppc;
    w.pc = piece - w.ch * ppc;
    w.code = w.h * code_stride_h + (w.t * sn + w.ch) * s;
    return w;
}

// Any types, any s: one pair at a time.
template <typename TD, typename TI, typename TC, typename TO>
__global__ __launch_bounds__(256) void reconstruct_kernel(const TD *__restrict__ Dict, const TI *__restrict__ idx,
                                                          const TC *__restrict__ coef, TO *__restrict__ out, int64_t T,
                                                          int32_t d, int32_t N, int32_t s, int32_t sn, int32_t dict_count,
                                                          int64_t code_stride_h, int64_t out_stride_h,
                                                          int64_t out_stride_t, int64_t total)
{
    const int pieces = d >> 3;             // lanes per vector
    const int dc = d / sn, ppc = dc >> 3;  // dimensions / pieces per chunk
    const int64_t e = xcd_contiguous_block() * 256 + threadIdx.x;
    if (e >= total) return;
    const Where w = locate(e, pieces, ppc, T, sn, s, code_stride_h);
    const TD *Dh = Dict + ((int64_t)(w.h % dict_count) * sn + w.ch) * N * dc + w.pc * 8;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
    for (int j = 0; j < s; ++j) {
        const int n = load_idx(idx + w.code + j);
        const float c = load_coef(coef + w.code + j);
        float row[8];
        load8f<TD>(Dh + (int64_t)n * dc, row);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = fmaf(c, row[k], acc[k]);
    }
    store8f(out + w.h * out_stride_h + w.t * out_stride_t + (w.ch * ppc + w.pc) * 8, acc);
}

// The paper's storage (16-bit indices, fp16 coefficients) with s = 8 G pairs: a lane reads eight pairs with one
// 16-byte load per stream and has the eight atom-row pieces of a group in flight together; same sum order.
template <typename TD, typename TO, int G>
__global__ __launch_bounds__(256) void reconstruct_vec_kernel(const TD *__restrict__ Dict, const uint16_t *__restrict__ idx,
                                                              const __half *__restrict__ coef, TO *__restrict__ out,
                                                              int64_t T, int32_t d, int32_t N, int32_t sn,
                                                              int32_t dict_count, int64_t code_stride_h,
                                                              int64_t out_stride_h, int64_t out_stride_t, int64_t total)
{
    const int pieces = d >> 3;
    const int dc = d / sn, ppc = dc >> 3;
    const int64_t e = xcd_contiguous_block() * 256 + threadIdx.x;
    if (e >= total) return;
    const Where w = locate(e, pieces, ppc, T, sn, 8 * G, code_stride_h);
    uint4 qi[G], qc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        qi[g] = *reinterpret_cast<const uint4 *>(idx + w.code + 8 * g);
        qc[g] = *reinterpret_cast<const uint4 *>(coef + w.code + 8 * g);
    }
    const TD *Dh = Dict + ((int64_t)(w.h % dict_count) * sn + w.ch) * N * dc + w.pc * 8;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint32_t iw[4] = {qi[g].x, qi[g].y, qi[g].z, qi[g].w};
        const __half2 *h2 = reinterpret_cast<const __half2 *>(&qc[g]);
        float row[8][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int n = (j & 1) ? (int)(iw[j >> 1] >> 16) : (int)(iw[j >> 1] & 0xffffu);
            load8f<TD>(Dh + (int64_t)n * dc, row[j]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float2 cf = __half22float2(h2[j >> 1]);
            const float c = (j & 1) ? cf.y : cf.x;
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] = fmaf(c, row[j][k], acc[k]);
        }
    }
    store8f(out + w.h * out_stride_h + w.t * out_stride_t + (w.ch * ppc + w.pc) * 8, acc);
}

template <typename TD, typename TI, typename TC, typename TO>
hipError_t launch_t(const ReconstructArgs &a)
{
    const int64_t total = (int64_t)a.H * a.T * (a.d / 8);
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    if constexpr (sizeof(TI) == 2 && sizeof(TC) == 2) {
        const bool vec = a.s % 8 == 0 && a.code_stride_h % 8 == 0 && (reinterpret_cast<uintptr_t>(a.idx) % 16) == 0 &&
                         (reinterpret_cast<uintptr_t>(a.coef) % 16) == 0;
        if (vec) {
#define CSR_REC_VEC(G)                                                                                              \
    hipLaunchKernelGGL((reconstruct_vec_kernel<TD, TO, G>), grid, dim3(256), 0, a.stream, (const TD *)a.D,          \
                       (const uint16_t *)a.idx, (const __half *)a.coef, (TO *)a.out, a.T, a.d, a.N, a.sn,           \
                       a.dict_count, a.code_stride_h, a.out_stride_h, a.out_stride_t, total)
            switch (a.s / 8) {
                case 1: CSR_REC_VEC(1); break;
                case 2: CSR_REC_VEC(2); break;
                case 3: CSR_REC_VEC(3); break;
                default: CSR_REC_VEC(4); break;
            }
#undef CSR_REC_VEC
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((reconstruct_kernel<TD, TI, TC, TO>), grid, dim3(256), 0, a.stream, (const TD *)a.D,
                       (const TI *)a.idx, (const TC *)a.coef, (TO *)a.out, a.T, a.d, a.N, a.s, a.sn, a.dict_count,
                       a.code_stride_h, a.out_stride_h, a.out_stride_t, total);
    return hipGetLastError();
}

template <typename TD, typename TI, typename TC>
hipError_t launch_o(const ReconstructArgs &a)
{
    return a.out16 ? launch_t<TD, TI, TC, __half>(a) : launch_t<TD, TI, TC, float>(a);
}
template <typename TD, typename TI>
hipError_t launch_c(const ReconstructArgs &a)
{
    return a.coef16 ? launch_o<TD, TI, __half>(a) : launch_o<TD, TI, float>(a);
}
template <typename TD>
hipError_t launch_i(const ReconstructArgs &a)
{
    return a.idx16 ? launch_c<TD, uint16_t>(a) : launch_c<TD, int32_t>(a);
}

}  // namespace

hipError_t launch_reconstruct(const ReconstructArgs &a)
{
    return a.dict16 ? launch_i<__half>(a) : launch_i<float>(a);
}

}  // namespace csr
