// Device helpers and launch constants shared by the decode kernels (decode.hip, decode_rope.hip).
#pragma once
#include "csr_internal.h"

namespace csr {
namespace dec {

constexpr int kStreamThreads = 1024;  // 16 waves: enough loads in flight with one workgroup per CU
constexpr int kStreamWaves = kStreamThreads / 64;
constexpr int kMaxDevices = 64;      // devices a process may use this library on
constexpr int kMaxTPT = 16;           // tokens per thread and chunk: their scores stay in registers
constexpr int kMaxChunks = 64;
// The rotary-key kernel (decode_rope.hip).  One query head at a time: 16 waves with 128 registers each; a query group
// keeps a rebuilt key and the group's scores in registers: 8 waves with 256 each.
constexpr int rope_threads(int GB) { return GB >= 2 ? 512 : 1024; }  // tokens per round
// rounds a chunk may have: one score per round and query head stays in registers
constexpr int rope_rounds(int GB) { return GB == 2 ? 16 : 8; }
constexpr size_t kRopeTableBytes = 8 * 32 * 4 + 8 * 4 * 8 * 4 + 64 * 8;  // rotation constants, a group's query pairs, theta
constexpr size_t kLdsBudget = 150 * 1024;

__device__ __forceinline__ float h2f(__half v) { return __half2float(v); }

template <typename T> __device__ __forceinline__ void load8(const T *p, float (&o)[8]);
template <> __device__ __forceinline__ void load8<__half>(const __half *p, float (&o)[8])
{
    const uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 f = __half22float2(h2[j]);
        o[2 * j] = f.x;
        o[2 * j + 1] = f.y;
    }
}
template <> __device__ __forceinline__ void load8<float>(const float *p, float (&o)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// ---------------------------------------------------------------------------------------------
// Code-stream loads: PV pairs of one token at a time, widened to int / float registers.
template <typename TI, int PV> struct IdxLoad;
template <> struct IdxLoad<uint16_t, 8> {
    static __device__ __forceinline__ void ld(const uint16_t *p, int (&o)[8]) {
        const uint4 r = *reinterpret_cast<const uint4 *>(p);
        o[0] = r.x & 0xffff; o[1] = r.x >> 16; o[2] = r.y & 0xffff; o[3] = r.y >> 16;
        o[4] = r.z & 0xffff; o[5] = r.z >> 16; o[6] = r.w & 0xffff; o[7] = r.w >> 16;
    }
};
template <> struct IdxLoad<uint16_t, 4> {
    static __device__ __forceinline__ void ld(const uint16_t *p, int (&o)[4]) {
        const uint2 r = *reinterpret_cast<const uint2 *>(p);
        o[0] = r.x & 0xffff; o[1] = r.x >> 16; o[2] = r.y & 0xffff; o[3] = r.y >> 16;
    }
};
template <> struct IdxLoad<uint16_t, 1> {
    static __device__ __forceinline__ void ld(const uint16_t *p, int (&o)[1]) { o[0] = p[0]; }
};
template <> struct IdxLoad<int32_t, 8> {
    static __device__ __forceinline__ void ld(const int32_t *p, int (&o)[8]) {
        const int4 a = *reinterpret_cast<const int4 *>(p);
        const int4 b = *reinterpret_cast<const int4 *>(p + 4);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};
template <> struct IdxLoad<int32_t, 4> {
    static __device__ __forceinline__ void ld(const int32_t *p, int (&o)[4]) {
        const int4 a = *reinterpret_cast<const int4 *>(p);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    }
};
template <> struct IdxLoad<int32_t, 1> {
    static __device__ __forceinline__ void ld(const int32_t *p, int (&o)[1]) { o[0] = p[0]; }
};

template <typename TC, int PV> struct CoefLoad;
template <> struct CoefLoad<__half, 8> {
    static __device__ __forceinline__ void ld(const __half *p, float (&o)[8]) { load8<__half>(p, o); }
};
template <> struct CoefLoad<__half, 4> {
    static __device__ __forceinline__ void ld(const __half *p, float (&o)[4]) {
        const uint2 raw = *reinterpret_cast<const uint2 *>(p);
        const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
        const float2 f0 = __half22float2(h2[0]), f1 = __half22float2(h2[1]);
        o[0] = f0.x; o[1] = f0.y; o[2] = f1.x; o[3] = f1.y;
    }
};
template <> struct CoefLoad<__half, 1> {
    static __device__ __forceinline__ void ld(const __half *p, float (&o)[1]) { o[0] = h2f(p[0]); }
};
template <> struct CoefLoad<float, 8> {
    static __device__ __forceinline__ void ld(const float *p, float (&o)[8]) { load8<float>(p, o); }
};
template <> struct CoefLoad<float, 4> {
    static __device__ __forceinline__ void ld(const float *p, float (&o)[4]) {
        const float4 a = *reinterpret_cast<const float4 *>(p);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    }
};
template <> struct CoefLoad<float, 1> {
    static __device__ __forceinline__ void ld(const float *p, float (&o)[1]) { o[0] = p[0]; }
};

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// x as a 64-bit fixed-point number in units of 2^-32 (two's complement); needs |x| < 2^31.
// x - floor(x) is exact in fp32.  The caller scales p * c by a power of two first (see stream_kernel),
// so that the unit follows the data and the result does not depend on the scale of the coefficients.
__device__ __forceinline__ unsigned long long to_fixed(float x)
{
    const float fl = floorf(x);
    const int hi = (int)fl;
    const unsigned lo = (unsigned)((x - fl) * 4294967296.0f);
    return ((unsigned long long)(unsigned)hi << 32) | lo;
}
__device__ __forceinline__ float from_fixed(unsigned long long v)
{
    return (float)(int)(unsigned)(v >> 32) + (float)(unsigned)(v & 0xffffffffull) * 2.3283064365386963e-10f;
}

}  // namespace dec
}  // namespace csr
