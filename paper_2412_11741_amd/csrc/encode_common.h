// Device helpers and the screening bound shared by the matrix-core Matching Pursuit encoders (encode_mfma.hip,
// encode_resident.hip, encode_split.hip, encode_gram.hip, encode_gramstep.hip).
#pragma once
#include "csr_internal.h"

namespace csr {
namespace enc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// fp32 accumulation error of a 128-term dot product of exact fp16 products, relative to |hi||d|:
// 129 roundings of at most 2^-23 each (this also covers accumulators that truncate).
constexpr float kGammaAcc = 1.6e-5f;

// The bound of the screening sweep (Eq.2-3 decided on hi . d_n instead of R . d_n, R = hi + lo):
//   |hi . d_n - R . d_n| <= |lo| |d_n| + kGammaAcc |R| |d_n|  =: delta / 2  for every atom n,
// so the atom of largest true |correlation| lies within delta of the largest screened value.  dmax: the largest
// atom norm of the dictionary; lo2 = |lo|^2, r2 = |R|^2.
__device__ __forceinline__ float screen_delta(float dmax, float lo2, float r2)
{
    return 2.0f * dmax * (sqrtf(lo2) + kGammaAcc * sqrtf(r2));
}

__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c)
{
    return max(min(a, b), min(max(a, b), c));
}

// value of the other lane of the pair (lane ^ 32)
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

// 8 dimensions of a dot product: a (fp16 x 8) . d (fp16 x 8), two fp32 accumulators; the products of fp16 pairs
// are exact in fp32
__device__ __forceinline__ void dot8(const half8 &a, const half8 &d, float &s0, float &s1)
{
    s0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(d, d, 0, 1), s0, false);
    s1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(d, d, 2, 3), s1, false);
    s0 = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(d, d, 4, 5), s0, false);
    s1 = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(d, d, 6, 7), s1, false);
}

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// waits until at most `n` of this wave's vector memory operations are still in flight
template <int N_LEFT>
__device__ __forceinline__ void wait_vmem_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_LEFT) : "memory"); }

// LDS traffic inside one wave needs no barrier (the LDS executes a wave's instructions in order),
// only that the compiler keeps the order and waits for the data.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// (|c|, atom, c) candidates: larger |c| wins, the lower atom on equal |c| (the tie rule of Eq.3)
__device__ __forceinline__ void take_better(float &ba, int &bi, float &bc, float oa, int oi, float oc)
{
    if (oa > ba || (oa == ba && oi < bi)) { ba = oa; bi = oi; bc = oc; }
}

}  // namespace enc
}  // namespace csr
