// Checks a caller can run before the hot path, which itself checks nothing of this kind.
//
// Squared norms of dictionary atoms.  Section "Sparse representation" takes the atoms to have unit Euclidean norm;
// the encoders do not check it (they stay correct for other norms, Eq.4 is then no longer a projection), and the
// Gram-update encoder needs the norms to stay below 250.  This lets a caller look before it encodes.
#include "csr_internal.h"

namespace csr {
namespace {

template <typename T> __device__ __forceinline__ float ld(const T *p);
template <> __device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld<__half>(const __half *p) { return __half2float(*p); }

// one wave per atom: lanes stride over the d elements, fp32 sum, butterfly
template <typename T>
__global__ __launch_bounds__(256) void atom_norm2_kernel(const T *__restrict__ D, float *__restrict__ out, int64_t n_atoms, int32_t d)
{
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= n_atoms) return;  // (wave-uniform)
    const T *row = D + n * d;
    float ss = 0.0f;
    for (int k = lane; k < d; k += 64) {
        const float v = ld<T>(row + k);
        ss = fmaf(v, v, ss);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
    if (lane == 0) out[n] = ss;
}

// Atom indices of a code stream outside [0, N): decode and reconstruct use an index as it is (an index >= N reads
// outside the score table or the dictionary), so a cache of codes that comes from elsewhere can be looked at first.
__global__ void zero_count_kernel(unsigned long long *bad) { *bad = 0ull; }

template <typename TI>
__global__ __launch_bounds__(256) void check_codes_kernel(const TI *__restrict__ idx, int64_t count, uint32_t N,
                                                          unsigned long long *__restrict__ bad)
{
    unsigned mine = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        // 16-bit indices are unsigned; a negative 32-bit index is a huge unsigned one
        const uint32_t v = sizeof(TI) == 2 ? (uint32_t)(uint16_t)idx[e] : (uint32_t)idx[e];
        mine += v >= N;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mine += __shfl_xor((int)mine, m, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(bad, (unsigned long long)mine);
}

}  // namespace

hipError_t launch_check_codes(const void *idx, bool idx16, int64_t count, int32_t N, int64_t *bad, hipStream_t stream)
{
    unsigned long long *out = reinterpret_cast<unsigned long long *>(bad);
    hipLaunchKernelGGL(zero_count_kernel, dim3(1), dim3(1), 0, stream, out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || count == 0) return e;
    const int64_t want = (count + 256 * 16 - 1) / (256 * 16);
    const unsigned groups = (unsigned)(want < 4096 ? want : 4096);
    if (idx16)
        hipLaunchKernelGGL(check_codes_kernel<uint16_t>, dim3(groups), dim3(256), 0, stream, (const uint16_t *)idx, count, (uint32_t)N, out);
    else
        hipLaunchKernelGGL(check_codes_kernel<int32_t>, dim3(groups), dim3(256), 0, stream, (const int32_t *)idx, count, (uint32_t)N, out);
    return hipGetLastError();
}

hipError_t launch_atom_norms2(const void *D, bool f16, int64_t n_atoms, int32_t d, float *out, hipStream_t stream)
{
    const int64_t groups = (n_atoms + 3) / 4;
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    if (f16)
        hipLaunchKernelGGL(atom_norm2_kernel<__half>, dim3((unsigned)groups), dim3(256), 0, stream, (const __half *)D, out, n_atoms, d);
    else
        hipLaunchKernelGGL(atom_norm2_kernel<float>, dim3((unsigned)groups), dim3(256), 0, stream, (const float *)D, out, n_atoms, d);
    return hipGetLastError();
}

}  // namespace csr
