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

}  // namespace

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
