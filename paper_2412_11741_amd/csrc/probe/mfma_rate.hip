// What this chip sustains on the matrix cores alone: a stand-alone probe, not part of the library.
//
// Every wave runs nothing but v_mfma_f32_32x32x16_f16 on operands held in registers (no memory traffic, no LDS, no
// vector-ALU work): 2 waves per SIMD, four independent accumulator chains per wave, for about 20 ms.  Three operand
// patterns: "random" (both operands unit Gaussians, accumulated without end), "smooth" (all operands equal) and
// "encoder_like" (one operand drawn like unit-norm atoms of 128 dimensions, the other like residuals scaled into
// [2^11, 2^12), every accumulation restarted from zero after 8 instructions: the encoder's sweep of one 32-atom
// tile).  MI355X is power-limited under matrix-core load and the clock it settles at depends on how many bits
// toggle, so the rate on such operands - not the nominal 2.5 PFLOP/s - is the ceiling a kernel that feeds the
// matrix cores real data can reach; bench.py reports the encoder's rate against it.
//
//   mfma_rate.bin            prints one JSON line: {"mfma_only_tflops_random": .., "mfma_only_tflops_smooth": ..,
//                            "mfma_only_tflops_encoder_like": ..}
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kChains = 4;

template <bool RESTART>
__global__ __launch_bounds__(512) void mfma_loop(const _Float16 *__restrict__ operands, float *__restrict__ sink, int iters)
{
    const int lane = threadIdx.x & 63;
    half8 a[kChains], b[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
        a[c] = *reinterpret_cast<const half8 *>(operands + ((size_t)(2 * c) * 64 + lane) * 8);
        b[c] = *reinterpret_cast<const half8 *>(operands + ((size_t)(2 * c + 1) * 64 + lane) * 8);
    }
    floatx16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
    float keep = 0.0f;
    if constexpr (RESTART) {
        for (int i = 0; i < iters; i += 8) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) {
                floatx16 t;
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) t = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[c], b[(c + j) % kChains], t, 0, 0, 0);
                keep = fmaxf(keep, t[0]);   // one instruction per 8 MFMAs keeps the results alive
            }
        }
    } else {
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[c], b[c], acc[c], 0, 0, 0);
        }
    }
    float s = keep;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 12345.678f) sink[0] = s;  // keeps the loop alive
}

static double run(const std::vector<_Float16> &host, int cus, bool restart = false)
{
    auto kern = restart ? mfma_loop<true> : mfma_loop<false>;
    _Float16 *dev = nullptr;
    float *sink = nullptr;
    if (hipMalloc(&dev, host.size() * sizeof(_Float16)) != hipSuccess || hipMalloc(&sink, 64) != hipSuccess) return -1.0;
    (void)hipMemcpy(dev, host.data(), host.size() * sizeof(_Float16), hipMemcpyHostToDevice);
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    const int iters = 40000;
    const dim3 grid(cus), block(512);  // 8 waves per CU: two per SIMD
    hipLaunchKernelGGL(kern, grid, block, 0, 0, dev, sink, 2000);  // warm-up
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0, 0);
    hipLaunchKernelGGL(kern, grid, block, 0, 0, dev, sink, iters);
    (void)hipEventRecord(e1, 0);
    (void)hipEventSynchronize(e1);
    float ms = 0.0f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipFree(dev);
    (void)hipFree(sink);
    const double flop = 2.0 * 32 * 32 * 16 * (double)kChains * iters * 8.0 * cus;
    return flop / (ms * 1e-3) / 1e12;
}

int main()
{
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0) != hipSuccess || cus <= 0) {
        std::fprintf(stderr, "mfma_rate: no GPU\n");
        return 1;
    }
    std::vector<_Float16> rnd(2 * kChains * 64 * 8), smooth(rnd.size(), (_Float16)1.0f);
    uint64_t s = 0x9E3779B97F4A7C15ull;
    for (auto &v : rnd) {  // sum of four uniforms: close enough to a Gaussian, seeded
        float acc = 0.0f;
        for (int k = 0; k < 4; ++k) {
            s = s * 6364136223846793005ull + 1442695040888963407ull;
            acc += (float)((s >> 40) & 0xffffff) / 16777216.0f - 0.5f;
        }
        v = (_Float16)(acc * 1.732f);
    }
    // A operands (even slots): atoms, unit Gaussians / sqrt(128); B operands (odd slots): residuals of scale 2^10
    std::vector<_Float16> enc(rnd.size());
    for (size_t i = 0; i < enc.size(); ++i)
        enc[i] = (_Float16)((float)rnd[i] * (((i / (64 * 8)) & 1) ? 1024.0f : 0.0883883f));
    const double r = run(rnd, cus), m = run(smooth, cus), e = run(enc, cus, true);
    std::printf("{\"mfma_only_tflops_random\": %.1f, \"mfma_only_tflops_smooth\": %.1f, \"mfma_only_tflops_encoder_like\": %.1f, "
                "\"compute_units\": %d, \"instruction\": \"v_mfma_f32_32x32x16_f16\", \"waves_per_simd\": 2}\n", r, m, e, cus);
    return 0;
}
