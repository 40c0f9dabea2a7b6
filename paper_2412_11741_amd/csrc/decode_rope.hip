// Decode attention on codes whose KEYS were sparsely represented before the rotary position embedding
// (Section "Position embedding makes nonstationary Keys": the key cache is processed ahead of the embedding,
// so attention has to rotate the rebuilt key K~_t = D_K r_t of Eq.12 to its position t).
//
// The rotation depends on the token, so the one score table q . d_n of the position-free path no longer
// exists.  What survives is the transposition: (Rot(t) K~_t) . q = K~_t . (Rot(-t) q) = sum_j c_j d_{i_j} . q~_t,
// i.e. s gathered atom rows dotted with a query turned back by the token's position.  That is d multiply-adds
// per pair instead of one, so it only pays while the atom rows come from LDS: the kernel keeps the whole key
// dictionary of its KV head there (N * d * 2 bytes <= 128 KB, the paper's own dictionary sizes) and is bound by
// the vector ALU, not by HBM.  Values carry no position: the V side is the same histogram scatter as in
// stream_kernel, and out_kernel / finalize_kernel run unchanged on its results.
//
// Mapping of pass 1.  A wave handles 64 consecutive tokens per round; lane l owns token l (it loads that token's
// codes, coalesced, and keeps its score).  The 16 lanes of a quarter wave share the work of one token at a time:
// sub-lane j holds frequency pairs 4j .. 4j+3 of the turned-back query (8 numbers) and reads the matching
// 16 bytes of every gathered atom row, so a quarter reads one whole 256-byte row per load: all 64 banks once.
// In step u the quarter works on its token 16*quarter + u, whose codes come from the owner lane by a lane
// permute; the 16 partial scores meet in a 4-step butterfly.  From step to step the query is turned by one more
// position (a fixed rotation per pair), from round to round by the rest of the 1024-token stride; the starting
// angle of every lane is reduced in double precision, so positions in the hundreds of thousands stay accurate.
#include <atomic>
#include <cmath>

#include "csr_internal.h"
#include "decode_common.h"

namespace csr {
namespace {

using namespace dec;

typedef _Float16 half2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(*reinterpret_cast<const half2v *>(&a), *reinterpret_cast<const half2v *>(&b), c, false);
}

__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    const __half2 h = __floats2half2_rn(a, b);
    return *reinterpret_cast<const uint32_t *>(&h);
}

// LDS: atom rows of D_K[h], 256 bytes each, the two members of every frequency pair side by side (pass 1);
// the 64-bit histogram [GB][NV] (pass 2) | red[waves][GB] | red[waves]
template <int GB, int PVK, int PV>
__global__ __launch_bounds__(kStreamThreads) void stream_rope_kernel(
    const __half *__restrict__ q, const __half *__restrict__ DK, const uint16_t *__restrict__ idxK,
    const __half *__restrict__ coefK, const uint16_t *__restrict__ idxV, const __half *__restrict__ coefV,
    const int32_t *__restrict__ seq_lens, float *__restrict__ part_hist, float *__restrict__ part_ml, int32_t Hq,
    int32_t Hkv, int32_t G, int32_t ngs, int64_t T, int32_t N, int32_t sK, int32_t sV, int32_t snV, float scale,
    float rope_base, int32_t layout, int64_t pos0, int64_t chunk_tokens, int32_t nchunks, uint32_t tab_bytes)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    unsigned long long *hist = reinterpret_cast<unsigned long long *>(smem_raw);
    float *red = reinterpret_cast<float *>(smem_raw + tab_bytes);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 15, quarter = lane >> 4;
    const int c = blockIdx.x;
    const int h = blockIdx.y / ngs, gs = blockIdx.y % ngs;
    const int b = blockIdx.z;
    const int NV = snV * N, sVt = snV * sV;

    int64_t len = T;
    if (seq_lens) {
        const int32_t l = seq_lens[b];
        len = l < 0 ? 0 : (l > T ? T : l);
    }
    const int64_t t0 = (int64_t)c * chunk_tokens;
    const int64_t t_end = min(t0 + chunk_tokens, len);
    const int64_t slot = (((int64_t)b * Hkv + h) * ngs + gs) * nchunks + c;
    float *ml = part_ml + slot * (2 * GB);
    if (t_end <= t0) {  // nothing cached in this chunk: weight zero, histogram never read
        if (tid < GB) { ml[2 * tid] = -INFINITY; ml[2 * tid + 1] = 0.0f; }
        return;
    }
    const int64_t code_row = ((int64_t)b * Hkv + h) * T;
    const int n_mine = (int)((t_end - t0 + kStreamThreads - 1) / kStreamThreads);  // rounds of 1024 tokens

    // ---- the key dictionary into LDS, frequency pairs made adjacent -----------------------------------------
    {
        const __half *src = DK + (int64_t)h * N * 128;
        for (int e = tid; e < N * 16; e += kStreamThreads) {
            const int row = e >> 4, j = e & 15;
            uint4 v;
            if (layout == 0) {  // pair k = dimensions (k, k + 64): take 4 + 4 and interleave
                const uint2 lo = *reinterpret_cast<const uint2 *>(src + row * 128 + 4 * j);
                const uint2 hi = *reinterpret_cast<const uint2 *>(src + row * 128 + 64 + 4 * j);
                v.x = (lo.x & 0xffffu) | (hi.x << 16);
                v.y = (lo.x >> 16) | (hi.x & 0xffff0000u);
                v.z = (lo.y & 0xffffu) | (hi.y << 16);
                v.w = (lo.y >> 16) | (hi.y & 0xffff0000u);
            } else {            // pair k = dimensions (2k, 2k + 1): already adjacent
                v = *reinterpret_cast<const uint4 *>(src + row * 128 + 8 * j);
            }
            *reinterpret_cast<uint4 *>(smem_raw + row * 256 + j * 16) = v;
        }
    }

    // ---- this lane's four frequency pairs: the query turned back to the lane's first position ---------------
    // position of the token the quarter handles in step 0 of round 0
    const int64_t pos_start = pos0 + t0 + wave * 64 + quarter * 16;
    float c1[4], s1[4], cj[4], sj[4];  // one position further; the rest of the stride between rounds
    float qa[GB][4], qb[GB][4];        // q~ pairs, fp32
    {
        const double l2b = log2((double)rope_base);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int k = 4 * sub + p;
            const double theta = exp2(-(2.0 * k / 128.0) * l2b);
            auto reduced = [&](double turns_of) {
                const double a = turns_of * theta;
                return (float)(a - 6.283185307179586476925 * rint(a * 0.15915494309189533577));
            };
            float a1 = reduced(1.0), aj = reduced((double)(kStreamThreads - 16)), a0 = reduced((double)pos_start);
            c1[p] = cosf(a1); s1[p] = sinf(a1);
            cj[p] = cosf(aj); sj[p] = sinf(aj);
            const float c0 = cosf(a0), s0 = sinf(a0);
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                const __half *qp = q + ((int64_t)b * Hq + (int64_t)h * G + gs * GB + g) * 128;
                const float a = scale * h2f(layout == 0 ? qp[k] : qp[2 * k]);
                const float bb = scale * h2f(layout == 0 ? qp[k + 64] : qp[2 * k + 1]);
                // Rot(-pos) (a, b)
                qa[g][p] = a * c0 + bb * s0;
                qb[g][p] = bb * c0 - a * s0;
            }
        }
    }
    __syncthreads();

    // ---- pass 1 ---------------------------------------------------------------------------------------------
    float cm = 0.0f;
    float sc[kMaxTPT][GB];
    float mx[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) mx[g] = -INFINITY;
    const unsigned char *my_rows = smem_raw + sub * 16;
#pragma unroll
    for (int i = 0; i < kMaxTPT; ++i) {
#pragma unroll
        for (int g = 0; g < GB; ++g) sc[i][g] = -INFINITY;
        // (a wave whose 64 tokens of this round all lie past the end has none in later rounds either)
        if (i < n_mine && t0 + (int64_t)i * kStreamThreads + wave * 64 < t_end) {
            const int64_t t = t0 + (int64_t)i * kStreamThreads + tid;  // the token this lane owns in round i
            const bool have = t < t_end;
            if (i == 0 && have) {  // sample the value coefficients for the histogram unit (see stream_kernel)
                const __half *vp = coefV + (code_row + t) * sVt;
                for (int j0 = 0; j0 < sVt; j0 += PV) {
                    float cf[PV];
                    CoefLoad<__half, PV>::ld(vp + j0, cf);
#pragma unroll
                    for (int j = 0; j < PV; ++j) cm = fmaxf(cm, fabsf(cf[j]));
                }
            }
            float mine[GB];
#pragma unroll
            for (int g = 0; g < GB; ++g) mine[g] = 0.0f;
            for (int j0 = 0; j0 < sK; j0 += PVK) {
                // the owner's PVK pairs: indices and coefficients as packed 16-bit words (absent tokens: zeros)
                uint32_t wi[PVK / 2], wc[PVK / 2];
#pragma unroll
                for (int w = 0; w < PVK / 2; ++w) wi[w] = wc[w] = 0u;
                if (have) {
                    const uint16_t *ip = idxK + (code_row + t) * sK + j0;
                    const __half *cp = coefK + (code_row + t) * sK + j0;
                    if constexpr (PVK == 8) {
                        const uint4 a = *reinterpret_cast<const uint4 *>(ip);
                        const uint4 bq = *reinterpret_cast<const uint4 *>(cp);
                        wi[0] = a.x; wi[1] = a.y; wi[2] = a.z; wi[3] = a.w;
                        wc[0] = bq.x; wc[1] = bq.y; wc[2] = bq.z; wc[3] = bq.w;
                    } else {
                        const uint2 a = *reinterpret_cast<const uint2 *>(ip);
                        const uint2 bq = *reinterpret_cast<const uint2 *>(cp);
                        wi[0] = a.x; wi[1] = a.y;
                        wc[0] = bq.x; wc[1] = bq.y;
                    }
                }
                // the turned-back query of this round's first step (kept across the pair blocks of a token by
                // re-deriving it: the step rotations below run on copies)
                float ra[GB][4], rb[GB][4];
#pragma unroll
                for (int g = 0; g < GB; ++g) {
#pragma unroll
                    for (int p = 0; p < 4; ++p) { ra[g][p] = qa[g][p]; rb[g][p] = qb[g][p]; }
                }
#pragma unroll 1
                for (int u = 0; u < 16; ++u) {
                    const int owner = (lane & 48) | u;
                    uint32_t ti[PVK / 2], tc[PVK / 2];
#pragma unroll
                    for (int w = 0; w < PVK / 2; ++w) {
                        ti[w] = (uint32_t)__shfl((int)wi[w], owner, 64);
                        tc[w] = (uint32_t)__shfl((int)wc[w], owner, 64);
                    }
                    uint32_t qp[GB][4];
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
#pragma unroll
                        for (int p = 0; p < 4; ++p) qp[g][p] = pack_half2(ra[g][p], rb[g][p]);
                    }
                    float acc[GB];
#pragma unroll
                    for (int g = 0; g < GB; ++g) acc[g] = 0.0f;
#pragma unroll
                    for (int jj = 0; jj < PVK; ++jj) {
                        const uint32_t id = (jj & 1) ? (ti[jj >> 1] >> 16) : (ti[jj >> 1] & 0xffffu);
                        const uint32_t cw = (jj & 1) ? (tc[jj >> 1] >> 16) : (tc[jj >> 1] & 0xffffu);
                        const uint16_t cs = (uint16_t)cw;
                        const float cf = h2f(*reinterpret_cast<const __half *>(&cs));
                        const uint4 dv = *reinterpret_cast<const uint4 *>(my_rows + id * 256u);
#pragma unroll
                        for (int g = 0; g < GB; ++g) {
                            float part = dot2(qp[g][0], dv.x, 0.0f);
                            part = dot2(qp[g][1], dv.y, part);
                            part = dot2(qp[g][2], dv.z, part);
                            part = dot2(qp[g][3], dv.w, part);
                            acc[g] = fmaf(cf, part, acc[g]);
                        }
                    }
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
                        float v = acc[g];
                        v += __shfl_xor(v, 1, 64);
                        v += __shfl_xor(v, 2, 64);
                        v += __shfl_xor(v, 4, 64);
                        v += __shfl_xor(v, 8, 64);
                        if (sub == u) mine[g] += v;
                    }
                    // one position further
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            const float a = ra[g][p], bb = rb[g][p];
                            ra[g][p] = a * c1[p] + bb * s1[p];
                            rb[g][p] = bb * c1[p] - a * s1[p];
                        }
                    }
                }
                if (j0 + PVK >= sK) {  // last pair block: carry the query on to the next round's first position
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            const float a = ra[g][p], bb = rb[g][p];
                            qa[g][p] = a * cj[p] + bb * sj[p];
                            qb[g][p] = bb * cj[p] - a * sj[p];
                        }
                    }
                }
            }
            if (have) {
#pragma unroll
                for (int g = 0; g < GB; ++g) { sc[i][g] = mine[g]; mx[g] = fmaxf(mx[g], mine[g]); }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        const float wm = wave_max(mx[g]);
        if (lane == 0) red[wave * GB + g] = wm;
    }
    cm = wave_max(cm);
    if (lane == 0) red[kStreamWaves * GB + wave] = cm;
    __syncthreads();  // every score is computed: the dictionary rows are free
    float m_c[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        float v = red[g];
#pragma unroll
        for (int w = 1; w < kStreamWaves; ++w) v = fmaxf(v, red[w * GB + g]);
        m_c[g] = v;
    }
    float c_est = red[kStreamWaves * GB];
#pragma unroll
    for (int w = 1; w < kStreamWaves; ++w) c_est = fmaxf(c_est, red[kStreamWaves * GB + w]);
    int unit_exp = -32;
    if (c_est > 0.0f && c_est < INFINITY) {
        int e2;
        (void)frexpf(c_est, &e2);
        unit_exp = e2 - 1 - 30;
    }
    const int k_units = -unit_exp - 32;
    float m_eff[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) m_eff[g] = m_c[g] - (float)k_units * 0.69314718f;
    const int bins = NV * GB;
    for (int e = tid; e < bins; e += kStreamThreads) hist[e] = 0ull;
    __syncthreads();

    // ---- pass 2: p = exp(score - max) in histogram units, scatter p * c of the V codes -----------------------
    float l_thr[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) l_thr[g] = 0.0f;
#pragma unroll
    for (int i = 0; i < kMaxTPT; ++i) {
        if (i < n_mine) {
            const int64_t t = t0 + (int64_t)i * kStreamThreads + tid;
            if (t < t_end) {
                float p[GB];
#pragma unroll
                for (int g = 0; g < GB; ++g) { p[g] = __expf(sc[i][g] - m_eff[g]); l_thr[g] += p[g]; }
                const uint16_t *ip = idxV + (code_row + t) * sVt;
                const __half *cp = coefV + (code_row + t) * sVt;
                unsigned long long *hb = hist;
                for (int ch = 0; ch < snV; ++ch, hb += N, ip += sV, cp += sV) {
                    for (int j0 = 0; j0 < sV; j0 += PV) {
                        int id[PV];
                        float cf[PV];
                        IdxLoad<uint16_t, PV>::ld(ip + j0, id);
                        CoefLoad<__half, PV>::ld(cp + j0, cf);
#pragma unroll
                        for (int j = 0; j < PV; ++j) {
#pragma unroll
                            for (int g = 0; g < GB; ++g) atomicAdd(&hb[g * NV + id[j]], to_fixed(p[g] * cf[j]));
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

#pragma unroll
    for (int g = 0; g < GB; ++g) {
        const float ws = wave_sum(l_thr[g]);
        if (lane == 0) red[wave * GB + g] = ws;
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        if (tid == g) {
            float l = 0.0f;
            for (int w = 0; w < kStreamWaves; ++w) l += red[w * GB + g];
            ml[2 * g] = m_c[g];
            ml[2 * g + 1] = ldexpf(l, -k_units);
        }
    }
    float *dst = part_hist + slot * (int64_t)bins;
    const float from_units = ldexpf(1.0f, unit_exp + 32);
    for (int e = tid; e < bins; e += kStreamThreads) dst[e] = from_fixed(hist[e]) * from_units;
}

template <int GB, int PVK, int PV>
hipError_t launch_rope_t(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    auto kern = stream_rope_kernel<GB, PVK, PV>;
    static std::atomic<bool> attr_set[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kLdsBudget);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    const size_t red_bytes = (size_t)kStreamWaves * (GB + 1) * sizeof(float);
    const uint32_t tab_bytes = (uint32_t)(p.lds_bytes - red_bytes);
    const dim3 grid((unsigned)p.nchunks, (unsigned)(a.Hkv * p.ngs), (unsigned)a.B);
    hipLaunchKernelGGL(kern, grid, dim3(kStreamThreads), p.lds_bytes, a.stream, (const __half *)a.q,
                       (const __half *)a.DK, (const uint16_t *)a.idxK, (const __half *)a.coefK,
                       (const uint16_t *)a.idxV, (const __half *)a.coefV, a.seq_lens, hist, ml, a.Hq, a.Hkv, a.G, p.ngs,
                       a.T, a.N, a.sK, a.sV, a.snV, a.scale, a.rope_base, a.rope_layout, a.rope_pos0, p.chunk_tokens,
                       p.nchunks, tab_bytes);
    return hipGetLastError();
}

template <int GB, int PVK>
hipError_t launch_rope_pv(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    if (a.sV % 8 == 0) return launch_rope_t<GB, PVK, 8>(a, p, hist, ml);
    if (a.sV % 4 == 0) return launch_rope_t<GB, PVK, 4>(a, p, hist, ml);
    return launch_rope_t<GB, PVK, 1>(a, p, hist, ml);
}

template <int GB>
hipError_t launch_rope_gb(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    if (a.sK % 8 == 0) return launch_rope_pv<GB, 8>(a, p, hist, ml);
    return launch_rope_pv<GB, 4>(a, p, hist, ml);
}

}  // namespace

bool decode_rope_shape_supported(int32_t d, int32_t N, int32_t sK, int32_t snK)
{
    return d == 128 && snK == 1 && sK % 4 == 0 && (size_t)N * 256 <= 128 * 1024;
}

hipError_t launch_stream_rope(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    switch (p.GB) {
        case 2: return launch_rope_gb<2>(a, p, hist, ml);
        case 1: return launch_rope_gb<1>(a, p, hist, ml);
    }
    return hipErrorInvalidValue;
}

}  // namespace csr
