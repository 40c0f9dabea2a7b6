// Decode attention on codes whose KEYS were sparsely represented before the rotary position embedding
// (Section "Position embedding makes nonstationary Keys": the key cache is processed ahead of the embedding,
// so attention has to rotate the rebuilt key K~_t = D_K r_t of Eq.12 to its position t).
//
// The rotation depends on the token, so the one score table q . d_n of the position-free path no longer
// exists: every (token, pair) costs a gathered atom row and d multiply-adds instead of one table entry.  That
// only pays while the atom rows come from LDS: the kernel keeps the whole key dictionary of its KV head there
// (N * d * 2 bytes <= 128 KB, the paper's own dictionary sizes) and is bound by the vector ALU (the count of its
// instructions), not by HBM.  Values carry no position: the V side is the same histogram scatter as in stream_kernel, and out_kernel /
// finalize_kernel run unchanged on its results.
//
// Two ways to spend the multiply-adds, chosen by the number of query heads that share the KV head:
//   one query head:  (Rot(t) K~_t) . q = K~_t . (Rot(-t) q) = sum_j c_j (d_{i_j} . q~_t): the query is turned back
//                    to the token's position and dotted with each gathered row (packed fp16 dot products);
//   a query group:   K~_t is rebuilt in fp32 from the gathered rows, turned to its position once and dotted with
//                    every query of the group.
//
// Mapping of pass 1.  A wave handles 64 consecutive tokens per round.  The 8 lanes of an eighth of the wave share the
// work of one token at a time: each holds 8 of the 64 frequency pairs and reads the matching two 16-byte pieces of
// every gathered row.  In step u eighth e works on token 8u + e of the wave's 64: all its lanes read that token's
// codes straight from memory (the same 16 bytes; the eighths' tokens are neighbours, so the wave reads one
// 128-byte line per stream and step, requested one step ahead), the 8 partial scores meet in a 3-step butterfly of
// cross-lane adds, and lane (e, u) keeps the score: it is the lane that handles this token's value codes in
// pass 2.  From step to step the rotation advances by 8 positions (a fixed rotation per pair, fp32), from round to
// round by the rest of the round's stride; the starting angle of every lane is reduced in double precision, so
// positions in the hundreds of thousands stay accurate.
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

__device__ __forceinline__ float lo_half(uint32_t w)
{
    const uint16_t v = (uint16_t)(w & 0xffffu);
    return h2f(*reinterpret_cast<const __half *>(&v));
}
__device__ __forceinline__ float hi_half(uint32_t w)
{
    const uint16_t v = (uint16_t)(w >> 16);
    return h2f(*reinterpret_cast<const __half *>(&v));
}

// v + (v of the lane whose number differs in bit 0 / 1 / 2): cross-lane adds inside a row of 16 lanes
template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(o);
}
__device__ __forceinline__ float sum8(float v)
{
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror: lane i of every 8 with lane 7 - i, which lies in the other quad
    return v;
}

// LDS: atom rows of D_K[h], 256 bytes each, the two members of every frequency pair side by side (pass 1), later the
// fixed-point histogram (pass 2, finish_chunk) | reduction scratch | rotation constants [8 lane classes][32] |
// the group's query pairs, packed fp16 [8 lane classes][4][8] (ROTK only) | theta_k as doubles [64]
// TPT: rounds of rope_threads(GB) tokens a chunk may have (a lane keeps one score per round and query head).
// ONEB: a key code is exactly one block of PVK pairs.
// GLOBAL: the key dictionary does not fit the LDS (more than 512 atoms): every gathered row piece then comes from
// device memory - the L2 for dictionaries of a few MB - instead, brought into the same pair-adjacent form in
// registers.  The arithmetic is the same; the call is then bound by those gathers (256 bytes per code pair).
template <int GB, bool ROTK, int PVK, bool ONEB, int PV, int TPT, bool GLOBAL>
__global__ __launch_bounds__(rope_threads(GB)) void stream_rope_kernel(
    const __half *__restrict__ q, const __half *__restrict__ DK, const uint16_t *__restrict__ idxK,
    const __half *__restrict__ coefK, const uint16_t *__restrict__ idxV, const __half *__restrict__ coefV,
    const int32_t *__restrict__ seq_lens, float *__restrict__ part_hist, float *__restrict__ part_ml, int32_t Hq,
    int32_t Hkv, int32_t G, int32_t ngs, int64_t T, int32_t N, int32_t sK, int32_t sV, int32_t snV, float scale,
    float rope_base, int32_t layout, int64_t pos0, int64_t chunk_tokens, int32_t nchunks, uint32_t tab_bytes)
{
    constexpr int THREADS = rope_threads(GB);
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float *red = reinterpret_cast<float *>(smem_raw + tab_bytes);
    float *ctab = red + kRedBytes / sizeof(float);  // [8][32]: cos, sin of a step; cos, sin of the round jump
    uint32_t *qtab = reinterpret_cast<uint32_t *>(ctab + 8 * 32);  // [8][GB][8]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 7, eighth = lane >> 3;
    const int c = blockIdx.x;
    const int h = blockIdx.y / ngs, gs = blockIdx.y % ngs;
    const int b = blockIdx.z;

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
    const int n_mine = (int)((t_end - t0 + THREADS - 1) / THREADS);  // rounds of THREADS tokens

    // ---- the key dictionary into LDS, frequency pairs made adjacent -----------------------------------------
    if constexpr (!GLOBAL) {
        const __half *src = DK + (int64_t)h * N * 128;
        for (int e = tid; e < N * 16; e += THREADS) {
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

    // ---- frequency pairs of a lane: slot e < 4 lives in row piece `sub`, e >= 4 in piece 8 + sub (128 bytes
    // further); piece p holds pairs 4p .. 4p+3.  What depends on `sub` only goes to LDS, computed once. --------
    // theta_k of all 64 pairs, in double, once per workgroup
    double *theta = reinterpret_cast<double *>(qtab + 8 * 4 * 8);  // [64]
    if (tid < 64) theta[tid] = exp2(-(2.0 * tid / 128.0) * log2((double)rope_base));
    __syncthreads();
    auto pair_of = [](int sb, int e) { return 4 * (e < 4 ? sb : sb + 8) + (e & 3); };
    // cos and sin of positions * theta_k: the angle is reduced to [-1/2, 1/2] revolutions in double, then the
    // hardware sine and cosine (which take revolutions) are accurate to about 1e-6
    auto cos_sin = [&](int k, double positions, float &co, float &si) {
        const double r = positions * theta[k] * 0.15915494309189533577;
        const float f = (float)(r - rint(r));
        co = __builtin_amdgcn_cosf(f);
        si = __builtin_amdgcn_sinf(f);
    };
    // the step constants are applied dozens of times in a row, so their angles get the library's accurate sine and
    // cosine (one thread per constant, once per workgroup); a lane's starting phase above is applied once
    auto cos_sin_exact = [&](int k, double positions, float &co, float &si) {
        const double r = positions * theta[k] * 0.15915494309189533577;
        const double a = (r - rint(r)) * 6.283185307179586476925;
        co = (float)cos(a);
        si = (float)sin(a);
    };
    if (tid < 64) {
        const int sb = tid >> 3, e = tid & 7, k = pair_of(sb, e);
        cos_sin_exact(k, 8.0, ctab[sb * 32 + e], ctab[sb * 32 + 8 + e]);
        cos_sin_exact(k, (double)(THREADS - 64), ctab[sb * 32 + 16 + e], ctab[sb * 32 + 24 + e]);
        if constexpr (ROTK) {
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                const __half *qp = q + ((int64_t)b * Hq + (int64_t)h * G + gs * GB + g) * 128;
                const __half2 pk = __halves2half2(layout == 0 ? qp[k] : qp[2 * k], layout == 0 ? qp[k + 64] : qp[2 * k + 1]);
                qtab[(sb * GB + g) * 8 + e] = *reinterpret_cast<const uint32_t *>(&pk);
            }
        }
    }
    const unsigned char *rows0 = smem_raw + sub * 16;
    // GLOBAL: this lane's two 16-byte pieces (pairs 4 sub .. 4 sub + 3 and 32 + 4 sub .. + 3) of the atom row at byte
    // offset `off` of the head's dictionary, the members of every pair made adjacent
    const unsigned char *grow = reinterpret_cast<const unsigned char *>(DK + (int64_t)h * N * 128);
    auto global_pieces = [&](uint32_t off, uint4 &d0, uint4 &d1) {
        if (layout == 0) {  // pair k = dimensions (k, k + 64): 4 + 4 halves from both halves of the row, interleaved
            auto weave = [](const uint2 &lo, const uint2 &hi) {
                return make_uint4((lo.x & 0xffffu) | (hi.x << 16), (lo.x >> 16) | (hi.x & 0xffff0000u),
                                  (lo.y & 0xffffu) | (hi.y << 16), (lo.y >> 16) | (hi.y & 0xffff0000u));
            };
            const unsigned char *r = grow + off + sub * 8;
            const uint2 a0 = *reinterpret_cast<const uint2 *>(r), b0 = *reinterpret_cast<const uint2 *>(r + 128);
            const uint2 a1 = *reinterpret_cast<const uint2 *>(r + 64), b1 = *reinterpret_cast<const uint2 *>(r + 192);
            d0 = weave(a0, b0);
            d1 = weave(a1, b1);
        } else {            // pair k = dimensions (2k, 2k + 1): already adjacent
            d0 = *reinterpret_cast<const uint4 *>(grow + off + sub * 16);
            d1 = *reinterpret_cast<const uint4 *>(grow + off + 128 + sub * 16);
        }
    };
    const float *my_c = ctab + sub * 32;
    const uint32_t *my_q = qtab + sub * GB * 8;
    // the rotating state, at the position of the first token this eighth handles (step 0 of the first pass over 64).
    // ROTK: (ra, rb) = (cos, sin) of position * theta; else: the query pair turned back by that angle, scaled
    constexpr int NR = ROTK ? 1 : GB;
    float ra[NR][8], rb[NR][8];
    {
        const int64_t pos_start = pos0 + t0 + wave * 64 + eighth;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = pair_of(sub, e);
            float c0, s0;
            cos_sin(k, (double)pos_start, c0, s0);
            if constexpr (ROTK) {
                ra[0][e] = c0;
                rb[0][e] = s0;
            } else {
#pragma unroll
                for (int g = 0; g < GB; ++g) {  // Rot(-pos) (a, b)
                    const __half *qp = q + ((int64_t)b * Hq + (int64_t)h * G + gs * GB + g) * 128;
                    const float a = scale * h2f(layout == 0 ? qp[k] : qp[2 * k]);
                    const float bb = scale * h2f(layout == 0 ? qp[k + 64] : qp[2 * k + 1]);
                    ra[g][e] = a * c0 + bb * s0;
                    rb[g][e] = bb * c0 - a * s0;
                }
            }
        }
    }
    __syncthreads();

    // turn the state on by the angles whose cosines and sines sit at `cs` (8 + 8 floats)
    auto advance = [&](const float *cs) {
        float cc[8], ss[8];
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            *reinterpret_cast<float4 *>(&cc[e]) = *reinterpret_cast<const float4 *>(cs + e);
            *reinterpret_cast<float4 *>(&ss[e]) = *reinterpret_cast<const float4 *>(cs + 8 + e);
        }
#pragma unroll
        for (int g = 0; g < NR; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float a = ra[g][e], bb = rb[g][e];
                if constexpr (ROTK) {  // (cos, sin) forward
                    ra[g][e] = a * cc[e] - bb * ss[e];
                    rb[g][e] = bb * cc[e] + a * ss[e];
                } else {               // the query further back
                    ra[g][e] = a * cc[e] + bb * ss[e];
                    rb[g][e] = bb * cc[e] - a * ss[e];
                }
            }
        }
    };

    // ---- pass 1 ---------------------------------------------------------------------------------------------
    const int nblk = ONEB ? 1 : sK / PVK;  // pair blocks per token (ONEB: known to be one)
    float sc[TPT][GB];
    float mx[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) mx[g] = -INFINITY;
#pragma unroll
    for (int i = 0; i < TPT; ++i) {
#pragma unroll
        for (int g = 0; g < GB; ++g) sc[i][g] = -INFINITY;
        // (a wave whose 64 tokens of this round all lie past the end has none in later rounds either)
        if (i < n_mine && t0 + (int64_t)i * THREADS + wave * 64 < t_end) {
            // the token whose score this lane keeps in round i: the one its eighth handles in step `sub`
            const int64_t t = t0 + (int64_t)i * THREADS + wave * 64 + 8 * sub + eighth;
            const bool have = t < t_end;
            float mine[GB];
#pragma unroll
            for (int g = 0; g < GB; ++g) mine[g] = 0.0f;
            // PVK pairs of the token of step u, read by all 8 lanes of the eighth (one 16-byte piece, and the 8
            // eighths' tokens are neighbours: a wave reads 128 contiguous bytes per stream and step); indices and
            // coefficients as packed 16-bit words.  Requested one block ahead of its use.
            const int64_t tw = t0 + (int64_t)i * THREADS + wave * 64 + eighth;  // + 8 u
            uint32_t ni[PVK / 2], nc[PVK / 2];
            auto fetch = [&](int u, int jb) {
                const int64_t tu = min(tw + 8 * u, t_end - 1);  // past the end: the last token again, score unused
                const uint16_t *ip = idxK + (code_row + tu) * sK + jb * PVK;
                const __half *cp = coefK + (code_row + tu) * sK + jb * PVK;
                if constexpr (PVK == 8) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(ip);
                    const uint4 bq = *reinterpret_cast<const uint4 *>(cp);
                    ni[0] = a.x; ni[1] = a.y; ni[2] = a.z; ni[3] = a.w;
                    nc[0] = bq.x; nc[1] = bq.y; nc[2] = bq.z; nc[3] = bq.w;
                } else {
                    const uint2 a = *reinterpret_cast<const uint2 *>(ip);
                    const uint2 bq = *reinterpret_cast<const uint2 *>(cp);
                    ni[0] = a.x; ni[1] = a.y;
                    nc[0] = bq.x; nc[1] = bq.y;
                }
            };
            fetch(0, 0);
#pragma unroll 1
            for (int u = 0; u < 8; ++u) {
                float part[GB];
                float ka[ROTK ? 8 : 1], kb[ROTK ? 8 : 1];  // ROTK: K~ of this lane's 8 pairs, fp32
                uint32_t qp[ROTK ? 1 : GB][8];             // else: the turned-back queries as fp16 pairs
                if constexpr (ROTK) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) ka[e] = kb[e] = 0.0f;
                } else {
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
                        part[g] = 0.0f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) qp[g][e] = pack_half2(ra[g][e], rb[g][e]);
                    }
                }
#pragma unroll 1
                for (int jb = 0; jb < nblk; ++jb) {
                    uint32_t to[PVK], tc[PVK / 2];
#pragma unroll
                    for (int jj = 0; jj < PVK; ++jj) to[jj] = ((jj & 1) ? (ni[jj >> 1] >> 16) : (ni[jj >> 1] & 0xffffu)) * 256u;
#pragma unroll
                    for (int w = 0; w < PVK / 2; ++w) tc[w] = nc[w];
                    if (jb + 1 < nblk) fetch(u, jb + 1);
                    else if (u < 7) fetch(u + 1, 0);
#pragma unroll
                    for (int jj = 0; jj < PVK; ++jj) {
                        const float cf = (jj & 1) ? hi_half(tc[jj >> 1]) : lo_half(tc[jj >> 1]);
                        uint4 d0, d1;
                        if constexpr (GLOBAL) {
                            global_pieces(to[jj], d0, d1);
                        } else {
                            d0 = *reinterpret_cast<const uint4 *>(rows0 + to[jj]);
                            d1 = *reinterpret_cast<const uint4 *>(rows0 + to[jj] + 128);
                        }
                        if constexpr (ROTK) {
                            const uint32_t dw[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                ka[e] = fmaf(cf, lo_half(dw[e]), ka[e]);
                                kb[e] = fmaf(cf, hi_half(dw[e]), kb[e]);
                            }
                        } else {
#pragma unroll
                            for (int g = 0; g < GB; ++g) {
                                float p = dot2(qp[g][0], d0.x, 0.0f);
                                p = dot2(qp[g][1], d0.y, p);
                                p = dot2(qp[g][2], d0.z, p);
                                p = dot2(qp[g][3], d0.w, p);
                                p = dot2(qp[g][4], d1.x, p);
                                p = dot2(qp[g][5], d1.y, p);
                                p = dot2(qp[g][6], d1.z, p);
                                p = dot2(qp[g][7], d1.w, p);
                                part[g] = fmaf(cf, p, part[g]);
                            }
                        }
                    }
                }
                if constexpr (ROTK) {
                    // turned to the token's position, rounded to fp16 pairs, dotted with every query of the group
                    uint32_t kp[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        kp[e] = pack_half2(ka[e] * ra[0][e] - kb[e] * rb[0][e], kb[e] * ra[0][e] + ka[e] * rb[0][e]);
#pragma unroll
                    for (int g = 0; g < GB; ++g) {
                        const uint4 q0 = *reinterpret_cast<const uint4 *>(my_q + g * 8);
                        const uint4 q1 = *reinterpret_cast<const uint4 *>(my_q + g * 8 + 4);
                        float p = dot2(q0.x, kp[0], 0.0f);
                        p = dot2(q0.y, kp[1], p);
                        p = dot2(q0.z, kp[2], p);
                        p = dot2(q0.w, kp[3], p);
                        p = dot2(q1.x, kp[4], p);
                        p = dot2(q1.y, kp[5], p);
                        p = dot2(q1.z, kp[6], p);
                        p = dot2(q1.w, kp[7], p);
                        part[g] = p;
                    }
                }
#pragma unroll
                for (int g = 0; g < GB; ++g) {
                    const float v = sum8(part[g]);
                    if (sub == u) mine[g] += v;
                }
                advance(my_c);  // 8 positions on: the next step's token
            }
            advance(my_c + 16);  // the rest of the round's stride
            if (have) {
#pragma unroll
                for (int g = 0; g < GB; ++g) {
                    const float v = ROTK ? mine[g] * scale : mine[g];
                    sc[i][g] = v;
                    mx[g] = fmaxf(mx[g], v);
                }
            }
        }
    }
    finish_chunk<GB, uint16_t, __half, PV, true, TPT, THREADS, 0>(smem_raw, red, sc, mx, n_mine, t0, t_end, code_row,
                                                                  wave * 64 + 8 * sub + eighth, idxV, coefV, N, sV, snV, ml,
                                                                  part_hist, slot);
}

template <int GB, bool ROTK, int PVK, bool ONEB, int PV, bool GLOBAL>
hipError_t launch_rope_t(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    auto kern = stream_rope_kernel<GB, ROTK, PVK, ONEB, PV, rope_rounds(GB), GLOBAL>;
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
    // the plan's LDS size = dictionary / histogram | reductions | constant tables (see plan_decode)
    const uint32_t tab_bytes = (uint32_t)(p.lds_bytes - kRedBytes - kRopeTableBytes);
    const dim3 grid((unsigned)p.nchunks, (unsigned)(a.Hkv * p.ngs), (unsigned)a.B);
    hipLaunchKernelGGL(kern, grid, dim3(rope_threads(GB)), p.lds_bytes, a.stream, (const __half *)a.q,
                       (const __half *)a.DK, (const uint16_t *)a.idxK, (const __half *)a.coefK,
                       (const uint16_t *)a.idxV, (const __half *)a.coefV, a.seq_lens, hist, ml, a.Hq, a.Hkv, a.G, p.ngs,
                       a.T, a.N, a.sK, a.sV, a.snV, a.scale, a.rope_base, a.rope_layout, a.rope_pos0, p.chunk_tokens,
                       p.nchunks, tab_bytes);
    return hipGetLastError();
}

template <int GB, bool ROTK, int PVK, bool ONEB, bool GLOBAL>
hipError_t launch_rope_pv(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    if (a.sV % 8 == 0) return launch_rope_t<GB, ROTK, PVK, ONEB, 8, GLOBAL>(a, p, hist, ml);
    if (a.sV % 4 == 0) return launch_rope_t<GB, ROTK, PVK, ONEB, 4, GLOBAL>(a, p, hist, ml);
    return launch_rope_t<GB, ROTK, PVK, ONEB, 1, GLOBAL>(a, p, hist, ml);
}

template <int GB, bool ROTK>
hipError_t launch_rope_gb(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    if (!rope_dictionary_fits_lds(a.N)) {  // rows gathered from device memory
        if (a.sK % 8 == 0) return launch_rope_pv<GB, ROTK, 8, false, true>(a, p, hist, ml);
        return launch_rope_pv<GB, ROTK, 4, false, true>(a, p, hist, ml);
    }
    if (a.sK == 8) return launch_rope_pv<GB, ROTK, 8, true, false>(a, p, hist, ml);  // the paper's key codes
    if (a.sK % 8 == 0) return launch_rope_pv<GB, ROTK, 8, false, false>(a, p, hist, ml);
    return launch_rope_pv<GB, ROTK, 4, false, false>(a, p, hist, ml);
}

}  // namespace

bool decode_rope_shape_supported(int32_t d, int32_t N, int32_t sK, int32_t snK)
{
    return d == 128 && snK == 1 && sK % 4 == 0 && N <= 65536;
}

hipError_t launch_stream_rope(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml)
{
    switch (p.GB) {
        case 4: return launch_rope_gb<4, true>(a, p, hist, ml);
        case 2: return launch_rope_gb<2, true>(a, p, hist, ml);
        case 1: return launch_rope_gb<1, false>(a, p, hist, ml);
    }
    return hipErrorInvalidValue;
}

}  // namespace csr
