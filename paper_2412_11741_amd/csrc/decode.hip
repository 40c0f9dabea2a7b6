// Decode attention computed directly on (index, coefficient) codes.
//
// The paper rebuilds X~ = D r (Eq.12) and runs ordinary attention on it.  Because the rebuild is
// linear, the same numbers come out of the code domain:
//     score_t = q . (D_K r_t)      = sum_j coefK[t][j] * (q . d^K_{idxK[t][j]})
//     out     = sum_t p_t D_V r_t  = D_V^T hist,   hist[n] = sum_{t,j: idxV[t][j]=n} p_t coefV[t][j]
// so per cached token only its 2s-odd code pairs are read from HBM instead of 2d values.
//
// Four launches on the caller's stream:
//   score table      qd[b][h][n][g] = scale * q[b][hg] . d^K_n: qd_rows_kernel (few queries per KV head: a plain read
//                    of the dictionary with packed dot products), qd_mfma_kernel (matrix cores), qd_kernel (fp32)
//   stream_kernel    one workgroup per (token chunk, KV head x group slice, sequence), two passes over
//                    its tokens.  Pass 1: the score table qd sits in LDS as [N][GB]; the K code stream
//                    is read once, coalesced, and every thread keeps the scores of its tokens in
//                    registers; one reduction gives the chunk's maximum.  Pass 2 (finish_chunk in
//                    decode_common.h): the same LDS now holds the histogram; p = exp(score - max) and the V
//                    code stream is scattered into it with integer LDS atomics - fixed point, 32-bit
//                    sign-split bins with a check after the scatter and a 64-bit form to fall back on: on
//                    this chip the LDS float atomic add is serialised lane by lane and runs about
//                    thirty times slower than the integer one, and integer sums are exact, so the
//                    result does not depend on the order of the adds.  The chunk's histogram (as
//                    fp32), maximum and sum go to scratch.
//   D_V x histogram  combines chunk histograms with exp(m_c - M) weights and multiplies by a slice of D_V:
//                    out_rows_kernel (one pair per KV head), out_kernel (up to eight (sequence, query head) pairs
//                    of a KV head at once), out_mfma_kernel (up to 32, on the matrix cores in fp32); one partial
//                    output per slice goes to scratch (no float atomics anywhere: the result is the same
//                    bits on every run)
//   finalize_kernel  adds the slices' partial outputs, divides by the softmax denominator and
//                    stores in the output type.  (Folding this into the last workgroup per
//                    head was tried: the device-scope fences it needs cost more than the launch.)
#include <atomic>
#include <cmath>

#include "csr_internal.h"
#include "decode_common.h"

namespace csr {
namespace {

using namespace dec;

constexpr int kOutAtomsF16 = 128;     // atoms of D_V per out_kernel workgroup, fp16 dictionary
constexpr int kOutAtomsF32 = 64;      // same, fp32 dictionary (the slice sits in LDS in its own type)
constexpr int kQdAtoms = 64;          // atoms of D_K per qd_kernel workgroup
constexpr int kQdTiles = 2;           // 32-atom tiles per wave of qd_mfma_kernel (1 where that leaves CUs without a workgroup)
constexpr int kQTile = 32;            // queries staged in LDS at a time by qd_kernel

// ---------------------------------------------------------------------------------------------
// qd[b][h][gs][n][gg] = scale * q[b][h*G + gs*GB + gg] . DK[h][n]
// 16 lanes share one atom row (8 consecutive k each), so a wave reads 4 rows = 1 KiB per load.
template <typename TQ, typename TD>
__global__ __launch_bounds__(256) void qd_kernel(const TQ *__restrict__ q, const TD *__restrict__ DK,
                                                 float *__restrict__ qd,
                                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t G,
                                                 int32_t GB, int32_t N, float scale)
{
    __shared__ float q_s[kQTile][128];
    const int h = blockIdx.y;
    const int tid = threadIdx.x;
    const int sub = tid & 15, arow = tid >> 4;
    const int n_base = blockIdx.x * kQdAtoms;
    const int ngs = G / GB;

    float a[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = n_base + arow + 16 * i;
        if (n < N) load8<TD>(DK + ((int64_t)h * N + n) * 128 + sub * 8, a[i]);
        else {
#pragma unroll
            for (int j = 0; j < 8; ++j) a[i][j] = 0.0f;
        }
    }

    const int BG = B * G;
    for (int q0 = 0; q0 < BG; q0 += kQTile) {
        const int nq = min(kQTile, BG - q0);
        __syncthreads();
        for (int e = tid; e < nq * 128; e += 256) {
            const int qi = q0 + e / 128, k = e % 128;
            const int b = qi / G, g = qi % G;
            q_s[e / 128][k] = (float)q[((int64_t)b * Hq + h * G + g) * 128 + k];
        }
        __syncthreads();
        for (int ql = 0; ql < nq; ++ql) {
            float qv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) qv[j] = q_s[ql][sub * 8 + j];
            float dot[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc = fmaf(a[i][j], qv[j], acc);
                dot[i] = acc;
            }
#pragma unroll
            for (int m = 8; m >= 1; m >>= 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) dot[i] += __shfl_xor(dot[i], m, 64);
            }
            if (sub == 0) {
                const int qi = q0 + ql;
                const int b = qi / G, g = qi % G;
                const int gs = g / GB, gg = g % GB;
                float *dst = qd + (((int64_t)b * Hkv + h) * ngs + gs) * (int64_t)N * GB;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int n = n_base + arow + 16 * i;
                    if (n < N) dst[(int64_t)n * GB + gg] = scale * dot[i];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The same product on the matrix cores, fp16 queries and dictionary (fp16 products are exact, fp32
// accumulation).  Per 32-atom tile: queries are the M rows of v_mfma_f32_32x32x16_f16, atoms
// the N columns, so a lane ends up with one atom and, per group of four accumulators, four
// consecutive queries - the [n][gg] order of the table.  Fragment j of lane half hf holds dimensions
// 16 j + 8 hf .. + 7, so the two lanes of a row read 32 contiguous bytes per instruction.
typedef _Float16 qd_half8 __attribute__((ext_vector_type(8)));
typedef float qd_floatx16 __attribute__((ext_vector_type(16)));

template <int TILES>
__global__ __launch_bounds__(256) void qd_mfma_kernel(const __half *__restrict__ q, const __half *__restrict__ DK,
                                                      float *__restrict__ qd, int32_t B, int32_t Hq, int32_t Hkv,
                                                      int32_t G, int32_t GB, int32_t N, int32_t sn, float scale)
{
    // With chunks (sn > 1) the table has sn * N entries: entry c * N + n is q's chunk c times atom n of chunk
    // dictionary c, a dot product over dc = 128 / sn dimensions (dc / 16 of the eight MFMA steps carry data).  N is then a multiple of
    // 128, so a 32-atom tile never straddles two chunks.
    const int h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, hf = lane >> 5;
    const int ngs = G / GB;
    const int BG = B * G;
    const int NT = sn * N;       // table entries
    const int dc = 128 / sn;     // dimensions per chunk
    const int nf = dc / 16;      // MFMA steps
    // a wave owns TILES consecutive 32-atom tiles; all their rows are requested before the first product
    const int n_first = (blockIdx.x * 4 + wave) * 32 * TILES;
    if (n_first >= NT) return;
    qd_half8 bfrag[TILES][8];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int v = min(n_first + t * 32 + col, NT - 1);  // row v of [Hkv][sn * N][dc]
        const __half *row = DK + ((int64_t)h * NT + v) * dc + hf * 8;
        const int j_first = (min(n_first + t * 32, NT - 1) / N) * nf;  // the tile's chunk (uniform over the wave)
        // step j multiplies dimensions 16 j .. 16 j + 15 of the query: the row sits at the steps of its chunk's
        // dimensions and is zero elsewhere
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint4 raw = make_uint4(0u, 0u, 0u, 0u);
            if (j >= j_first && j < j_first + nf) raw = *reinterpret_cast<const uint4 *>(row + 16 * (j - j_first));
            bfrag[t][j] = *reinterpret_cast<const qd_half8 *>(&raw);
        }
    }
    for (int q0 = 0; q0 < BG; q0 += 32) {
        const int bgq = q0 + col;  // this lane's query row of the A operand
        const bool have = bgq < BG;
        const __half *qrow = q + ((int64_t)(have ? bgq / G : 0) * Hq + h * G + (have ? bgq % G : 0)) * 128 + hf * 8;
        qd_half8 afrag[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint4 raw = make_uint4(0u, 0u, 0u, 0u);
            if (have) raw = *reinterpret_cast<const uint4 *>(qrow + 16 * j);
            afrag[j] = *reinterpret_cast<const qd_half8 *>(&raw);
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int v = n_first + t * 32 + col;
            qd_floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag[j], bfrag[t][j], acc, 0, 0, 0);
            if (v < NT) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int bg = q0 + 8 * r4 + 4 * hf;  // first of four consecutive queries
                    if (GB == 4 && bg + 3 < BG) {          // G is a multiple of 4: same sequence, same group slice
                        const int b = bg / G, g = bg % G;
                        float *dst = qd + ((((int64_t)b * Hkv + h) * ngs + g / 4) * (int64_t)NT + v) * 4;
                        *reinterpret_cast<float4 *>(dst) = make_float4(scale * acc[4 * r4], scale * acc[4 * r4 + 1],
                                                                       scale * acc[4 * r4 + 2], scale * acc[4 * r4 + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (bg + e < BG) {
                                const int b = (bg + e) / G, g = (bg + e) % G;
                                qd[((((int64_t)b * Hkv + h) * ngs + g / GB) * (int64_t)NT + v) * GB + g % GB] = scale * acc[4 * r4 + e];
                            }
                        }
                    }
                }
            }
        }
    }
}
// ---------------------------------------------------------------------------------------------
// The same table for few queries per KV head (at most 8: short batches without query groups), fp16 queries and
// dictionary.  With so few rows the matrix cores have nothing to do and what counts is how the dictionary is read:
// here 16 lanes share an atom row (16 bytes each, so a wave instruction reads four whole rows, 1 KiB contiguous),
// all eight row requests of a thread are issued before the first is used, the products are packed fp16 dot products
// with fp32 accumulation (exact products, as on the matrix cores) and the 16 partial sums of a row meet in four
// cross-lane adds.  Whole-vector codes only (the chunked table stays with qd_mfma_kernel).
typedef _Float16 qd_half2 __attribute__((ext_vector_type(2)));
template <int NQ>
__global__ __launch_bounds__(256) void qd_rows_kernel(const __half *__restrict__ q, const __half *__restrict__ DK,
                                                      float *__restrict__ qd, int32_t B, int32_t Hq, int32_t Hkv,
                                                      int32_t G, int32_t GB, int32_t N, float scale)
{
    constexpr int kRows = 8;                      // atom rows per thread; 16 threads per row: 128 atoms per workgroup
    const int h = blockIdx.y;
    const int tid = threadIdx.x;
    const int sub = tid & 15, arow = tid >> 4;
    const int n_base = blockIdx.x * (16 * kRows);
    const int ngs = G / GB;
    const int BG = B * G;                         // <= NQ
    uint4 a[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        const int n = n_base + arow + 16 * i;
        a[i] = make_uint4(0u, 0u, 0u, 0u);
        if (n < N) a[i] = *reinterpret_cast<const uint4 *>(DK + ((int64_t)h * N + n) * 128 + sub * 8);
    }
    uint4 qv[NQ];
#pragma unroll
    for (int r = 0; r < NQ; ++r) {
        qv[r] = make_uint4(0u, 0u, 0u, 0u);
        if (r < BG) qv[r] = *reinterpret_cast<const uint4 *>(q + ((int64_t)(r / G) * Hq + h * G + r % G) * 128 + sub * 8);
    }
    auto dot8 = [](const uint4 &x, const uint4 &y) {
        const qd_half2 *xp = reinterpret_cast<const qd_half2 *>(&x), *yp = reinterpret_cast<const qd_half2 *>(&y);
        float acc = __builtin_amdgcn_fdot2(xp[0], yp[0], 0.0f, false);
        acc = __builtin_amdgcn_fdot2(xp[1], yp[1], acc, false);
        acc = __builtin_amdgcn_fdot2(xp[2], yp[2], acc, false);
        return __builtin_amdgcn_fdot2(xp[3], yp[3], acc, false);
    };
    // lane `sub` of a row keeps query `sub`'s product, so that one store instruction per row writes all queries
    const int64_t my_off = sub < BG ? ((((int64_t)(sub / G) * Hkv + h) * ngs + (sub % G) / GB) * (int64_t)N) * GB + (sub % G) % GB : 0;
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        const int n = n_base + arow + 16 * i;
        float mine = 0.0f;
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
            const float d = row_reduce<16>(dot8(a[i], qv[r]), OpAdd());
            if (sub == r) mine = d;
        }
        if (sub < BG && n < N) qd[my_off + (int64_t)n * GB] = scale * mine;
    }
}

// One workgroup: chunk c of the tokens of (sequence b, KV head h, group slice gs).
// LDS: the table of scores q.d, fp32 [N][GB] (pass 1), then the fixed-point histogram (pass 2, see finish_chunk) |
// reduction scratch.
// TPT: rounds of stream_threads(GB) tokens a chunk may have; a thread keeps the scores of its tokens (one per round) in registers.
// VL > 0: a token's key code and its value code are VL 16-byte vectors of indices and of coefficients each (16-bit
// indices, fp16 coefficients, whole-vector codes, s = 8 VL): the vectors are requested ahead of their use - the
// first rounds' before the score table is loaded - so that several round trips to memory overlap.
template <int GB, typename TI, typename TC, int PV, bool CH, int TPT, int VL, int THREADS = kStreamThreads>
__global__ __launch_bounds__(THREADS) void stream_kernel(
    const float *__restrict__ qd, const TI *__restrict__ idxK, const TC *__restrict__ coefK,
    const TI *__restrict__ idxV, const TC *__restrict__ coefV, const int32_t *__restrict__ seq_lens,
    float *__restrict__ part_hist, float *__restrict__ part_ml, int32_t Hkv, int32_t ngs, int64_t T,
    int32_t N, int32_t sK, int32_t sV, int32_t snK_arg, int32_t snV_arg, int64_t chunk_tokens, int32_t nchunks,
    uint32_t tab_bytes)
{
    // CH = false: whole-vector codes, the chunk loops below have one trip known at compile time
    const int snK = CH ? snK_arg : 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float *qd_s = reinterpret_cast<float *>(smem_raw);
    // With chunked codes (sn > 1) a token carries sn * s pairs; pair j of chunk c addresses entry c * N + idx of a
    // table of sn * N entries - the same kernel on a block-diagonal dictionary that is never built.
    const int NK = snK * N;    // entries of the score table
    const int sKt = snK * sK;  // pairs per token
    float *red = reinterpret_cast<float *>(smem_raw + tab_bytes);

    const int tid = threadIdx.x;
    // (KV head, group slice) is the fastest grid dimension: workgroups are dealt to the 8 XCDs round-robin in that
    // order, so the chunks of one (sequence, KV head) - which load the same score table - tend to share an L2
    const int c = blockIdx.y;
    const int h = blockIdx.x / ngs, gs = blockIdx.x % ngs;
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

    static_assert(VL == 0 || (sizeof(TI) == 2 && sizeof(TC) == 2 && PV == 8 && !CH), "16-byte code vectors");
    const int64_t tok0 = t0 + tid;  // this thread's token of round 0
    constexpr int PF = prefetch_rounds<GB, TPT, VL>();
    CodeVec<VL> ring[PF + 1];  // round i reads slot i % (PF + 1) while round i + PF is requested into the slot round i - 1 left
    CodeWalk<VL, THREADS> walk(idxK, coefK, code_row + t0, tid);  // walks PF rounds ahead of the current one
    if constexpr (VL > 0) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            fetch_codes<VL, THREADS>(ring[k], walk, k < n_mine && tok0 + (int64_t)k * THREADS < t_end);
            walk.next();
        }
    }
    const int table = NK * GB;
    {
        const float *src = qd + (((int64_t)b * Hkv + h) * ngs + gs) * (int64_t)table;
        constexpr int U = 4;   // 16-byte pieces a thread requests together: one round trip to L2 instead of four
        const int whole = table & ~3;
        for (int e0 = tid * 4; e0 < whole; e0 += U * THREADS * 4) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {   // past the end: the first piece again, not stored (no load under a branch)
                const int e = e0 + u * THREADS * 4;
                v[u] = *reinterpret_cast<const float4 *>(src + (e < whole ? e : 0));
            }
            // all four pieces are live here: the requests above cannot be strung out between the stores below
            asm volatile("" : "+v"(v[0].x), "+v"(v[0].y), "+v"(v[0].z), "+v"(v[0].w), "+v"(v[1].x), "+v"(v[1].y), "+v"(v[1].z),
                              "+v"(v[1].w), "+v"(v[2].x), "+v"(v[2].y), "+v"(v[2].z), "+v"(v[2].w), "+v"(v[3].x), "+v"(v[3].y),
                              "+v"(v[3].z), "+v"(v[3].w));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + u * THREADS * 4;
                if (e < whole) *reinterpret_cast<float4 *>(qd_s + e) = v[u];
            }
        }
        if (tid < table - whole) qd_s[whole + tid] = src[whole + tid];
    }
    __syncthreads();

    // ---- pass 1: scores of this thread's tokens (token t0 + i * THREADS + tid in round i) --------
    float sc[TPT][GB];
    float mx[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) mx[g] = -INFINITY;
#pragma unroll
    for (int i = 0; i < TPT; ++i) {
#pragma unroll
        for (int g = 0; g < GB; ++g) sc[i][g] = -INFINITY;
    }
    auto pairs = [&](const float *tab, const int (&id)[PV], const float (&cf)[PV], float (&acc)[GB]) {
#pragma unroll
        for (int j = 0; j < PV; ++j) {
            if constexpr (GB == 4) {
                const float4 t4 = *reinterpret_cast<const float4 *>(tab + id[j] * 4);
                acc[0] = fmaf(cf[j], t4.x, acc[0]); acc[1] = fmaf(cf[j], t4.y, acc[1]);
                acc[2] = fmaf(cf[j], t4.z, acc[2]); acc[3] = fmaf(cf[j], t4.w, acc[3]);
            } else if constexpr (GB == 2) {
                const float2 t2 = *reinterpret_cast<const float2 *>(tab + id[j] * 2);
                acc[0] = fmaf(cf[j], t2.x, acc[0]); acc[1] = fmaf(cf[j], t2.y, acc[1]);
            } else {
                acc[0] = fmaf(cf[j], tab[id[j]], acc[0]);
            }
        }
    };
#pragma unroll
    for (int i = 0; i < TPT; ++i) {
        if (i < n_mine) {
            round_fence();
            const int64_t t = tok0 + (int64_t)i * THREADS;
            CodeVec<VL> &cur = ring[i % (PF + 1)];
            if constexpr (VL > 0) {
                await_codes<VL>(cur);
                if (i + PF < TPT) {
                    fetch_codes<VL, THREADS>(ring[(i + PF) % (PF + 1)], walk, i + PF < n_mine && t + (int64_t)PF * THREADS < t_end);
                    walk.next();
                }
            }
            if (t < t_end) {
                float acc[GB];
#pragma unroll
                for (int g = 0; g < GB; ++g) acc[g] = 0.0f;
                if constexpr (VL > 0) {
#pragma unroll
                    for (int v = 0; v < VL; ++v) {
                        int id[8];
                        float cf[8];
                        unpack8(cur.i[v], cur.c[v], id, cf);
                        pairs(qd_s, id, cf, acc);
                    }
                } else {
                    const TI *ip = idxK + (code_row + t) * sKt;
                    const TC *cp = coefK + (code_row + t) * sKt;
                    const float *tab = qd_s;
                    for (int ch = 0; ch < snK; ++ch, tab += N * GB, ip += sK, cp += sK) {
                        for (int j0 = 0; j0 < sK; j0 += PV) {  // PV divides sK: a vector load stays in its chunk
                            int id[PV];
                            float cf[PV];
                            IdxLoad<TI, PV>::ld(ip + j0, id);
                            CoefLoad<TC, PV>::ld(cp + j0, cf);
                            pairs(tab, id, cf, acc);
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < GB; ++g) { sc[i][g] = acc[g]; mx[g] = fmaxf(mx[g], acc[g]); }
            }
        }
    }
    finish_chunk<GB, TI, TC, PV, CH, TPT, THREADS, VL>(smem_raw, red, sc, mx, n_mine, t0, t_end, code_row, tid, idxV,
                                                             coefV, N, sV, snV_arg, ml, part_hist, slot);
}

// ---------------------------------------------------------------------------------------------
// The same product for many (sequence, query head) pairs per KV head (grouped queries, batches of sequences): a
// 128-atom slice of D_V times the combined histograms of up to 32 pairs on the matrix cores, in fp32
// (v_mfma_f32_32x32x2_f32: the histogram needs all 24 bits).  The slice is staged once per 32 pairs instead of once
// per 8, and an LDS read feeds 32 x 32 multiply-adds instead of 4.  Pairs are the M rows (the histogram sits in LDS
// atom-major, [atom][pair], so the 32 lanes of a k-step read one row), dimensions the N columns: a lane reads the
// two neighbouring halves (dimensions 2n, 2n + 1 of a 64-dimension half) of an atom row as one 32-bit word and
// feeds them to two accumulator tiles.  Wave w takes dimension half w & 1 and atom half w >> 1 of the slice; the two
// atom halves meet in LDS.  fp16 dictionary, whole-vector value codes, N a multiple of 128.
// kBatch: chunk histograms in flight together (4: contexts of at most 4 chunks, fewer registers; 8: long ones).
constexpr int kOutMfmaPairs = 32;
template <int kBatch>
__global__ __launch_bounds__(256) void out_mfma_kernel(const __half *__restrict__ DV, const float *__restrict__ part_hist,
                                                       const float *__restrict__ part_ml, float *__restrict__ part_out,
                                                       int32_t B, int32_t Hkv, int32_t G, int32_t GB, int32_t N,
                                                       int32_t nchunks)
{
    constexpr int ATOMS = 128, P = kOutMfmaPairs, kPad = P + 1;
    // the D_V slice as fp16 [atom][dimension]; afterwards the second atom half's partial result, fp32 [pair][dimension]
    __shared__ __attribute__((aligned(16))) unsigned char dv_raw[ATOMS * 128 * sizeof(__half)];
    __shared__ float hist_t[ATOMS][kPad];   // combined histogram, [atom][pair]; one word of padding per row
    __shared__ float w_s[P][kBatch > 4 ? kMaxChunks : 4];   // chunk weights
    __half(*dv_s)[128] = reinterpret_cast<__half(*)[128]>(dv_raw);
    float(*red_s)[128] = reinterpret_cast<float(*)[128]>(dv_raw);
    static_assert(P * 128 * sizeof(float) <= sizeof(dv_raw), "partial result fits the slice's space");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * ATOMS;
    const int h = blockIdx.y;
    const int ngs = G / GB;
    const int nslices = gridDim.x;
    const int BG = B * G;
    const int bg0 = blockIdx.z * P;
    const int nbg = min(P, BG - bg0);
    constexpr int kLoads = ATOMS * 16 / 256;      // 16-byte pieces of the slice per thread
    constexpr int kQuads = P * ATOMS / 4 / 256;   // (pair, four atoms) histogram entries per thread

    uint4 dv_r[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = i * 256 + tid;
        dv_r[i] = *reinterpret_cast<const uint4 *>(DV + ((int64_t)h * N + n0 + e / 16) * 128 + (e % 16) * 8);
    }
    // quad i of this thread: pair q / 32, atoms 4 (q % 32) .. + 3 with q = i * 256 + tid
    const float *ph[kQuads];
#pragma unroll
    for (int i = 0; i < kQuads; ++i) {
        const int q = i * 256 + tid;
        const int bgl = q / (ATOMS / 4), a4 = (q % (ATOMS / 4)) * 4;
        ph[i] = nullptr;
        if (bgl < nbg) {
            const int b = (bg0 + bgl) / G, g = (bg0 + bgl) % G;
            ph[i] = part_hist + ((((int64_t)b * Hkv + h) * ngs + g / GB) * nchunks) * (int64_t)N * GB +
                    (int64_t)(g % GB) * N + (n0 + a4);
        }
    }
    auto request = [&](float4 (&v)[kQuads][kBatch], int c0) {
#pragma unroll
        for (int i = 0; i < kQuads; ++i)
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                v[i][u] = (ph[i] && c0 + u < nchunks) ? *reinterpret_cast<const float4 *>(ph[i] + (int64_t)(c0 + u) * N * GB)
                                                      : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    };
    float4 first[kQuads][kBatch];
    request(first, 0);
    if (tid < nbg) {
        const int b = (bg0 + tid) / G, g = (bg0 + tid) % G;
        const int gs = g / GB, gg = g % GB;
        const float *ml = part_ml + ((((int64_t)b * Hkv + h) * ngs + gs) * nchunks) * (2 * GB);
        float M = -INFINITY;
        for (int c = 0; c < nchunks; ++c) M = fmaxf(M, ml[c * 2 * GB + 2 * gg]);
        for (int c = 0; c < nchunks; ++c) {
            const float m = ml[c * 2 * GB + 2 * gg];
            w_s[tid][c] = (m > -INFINITY) ? __expf(m - M) : 0.0f;
        }
    }
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = i * 256 + tid;
        *reinterpret_cast<uint4 *>(&dv_s[e / 16][(e % 16) * 8]) = dv_r[i];
    }
    __syncthreads();
    float4 hacc[kQuads];
#pragma unroll
    for (int i = 0; i < kQuads; ++i) hacc[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    // a chunk without tokens has weight 0 and a histogram that was never written: skipped, not multiplied
    auto combine = [&](const float4 (&v)[kQuads][kBatch], int c0) {
#pragma unroll
        for (int i = 0; i < kQuads; ++i) {
            const int bgl = (i * 256 + tid) / (ATOMS / 4);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const float w = (ph[i] && c0 + u < nchunks) ? w_s[bgl][c0 + u] : 0.0f;
                if (w > 0.0f) {
                    hacc[i].x = fmaf(w, v[i][u].x, hacc[i].x); hacc[i].y = fmaf(w, v[i][u].y, hacc[i].y);
                    hacc[i].z = fmaf(w, v[i][u].z, hacc[i].z); hacc[i].w = fmaf(w, v[i][u].w, hacc[i].w);
                }
            }
        }
    };
    combine(first, 0);
    if constexpr (kBatch > 4) {   // launched only then: more chunks than one batch
        for (int c0 = kBatch; c0 < nchunks; c0 += kBatch) {
            request(first, c0);
            combine(first, c0);
        }
    }
#pragma unroll
    for (int i = 0; i < kQuads; ++i) {
        const int q = i * 256 + tid;
        const int bgl = q / (ATOMS / 4), a4 = (q % (ATOMS / 4)) * 4;
        hist_t[a4][bgl] = hacc[i].x; hist_t[a4 + 1][bgl] = hacc[i].y;
        hist_t[a4 + 2][bgl] = hacc[i].z; hist_t[a4 + 3][bgl] = hacc[i].w;
    }
    __syncthreads();

    const int col = lane & 31, kk = lane >> 5;
    const int dh = wave & 1, ah = wave >> 1;
    qd_floatx16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.0f;
#pragma unroll 8
    for (int st = 0; st < ATOMS / 4; ++st) {
        const int k = ah * (ATOMS / 2) + 2 * st + kk;
        const float a = hist_t[k][col];
        const __half2 d2 = *reinterpret_cast<const __half2 *>(&dv_s[k][64 * dh + 2 * col]);
        const float2 df = __half22float2(d2);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, df.x, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, df.y, acc1, 0, 0, 0);
    }
    __syncthreads();  // every wave is done with the slice: its space takes the second atom half's result
    // accumulator r of a lane: pair 8 (r / 4) + 4 kk + r % 4, dimensions 64 dh + 2 col (acc0) and + 1 (acc1)
    if (ah == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int pr = 8 * (r >> 2) + 4 * kk + (r & 3);
            *reinterpret_cast<float2 *>(&red_s[pr][64 * dh + 2 * col]) = make_float2(acc0[r], acc1[r]);
        }
    }
    __syncthreads();
    if (ah == 0) {
        float *dst = part_out + (((int64_t)h * nslices + blockIdx.x) * BG + bg0) * 128;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int pr = 8 * (r >> 2) + 4 * kk + (r & 3);
            if (pr < nbg) {
                const float2 o = *reinterpret_cast<const float2 *>(&red_s[pr][64 * dh + 2 * col]);
                *reinterpret_cast<float2 *>(dst + (int64_t)pr * 128 + 64 * dh + 2 * col) = make_float2(acc0[r] + o.x, acc1[r] + o.y);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// part_out[h][slice][b*G+g][k] = sum_{n in slice} (sum_c w_c hist_c[n][g]) * DV[h][n][k].
// One workgroup: a slice of D_V (ATOMS atoms) times the histograms of up to NQ (sequence, query head)
// pairs of KV head h.  All global loads - the slice, the chunk maxima, the chunk histograms - are issued
// at once; the weights are applied when they have arrived.  Thread (half, k) owns output dimension k
// over half of the slice's atoms; the halves meet in LDS.
template <typename TD, int ATOMS, int NQ>
__global__ __launch_bounds__(256) void out_kernel(const TD *__restrict__ DV, const float *__restrict__ part_hist,
                                                  const float *__restrict__ part_ml, float *__restrict__ part_out,
                                                  int32_t B, int32_t Hkv, int32_t G, int32_t GB, int32_t N,
                                                  int32_t snV, int32_t nchunks)
{
    // Chunked values (snV > 1): the slice lies in one chunk c (ATOMS divides N), whose atoms have dc = 128 / snV
    // elements and fill columns [c * dc, (c + 1) * dc) of the output; the other columns of the slice are zero.
    __shared__ __attribute__((aligned(16))) TD dv_s[ATOMS][128];
    __shared__ __attribute__((aligned(16))) float hist_s[NQ][ATOMS];
    __shared__ float w_s[NQ][kMaxChunks];
    __shared__ float half_s[NQ][128];
    const int tid = threadIdx.x;
    const int n0 = blockIdx.x * ATOMS;
    const int h = blockIdx.y;
    const int ngs = G / GB;
    const int nslices = gridDim.x;
    const int BG = B * G;
    const int bg0 = blockIdx.z * NQ;
    const int nbg = min(NQ, BG - bg0);
    constexpr int kVec = 16 / sizeof(TD);               // elements per 16-byte load
    constexpr int kLoads = ATOMS * (128 / kVec) / 256;  // 16-byte loads per thread
    constexpr int kElems = (NQ * ATOMS + 255) / 256;    // (query, atom) histogram entries per thread
    constexpr int kEarly = 8;                           // chunks whose histograms are requested up front (one round trip
                                                        // for the 8 chunks a long grouped-query context has)
    const int NV = snV * N, dc = 128 / snV;
    const int col0 = (n0 / N) * dc;

    uint4 dv_r[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = i * 256 + tid;
        const int r = e / (128 / kVec), cch = e % (128 / kVec);
        const int col = cch * kVec - col0;
        dv_r[i] = make_uint4(0u, 0u, 0u, 0u);
        if (n0 + r < NV && col >= 0 && col < dc)
            dv_r[i] = *reinterpret_cast<const uint4 *>(DV + ((int64_t)h * NV + n0 + r) * dc + col);
    }
    // entry i of this thread: query bgl = e / ATOMS, atom nn = e % ATOMS with e = i * 256 + tid
    const float *ph[kElems];
    float early[kElems][kEarly];
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = i * 256 + tid;
        const int bgl = e / ATOMS, nn = e % ATOMS;
        ph[i] = nullptr;
        if (e < NQ * ATOMS && bgl < nbg && n0 + nn < NV) {
            const int b = (bg0 + bgl) / G, g = (bg0 + bgl) % G;
            ph[i] = part_hist + ((((int64_t)b * Hkv + h) * ngs + g / GB) * nchunks) * (int64_t)NV * GB +
                    (int64_t)(g % GB) * NV + (n0 + nn);
        }
#pragma unroll
        for (int c = 0; c < kEarly; ++c)
            early[i][c] = (ph[i] && c < nchunks) ? ph[i][(int64_t)c * NV * GB] : 0.0f;
    }
    if (tid < nbg) {
        const int b = (bg0 + tid) / G, g = (bg0 + tid) % G;
        const int gs = g / GB, gg = g % GB;
        const float *ml = part_ml + ((((int64_t)b * Hkv + h) * ngs + gs) * nchunks) * (2 * GB);
        float M = -INFINITY;
        for (int c = 0; c < nchunks; ++c) M = fmaxf(M, ml[c * 2 * GB + 2 * gg]);
        for (int c = 0; c < nchunks; ++c) {
            const float m = ml[c * 2 * GB + 2 * gg];
            w_s[tid][c] = (m > -INFINITY) ? __expf(m - M) : 0.0f;
        }
    }
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int e = i * 256 + tid;
        *reinterpret_cast<uint4 *>(&dv_s[e / (128 / kVec)][(e % (128 / kVec)) * kVec]) = dv_r[i];
    }
    __syncthreads();
    float hacc[kElems];
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = i * 256 + tid;
        const int bgl = e / ATOMS;
        float acc = 0.0f;
        if (ph[i]) {
            // a chunk without tokens has weight 0 and a histogram that was never written: skip, not multiply
#pragma unroll
            for (int c = 0; c < kEarly; ++c) {
                const float w = c < nchunks ? w_s[bgl][c] : 0.0f;
                if (w > 0.0f) acc = fmaf(w, early[i][c], acc);
            }
        }
        hacc[i] = acc;
    }
    // the remaining chunks, four at a time: all their loads are requested before the first is used (a histogram that
    // was never written is read too, and dropped with its zero weight)
    for (int c0 = kEarly; c0 < nchunks; c0 += 4) {
        float v[kElems][4];
#pragma unroll
        for (int i = 0; i < kElems; ++i) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[i][u] = (ph[i] && c0 + u < nchunks) ? ph[i][(int64_t)(c0 + u) * NV * GB] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kElems; ++i) {
            const int bgl = (i * 256 + tid) / ATOMS;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float w = (ph[i] && c0 + u < nchunks) ? w_s[bgl][c0 + u] : 0.0f;
                if (w > 0.0f) hacc[i] = fmaf(w, v[i][u], hacc[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = i * 256 + tid;
        if (e < NQ * ATOMS) hist_s[e / ATOMS][e % ATOMS] = hacc[i];
    }
    __syncthreads();
    const int k = tid & 127, half = tid >> 7;
    float acc[NQ];
#pragma unroll
    for (int r = 0; r < NQ; ++r) acc[r] = 0.0f;
    // four atoms at a time: four reads of this thread's column, one 16-byte broadcast read per query
#pragma unroll 2
    for (int nn = half * (ATOMS / 2); nn < (half + 1) * (ATOMS / 2); nn += 4) {
        const float d0 = (float)dv_s[nn][k], d1 = (float)dv_s[nn + 1][k], d2 = (float)dv_s[nn + 2][k],
                    d3 = (float)dv_s[nn + 3][k];
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
            const float4 hv = *reinterpret_cast<const float4 *>(&hist_s[r][nn]);
            acc[r] = fmaf(hv.x, d0, fmaf(hv.y, d1, fmaf(hv.z, d2, fmaf(hv.w, d3, acc[r]))));
        }
    }
    if (half == 1) {
#pragma unroll
        for (int r = 0; r < NQ; ++r) half_s[r][k] = acc[r];
    }
    __syncthreads();
    if (half == 0) {
        float *dst = part_out + (((int64_t)h * nslices + blockIdx.x) * BG + bg0) * 128;
#pragma unroll
        for (int r = 0; r < NQ; ++r)
            if (r < nbg) dst[(int64_t)r * 128 + k] = acc[r] + half_s[r][k];
    }
}

// The same for fp16 dictionaries, whole-vector values and ONE (sequence, query head) pair per KV head (a single
// sequence without query groups; with more pairs out_kernel's LDS-staged slice is the faster form), with the slice read the way qd_rows_kernel reads D_K: 16 lanes
// share an atom row (16 bytes each), all eight row requests of a thread are issued ahead of everything else, and the
// slice never passes through LDS.  Thread (arow, sub) owns dimensions 8 sub .. 8 sub + 7 of atoms arow + 16 i; it takes
// the combined histogram values of its atoms from LDS (one value per atom and pair, shared by the 16 lanes of the
// row), and the 16 atom groups meet through lane exchanges inside a wave and LDS across the four waves.
template <int NQ>
__global__ __launch_bounds__(256) void out_rows_kernel(const __half *__restrict__ DV, const float *__restrict__ part_hist,
                                                       const float *__restrict__ part_ml, float *__restrict__ part_out,
                                                       int32_t B, int32_t Hkv, int32_t G, int32_t GB, int32_t N, int32_t nchunks)
{
    constexpr int ATOMS = kOutAtomsF16, kRows = ATOMS / 16;
    __shared__ __attribute__((aligned(16))) float hist_s[NQ][ATOMS];
    __shared__ float w_s[NQ][kMaxChunks];
    __shared__ __attribute__((aligned(16))) float red_s[4][NQ][128];
    const int tid = threadIdx.x;
    const int sub = tid & 15, arow = tid >> 4;
    const int n0 = blockIdx.x * ATOMS;
    const int h = blockIdx.y;
    const int ngs = G / GB;
    const int nslices = gridDim.x;
    const int BG = B * G;
    const int bg0 = blockIdx.z * NQ;
    const int nbg = min(NQ, BG - bg0);
    constexpr int kElems = (NQ * ATOMS + 255) / 256;
    constexpr int kEarly = 4;

    uint4 raw[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        const int n = n0 + arow + 16 * i;
        raw[i] = make_uint4(0u, 0u, 0u, 0u);
        if (n < N) raw[i] = *reinterpret_cast<const uint4 *>(DV + ((int64_t)h * N + n) * 128 + sub * 8);
    }
    const float *ph[kElems];
    float early[kElems][kEarly];
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = i * 256 + tid;
        const int bgl = e / ATOMS, nn = e % ATOMS;
        ph[i] = nullptr;
        if (e < NQ * ATOMS && bgl < nbg && n0 + nn < N) {
            const int b = (bg0 + bgl) / G, g = (bg0 + bgl) % G;
            ph[i] = part_hist + ((((int64_t)b * Hkv + h) * ngs + g / GB) * nchunks) * (int64_t)N * GB +
                    (int64_t)(g % GB) * N + (n0 + nn);
        }
#pragma unroll
        for (int c = 0; c < kEarly; ++c)
            early[i][c] = (ph[i] && c < nchunks) ? ph[i][(int64_t)c * N * GB] : 0.0f;
    }
    if (tid < nbg) {
        const int b = (bg0 + tid) / G, g = (bg0 + tid) % G;
        const int gs = g / GB, gg = g % GB;
        const float *ml = part_ml + ((((int64_t)b * Hkv + h) * ngs + gs) * nchunks) * (2 * GB);
        float M = -INFINITY;
        for (int c = 0; c < nchunks; ++c) M = fmaxf(M, ml[c * 2 * GB + 2 * gg]);
        for (int c = 0; c < nchunks; ++c) {
            const float m = ml[c * 2 * GB + 2 * gg];
            w_s[tid][c] = (m > -INFINITY) ? __expf(m - M) : 0.0f;
        }
    }
    __syncthreads();
    float hacc[kElems];
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int bgl = (i * 256 + tid) / ATOMS;
        float acc = 0.0f;
        if (ph[i]) {
            // a chunk without tokens has weight 0 and a histogram that was never written: skip, not multiply
#pragma unroll
            for (int c = 0; c < kEarly; ++c) {
                const float w = c < nchunks ? w_s[bgl][c] : 0.0f;
                if (w > 0.0f) acc = fmaf(w, early[i][c], acc);
            }
        }
        hacc[i] = acc;
    }
    for (int c0 = kEarly; c0 < nchunks; c0 += 4) {
        float v[kElems][4];
#pragma unroll
        for (int i = 0; i < kElems; ++i) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[i][u] = (ph[i] && c0 + u < nchunks) ? ph[i][(int64_t)(c0 + u) * N * GB] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kElems; ++i) {
            const int bgl = (i * 256 + tid) / ATOMS;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float w = (ph[i] && c0 + u < nchunks) ? w_s[bgl][c0 + u] : 0.0f;
                if (w > 0.0f) hacc[i] = fmaf(w, v[i][u], hacc[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = i * 256 + tid;
        if (e < NQ * ATOMS) hist_s[e / ATOMS][e % ATOMS] = hacc[i];
    }
    __syncthreads();
    float acc[NQ][8];
#pragma unroll
    for (int r = 0; r < NQ; ++r)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[r][k] = 0.0f;
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        float d[8];
        load8_raw(raw[i], d);
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
            const float hv = hist_s[r][arow + 16 * i];
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[r][k] = fmaf(hv, d[k], acc[r][k]);
        }
    }
    // the four atom groups of a wave (rows of 16 lanes) meet through two lane exchanges, the waves through LDS
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int r = 0; r < NQ; ++r) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float v = acc[r][k];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            acc[r][k] = v;
        }
    }
    if (lane < 16) {
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
            *reinterpret_cast<float4 *>(&red_s[wave][r][8 * sub]) = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
            *reinterpret_cast<float4 *>(&red_s[wave][r][8 * sub + 4]) = make_float4(acc[r][4], acc[r][5], acc[r][6], acc[r][7]);
        }
    }
    __syncthreads();
    float *dst = part_out + (((int64_t)h * nslices + blockIdx.x) * BG + bg0) * 128;
    for (int e = tid; e < nbg * 128; e += 256) {
        const int r = e >> 7, k = e & 127;
        dst[e] = (red_s[0][r][k] + red_s[1][r][k]) + (red_s[2][r][k] + red_s[3][r][k]);
    }
}

// out[b][hq][k] = (sum over slices of part_out) / softmax denominator.  Thread (half, k): the slices of one
// parity, eight loads in flight; the order of the additions is fixed, so the result is reproducible.
template <typename TO>
__global__ __launch_bounds__(256) void finalize_kernel(const float *__restrict__ part_out,
                                                       const float *__restrict__ part_ml, TO *__restrict__ out,
                                                       int32_t B, int32_t Hq, int32_t Hkv, int32_t G, int32_t GB,
                                                       int32_t nchunks, int32_t nslices)
{
    __shared__ float half_s[128];
    const int hq = blockIdx.x % Hq, b = blockIdx.x / Hq;
    const int h = hq / G, g = hq % G;
    const int ngs = G / GB, gs = g / GB, gg = g % GB;
    const int k = threadIdx.x & 127, half = threadIdx.x >> 7;
    const int BG = B * G;
    const int64_t stride = (int64_t)BG * 128;
    const float *src = part_out + ((int64_t)h * nslices * BG + (b * G + g)) * 128 + k;
    float acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[r] = 0.0f;
    int sl = half;
    for (; sl + 14 < nslices; sl += 16) {
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] += src[(int64_t)(sl + 2 * r) * stride];
    }
    for (; sl < nslices; sl += 2) acc[0] += src[(int64_t)sl * stride];
    const float sum = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
    if (half == 1) half_s[k] = sum;
    const float *ml = part_ml + ((((int64_t)b * Hkv + h) * ngs + gs) * nchunks) * (2 * GB);
    float M = -INFINITY;
    for (int c = 0; c < nchunks; ++c) M = fmaxf(M, ml[c * 2 * GB + 2 * gg]);
    float L = 0.0f;
    for (int c = 0; c < nchunks; ++c) {
        const float m = ml[c * 2 * GB + 2 * gg];
        if (m > -INFINITY) L = fmaf(__expf(m - M), ml[c * 2 * GB + 2 * gg + 1], L);
    }
    __syncthreads();
    if (half == 0) {
        const float v = L > 0.0f ? (sum + half_s[k]) / L : 0.0f;
        out[((int64_t)b * Hq + hq) * 128 + k] = (TO)v;
    }
}

template <int GB, typename TI, typename TC, int PV, bool CH, int TPT = max_rounds(GB), int VL = 0, int THREADS = kStreamThreads>
hipError_t launch_stream_t(const DecodeArgs &a, const DecodePlan &p, float *qd, float *hist, float *ml)
{
    auto kern = stream_kernel<GB, TI, TC, PV, CH, TPT, VL, THREADS>;
    // raising the dynamic-LDS limit is needed once per kernel and device
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
    const dim3 grid((unsigned)(a.Hkv * p.ngs), (unsigned)p.nchunks, (unsigned)a.B);
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), p.lds_bytes, a.stream, qd, (const TI *)a.idxK,
                       (const TC *)a.coefK, (const TI *)a.idxV, (const TC *)a.coefV, a.seq_lens, hist, ml,
                       a.Hkv, p.ngs, a.T, a.N, a.sK, a.sV, a.snK, a.snV, p.chunk_tokens, p.nchunks,
                       (uint32_t)(p.lds_bytes - kRedBytes));
    return hipGetLastError();
}

template <int GB, typename TI, typename TC>
hipError_t launch_stream_pv(const DecodeArgs &a, const DecodePlan &p, float *qd, float *hist, float *ml)
{
    if (a.snK > 1 || a.snV > 1) {
        if (a.sK % 8 == 0 && a.sV % 8 == 0) return launch_stream_t<GB, TI, TC, 8, true>(a, p, qd, hist, ml);
        if (a.sK % 4 == 0 && a.sV % 4 == 0) return launch_stream_t<GB, TI, TC, 4, true>(a, p, qd, hist, ml);
        return launch_stream_t<GB, TI, TC, 1, true>(a, p, qd, hist, ml);
    }
    if constexpr (sizeof(TI) == 2 && sizeof(TC) == 2) {
        // the paper's storage (16-bit indices, fp16 coefficients) with 8 or 16 pairs per code: 16-byte code vectors
        // requested ahead; chunks of at most 1024 tokens (short contexts) keep one score per thread
        if constexpr (GB == 4) {
            if (p.threads == kLongThreads4)
                return launch_stream_t<GB, TI, TC, 8, false, kLongRounds4, 1, kLongThreads4>(a, p, qd, hist, ml);
        }
        const int rounds = (int)(p.chunk_tokens / kStreamThreads);
        if (a.sK == 8 && a.sV == 8)
            return rounds == 1 ? launch_stream_t<GB, TI, TC, 8, false, 1, 1>(a, p, qd, hist, ml)
                 : rounds <= 8 ? launch_stream_t<GB, TI, TC, 8, false, 8, 1>(a, p, qd, hist, ml)
                               : launch_stream_t<GB, TI, TC, 8, false, max_rounds(GB), 1>(a, p, qd, hist, ml);
        if (a.sK == 16 && a.sV == 16)
            return rounds == 1 ? launch_stream_t<GB, TI, TC, 8, false, 1, 2>(a, p, qd, hist, ml)
                 : rounds <= 8 ? launch_stream_t<GB, TI, TC, 8, false, 8, 2>(a, p, qd, hist, ml)
                               : launch_stream_t<GB, TI, TC, 8, false, max_rounds(GB), 2>(a, p, qd, hist, ml);
    }
    if (a.sK % 8 == 0 && a.sV % 8 == 0) return launch_stream_t<GB, TI, TC, 8, false>(a, p, qd, hist, ml);
    if (a.sK % 4 == 0 && a.sV % 4 == 0) return launch_stream_t<GB, TI, TC, 4, false>(a, p, qd, hist, ml);
    return launch_stream_t<GB, TI, TC, 1, false>(a, p, qd, hist, ml);
}

template <int GB>
hipError_t launch_stream_gb(const DecodeArgs &a, const DecodePlan &p, float *qd, float *hist, float *ml)
{
    if (a.idx16) {
        if (a.coef16) return launch_stream_pv<GB, uint16_t, __half>(a, p, qd, hist, ml);
        return launch_stream_pv<GB, uint16_t, float>(a, p, qd, hist, ml);
    }
    if (a.coef16) return launch_stream_pv<GB, int32_t, __half>(a, p, qd, hist, ml);
    return launch_stream_pv<GB, int32_t, float>(a, p, qd, hist, ml);
}

}  // namespace

bool plan_decode(int32_t B, int32_t Hq, int32_t Hkv, int64_t T, int32_t d, int32_t N, int32_t snK, int32_t snV,
                 bool rope, int code_vecs, DecodePlan *p)
{
    const size_t NK = (size_t)snK * N, NV = (size_t)snV * N;  // entries of the score table / of a histogram
    const int G = Hq / Hkv;
    int GB = 0;
    for (int cand : {4, 2, 1}) {
        if (G % cand != 0) continue;
        // score table (fp32; with rotary keys the dictionary itself, fp16 rows) and histogram (64-bit) share the
        // space: the larger one counts
        const size_t first = rope ? (rope_dictionary_fits_lds(N) ? (size_t)N * d * 2 : 0) : NK * 4 * cand;
        const size_t tab = ((first > NV * 8 * cand ? first : NV * 8 * cand) + 15) & ~size_t(15);
        const size_t lds = tab + kRedBytes + (rope ? kRopeTableBytes : 0);
        if (lds <= kLdsBudget) { GB = cand; p->lds_bytes = lds; break; }
    }
    if (!GB) return false;
    p->GB = GB;
    p->ngs = G / GB;
    // Split the token axis until every CU has a workgroup (two per CU was measured slower); every extra chunk costs one histogram
    // round trip through scratch, so no more than that, except that a chunk holds at most
    // max_rounds x stream_threads tokens (a thread keeps its tokens' scores in registers).
    const int64_t groups = (int64_t)(B > 0 ? B : 1) * Hkv * p->ngs;
    int64_t want = (256 + groups - 1) / groups;
    int64_t threads = rope ? rope_threads(GB) : kStreamThreads;  // tokens per round of the streaming kernel
    int64_t tpt = rope ? rope_rounds(GB) : max_rounds(GB);       // rounds per chunk
    // four query heads, 8 pairs per code in the paper's storage types, a context too long for `want` chunks of the
    // 16-wave shape: the 8-wave shape with four times the rounds
    if (!rope && GB == 4 && code_vecs == 1 && T > want * tpt * threads) { threads = kLongThreads4; tpt = kLongRounds4; }
    p->threads = (int32_t)threads;
    const int64_t most = T > 0 ? (T + threads - 1) / threads : 1;
    const int64_t least = T > 0 ? (T + tpt * threads - 1) / (tpt * threads) : 1;
    if (want > most) want = most;
    if (want > kMaxChunks) want = kMaxChunks;
    if (want < least) want = least;
    if (want > kMaxChunks) return false;  // T beyond kMaxChunks chunks of the most tokens a chunk can hold
    if (want < 1) want = 1;
    int64_t ct = T > 0 ? (T + want - 1) / want : threads;
    ct = (ct + threads - 1) / threads * threads;
    p->chunk_tokens = ct;
    p->nchunks = T > 0 ? (int32_t)((T + ct - 1) / ct) : 1;
    auto r256 = [](size_t v) { return (v + 255) & ~size_t(255); };
    const size_t BHq = (size_t)(B > 0 ? B : 1) * Hq;
    size_t off = 0;
    p->off_qd = off;   off += r256(BHq * NK * sizeof(float));
    p->off_hist = off; off += r256(BHq * NV * sizeof(float) * p->nchunks);
    p->off_ml = off;   off += r256(BHq * 2 * sizeof(float) * p->nchunks);
    p->off_acc = off;  off += r256(BHq * 128 * sizeof(float) * ((NV + kOutAtomsF32 - 1) / kOutAtomsF32));
    p->total_bytes = off;
    return true;
}

hipError_t launch_decode(const DecodeArgs &a, const DecodePlan &p)
{
    char *ws = static_cast<char *>(a.workspace);
    float *qd = reinterpret_cast<float *>(ws + p.off_qd);
    float *hist = reinterpret_cast<float *>(ws + p.off_hist);
    float *ml = reinterpret_cast<float *>(ws + p.off_ml);
    float *acc = reinterpret_cast<float *>(ws + p.off_acc);

    if (a.rope_base > 0.0f) {
        const hipError_t e = launch_stream_rope(a, p, hist, ml);
        if (e != hipSuccess) return e;
    } else {
    {
        const dim3 grid((unsigned)((a.N + kQdAtoms - 1) / kQdAtoms), (unsigned)a.Hkv);
#define CSR_QD(TQ, TD)                                                                              \
    hipLaunchKernelGGL((qd_kernel<TQ, TD>), grid, dim3(256), 0, a.stream, (const TQ *)a.q,          \
                       (const TD *)a.DK, qd, a.B, a.Hq, a.Hkv, a.G, p.GB, a.N, a.scale)
        const int BG = a.B * a.G;
        if (a.q16 && a.dict16 && a.snK == 1 && BG <= 8) {
            const dim3 rgrid((unsigned)((a.N + 127) / 128), (unsigned)a.Hkv);
#define CSR_QDR(NQ)                                                                                        \
    hipLaunchKernelGGL((qd_rows_kernel<NQ>), rgrid, dim3(256), 0, a.stream, (const __half *)a.q,           \
                       (const __half *)a.DK, qd, a.B, a.Hq, a.Hkv, a.G, p.GB, a.N, a.scale)
            if (BG <= 1) CSR_QDR(1); else if (BG <= 2) CSR_QDR(2); else if (BG <= 4) CSR_QDR(4); else CSR_QDR(8);
#undef CSR_QDR
        } else if (a.q16 && a.dict16) {
            const int NT = a.snK * a.N;
            if ((int64_t)((NT + 128 * kQdTiles - 1) / (128 * kQdTiles)) * a.Hkv >= 256) {
                const dim3 mgrid((unsigned)((NT + 128 * kQdTiles - 1) / (128 * kQdTiles)), (unsigned)a.Hkv);
                hipLaunchKernelGGL(qd_mfma_kernel<kQdTiles>, mgrid, dim3(256), 0, a.stream, (const __half *)a.q,
                                   (const __half *)a.DK, qd, a.B, a.Hq, a.Hkv, a.G, p.GB, a.N, a.snK, a.scale);
            } else {   // few KV heads: one tile per wave, twice the workgroups
                const dim3 mgrid((unsigned)((NT + 127) / 128), (unsigned)a.Hkv);
                hipLaunchKernelGGL(qd_mfma_kernel<1>, mgrid, dim3(256), 0, a.stream, (const __half *)a.q,
                                   (const __half *)a.DK, qd, a.B, a.Hq, a.Hkv, a.G, p.GB, a.N, a.snK, a.scale);
            }
        } else if (a.q16) CSR_QD(__half, float);
        else if (a.dict16) CSR_QD(float, __half);
        else CSR_QD(float, float);
#undef CSR_QD
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        hipError_t e;
        switch (p.GB) {
            case 4: e = launch_stream_gb<4>(a, p, qd, hist, ml); break;
            case 2: e = launch_stream_gb<2>(a, p, qd, hist, ml); break;
            default: e = launch_stream_gb<1>(a, p, qd, hist, ml); break;
        }
        if (e != hipSuccess) return e;
    }
    }
    const int out_atoms = a.dict16 ? kOutAtomsF16 : kOutAtomsF32;
    const int nslices = (a.snV * a.N + out_atoms - 1) / out_atoms;
    {
        const int BG = a.B * a.G;
        const int nq = BG >= 8 ? 8 : (BG >= 4 ? 4 : (BG >= 2 ? 2 : 1));
        const dim3 grid((unsigned)nslices, (unsigned)a.Hkv, (unsigned)((BG + nq - 1) / nq));
#define CSR_OUT(TD, ATOMS, NQ)                                                                                   \
    hipLaunchKernelGGL((out_kernel<TD, ATOMS, NQ>), grid, dim3(256), 0, a.stream, (const TD *)a.DV, hist, ml, acc, \
                       a.B, a.Hkv, a.G, p.GB, a.N, a.snV, p.nchunks)
#define CSR_OUT_NQ(TD, ATOMS)                                                                                    \
    switch (nq) {                                                                                                \
        case 8: CSR_OUT(TD, ATOMS, 8); break;                                                                    \
        case 4: CSR_OUT(TD, ATOMS, 4); break;                                                                    \
        case 2: CSR_OUT(TD, ATOMS, 2); break;                                                                    \
        default: CSR_OUT(TD, ATOMS, 1); break;                                                                   \
    }
#define CSR_OUTR(NQ)                                                                                              \
    hipLaunchKernelGGL((out_rows_kernel<NQ>), grid, dim3(256), 0, a.stream, (const __half *)a.DV, hist, ml, acc, a.B, \
                       a.Hkv, a.G, p.GB, a.N, p.nchunks)
        if (a.dict16 && a.snV == 1 && BG >= 16 && a.N % 128 == 0) {   // many pairs per KV head: matrix cores
            const dim3 mgrid((unsigned)nslices, (unsigned)a.Hkv, (unsigned)((BG + kOutMfmaPairs - 1) / kOutMfmaPairs));
            if (p.nchunks <= 4)
                hipLaunchKernelGGL(out_mfma_kernel<4>, mgrid, dim3(256), 0, a.stream, (const __half *)a.DV, hist, ml, acc,
                                   a.B, a.Hkv, a.G, p.GB, a.N, p.nchunks);
            else
                hipLaunchKernelGGL(out_mfma_kernel<8>, mgrid, dim3(256), 0, a.stream, (const __half *)a.DV, hist, ml, acc,
                                   a.B, a.Hkv, a.G, p.GB, a.N, p.nchunks);
        } else if (a.dict16 && a.snV == 1 && nq == 1) {   // measured faster for one pair per KV head only
            CSR_OUTR(1);
        } else if (a.dict16) { CSR_OUT_NQ(__half, kOutAtomsF16) } else { CSR_OUT_NQ(float, kOutAtomsF32) }
#undef CSR_OUTR
#undef CSR_OUT_NQ
#undef CSR_OUT
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        const dim3 grid((unsigned)(a.B * a.Hq));
        if (a.out16)
            hipLaunchKernelGGL((finalize_kernel<__half>), grid, dim3(256), 0, a.stream, acc, ml, (__half *)a.out,
                               a.B, a.Hq, a.Hkv, a.G, p.GB, p.nchunks, nslices);
        else
            hipLaunchKernelGGL((finalize_kernel<float>), grid, dim3(256), 0, a.stream, acc, ml, (float *)a.out,
                               a.B, a.Hq, a.Hkv, a.G, p.GB, p.nchunks, nslices);
        return hipGetLastError();
    }
}

}  // namespace csr
