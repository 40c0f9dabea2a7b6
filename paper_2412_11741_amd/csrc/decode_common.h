// Device helpers and launch constants shared by the decode kernels (decode.hip, decode_rope.hip).
#pragma once
#include <type_traits>

#include "csr_internal.h"

namespace csr {
namespace dec {

// Threads of a workgroup of the position-free streaming kernel = tokens per round: 16 waves (enough loads in flight
// with one workgroup per CU) of 128 registers each.
constexpr int kStreamThreads = 1024;
constexpr int kMaxDevices = 64;      // devices a process may use this library on
// Rounds per chunk: a thread keeps the scores of its tokens (one per round and query head) in registers.  With four
// query heads per workgroup only 8 (32 of the 128 registers) ...
constexpr int max_rounds(int GB) { return GB == 4 ? 8 : 16; }
// ... which makes long contexts many short chunks, and every chunk costs a fixed 10 us (dispatch, table load, histogram
// clear and read-out, checks).  For those the four-head kernel has a second shape: 8 waves of 256 registers keep 32
// rounds - chunks of 16384 tokens, like the other variants' (measured at 8 sequences x 8 KV heads x 131072 tokens:
// 185 against 211 us per call).  Built for the paper's storage types with 8 pairs per code.
constexpr int kLongThreads4 = 512;
constexpr int kLongRounds4 = 32;
constexpr int kMaxChunks = 128;
// The rotary-key kernel (decode_rope.hip).  One query head at a time: 16 waves with 128 registers each; a query group
// keeps a rebuilt key and the group's scores in registers: 8 waves with 256 each.
constexpr int rope_threads(int GB) { return GB >= 2 ? 512 : 1024; }  // tokens per round
// rounds a chunk may have: one score per round and query head stays in registers
constexpr int rope_rounds(int GB) { return GB == 2 ? 16 : 8; }
// the rotary-key kernel keeps the key dictionary of its KV head in LDS when it fits (at most 512 atoms of 128 halves)
constexpr bool rope_dictionary_fits_lds(int N) { return (size_t)N * 256 <= 128 * 1024; }
constexpr size_t kRopeTableBytes = 8 * 32 * 4 + 8 * 4 * 8 * 4 + 64 * 8;  // rotation constants, a group's query pairs, theta
constexpr size_t kLdsBudget = 150 * 1024;
// Reduction scratch of the streaming kernels, in 4-byte words behind the table / histogram (WAVES <= 16, GB <= 4):
constexpr int kRedMax = 0;     // [WAVES][GB]  wave maxima of the scores
constexpr int kRedCm = 64;     // [WAVES]      wave maxima of the sampled |value coefficients|
constexpr int kRedL = 80;      // [WAVES][GB]  wave sums of p
constexpr int kRedChk = 144;   // [WAVES][12]  the scatter's self-check: see finish_chunk
constexpr int kRedWords = 144 + 16 * 12;
constexpr size_t kRedBytes = 2048;
static_assert(kRedWords * 4 <= kRedBytes, "reduction scratch");

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
__device__ __forceinline__ void load8_raw(const uint4 &raw, float (&o)[8])   // 8 packed halves, already in registers
{
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

// Cross-lane reductions without the LDS (whose time these kernels are short of): data-parallel-primitive moves
// inside a row of 16 lanes, lane reads across the four rows.  The order of the operations is fixed.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_mov(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) { return __uint_as_float(dpp_mov<CTRL>(__float_as_uint(v))); }
template <int CTRL> __device__ __forceinline__ unsigned long long dpp_mov(unsigned long long v)
{
    return ((unsigned long long)dpp_mov<CTRL>((uint32_t)(v >> 32)) << 32) | dpp_mov<CTRL>((uint32_t)v);
}
// every lane gets op over its group of LANES (4, 8 or 16) neighbouring lanes
template <int LANES, typename T, typename Op> __device__ __forceinline__ T row_reduce(T v, Op op)
{
    v = op(v, dpp_mov<0xB1>(v));                            // quad_perm [1,0,3,2]
    v = op(v, dpp_mov<0x4E>(v));                            // quad_perm [2,3,0,1]
    if constexpr (LANES >= 8) v = op(v, dpp_mov<0x141>(v));  // row_half_mirror: the other quad of every 8
    if constexpr (LANES >= 16) v = op(v, dpp_mov<0x140>(v)); // row_mirror: the other half of the row
    return v;
}
__device__ __forceinline__ uint32_t lane_read(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }
__device__ __forceinline__ float lane_read(float v, int l) { return __uint_as_float(lane_read(__float_as_uint(v), l)); }
__device__ __forceinline__ unsigned long long lane_read(unsigned long long v, int l)
{
    return ((unsigned long long)lane_read((uint32_t)(v >> 32), l) << 32) | lane_read((uint32_t)v, l);
}
template <typename T, typename Op> __device__ __forceinline__ T wave_reduce(T v, Op op)
{
    v = row_reduce<16>(v, op);
    return op(op(lane_read(v, 0), lane_read(v, 16)), op(lane_read(v, 32), lane_read(v, 48)));
}
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpAdd { template <typename T> __device__ __forceinline__ T operator()(T a, T b) const { return a + b; } };
struct OpOr { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a | b; } };
__device__ __forceinline__ float wave_max(float v) { return wave_reduce(v, OpMax()); }
__device__ __forceinline__ float wave_sum(float v) { return wave_reduce(v, OpAdd()); }

// x as a 64-bit fixed-point number in units of 2^-32 (two's complement), rounded to the nearest unit; |x| must
// stay below 2^31 (the integer part is saturated there rather than wrapped).  fl = floor(x) and x - fl are exact in
// fp32, but x - fl can be exactly 1 (a tiny negative x), so the scaled fraction is kept below 2^32 before the
// conversion; adding one half only matters where the scaled fraction still has fraction bits (below 2^23).  The
// caller scales p * c by a power of two first (see stream_kernel), so that the unit follows the data and the
// result does not depend on the scale of the coefficients.
__device__ __forceinline__ unsigned long long to_fixed(float x)
{
    const float fl = floorf(fminf(fmaxf(x, -2147483648.0f), 2147483520.0f));
    const int hi = (int)fl;
    const unsigned lo = (unsigned)fminf((x - fl) * 4294967296.0f + 0.5f, 4294967040.0f);
    return ((unsigned long long)(unsigned)hi << 32) | lo;
}
__device__ __forceinline__ float from_fixed(unsigned long long v)
{
    return (float)(int)(unsigned)(v >> 32) + (float)(unsigned)(v & 0xffffffffull) * 2.3283064365386963e-10f;
}

// ---------------------------------------------------------------------------------------------
// The V side of a chunk, common to the streaming kernels (position-free and rotary keys): softmax weights of
// the chunk's tokens, the scatter of p * c of the value codes into the LDS histogram (D4), and the chunk's
// histogram (fp32), maximum and sum of weights to scratch.
//
// The histogram is fixed point, summed with integer LDS atomics: integer sums are exact, so the result does
// not depend on the order in which the hardware serves the adds, and the float atomic add of this LDS is
// serialised lane by lane.  Fast form: 32-bit adds (1.7 times the rate of 64-bit ones).  Every query head has
// bins [n][sign]: p >= 0, so the sign of an add is the sign of its coefficient, and with the magnitudes of the
// two signs kept apart every bin only grows - an overflow (a wrap, or a bin beyond 2^31) cannot cancel and is
// found exactly: the bins' total is compared with the total the threads add up themselves (in fp32, to 2^-17
// relative: a wrap is off by 2^32), and every bin is looked at when it is read out.  The unit is a power of two
// per query head chosen BEFORE the scatter from what is known then - the sum l of the weights and the largest
// |coefficient| among the chunk's first tokens: 2^-28 .. 2^-27 of c_est * max(1, l s / N) (the |p c| an average bin
// would collect if every coefficient were the largest sampled one), which leaves 8- to 16-fold headroom over that.
// After the scatter two things are checked:
//   * no overflow (above);
//   * resolution: the rounding of the n adds to the unit (each within half a unit, signs random) perturbs the
//     histogram by about unit * sqrt(n / 12) in the 2-norm; that must stay below 2^-15 of the histogram's own
//     2-norm (taken at the read-out): 3e-5, a thirtieth of the tolerance of the whole call.
// If either fails - coefficients far larger than the sampled ones, a hot atom hit by most tokens, weights and
// coefficients spanning more than the 32 bits can hold - the scatter is repeated ONCE in the wide form: 64-bit
// bins [n] in units of 2^-62 .. 2^-61 of the total |p c| just measured, which can neither overflow nor lose
// anything an fp32 product carries.  The decision depends on exact sums and on fp32 sums formed in a fixed
// order, so it is the same on every run, and so are the output bits.
//
// sc[i][g]: score of the token this thread owns in round i (token t0 + i * THREADS + owner_off), -inf if none.
// VL > 0: the value code of a token is VL 16-byte vectors of indices and of coefficients (16-bit indices, fp16
// coefficients, whole-vector codes): they are then requested PF rounds ahead of their use.
template <int VL> struct CodeVec { uint4 i[VL > 0 ? VL : 1], c[VL > 0 ? VL : 1]; };
// Rounds whose code vectors are requested ahead: two where the registers allow it without spilling (one query head
// per workgroup, one vector per code: what bounds that kernel is the number of bytes in flight per CU), else one.
template <int GB, int TPT, int VL> constexpr int prefetch_rounds() { return GB == 1 && VL == 1 && TPT >= 4 ? 2 : 1; }

// The code streams of a thread's tokens, walked round by round: two workgroup-uniform base addresses (the code
// vectors of the chunk's first token) and one 32-bit offset per thread, in 16-byte vectors.  The offset passes
// through an empty asm statement at every step, so that the compiler cannot work out all rounds' addresses ahead of
// time (they would occupy registers from the start of the loop).
template <int VL, int THREADS> struct CodeWalk {
    const uint4 *ib, *cb;   // uniform
    uint32_t off;           // this thread's token of the round the walk stands at, times VL
    __device__ __forceinline__ CodeWalk(const void *idx, const void *coef, int64_t first_token, int owner_off)
        : ib(reinterpret_cast<const uint4 *>(idx) + first_token * (VL > 0 ? VL : 1)),
          cb(reinterpret_cast<const uint4 *>(coef) + first_token * (VL > 0 ? VL : 1)),
          off((uint32_t)owner_off * (VL > 0 ? VL : 1)) {}
    __device__ __forceinline__ void next()
    {
        off += THREADS * (VL > 0 ? VL : 1);
        asm volatile("" : "+v"(off));
    }
};
// Requests the 16-byte code vectors of the token the walk stands at.  Without such a token (`have` false: past the
// end of the chunk) the chunk's first token is requested instead and the caller ignores what arrives: a request
// under a branch would make the destination registers the meeting point of two paths, and the compiler then copies
// them - and waits for the request - right behind it.
template <int VL, int THREADS>
__device__ __forceinline__ void fetch_codes(CodeVec<VL> &r, const CodeWalk<VL, THREADS> &w, bool have)
{
    const uint32_t o = have ? w.off : 0u;
#pragma unroll
    for (int v = 0; v < (VL > 0 ? VL : 1); ++v) {
        if constexpr (VL > 0) { r.i[v] = w.ib[o + v]; r.c[v] = w.cb[o + v]; }
        else r.i[v] = r.c[v] = make_uint4(0u, 0u, 0u, 0u);
    }
}
// The code vectors of the current round must have arrived BEFORE a later round's request is issued: the empty asm
// statements make the compiler place the wait for them here, where only older requests are outstanding, instead of
// behind the new request, where it would wait for both.
template <int VL>
__device__ __forceinline__ void await_codes(CodeVec<VL> &cur)
{
#pragma unroll
    for (int v = 0; v < (VL > 0 ? VL : 1); ++v) {
        asm volatile("" : "+v"(cur.i[v].x), "+v"(cur.i[v].y), "+v"(cur.i[v].z), "+v"(cur.i[v].w));
        asm volatile("" : "+v"(cur.c[v].x), "+v"(cur.c[v].y), "+v"(cur.c[v].z), "+v"(cur.c[v].w));
    }
}
__device__ __forceinline__ void unpack8(const uint4 &ri, const uint4 &rc, int (&id)[8], float (&cf)[8])
{
    id[0] = ri.x & 0xffff; id[1] = ri.x >> 16; id[2] = ri.y & 0xffff; id[3] = ri.y >> 16;
    id[4] = ri.z & 0xffff; id[5] = ri.z >> 16; id[6] = ri.w & 0xffff; id[7] = ri.w >> 16;
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&rc);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 f = __half22float2(h2[j]);
        cf[2 * j] = f.x;
        cf[2 * j + 1] = f.y;
    }
}

// A thread keeps one value per round and query head in registers, sc[round][head]: the loops over the rounds are
// fully unrolled (registers cannot be indexed by a loop counter).  Left alone, the compiler then pulls the loads and
// address arithmetic of all rounds ahead until it spills; round_fence() between two rounds keeps memory accesses on
// their side of it, so that only the explicitly requested vectors (fetch_codes) are in flight.
__device__ __forceinline__ void round_fence() { asm volatile("" ::: "memory"); }

template <int GB, typename TI, typename TC, int PV, bool CH, int TPT, int THREADS, int VL>
__device__ __forceinline__ void finish_chunk(unsigned char *smem_raw, float *red, float (&sc)[TPT][GB], const float (&mx)[GB],
                                             int n_mine, int64_t t0, int64_t t_end, int64_t code_row, int owner_off,
                                             const TI *__restrict__ idxV, const TC *__restrict__ coefV, int32_t N,
                                             int32_t sV, int32_t snV_arg, float *ml, float *part_hist, int64_t slot)
{
    constexpr int WAVES = THREADS / 64;
    static_assert(WAVES <= 16 && GB <= 4, "layout of the reduction scratch");
    static_assert(VL == 0 || (sizeof(TI) == 2 && sizeof(TC) == 2 && PV == 8 && !CH), "16-byte code vectors");
    const int snV = CH ? snV_arg : 1;
    // 32-bit form: |sum| of c > 0 and of c < 0 per (query head, atom).  [g][n][sign]; for an even number of heads
    // [g / 2][n][sign][g % 2]: the bins of two heads side by side, so that ONE 64-bit add serves both (a loop of 16
    // ds_add_u64 takes 8 % less LDS time than one of 32 ds_add_u32, and the second head needs no address).  A bin that
    // wraps then carries into its neighbour's - which the check of the totals finds like any other wrap (the sum of
    // all bins is off by 2^32 - 1).
    constexpr bool PAIRED = GB % 2 == 0;
    uint32_t *h32 = reinterpret_cast<uint32_t *>(smem_raw);
    unsigned long long *h64 = reinterpret_cast<unsigned long long *>(smem_raw);  // wide form: [GB][NV]
    uint32_t *redw = reinterpret_cast<uint32_t *>(red);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NV = snV * N, sVt = snV * sV;
    const int bins = NV * GB;
    const int64_t tok0 = t0 + owner_off;  // this thread's token of round 0

    // ---- the chunk's maximum; a sample of the value coefficients (the first round's tokens) ---------------
    float cm = 0.0f;
    constexpr int PF = prefetch_rounds<GB, TPT, VL>();
    CodeVec<VL> ring[PF + 1];  // round i reads slot i % (PF + 1) while round i + PF is requested into the slot round i - 1 left
    auto prime = [&](CodeWalk<VL, THREADS> &w) {   // requests rounds 0 .. PF-1, leaves w at round PF
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            fetch_codes<VL, THREADS>(ring[k], w, k < n_mine && tok0 + (int64_t)k * THREADS < t_end);
            w.next();
        }
    };
    if constexpr (VL > 0) {
        CodeWalk<VL, THREADS> w0(idxV, coefV, code_row + t0, owner_off);
        prime(w0);
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        const float wm = wave_max(mx[g]);
        if (lane == 0) red[kRedMax + wave * GB + g] = wm;
    }
    if constexpr (VL > 0) {
#pragma unroll
        for (int v = 0; v < VL; ++v) {
            int id[8];
            float cf[8];
            unpack8(ring[0].i[v], ring[0].c[v], id, cf);
            if (n_mine > 0 && tok0 < t_end) {   // else the vectors are not this thread's
#pragma unroll
                for (int j = 0; j < 8; ++j) cm = fmaxf(cm, fabsf(cf[j]));
            }
        }
    } else {
        if (n_mine > 0 && tok0 < t_end) {
            const TC *vp = coefV + (code_row + tok0) * sVt;
            for (int j0 = 0; j0 < sVt; j0 += PV) {
                float cf[PV];
                CoefLoad<TC, PV>::ld(vp + j0, cf);
#pragma unroll
                for (int j = 0; j < PV; ++j) cm = fmaxf(cm, fabsf(cf[j]));
            }
        }
    }
    cm = wave_max(cm);
    if (lane == 0) red[kRedCm + wave] = cm;
    __syncthreads();  // every score is computed: the table (or the dictionary rows) is free
    // the waves' partial results meet: lane l takes wave l % WAVES's, a reduction inside rows of WAVES lanes follows
    const int wsel = lane & (WAVES - 1);
    float m_c[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) m_c[g] = row_reduce<WAVES>(red[kRedMax + wsel * GB + g], OpMax());
    const float c_est = row_reduce<WAVES>(red[kRedCm + wsel], OpMax());

    // ---- p = exp(score - max) in place of the scores, their sum; the histogram cleared -------------------
    float l_thr[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) l_thr[g] = 0.0f;
#pragma unroll
    for (int i = 0; i < TPT; ++i) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            const float p = (i < n_mine && sc[i][g] > -INFINITY) ? __expf(sc[i][g] - m_c[g]) : 0.0f;
            sc[i][g] = p;
            l_thr[g] += p;
        }
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        const float ws = wave_sum(l_thr[g]);
        if (lane == 0) red[kRedL + wave * GB + g] = ws;
    }
    {
        uint4 *z = reinterpret_cast<uint4 *>(smem_raw);
        const int n16 = (bins * 8 + 15) / 16;  // the table region is a multiple of 16 bytes
        for (int e = tid; e < n16; e += THREADS) z[e] = make_uint4(0u, 0u, 0u, 0u);
    }
    __syncthreads();
    int k_exp[GB];   // p is scattered as p * 2^k_exp
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        const float l = row_reduce<WAVES>(red[kRedL + wsel * GB + g], OpAdd());
        if (tid == g) { ml[2 * g] = m_c[g]; ml[2 * g + 1] = l; }
        const float b_est = c_est * fmaxf(1.0f, l * (float)sVt / (float)NV);
        k_exp[g] = 20;  // nothing sampled (or nothing finite): any unit will do, the checks below decide
        if (b_est > 0.0f && b_est < INFINITY) {
            int e2;
            (void)frexpf(b_est, &e2);  // b_est in [2^(e2-1), 2^e2)
            k_exp[g] = 28 - e2;        // b_est * 2^k in [2^27, 2^28)
        }
    }

    // ---- scatter ----------------------------------------------------------------------------------------
    float *dst = part_hist + slot * (int64_t)bins;
    const float n_adds = (float)(t_end - t0) * (float)sVt;
    bool wide = false;
#pragma unroll 1
    for (int attempt = 0; attempt < 2; ++attempt) {
        float scale[GB];
#pragma unroll
        for (int g = 0; g < GB; ++g) scale[g] = ldexpf(1.0f, k_exp[g]);
        float s_thr = 0.0f, m_thr = 0.0f;  // sum and maximum of p' * sum_j |c_j| over this thread's tokens and heads
        CodeWalk<VL, THREADS> walk(idxV, coefV, code_row + t0, owner_off);  // walks PF rounds ahead of the current one
        if constexpr (VL > 0) {
            if (attempt > 0) prime(walk);
            else {
#pragma unroll
                for (int k = 0; k < PF; ++k) walk.next();
            }
        }
        auto rounds = [&](auto wide_c) {
            constexpr bool WIDE = decltype(wide_c)::value;
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
                        float pp[GB];
#pragma unroll
                        for (int g = 0; g < GB; ++g) pp[g] = sc[i][g] * scale[g];
                        float a_t = 0.0f;
                        auto pairs = [&](int base, const int (&id)[PV], const float (&cf)[PV]) {
#pragma unroll
                            for (int j = 0; j < PV; ++j) {
                                const float ac = fabsf(cf[j]);
                                a_t += ac;
                                if constexpr (WIDE) {
#pragma unroll
                                    for (int g = 0; g < GB; ++g) atomicAdd(&h64[g * NV + base + id[j]], to_fixed(pp[g] * cf[j]));
                                } else {
                                    const int cell = 2 * (base + id[j]) + (int)(__float_as_uint(cf[j]) >> 31);
                                    if constexpr (PAIRED) {
#pragma unroll
                                        for (int g = 0; g < GB; g += 2) {
                                            const uint32_t a0 = __float2uint_rz(fmaf(pp[g], ac, 0.5f));
                                            const uint32_t a1 = __float2uint_rz(fmaf(pp[g + 1], ac, 0.5f));
                                            atomicAdd(h64 + cell + g * NV, ((unsigned long long)a1 << 32) | a0);
                                        }
                                    } else {
#pragma unroll
                                        for (int g = 0; g < GB; ++g)
                                            atomicAdd(h32 + cell + 2 * g * NV, __float2uint_rz(fmaf(pp[g], ac, 0.5f)));
                                    }
                                }
                                // one pair after the other (the next pair's products depend on this statement), so
                                // that the values of all 8 x GB adds are not computed ahead and held in registers
#pragma unroll
                                for (int g = 0; g < GB; ++g) asm volatile("" : "+v"(pp[g]));
                            }
                        };
                        if constexpr (VL > 0) {
#pragma unroll
                            for (int v = 0; v < VL; ++v) {
                                int id[8];
                                float cf[8];
                                unpack8(cur.i[v], cur.c[v], id, cf);
                                pairs(0, id, cf);
                            }
                        } else {
                            const TI *ip = idxV + (code_row + t) * sVt;
                            const TC *cp = coefV + (code_row + t) * sVt;
                            int base = 0;
                            for (int ch = 0; ch < snV; ++ch, base += N, ip += sV, cp += sV) {
                                for (int j0 = 0; j0 < sV; j0 += PV) {  // PV divides sV: a vector load stays in its chunk
                                    int id[PV];
                                    float cf[PV];
                                    IdxLoad<TI, PV>::ld(ip + j0, id);
                                    CoefLoad<TC, PV>::ld(cp + j0, cf);
                                    pairs(base, id, cf);
                                }
                            }
                        }
#pragma unroll
                        for (int g = 0; g < GB; ++g) {
                            const float pa = pp[g] * a_t;
                            s_thr += pa;
                            m_thr = fmaxf(m_thr, pa);
                        }
                    }
                }
            }
        };
        if (wide) rounds(std::true_type{});
        else rounds(std::false_type{});
        __syncthreads();  // all atomics landed

        // ---- read-out: histogram to scratch as fp32; the checks' sums on the way ------------------------
        if (wide) {
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                const float from_units = ldexpf(1.0f, -k_exp[g]);
                for (int e = tid; e < NV; e += THREADS) dst[g * NV + e] = from_fixed(h64[g * NV + e]) * from_units;
            }
            break;
        }
        unsigned long long tot = 0ull;  // this thread's bins added up
        uint32_t high = 0u;             // OR of this thread's bins
        float h2[GB];                   // squares of this thread's histogram entries, per query head
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            h2[g] = 0.0f;
            const float from_units = ldexpf(1.0f, -k_exp[g]);
            constexpr int U = 4;   // bins read together: the LDS round trips of a thread overlap
            for (int e0 = tid; e0 < NV; e0 += U * THREADS) {
                uint2 pn[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {   // past the end: bin 0, ignored below (no load under a branch)
                    const int e = e0 + u * THREADS;
                    const int ec = e < NV ? e : 0;
                    if constexpr (PAIRED) {
                        const uint32_t *c2 = h32 + 4 * ((g >> 1) * NV + ec) + (g & 1);
                        pn[u] = make_uint2(c2[0], c2[2]);
                    } else {
                        pn[u] = *reinterpret_cast<const uint2 *>(h32 + 2 * (g * NV + ec));
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = e0 + u * THREADS;
                    if (e < NV) {
                        tot += (unsigned long long)pn[u].x + pn[u].y;
                        high |= pn[u].x | pn[u].y;
                        const float v = (float)(int)(pn[u].x - pn[u].y);  // exact while both stay below 2^31
                        h2[g] = fmaf(v, v, h2[g]);
                        dst[g * NV + e] = v * from_units;
                    }
                }
            }
        }
        // per wave: s - tot (as integers: the sums are exact from here on), max single add, high bits, |hist|^2
        unsigned long long dif = wave_reduce((unsigned long long)fminf(s_thr, 1.0e19f) - tot, OpAdd());
        high = wave_reduce(high, OpOr());
        m_thr = wave_max(m_thr);
        const float s_wave = wave_sum(fminf(s_thr, 1.0e19f));
#pragma unroll
        for (int g = 0; g < GB; ++g) h2[g] = wave_sum(h2[g]);
        if (lane == 0) {
            uint32_t *c = redw + kRedChk + wave * 12;
            c[0] = (uint32_t)dif; c[1] = (uint32_t)(dif >> 32);
            c[2] = __float_as_uint(s_wave);
            c[4] = __float_as_uint(m_thr); c[5] = high;
#pragma unroll
            for (int g = 0; g < GB; ++g) c[6 + g] = __float_as_uint(h2[g]);
        }
        __syncthreads();
        const uint32_t *c = redw + kRedChk + wsel * 12;
        const unsigned long long DIF = row_reduce<WAVES>(((unsigned long long)c[1] << 32) | c[0], OpAdd());
        const float M = row_reduce<WAVES>(__uint_as_float(c[4]), OpMax());
        const float S_f = row_reduce<WAVES>(__uint_as_float(c[2]), OpAdd());
        const uint32_t HIGH = row_reduce<WAVES>(c[5], OpOr());
        float H2[GB];
#pragma unroll
        for (int g = 0; g < GB; ++g) H2[g] = row_reduce<WAVES>(__uint_as_float(c[6 + g]), OpAdd());
        const long long diff = (long long)DIF;
        bool ok = HIGH < 0x80000000u && M < 2147483648.0f && diff < 2147483648ll && diff > -2147483648ll;
        // resolution: unit * sqrt(n / 12) against 2^-15 |hist|, both in units (an all-zero histogram passes)
#pragma unroll
        for (int g = 0; g < GB; ++g) ok = ok && (n_adds * (1.0f / 12.0f) * 1073741824.0f <= H2[g] || M == 0.0f);
        if (ok) break;
        // wide form: the integer part of an add counts 2^32 units; all adds of a head together stay below 2^30 of
        // them.  S is the total over the heads in units of 2^-k_exp (as a float it may have saturated: then the
        // maximum single add, which has not, gives the scale)
        wide = true;
        const float total = fmaxf(S_f, M) * 1.0001f;
        int e2 = 0;
        if (total > 0.0f && total < INFINITY) (void)frexpf(total, &e2);  // total < 2^e2
#pragma unroll
        for (int g = 0; g < GB; ++g) k_exp[g] += 30 - e2;
        {
            uint4 *z = reinterpret_cast<uint4 *>(smem_raw);
            const int n16 = (bins * 8 + 15) / 16;
            for (int e = tid; e < n16; e += THREADS) z[e] = make_uint4(0u, 0u, 0u, 0u);
        }
        __syncthreads();
    }
}

}  // namespace dec
}  // namespace csr
