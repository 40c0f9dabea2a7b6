// Matching Pursuit encoder with the Gram-matrix residual update for FEW vectors per LARGE dictionary (gfx950): the
// tokens generated in one decoding step, which Section "KV Decomposition and Sparse Storage" encodes like the
// prompt's (Eq.2-4 of Section "Sparse representation", s iterations).
//
// With one vector per dictionary every iteration of Eq.2 is a matrix-vector product that reads the whole dictionary
// (1 MB at N = 4096): s sweeps of every dictionary per generated token.  All correlations obey
//     C_{g+1}[n] = (R_g - c_g d_i) . d_n = C_g[n] - c_g G[i][n],        G = D D^T,
// so with G prepared once per dictionary (csr_gram_build: N x N fp16 in device memory, 32 MB at N = 4096) only the
// first iteration sweeps the dictionary; each later one reads ONE row of G (2 N bytes) per vector.
//
//   launch 1, sweep_kernel, workgroup (dictionary, 256-atom slice): C_1[n] = x . d_n for the dictionary's vectors
//       (exact fp16 products, fp32 sums) into scratch, and the slice's largest squared atom norm.  Up to 8 vectors
//       per dictionary on the vector ALU (the launch is bound by reading the dictionaries), more on the matrix cores.
//   launch 2, iterate_kernel, one workgroup per vector (8 waves when few vectors wait and the length of the chain
//       counts, 2 or 4 from 12 vectors per dictionary on, when instruction issue does): the correlations live in
//       registers (8 consecutive atoms per thread and round), the fp32 residual R in every wave.  Per iteration: block arg-max of |C|; the row of G and
//       of D of that atom are requested at once; every atom whose |C| lies within 2 delta of the maximum is a
//       candidate, and the candidates' R . d are evaluated in fp32 from the atoms themselves (largest wins, lowest
//       atom on ties) - the recursion only SCREENS, as the fp16 sweeps of the other encoders do:
//           |C_g[n] - R_g . d_n| <= delta_g,   delta_1 = gamma |x| dmax,
//           delta_{g+1} = delta_g + |c_g| (dmax^2 (2^-12 + gamma) + 2^-25) + 2^-22 rmax dmax
//       (gamma bounds the fp32 accumulation of a dot product of exact fp16 products; |G| <= dmax^2; 2^-25 covers
//       fp16-subnormal entries of G; rmax is the largest residual norm so far: the last term is the rounding of the
//       fp32 residual and of the recursion itself).  More candidates than the list holds (a residual that is almost orthogonal to
//       everything, a dictionary of equal atoms): all N atoms are evaluated.  Then Eq.4 on R with the unrounded
//       coefficient, and the recursion on C.
#include "csr_internal.h"
#include "encode_common.h"

namespace csr {
namespace {

using namespace enc;

constexpr int kSweepThreads = 256;
constexpr int kSliceAtoms = 256;        // atoms per sweep workgroup
constexpr int kIterThreadsMax = 512;     // threads of an iterate workgroup: 512 when few vectors wait (the chain of an
                                        // iteration is shortest), 128 or 256 from kThroughputVectors per dictionary on
                                        // (what every wave repeats - merge, coefficient, residual - is done by fewer)
constexpr int kThroughputVectors = 12;
constexpr int kMaxRounds = 4;           // rounds of 8 atoms per thread: N <= 512 * 8 * 4
constexpr int kMaxAtoms = kIterThreadsMax * 8 * kMaxRounds;  // 16384
constexpr int kMaxVectors = 128;        // per dictionary: a decoding step of up to 128 sequences
constexpr int kValuSweepVectors = 8;    // up to here the sweep is a matrix-vector product on the vector ALU
constexpr int kSweepTiles = 2;          // 32-atom tiles per wave of the matrix-core sweep (4 waves: 256 atoms)
static_assert(kSliceAtoms == (kSweepThreads / 64) * 32 * kSweepTiles, "a sweep workgroup covers one slice");
constexpr int kCand = 256;              // candidate list; beyond it every atom is evaluated

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(*reinterpret_cast<const half2v *>(&a), *reinterpret_cast<const half2v *>(&b), c, false);
}
__device__ __forceinline__ float dot8(const uint4 &a, const uint4 &b)
{
    return dot2(a.w, b.w, dot2(a.z, b.z, dot2(a.y, b.y, dot2(a.x, b.x, 0.0f))));
}
template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// sum over the LPR (8 or 16) consecutive lanes that hold one row; every one of them gets it
template <int LPR> __device__ __forceinline__ float row_sum(float v)
{
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror: lane i of every 8 with lane 7 - i
    if (LPR == 16) v = dpp_add<0x140>(v);  // row_mirror: lane i of every 16 with lane 15 - i
    return v;
}

// (a1 >= a2 >= 0), the two largest of a set, merged with those of the lane that the DPP pattern names (a disjoint set;
// rows outside ROWS keep their own): the two largest of the union
template <int CTRL, int ROWS> __device__ __forceinline__ void top2_dpp(float &a1, float &a2)
{
    const float o1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(a1), CTRL, ROWS, 0xf, false));
    const float o2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(a2), CTRL, ROWS, 0xf, false));
    a2 = fmaxf(fmaxf(a2, o2), fminf(a1, o1));
    a1 = fmaxf(a1, o1);
}
// R . d in fp32 for the row whose 8-dimension piece this lane holds (R the same piece); all LPR lanes get the sum
template <int LPR> __device__ __forceinline__ float exact_dot(const float (&R)[8], const uint4 &raw)
{
    float dn[8];
    unpack8(raw, dn);
    float c = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) c = fmaf(R[e], dn[e], c);
    return row_sum<LPR>(c);
}

// where vector m (0 .. M-1) of dictionary dct lives: blocks that share a dictionary are numbered one after the other
struct VecAt {
    int64_t x_off;   // elements from X to the chunk
    int64_t code;    // elements from idx / coef to its first pair
    int64_t norm;    // elements from res_norm2
};
__device__ __forceinline__ VecAt locate(int dct, int64_t m, int64_t T, int sn, int s, int DC, int dict_count, int64_t x_stride_h,
                                        int64_t x_stride_t, int64_t code_stride_h)
{
    const int dict = dct / sn, ch = dct - dict * sn;
    const int64_t rep = m / T, tok = m - rep * T;
    const int64_t h = rep * dict_count + dict;
    VecAt v;
    v.x_off = h * x_stride_h + tok * x_stride_t + (int64_t)ch * DC;
    v.code = h * code_stride_h + (tok * sn + ch) * s;
    v.norm = (h * T + tok) * sn + ch;
    return v;
}

// ---- G = D D^T, fp16, row-major [dictionary][N][N] -------------------------------------------------------------------
// v_mfma_f32_16x16x32_f16: lane (col = lane % 16, q = lane / 16) supplies dimensions 8 q .. 8 q + 7 of every
// 32-dimension slice of row col of both operands and receives the products of rows 4 q .. 4 q + 3 of A with row col
// of B.  A wave owns 16 rows i of G and walks the 16-atom tiles t of the columns.
template <int DC>
__global__ __launch_bounds__(256) void gram_build_kernel(const __half *__restrict__ Dict, __half *__restrict__ G, int32_t N)
{
    constexpr int kF = DC / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, q = lane >> 4;
    const int ntile = N >> 4;
    const int rb = blockIdx.x * 4 + wave;
    if (rb >= ntile) return;  // (wave-uniform; no barriers in this kernel)
    const __half *Dh = Dict + (int64_t)blockIdx.y * N * DC;
    __half *Gd = G + (int64_t)blockIdx.y * N * N;
    auto atom_frag = [&](int n, int f) { return *reinterpret_cast<const half8 *>(Dh + (int64_t)n * DC + 32 * f + 8 * q); };
    const int i = 16 * rb + col;
    half8 bfr[kF];
#pragma unroll
    for (int f = 0; f < kF; ++f) bfr[f] = atom_frag(i, f);
    for (int t = 0; t < ntile; ++t) {
        floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int f = 0; f < kF; ++f) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(atom_frag(16 * t + col, f), bfr[f], acc, 0, 0, 0);
        // acc[e] = d_n . d_i for n = 16 t + 4 q + e
        const __half2 p0 = __floats2half2_rn(acc[0], acc[1]), p1 = __floats2half2_rn(acc[2], acc[3]);
        uint2 w;
        w.x = *reinterpret_cast<const uint32_t *>(&p0);
        w.y = *reinterpret_cast<const uint32_t *>(&p1);
        *reinterpret_cast<uint2 *>(Gd + (int64_t)i * N + 16 * t + 4 * q) = w;
    }
}

// ---- launch 1: C_1 and the atom norms ----------------------------------------------------------------------------------
// LPR = DC / 8 lanes read one atom row (16 bytes each), 64 / LPR rows per wave and load.
template <int DC>
__global__ __launch_bounds__(kSweepThreads) void sweep_kernel(const __half *__restrict__ X, const __half *__restrict__ Dict,
                                                              float *__restrict__ Cbuf, float *__restrict__ dmax2_part, int64_t T,
                                                              int32_t M, int32_t N, int32_t s, int32_t sn, int64_t x_stride_h,
                                                              int64_t x_stride_t, int32_t dict_count, int32_t nslices)
{
    constexpr int LPR = DC / 8, RPW = 64 / LPR;
    __shared__ float red[kSweepThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int piece = lane % LPR, rg = lane / LPR;
    const int dct = blockIdx.x / nslices, sl = blockIdx.x - dct * nslices;
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    float nmax = 0.0f;
    for (int m0 = 0; m0 < M; m0 += 8) {
        uint4 xp[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            xp[j] = make_uint4(0u, 0u, 0u, 0u);
            if (m0 + j < M) {
                const VecAt v = locate(dct, m0 + j, T, sn, s, DC, dict_count, x_stride_h, x_stride_t, 0);
                xp[j] = *reinterpret_cast<const uint4 *>(X + v.x_off + 8 * piece);
            }
        }
        for (int r0 = sl * kSliceAtoms + wave * RPW; r0 < (sl + 1) * kSliceAtoms; r0 += (kSweepThreads / 64) * RPW) {
            const int r = r0 + rg;
            const int rc = r < N ? r : N - 1;  // the last slice may be ragged: those lanes recompute the last atom
            const uint4 dr = *reinterpret_cast<const uint4 *>(Dh + (int64_t)rc * DC + 8 * piece);
            if (m0 == 0) nmax = fmaxf(nmax, row_sum<LPR>(dot8(dr, dr)));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (m0 + j < M) {  // (uniform)
                    const float c = row_sum<LPR>(dot8(xp[j], dr));
                    if (piece == 0 && r < N) Cbuf[((int64_t)dct * M + m0 + j) * N + r] = c;
                }
            }
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) nmax = fmaxf(nmax, __shfl_xor(nmax, m, 64));
    if (lane == 0) red[wave] = nmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        float v = red[0];
        for (int w = 1; w < kSweepThreads / 64; ++w) v = fmaxf(v, red[w]);
        dmax2_part[(int64_t)dct * nslices + sl] = v;
    }
}

// The same launch for more than a handful of vectors per dictionary, on the matrix cores: v_mfma_f32_32x32x16_f16 with
// 32 vectors as the rows of A and 32 atoms as the columns of B.  Lane (col = lane % 32, hf = lane / 32) supplies
// dimensions 16 j + 8 hf .. + 7 of step j for vector col (A) and atom col (B) - 16 contiguous bytes of a row per step -
// and receives, in accumulator 4 r4 + e, the product of vector 8 r4 + 4 hf + e with atom col.  A wave keeps the rows
// of its kSweepTiles tiles in registers and walks the vectors 32 at a time.
template <int DC>
__global__ __launch_bounds__(kSweepThreads) void sweep_mfma_kernel(const __half *__restrict__ X, const __half *__restrict__ Dict,
                                                                   float *__restrict__ Cbuf, float *__restrict__ dmax2_part, int64_t T,
                                                                   int32_t M, int32_t N, int32_t s, int32_t sn, int64_t x_stride_h,
                                                                   int64_t x_stride_t, int32_t dict_count, int32_t nslices)
{
    constexpr int NF = DC / 16;  // matrix-core steps per product
    __shared__ float red[kSweepThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, hf = lane >> 5;
    const int dct = blockIdx.x / nslices, sl = blockIdx.x - dct * nslices;
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    const int n_first = sl * kSliceAtoms + wave * 32 * kSweepTiles;
    float nmax = 0.0f;
    half8 bfrag[kSweepTiles][NF];
#pragma unroll
    for (int t = 0; t < kSweepTiles; ++t) {
        const int n = n_first + 32 * t + col;
        const int nc = n < N ? n : N - 1;  // the last slice may be ragged: those lanes hold the last atom again
        float nn = 0.0f;
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)nc * DC + 16 * j + 8 * hf);
            bfrag[t][j] = *reinterpret_cast<const half8 *>(&raw);
            nn += dot8(raw, raw);
        }
        nn += __shfl_xor(nn, 32, 64);  // the other half of the atom's dimensions
        nmax = fmaxf(nmax, nn);
    }
    for (int v0 = 0; v0 < M; v0 += 32) {
        const int m = v0 + col;
        half8 afrag[NF];
        {
            const VecAt at = locate(dct, m < M ? m : M - 1, T, sn, s, DC, dict_count, x_stride_h, x_stride_t, 0);
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                uint4 raw = make_uint4(0u, 0u, 0u, 0u);
                if (m < M) raw = *reinterpret_cast<const uint4 *>(X + at.x_off + 16 * j + 8 * hf);
                afrag[j] = *reinterpret_cast<const half8 *>(&raw);
            }
        }
#pragma unroll
        for (int t = 0; t < kSweepTiles; ++t) {
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int j = 0; j < NF; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag[j], bfrag[t][j], acc, 0, 0, 0);
            const int n = n_first + 32 * t + col;
            if (n < N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int mv = v0 + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (mv < M) Cbuf[((int64_t)dct * M + mv) * N + n] = acc[r];
                }
            }
        }
    }
#pragma unroll
    for (int mm = 32; mm >= 1; mm >>= 1) nmax = fmaxf(nmax, __shfl_xor(nmax, mm, 64));
    if (lane == 0) red[wave] = nmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        float v = red[0];
        for (int w = 1; w < kSweepThreads / 64; ++w) v = fmaxf(v, red[w]);
        dmax2_part[(int64_t)dct * nslices + sl] = v;
    }
}

// ---- launch 2: the s iterations of one vector ------------------------------------------------------------------------------
template <int DC, int NR, int THREADS>
__global__ __launch_bounds__(THREADS) void iterate_kernel(const __half *__restrict__ X, const __half *__restrict__ Dict,
                                                               const __half *__restrict__ G, const float *__restrict__ Cbuf,
                                                               const float *__restrict__ dmax2_part, void *__restrict__ idx_out,
                                                               void *__restrict__ coef_out, int64_t T, int32_t M, int32_t N, int32_t s,
                                                               int32_t sn, int64_t x_stride_h, int64_t x_stride_t, int32_t dict_count,
                                                               int64_t code_stride_h, int32_t nslices, int32_t idx16, int32_t coef16,
                                                               float *__restrict__ res_norm2)
{
    constexpr int LPR = DC / 8, RPW = 64 / LPR;
    constexpr int kIterThreads = THREADS, kIterWaves = THREADS / 64;
    __shared__ float4 keys[2][kIterWaves];  // (by iteration parity: a wave may run one barrier ahead)
    __shared__ int cnt;
    __shared__ int cand[kCand];
    __shared__ float4 best[kIterWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int piece = lane % LPR, rg = lane / LPR;
    const int dct = blockIdx.x / M;
    const int m = blockIdx.x - dct * M;
    const VecAt at = locate(dct, m, T, sn, s, DC, dict_count, x_stride_h, x_stride_t, code_stride_h);
    const __half *Dh = Dict + (int64_t)dct * N * DC;
    const __half *Gd = G + (int64_t)dct * N * N;
    const float *Cv = Cbuf + ((int64_t)dct * M + m) * N;

    float dmax2 = 0.0f;
    for (int sl = 0; sl < nslices; ++sl) dmax2 = fmaxf(dmax2, dmax2_part[(int64_t)dct * nslices + sl]);
    const float dmax = sqrtf(dmax2);
    const float g_eps = dmax2 * (2.44140625e-4f + kGammaAcc) + 2.98023224e-8f;  // |G16 - G| <= g_eps

    // the residual: every group of LPR lanes holds all of it, 8 dimensions per lane, the same in all waves
    float R[8];
    {
        const uint4 raw = *reinterpret_cast<const uint4 *>(X + at.x_off + 8 * piece);
        unpack8(raw, R);
    }
    float r2 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) r2 = fmaf(R[e], R[e], r2);
    r2 = row_sum<LPR>(r2);
    const float xnorm = sqrtf(r2);

    // this thread's correlations: atoms 8 (tid + THREADS j) + e
    float C[NR][8];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int n0 = 8 * (tid + kIterThreads * j);
        float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
        if (n0 < N) {  // (N is a multiple of 8)
            lo = *reinterpret_cast<const float4 *>(Cv + n0);
            hi = *reinterpret_cast<const float4 *>(Cv + n0 + 4);
        }
        C[j][0] = lo.x; C[j][1] = lo.y; C[j][2] = lo.z; C[j][3] = lo.w;
        C[j][4] = hi.x; C[j][5] = hi.y; C[j][6] = hi.z; C[j][7] = hi.w;
    }
    float delta = kGammaAcc * xnorm * dmax;
    float rmax = xnorm;  // largest residual norm so far

    for (int g = 0; g < s; ++g) {
        const int p = g & 1;
        // ---- screen: the two largest |C| of the block and the atom of the largest --------------------------------------
        // (which of several EQUAL largest values is named does not matter: a tie sends the iteration down the
        // candidate path, where the atoms themselves decide)
        float a1 = 0.0f, a2 = 0.0f;
        int na = 8 * tid < N ? 8 * tid : 0;
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int n0 = 8 * (tid + kIterThreads * j);
            if (n0 < N) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = fabsf(C[j][e]);
                    a2 = fmaxf(a2, fminf(a1, v));
                    na = v > a1 ? n0 + e : na;
                    a1 = fmaxf(a1, v);
                }
            }
        }
        float w1 = a1, w2 = a2;
        top2_dpp<0xB1, 0xF>(w1, w2);   // quad_perm [1,0,3,2]
        top2_dpp<0x4E, 0xF>(w1, w2);   // quad_perm [2,3,0,1]
        top2_dpp<0x141, 0xF>(w1, w2);  // row_half_mirror
        top2_dpp<0x140, 0xF>(w1, w2);  // row_mirror: every lane has its row's two largest
        top2_dpp<0x142, 0xA>(w1, w2);  // row_bcast15: rows 1 and 3 take in the row before them
        top2_dpp<0x143, 0xC>(w1, w2);  // row_bcast31: row 3 takes in rows 0 and 1; lane 63 has the wave's
        w1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w1), 63));
        w2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w2), 63));
        {
            const unsigned long long holders = __ballot(a1 == w1);
            const int src = holders ? __ffsll((long long)holders) - 1 : 0;
            const int nw = __builtin_amdgcn_readlane(na, src);
            if (lane == 0) keys[p][wave] = make_float4(w1, w2, __int_as_float(nw), 0.0f);
        }
        __syncthreads();  // the only barrier of an iteration whose maximum stands clear of the rest
        float A1 = 0.0f, A2 = 0.0f;
        int n1 = 0;
#pragma unroll
        for (int w = 0; w < kIterWaves; ++w) {
            const float4 k = keys[p][w];
            A2 = fmaxf(A2, fmaxf(fminf(A1, k.x), k.y));
            n1 = k.x > A1 ? __float_as_int(k.z) : n1;
            A1 = fmaxf(A1, k.x);
        }
        const bool zero = !(r2 > 0.0f);

        // requested now, used after the decision (which is n1 almost always)
        uint4 gp[NR];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int n0 = 8 * (tid + kIterThreads * j);
            gp[j] = make_uint4(0u, 0u, 0u, 0u);
            if (n0 < N) gp[j] = *reinterpret_cast<const uint4 *>(Gd + (int64_t)n1 * N + n0);
        }
        const uint4 d1p = *reinterpret_cast<const uint4 *>(Dh + (int64_t)n1 * DC + 8 * piece);

        const float thr = A1 - 2.0f * delta;
        int best_n = n1;
        float best_c;
        if (zero || !(A2 >= thr)) {
            // ---- no other atom within 2 delta: every wave computes the coefficient itself ----------------------------------
            best_c = exact_dot<LPR>(R, d1p);
        } else {
            // ---- candidates: everything within 2 delta of the maximum -------------------------------------------------
            if (tid == 0) cnt = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < NR; ++j) {
                const int n0 = 8 * (tid + kIterThreads * j);
                if (n0 < N) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        if (n0 + e != n1 && fabsf(C[j][e]) >= thr) {
                            const int slot = atomicAdd(&cnt, 1);
                            if (slot < kCand) cand[slot] = n0 + e;
                        }
                    }
                }
            }
            __syncthreads();
            const int L = cnt;
            // exact R . d of the candidates, from the atoms themselves
            float ba = -1.0f, bc = 0.0f;
            int bn = 0x7fffffff;
            const bool all = L > kCand;
            const int total = all ? N : L + 1;  // list entry 0 is n1
            for (int base = 0; base < total; base += kIterWaves * RPW) {
                const int ci = base + wave * RPW + rg;
                const bool live = ci < total;
                int n = n1;
                if (live && all) n = ci;
                if (live && !all && ci > 0) n = cand[ci - 1];
                uint4 raw = d1p;
                if (n != n1) raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)n * DC + 8 * piece);
                const float c = exact_dot<LPR>(R, raw);
                if (live) take_better(ba, bn, bc, fabsf(c), n, c);
            }
#pragma unroll
            for (int mm = LPR; mm < 64; mm <<= 1) {
                const float oa = __shfl_xor(ba, mm, 64), oc = __shfl_xor(bc, mm, 64);
                const int on = __shfl_xor(bn, mm, 64);
                take_better(ba, bn, bc, oa, on, oc);
            }
            if (lane == 0) best[wave] = make_float4(ba, __int_as_float(bn), bc, 0.0f);
            __syncthreads();
            const float4 b0 = best[0];
            ba = b0.x; bn = __float_as_int(b0.y); bc = b0.z;
#pragma unroll
            for (int w = 1; w < kIterWaves; ++w) {
                const float4 b = best[w];
                take_better(ba, bn, bc, b.x, __float_as_int(b.y), b.z);
            }
            best_n = bn;
            best_c = bc;
            if (bn == 0x7fffffff) { best_n = n1; best_c = __uint_as_float(0x7fc00000u); }  // nothing compares: NaN in, NaN out
        }
        if (zero) { best_n = 0; best_c = 0.0f; }

        // ---- Eq.4 on the residual (unrounded c), the recursion on the correlations -----------------------------------
        {
            uint4 raw = d1p;
            if (best_n != n1) raw = *reinterpret_cast<const uint4 *>(Dh + (int64_t)best_n * DC + 8 * piece);  // (uniform)
            float dn[8];
            unpack8(raw, dn);
            float r2n = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                R[e] = fmaf(-best_c, dn[e], R[e]);
                r2n = fmaf(R[e], R[e], r2n);
            }
            r2 = row_sum<LPR>(r2n);
        }
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int n0 = 8 * (tid + kIterThreads * j);
            if (n0 < N) {
                uint4 raw = gp[j];
                if (best_n != n1) raw = *reinterpret_cast<const uint4 *>(Gd + (int64_t)best_n * N + n0);  // (uniform)
                float gv[8];
                unpack8(raw, gv);
#pragma unroll
                for (int e = 0; e < 8; ++e) C[j][e] = fmaf(-best_c, gv[e], C[j][e]);
            }
        }
        rmax = fmaxf(rmax, sqrtf(r2));  // (atoms longer than sqrt 2 can make a residual grow)
        delta += fabsf(best_c) * g_eps + 2.4e-7f * rmax * dmax;

        if (tid == 0) {
            const int64_t o = at.code + g;
            if (idx16) reinterpret_cast<uint16_t *>(idx_out)[o] = (uint16_t)best_n;
            else reinterpret_cast<int32_t *>(idx_out)[o] = best_n;
            if (coef16) reinterpret_cast<__half *>(coef_out)[o] = __float2half_rn(best_c);
            else reinterpret_cast<float *>(coef_out)[o] = best_c;
        }
    }
    if (res_norm2 && tid == 0) res_norm2[at.norm] = r2;
}

struct StepPlan {
    int64_t M;        // vectors per dictionary
    int64_t dicts;    // dictionaries (chunk dictionaries counted)
    int nslices;
    size_t c_bytes, total;
};

StepPlan plan_step(const EncodeArgs &a)
{
    StepPlan p{};
    p.M = (int64_t)(a.H / a.dict_count) * a.T;
    p.dicts = (int64_t)a.dict_count * a.sn;
    p.nslices = (a.N + kSliceAtoms - 1) / kSliceAtoms;
    p.c_bytes = ((size_t)p.dicts * p.M * a.N * sizeof(float) + 255) & ~size_t(255);
    p.total = p.c_bytes + (((size_t)p.dicts * p.nslices * sizeof(float) + 255) & ~size_t(255));
    return p;
}

template <int DC, int NR, int THREADS>
void launch_iterate(const EncodeArgs &a, const StepPlan &p, const float *Cbuf, const float *dpart)
{
    hipLaunchKernelGGL((iterate_kernel<DC, NR, THREADS>), dim3((unsigned)(p.dicts * p.M)), dim3(THREADS), 0, a.stream,
                       (const __half *)a.X, (const __half *)a.D, (const __half *)a.gram, Cbuf, dpart, a.idx, a.coef, a.T, (int32_t)p.M,
                       a.N, a.s, a.sn, a.x_stride_h, a.x_stride_t, a.dict_count, a.code_stride_h, p.nslices, (int32_t)a.idx16,
                       (int32_t)a.coef16, a.res_norm2);
}

template <int DC>
hipError_t launch_step_t(const EncodeArgs &a)
{
    const StepPlan p = plan_step(a);
    char *ws = static_cast<char *>(a.workspace);
    float *Cbuf = reinterpret_cast<float *>(ws);
    float *dpart = reinterpret_cast<float *>(ws + p.c_bytes);
    if (p.M <= kValuSweepVectors)
        hipLaunchKernelGGL(sweep_kernel<DC>, dim3((unsigned)(p.dicts * p.nslices)), dim3(kSweepThreads), 0, a.stream, (const __half *)a.X,
                           (const __half *)a.D, Cbuf, dpart, a.T, (int32_t)p.M, a.N, a.s, a.sn, a.x_stride_h, a.x_stride_t, a.dict_count,
                           p.nslices);
    else
        hipLaunchKernelGGL(sweep_mfma_kernel<DC>, dim3((unsigned)(p.dicts * p.nslices)), dim3(kSweepThreads), 0, a.stream,
                           (const __half *)a.X, (const __half *)a.D, Cbuf, dpart, a.T, (int32_t)p.M, a.N, a.s, a.sn, a.x_stride_h,
                           a.x_stride_t, a.dict_count, p.nslices);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.M >= kThroughputVectors && a.N <= 128 * 8 * kMaxRounds) launch_iterate<DC, 4, 128>(a, p, Cbuf, dpart);
    else if (p.M >= kThroughputVectors && a.N <= 256 * 8 * kMaxRounds) launch_iterate<DC, 4, 256>(a, p, Cbuf, dpart);
    else if (a.N <= 512 * 8) launch_iterate<DC, 1, 512>(a, p, Cbuf, dpart);
    else if (a.N <= 512 * 8 * 2) launch_iterate<DC, 2, 512>(a, p, Cbuf, dpart);
    else launch_iterate<DC, 4, 512>(a, p, Cbuf, dpart);
    return hipGetLastError();
}

}  // namespace

bool encode_gramstep_supported(const EncodeArgs &a)
{
    if (!(a.f16 && (a.d == 128 || a.d == 64) && a.N >= 32 && a.N % 32 == 0 && a.N <= kMaxAtoms)) return false;
    if (a.dict_count < 1 || a.H % a.dict_count != 0) return false;
    const int64_t M = (int64_t)(a.H / a.dict_count) * a.T;
    const int64_t dicts = (int64_t)a.dict_count * a.sn;
    const int64_t nslices = (a.N + kSliceAtoms - 1) / kSliceAtoms;
    return M <= kMaxVectors && dicts * nslices <= 0x7fffffffLL && dicts * M <= 0x7fffffffLL;
}

size_t encode_gramstep_workspace_bytes(const EncodeArgs &a) { return plan_step(a).total; }

hipError_t launch_encode_gramstep(const EncodeArgs &a)
{
    return a.d == 64 ? launch_step_t<64>(a) : launch_step_t<128>(a);
}

bool gram_build_supported(int32_t N, int32_t d) { return (d == 128 || d == 64) && N >= 32 && N % 32 == 0 && N <= kMaxAtoms; }

hipError_t launch_gram_build(const void *D, int32_t n_dicts, int32_t N, int32_t d, void *G, hipStream_t stream)
{
    const dim3 grid((unsigned)((N / 16 + 3) / 4), (unsigned)n_dicts);
    if (d == 64)
        hipLaunchKernelGGL(gram_build_kernel<64>, grid, dim3(256), 0, stream, (const __half *)D, (__half *)G, N);
    else
        hipLaunchKernelGGL(gram_build_kernel<128>, grid, dim3(256), 0, stream, (const __half *)D, (__half *)G, N);
    return hipGetLastError();
}

}  // namespace csr
