// Internal declarations shared by the host dispatch layer and the gfx950 kernels.
// Not part of the public ABI (that is include/csr.h).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "csr.h"

namespace csr {

constexpr int kWave = 64;  // CDNA wavefront width

// How the encoder kernels are told about the coefficients: bit 0 - stored as fp16 (else fp32); bit 1 - closed loop:
// Eq.4 subtracts the coefficient as it is stored.  Only fp16 storage rounds (the kernels' own coefficient is fp32).
constexpr int32_t kCoefF16 = 1, kCoefClosed = 2;
__host__ __device__ inline bool coef_is_f16(int32_t mode) { return (mode & kCoefF16) != 0; }
__host__ __device__ inline bool coef_rounds_in_loop(int32_t mode) { return (mode & (kCoefF16 | kCoefClosed)) == (kCoefF16 | kCoefClosed); }

// ---- encode ---------------------------------------------------------------------------------
struct EncodeArgs {
    const void *X;
    const void *D;
    void *idx;
    void *coef;
    int32_t H;
    int64_t T;
    int32_t d, N, s;                 // d = length of one chunk (the vector's length if sn == 1)
    int32_t sn;                      // chunks per vector (>= 1); chunk c of head h uses dictionary h * sn + c
    int64_t x_stride_h, x_stride_t;  // elements, already defaulted
    int32_t dict_count;              // block h uses dictionary h % dict_count (already defaulted to H)
    int64_t code_stride_h;           // elements between blocks' codes (already defaulted)
    bool f16;                        // X and D are fp16 (else fp32)
    bool coef16, idx16;
    bool closed_loop;                // Eq.4 subtracts the coefficient as it is stored (CSR_FLAG_CLOSED_LOOP)
    float *res_norm2;                // optional [H][T][sn] output, or nullptr
    const void *gram;                // optional Gram matrices [dict_count * sn][N][N] fp16 (csr_gram_build), or nullptr
    void *workspace;
    hipStream_t stream;
};

// fp32 vector-ALU encoder: any N, d in {32, 64, 128}.
hipError_t launch_encode_valu(const EncodeArgs &a);

// fp16 matrix-core encoder: chunks of 64 or 128 dimensions, fp16 inputs.
bool encode_mfma_supported(const EncodeArgs &a);
size_t encode_mfma_workspace_bytes(int32_t n_dicts, int64_t T, int32_t N, int32_t s);
hipError_t launch_encode_mfma(const EncodeArgs &a);

// fp16 matrix-core encoder for few vectors per dictionary (a decoding step): atoms split over workgroups,
// one launch per iteration.
bool encode_split_supported(const EncodeArgs &a);
size_t encode_split_workspace_bytes(const EncodeArgs &a);
hipError_t launch_encode_split(const EncodeArgs &a);

// fp16 matrix-core encoder for dictionaries that fit the LDS (at most 128 KB).
bool encode_resident_supported(const EncodeArgs &a);
hipError_t launch_encode_resident(const EncodeArgs &a);

// fp16 encoder for dictionaries of at most 256 atoms: Gram-matrix update of the correlations.
bool encode_gram_supported(const EncodeArgs &a);
hipError_t launch_encode_gram(const EncodeArgs &a);

// Gram update with the Gram matrices in device memory: a few vectors per dictionary of up to 16384 atoms.
bool encode_gramstep_supported(const EncodeArgs &a);
size_t encode_gramstep_workspace_bytes(const EncodeArgs &a);
hipError_t launch_encode_gramstep(const EncodeArgs &a);
bool gram_build_supported(int32_t N, int32_t d);
hipError_t launch_gram_build(const void *D, int32_t n_dicts, int32_t N, int32_t d, void *G, hipStream_t stream);

// ---- atom norms -----------------------------------------------------------------------------------------------------
hipError_t launch_atom_norms2(const void *D, bool f16, int64_t n_atoms, int32_t d, float *out, hipStream_t stream);
hipError_t launch_check_codes(const void *idx, bool idx16, int64_t count, int32_t N, int64_t *bad, hipStream_t stream);

// ---- reconstruct (Eq.12) --------------------------------------------------------------------
struct ReconstructArgs {
    const void *D;
    const void *idx;
    const void *coef;
    void *out;
    int32_t H;
    int64_t T;
    int32_t d, N, s, sn;  // d = whole vector length
    int32_t dict_count;
    int64_t code_stride_h, out_stride_h, out_stride_t;  // elements, already defaulted
    bool dict16, coef16, idx16, out16;
    hipStream_t stream;
};
hipError_t launch_reconstruct(const ReconstructArgs &a);

// ---- decode ---------------------------------------------------------------------------------
struct DecodePlan {
    int32_t GB;           // query heads of one KV head handled together by a block (1, 2 or 4)
    int32_t ngs;          // group slices per KV head = G / GB
    int32_t nchunks;      // split of the token axis
    int32_t threads;      // threads of a workgroup of the streaming kernel = tokens per round
    int64_t chunk_tokens; // tokens per chunk (multiple of the block's token step)
    size_t off_qd, off_hist, off_ml, off_acc, total_bytes;
    size_t lds_bytes;     // dynamic LDS of the streaming kernel
};

struct DecodeArgs {
    const void *q, *DK, *idxK, *coefK, *DV, *idxV, *coefV;
    const int32_t *seq_lens;
    void *out;
    int32_t B, Hq, Hkv, G;
    int64_t T;
    int32_t d, N, sK, sV;  // N atoms per (chunk) dictionary, sK / sV pairs per chunk
    int32_t snK, snV;      // chunks per head vector (>= 1)
    float scale;
    float rope_base;       // > 0: keys were coded before the rotary embedding (theta_k = rope_base^(-2k/d))
    int32_t rope_layout;   // 0: pair k = dimensions (k, k + d/2); 1: (2k, 2k + 1)
    int64_t rope_pos0;     // position of cache token 0
    bool q16, dict16, coef16, idx16, out16;
    void *workspace;
    hipStream_t stream;
};

// Fills the plan; returns false if no kernel configuration fits (e.g. N too large for LDS).
// rope: the plan is for the kernel that keeps the key dictionary in LDS (keys coded before the rotary embedding).
// code_vecs: 1 or 2 if key and value codes are whole-vector codes of 8 or 16 pairs in the paper's storage types
// (one or two 16-byte vectors per token and stream: the streaming kernel's fast variants), else 0.
bool plan_decode(int32_t B, int32_t Hq, int32_t Hkv, int64_t T, int32_t d, int32_t N, int32_t snK, int32_t snV,
                 bool rope, int code_vecs, DecodePlan *p);
hipError_t launch_decode(const DecodeArgs &a, const DecodePlan &p);

// Streaming kernel for keys coded before the rotary embedding (decode_rope.hip); fills the same chunk histograms,
// maxima and sums as the position-free one.
bool decode_rope_shape_supported(int32_t d, int32_t N, int32_t sK, int32_t snK);
hipError_t launch_stream_rope(const DecodeArgs &a, const DecodePlan &p, float *hist, float *ml);

}  // namespace csr
