/*
 * csr.h - C ABI of the MI355X (gfx950) implementation of the CSR sparse-representation
 * hot path (arXiv 2412.11741, "CSR: Achieving 1 Bit Key-Value Cache via Sparse
 * Representation").
 *
 * Two operations:
 *   csr_encode       greedy Matching Pursuit of dense per-head key/value vectors into s
 *                    (atom index, coefficient) pairs against a per-head dictionary
 *                    (Section "Sparse representation", Eq.2-4; Section "KV Decomposition and
 *                    Sparse Storage").
 *   csr_decode_attn  attention of one query token per sequence over the cached codes.  It
 *                    returns what ordinary softmax attention over the de-sparsified cache
 *                    X~ = D r (Eq.12, Section "De-Sparse to restore") returns, but never
 *                    builds X~: q.(D r) = (D^T q).r and sum_t p_t D r_t = D (sum_t p_t r_t).
 *
 * General rules
 *   - Every data pointer is DEVICE memory owned by the caller.  The library allocates
 *     nothing, frees nothing and keeps no pointer after a call returns.
 *   - Descriptors are plain host structs, read during the call only.
 *   - Calls enqueue work on the given HIP stream (a hipStream_t passed as void*; NULL is the
 *     default stream) and return without waiting for it.
 *   - No exception or abort crosses this boundary.  Argument problems are found on the host
 *     before anything is launched and reported as a status; csr_last_error() gives a message.
 *   - A dictionary is atom-major: D[h][n][k], n < N atoms, k < d contiguous.  Atoms must be
 *     unit L2 norm (up to storage rounding); this is not checked and nothing is renormalised.
 *   - Codes are two separate streams, idx[..][T][s] and coef[..][T][s], pair g of a vector being
 *     the atom and signed projection picked at iteration g.  The same atom may appear twice in
 *     one code; its coefficients then add (D r is the sum over the list).
 *   - 16-bit indices are unsigned (N <= 65536).
 */
#ifndef CSR_H
#define CSR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CSR_VERSION 100 /* major*10000 + minor*100 + patch */

typedef enum {
    CSR_OK = 0,
    CSR_ERR_INVALID_ARG = 1, /* null pointer, negative size, inconsistent descriptor      */
    CSR_ERR_UNSUPPORTED = 2, /* well-formed request this build has no kernel for           */
    CSR_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or smaller than the query says */
    CSR_ERR_DEVICE = 4       /* the HIP runtime reported an error while enqueuing          */
} csr_status;

typedef enum { CSR_F32 = 0, CSR_F16 = 1 } csr_dtype; /* vectors, dictionaries, coefficients */
typedef enum { CSR_I32 = 0, CSR_I16 = 1 } csr_itype; /* atom indices; I16 is unsigned        */

/* Which encoder kernel runs.  AUTO picks SPLIT when a dictionary serves few vectors (the tokens of one
 * decoding step; GRAM instead when the descriptor brings the dictionaries' Gram matrices and there are at
 * most 128), RESIDENT when the dictionary fits the LDS, MFMA when the shape allows it, else VALU. */
typedef enum {
    CSR_ENCODE_AUTO = 0,
    CSR_ENCODE_VALU = 1, /* fp32 vector-ALU correlation, any supported shape               */
    CSR_ENCODE_MFMA = 2, /* fp16 matrix-core screening pass + exact fp32 selection          */
    CSR_ENCODE_SPLIT = 3, /* few vectors per dictionary (at most 128): every dictionary's atoms are
                            split over several workgroups, one launch per iteration; fp16 inputs,
                            chunks of 64 or 128 dimensions, N a multiple of 32                   */
    CSR_ENCODE_RESIDENT = 4, /* small dictionaries (N * d/s_n * 2 bytes <= 128 KB, e.g. the 256 - 512 atoms per
                            head of the paper's experiments): the dictionary stays in LDS, exact
                            fp32-accumulated correlations on the matrix cores; same input types     */
    CSR_ENCODE_GRAM = 5  /* the correlations of all atoms are updated with the Gram matrix of the dictionary
                            (in fp16: atom norms must stay below 250) instead of being recomputed; same input
                            types.  Without csr_encode_desc.gram: at most 256 atoms, the matrix is built into LDS
                            by every workgroup; never picked by AUTO (on this chip it is slower than RESIDENT).
                            With csr_encode_desc.gram (csr_gram_build): up to 16384 atoms and at most 128 vectors
                            per dictionary, the decoding-step shape; AUTO picks it whenever gram is given and
                            the shape fits                                                               */
} csr_encode_algo;

/* csr_encode_desc.flags.  CLOSED_LOOP: Eq.4 subtracts the coefficient AS IT IS STORED - c_g is rounded to coef_dtype
 * first (Section "Analysis for CSR" stores fp16), so the residual the later iterations work on is exactly the error
 * of the stored code, and res_norm2 is the squared error of the stored code.  The default (flag clear) subtracts the
 * unrounded c_g and rounds on store only; with fp32 coefficients the two coincide.  Taken by the VALU, MFMA, SPLIT
 * and RESIDENT encoders (the Gram forms return CSR_ERR_UNSUPPORTED, and AUTO does not choose them with the flag). */
#define CSR_FLAG_CLOSED_LOOP 1u

/*
 * Matching Pursuit encode (Eq.2-4), H independent dictionaries with T vectors each.
 * For every vector x: R_1 = x; for g = 1..s: i_g = argmax_n |R_g . d_n| (lowest n on ties),
 * c_g = R_g . d_{i_g} (signed), R_{g+1} = R_g - c_g d_{i_g}.  The residual is kept in fp32 and
 * is updated with the unrounded c_g; rounding to coef_dtype happens on store only.  A zero
 * residual emits (0, 0).
 */
typedef struct {
    int32_t H;          /* vector blocks (e.g. sequences x KV heads x {K,V}); >= 0          */
    int64_t T;          /* vectors per dictionary; >= 0 (0 is a no-op)                     */
    int32_t d;          /* vector length; the chunk length d / s_n must be 32, 64 or 128 (VALU and, for
                           fp16, MFMA); the other encoders take fp16 chunks of 64 or 128        */
    int32_t N;          /* atoms per dictionary, 1..65536 (I16) or 1..2^24 (I32)            */
    int32_t s;          /* iterations = pairs per vector (per chunk), 1..32                 */
    int32_t s_n;        /* chunks per vector (Section "NeuralDict"): 0 or 1 = the vector is coded
                           whole; else 2, 4 or 8: dimensions c*d/s_n .. (c+1)*d/s_n - 1 form chunk
                           c, which is encoded on its own, on dictionary c, as a vector of its own */
    int32_t x_dtype;    /* csr_dtype of X                                                   */
    int32_t dict_dtype; /* csr_dtype of D; must equal x_dtype                               */
    int32_t coef_dtype; /* csr_dtype of coef                                                */
    int32_t idx_dtype;  /* csr_itype of idx                                                 */
    int64_t x_stride_h; /* elements between dictionaries' vector blocks; 0 = T*d            */
    int64_t x_stride_t; /* elements between consecutive vectors; 0 = d                      */
    int32_t dict_count; /* distinct dictionaries: block h uses dictionary h % dict_count (blocks ordered
                           sequence-major, head-minor share the heads' dictionaries); 0 = H, one each.
                           Must divide H                                                    */
    int64_t code_stride_h; /* elements between consecutive blocks' codes in idx and in coef; 0 = T*s_n*s.
                           With T = 1, idx / coef pointing at row t of a cache [H][T_max][s_n*s] and
                           code_stride_h = T_max*s_n*s the new token's codes are appended in place
                           (Section "KV Decomposition and Sparse Storage": a generated token is
                           encoded like the prompt's)                                       */
    int32_t algo;       /* csr_encode_algo                                                  */
    uint32_t flags;     /* 0 or CSR_FLAG_CLOSED_LOOP                                        */
    float *res_norm2;   /* optional device pointer, [H][T][s_n] fp32, or NULL: receives |R_{s+1}|^2, the
                           squared norm of what the s pairs leave of each vector (chunk) - by Eq.4 the
                           squared reconstruction error |x - D r|^2 with unrounded coefficients, i.e. the
                           vector's term of the dictionary-training loss of Section "NeuralDict"       */
    const void *gram;   /* optional device pointer, or NULL: the Gram matrices of D as csr_gram_build writes them
                           ([dict_count][N][N] fp16; chunked [dict_count][s_n][N][N]).  With them, CSR_ENCODE_GRAM -
                           and CSR_ENCODE_AUTO - encode up to 128 vectors per dictionary (the tokens of one decoding
                           step) with ONE sweep of each dictionary instead of s: later iterations read one row of
                           the Gram matrix per vector.  fp16 inputs, chunks of 64 or 128, N a multiple of 32, at
                           most 16384.  Results are those of the other encoders (the Gram recursion screens, the
                           decision is taken on the atoms).  Other explicit algos ignore it.  The matrices must
                           belong to exactly this D                                                      */
} csr_encode_desc;

/* Bytes of device scratch csr_encode needs for this descriptor (may be 0); (size_t)-1 if the
 * descriptor is invalid. */
size_t csr_encode_workspace_bytes(const csr_encode_desc *desc);

/*
 *   X    [H][T][d]  (strides as given)   in
 *   D    [dict_count][N][d]              in       (chunked: [dict_count][s_n][N][d/s_n])
 *   idx  [H][T][s]  idx_dtype            out      (chunked: [H][T][s_n][s], atom numbers 0..N-1 per chunk;
 *   coef [H][T][s]  coef_dtype           out       blocks code_stride_h elements apart)
 *   X and D must be 16-byte aligned; idx and coef to their element size.
 *   workspace: device memory, 256-byte aligned, >= csr_encode_workspace_bytes(); may be NULL
 *   when that is 0.  Contents are undefined before and after.
 */
csr_status csr_encode(const csr_encode_desc *desc, const void *X, const void *D, void *idx,
                      void *coef, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Decode attention on codes.  For every sequence b and query head hq (KV head h = hq / (Hq/Hkv)):
 *   score_t = scale * sum_j coefK[b][h][t][j] * (q[b][hq] . DK[h][idxK[b][h][t][j]])
 *   p       = softmax over the valid tokens t < len_b
 *   out     = DV[h]^T applied to hist, hist[n] = sum_{t,j : idxV = n} p_t * coefV[b][h][t][j]
 * which equals softmax attention over K~ = D_K r_K, V~ = D_V r_V of Eq.12.  No mask beyond the
 * sequence length; no position embedding (the paper's Section "KV cache in attention" sets it
 * aside) unless rope_base is set, see there.  A sequence with len_b = 0 yields zeros.  Accumulation is fp32, except the
 * V-side histogram, which is summed exactly in fixed point with integer atomics (per chunk of at most 16384 tokens: 32-bit
 * bins whose unit is fitted to the data, checked after the scatter for overflow and for resolution, and repeated in 64-bit
 * bins where the check fails), so the result does not depend on the order in which the hardware serves the scatter: the
 * same inputs give the same bits on every run.
 */
typedef struct {
    int32_t B;          /* sequences; >= 0                                                  */
    int32_t Hq;         /* query heads; multiple of Hkv, Hq/Hkv <= 8                        */
    int32_t Hkv;        /* KV heads                                                         */
    int64_t T;          /* code rows allocated per (b, h); 0 .. 2^20                        */
    int32_t d;          /* head dimension; supported: 128                                   */
    int32_t N;          /* atoms per dictionary                                             */
    int32_t sK, sV;     /* pairs per key / value code (per chunk), 1..32                    */
    int32_t snK, snV;   /* chunks per head vector for keys / values (the s_n of Section
                           "NeuralDict"); 0 or 1 = the vector is coded whole.  Supported: 1, 2, 4, 8
                           with fp16 q and dictionaries, N a multiple of 128 and sn * s <= 32         */
    float scale;        /* score scale; 0 means 1/sqrt(d)                                   */
    int32_t q_dtype;    /* csr_dtype of q                                                   */
    int32_t dict_dtype; /* csr_dtype of DK and DV                                           */
    int32_t coef_dtype; /* csr_dtype of coefK and coefV                                     */
    int32_t idx_dtype;  /* csr_itype of idxK and idxV                                       */
    int32_t out_dtype;  /* csr_dtype of out                                                 */
    uint32_t flags;     /* must be 0                                                        */
    float rope_base;    /* 0: the cached keys are in the frame of the query (no position embedding, or keys
                           coded after it).  > 1: the keys were coded BEFORE the rotary position embedding
                           (Section "Position embedding makes nonstationary Keys"): cache token t is rebuilt by
                           Eq.12 and turned to position rope_pos0 + t, frequency pair k by the angle
                           position * rope_base^(-2k/d); q is the query as attention receives it, already
                           turned at its own position.  Supported with the paper's storage types (fp16 q and
                           dictionaries, 16-bit indices, fp16 coefficients), whole-vector keys (snK <= 1) and
                           sK a multiple of 4.  A key dictionary of at most 128 KB (N <= 512, the paper's own
                           sizes) stays in LDS; a larger one is gathered row by row from device memory, which
                           is correct but several times slower (256 bytes per code pair instead of 4).
                           T is then at most 2^19 when Hq/Hkv is a multiple of 4.  Scores carry the rounding of the turned query (or key) to fp16, a
                           relative 2^-11 per component, instead of fp32 accuracy.                 */
    int32_t rope_layout; /* 0: pair k is dimensions (k, k + d/2); 1: dimensions (2k, 2k + 1)    */
    int64_t rope_pos0;  /* position of cache token 0 of every sequence; 0 .. 2^40              */
} csr_decode_desc;

/* Bytes of device scratch csr_decode_attn needs; (size_t)-1 if the descriptor is invalid. */
size_t csr_decode_workspace_bytes(const csr_decode_desc *desc);

/*
 *   q        [B][Hq][d]        in
 *   DK, DV   [Hkv][N][d]       in, shared by all sequences
 *   idxK, coefK [B][Hkv][T][sK]   in;   idxV, coefV [B][Hkv][T][sV]   in
 *   With chunks (snK, snV > 1; the value cache of the paper's experiments uses s = 4, s_n = 2): chunk c of a head
 *   vector is its dimensions c*d/sn .. (c+1)*d/sn - 1, coded on its own dictionary of N atoms of that length:
 *   DK [Hkv][snK][N][d/snK], idxK, coefK [B][Hkv][T][snK][sK], indices 0..N-1 per chunk; likewise for V.  The result
 *   is attention over the concatenation of the chunks' reconstructions (Eq.12 per chunk).
 *   seq_lens [B] int32 device pointer, or NULL for len_b = T.  Values must lie in [0, T];
 *            larger values are clamped to T, negative ones to 0.
 *   out      [B][Hq][d]        out
 *   workspace: device memory, 256-byte aligned, >= csr_decode_workspace_bytes().
 *   q, DK, DV, the four code streams and out must be 16-byte aligned.
 * Indices are not range-checked on the device: an index >= N reads outside the score table (csr_check_codes counts
 * such indices, off the hot path).
 */
csr_status csr_decode_attn(const csr_decode_desc *desc, const void *q, const void *DK,
                           const void *idxK, const void *coefK, const void *DV, const void *idxV,
                           const void *coefV, const int32_t *seq_lens, void *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/*
 * csr_decode_attn for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels, same results as
 * csr_decode_attn; the scratch is a static device array inside the library, CSR_STATIC_SCRATCH_BYTES per GPU, which
 * exists from the first use of the library on that GPU until the process ends.  The call allocates and frees
 * nothing (no hipMalloc, no hipFree, no allocating library routine); its first call on a device looks the array's
 * address up, every later call only enqueues.
 *   - A shape whose csr_decode_workspace_bytes() exceeds CSR_STATIC_SCRATCH_BYTES returns CSR_ERR_WORKSPACE (use
 *     csr_decode_attn with a workspace of the caller's).
 *   - All calls on one GPU share that GPU's array.  Calls on one stream, or ordered by events, follow each other
 *     safely (nothing in the scratch has to survive a call or start at zero); calls that may OVERLAP on one GPU -
 *     different streams without ordering, different host threads - race on it and give undefined results.
 *   - Every other rule of csr_decode_attn holds (device pointers owned by the caller, alignment, status codes).
 */
#define CSR_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
csr_status csr_decode_attn_static(const csr_decode_desc *desc, const void *q, const void *DK,
                                  const void *idxK, const void *coefK, const void *DV, const void *idxV,
                                  const void *coefV, const int32_t *seq_lens, void *out, void *hip_stream);

/*
 * De-sparse restore, Eq.12: out[h][t] = sum over the s pairs of coef * atom (per chunk with chunked codes, the
 * chunks' results side by side).  The dense vectors are what the paper feeds to ordinary attention;
 * csr_decode_attn does not need them, callers that post-process rebuilt keys or values do.
 * Accumulation is fp32 in pair order.  Indices are not range-checked on the device.
 */
typedef struct {
    int32_t H;          /* vector blocks; >= 0                                              */
    int64_t T;          /* vectors per block; >= 0                                          */
    int32_t d;          /* vector length: a multiple of 8 * s_n, at most 1024               */
    int32_t N;          /* atoms per (chunk) dictionary                                     */
    int32_t s;          /* pairs per vector (per chunk), 1..32                              */
    int32_t s_n;        /* chunks per vector; 0 or 1 = whole vectors; must divide d         */
    int32_t dict_dtype; /* csr_dtype of D                                                   */
    int32_t coef_dtype; /* csr_dtype of coef                                                */
    int32_t idx_dtype;  /* csr_itype of idx                                                 */
    int32_t out_dtype;  /* csr_dtype of out                                                 */
    int32_t dict_count; /* block h uses dictionary h % dict_count; 0 = H; must divide H     */
    int64_t code_stride_h; /* elements between blocks' codes; 0 = T*s_n*s                   */
    int64_t out_stride_h;  /* elements between blocks' vectors; 0 = T*out_stride_t          */
    int64_t out_stride_t;  /* elements between consecutive vectors; 0 = d; multiple of 8    */
    uint32_t flags;     /* must be 0                                                        */
} csr_reconstruct_desc;

/*
 *   D    [dict_count][N][d]  (chunked: [dict_count][s_n][N][d/s_n])   in
 *   idx, coef [H][T][s]      (chunked: [H][T][s_n][s])                in
 *   out  [H][T][d]           (strides as given), 16-byte aligned      out
 * No workspace.
 */
csr_status csr_reconstruct(const csr_reconstruct_desc *desc, const void *D, const void *idx, const void *coef,
                           void *out, void *hip_stream);

/*
 * Gram matrices G = D D^T of n_dicts dictionaries of N atoms with d elements each (fp16; with chunks, n_dicts counts
 * the chunk dictionaries and d is the chunk length): gram[k][i][n] = fp16(d_i . d_n), for csr_encode_desc.gram.
 * This is the "C - c G[i,:]" form of Eq.2-4's correlations; prepare it once per dictionary.
 *   D     device, [n_dicts][N][d] fp16, 16-byte aligned            in
 *   gram  device, csr_gram_bytes(n_dicts, N) bytes, 16-byte aligned  out
 * d must be 64 or 128, N a multiple of 32, at most 16384; n_dicts at most 65535.  No workspace.
 */
size_t csr_gram_bytes(int32_t n_dicts, int32_t N);
csr_status csr_gram_build(const void *D, int32_t n_dicts, int32_t N, int32_t d, void *gram, void *hip_stream);

/*
 * Squared Euclidean norms of dictionary atoms: norms2[n] = |D[n]|^2 (fp32 sum) for the n_atoms rows of d elements
 * of D - all dictionaries of a call are one such array, n_atoms = dictionaries * (chunks *) N.  Section "Sparse
 * representation" takes the atoms to have unit norm; csr_encode does not check it (the result is Eq.2-4 for
 * whatever atoms it is given), so a caller that wants the check runs this first.
 *   D       device, aligned to its element type     in
 *   norms2  device, [n_atoms] float                 out
 * n_atoms >= 0, 1 <= d <= 65536.  No workspace.
 */
csr_status csr_atom_norms2(const void *D, int32_t dict_dtype, int64_t n_atoms, int32_t d, float *norms2, void *hip_stream);

/*
 * Atom indices of a code stream that lie outside [0, N) (16-bit indices read unsigned; negative 32-bit ones count):
 * *bad receives their number.  Eq.12 addresses the dictionary with the stored index as it is: csr_decode_attn and
 * csr_reconstruct do not range-check on the device, so codes that were not written by csr_encode (a cache loaded
 * from elsewhere) can be looked at first.  One read of the index stream, off the hot path.
 *   idx    device, `count` indices of idx_dtype, contiguous      in
 *   bad    device, one int64, 8-byte aligned                     out (valid once the stream has run)
 */
csr_status csr_check_codes(const void *idx, int32_t idx_dtype, int64_t count, int32_t N, int64_t *bad, void *hip_stream);

/*
 * Storage accounting of Section "Analysis for CSR": bytes kept per head vector,
 * s * s_n * (index bytes + coefficient bytes).  Returns 0 on bad arguments.
 */
size_t csr_code_bytes(int32_t s, int32_t s_n, int32_t idx_dtype, int32_t coef_dtype);

/* Message for the last non-OK status returned on this thread ("" if none).  Static storage. */
const char *csr_last_error(void);

/* CSR_VERSION of the built library. */
int csr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CSR_H */
