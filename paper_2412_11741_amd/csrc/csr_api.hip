// Host side of the C ABI declared in include/csr.h: argument validation, kernel choice,
// workspace layout.  Nothing here allocates device memory or waits for the GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "csr_internal.h"

// Device scratch of csr_decode_attn_static: one array per GPU, held from the first use of the library's code
// on that GPU until the process ends.  Host code never uses this name as an address (on the host it is only a
// handle): static_scratch() asks the runtime for the array's device address, once per device.
constexpr size_t kStaticScratchBytes = CSR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[384] = "";

csr_status fail(csr_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

constexpr int kAlgoGramStep = 100;  // CSR_ENCODE_GRAM with the descriptor's Gram matrices (internal)

bool valid_dtype(int32_t v) { return v == CSR_F32 || v == CSR_F16; }
bool valid_itype(int32_t v) { return v == CSR_I32 || v == CSR_I16; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
size_t round256(size_t v) { return (v + 255) & ~size_t(255); }

// Checks everything about an encode descriptor that does not need the pointers; fills the shape part of the
// kernels' arguments and names the kernel that will run (AUTO resolved to one of the others).
csr_status check_encode_desc(const csr_encode_desc *d, csr::EncodeArgs *args, int *algo_out)
{
    if (!d) return fail(CSR_ERR_INVALID_ARG, "csr_encode: descriptor is NULL");
    if (d->H < 0 || d->T < 0) return fail(CSR_ERR_INVALID_ARG, "csr_encode: H=%d T=%lld must be >= 0", d->H, (long long)d->T);
    if ((d->flags & ~CSR_FLAG_CLOSED_LOOP) != 0) return fail(CSR_ERR_INVALID_ARG, "csr_encode: unknown flags 0x%x", d->flags);
    const bool closed = (d->flags & CSR_FLAG_CLOSED_LOOP) != 0;
    if (!valid_dtype(d->x_dtype) || !valid_dtype(d->dict_dtype) || !valid_dtype(d->coef_dtype) || !valid_itype(d->idx_dtype))
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: unknown dtype / index type");
    if (d->algo != CSR_ENCODE_AUTO && d->algo != CSR_ENCODE_VALU && d->algo != CSR_ENCODE_MFMA && d->algo != CSR_ENCODE_SPLIT &&
        d->algo != CSR_ENCODE_RESIDENT && d->algo != CSR_ENCODE_GRAM)
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: unknown algo %d", d->algo);
    if (d->s < 1 || d->s > 32) return fail(CSR_ERR_INVALID_ARG, "csr_encode: s=%d outside 1..32", d->s);
    if (d->N < 1) return fail(CSR_ERR_INVALID_ARG, "csr_encode: N=%d must be >= 1", d->N);
    if (d->d < 1) return fail(CSR_ERR_INVALID_ARG, "csr_encode: d=%d must be >= 1", d->d);
    if (d->idx_dtype == CSR_I16 && d->N > 65536)
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: N=%d does not fit unsigned 16-bit indices", d->N);
    if (d->N > (1 << 24)) return fail(CSR_ERR_UNSUPPORTED, "csr_encode: N=%d above 2^24", d->N);
    if (d->x_dtype != d->dict_dtype)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: vectors and dictionary must share one dtype");
    const int sn = d->s_n ? d->s_n : 1;
    if (sn != 1 && sn != 2 && sn != 4 && sn != 8)
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: s_n=%d must be 0, 1, 2, 4 or 8", d->s_n);
    if (d->d % sn != 0) return fail(CSR_ERR_INVALID_ARG, "csr_encode: d=%d is not a multiple of s_n=%d", d->d, sn);
    const int dc = d->d / sn;
    if (dc != 32 && dc != 64 && dc != 128)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: chunk length d/s_n=%d not supported (32, 64, 128)", dc);
    if ((int64_t)d->H * sn > 0x7fffffffLL) return fail(CSR_ERR_UNSUPPORTED, "csr_encode: H*s_n too large");
    if (d->dict_count < 0 || (d->dict_count > 0 && (d->H % d->dict_count != 0)))
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: dict_count=%d must be 0 or divide H=%d", d->dict_count, d->H);
    const int64_t st = d->x_stride_t ? d->x_stride_t : d->d;
    const int64_t sh = d->x_stride_h ? d->x_stride_h : d->T * st;
    const int64_t vec = d->x_dtype == CSR_F16 ? 8 : 4;  // elements per 16-byte load
    if (st < d->d || st % vec != 0 || sh % vec != 0 || sh < 0)
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: strides (h=%lld, t=%lld) must be >= d and multiples of 16 bytes",
                    (long long)sh, (long long)st);
    if (d->T > 0 && d->H > 1 && sh < (d->T - 1) * st + d->d)
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: x_stride_h=%lld makes dictionaries' vector blocks overlap", (long long)sh);
    const int64_t code_block = d->T * sn * d->s;
    if (d->code_stride_h < 0 || (d->code_stride_h > 0 && d->code_stride_h < code_block))
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: code_stride_h=%lld is smaller than one block's codes (%lld elements)",
                    (long long)d->code_stride_h, (long long)code_block);
    if ((d->T + 63) / 64 * (int64_t)d->H * sn > 0x7fffffffLL)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: H*T too large for one launch");
    csr::EncodeArgs a{};
    a.H = d->H; a.T = d->T; a.d = dc; a.sn = sn; a.N = d->N; a.s = d->s;
    a.x_stride_t = st; a.x_stride_h = sh;
    a.dict_count = d->dict_count ? d->dict_count : d->H;
    a.code_stride_h = d->code_stride_h ? d->code_stride_h : code_block;
    a.f16 = d->x_dtype == CSR_F16;
    a.coef16 = d->coef_dtype == CSR_F16;
    a.idx16 = d->idx_dtype == CSR_I16;
    const bool mfma_ok = csr::encode_mfma_supported(a), split_ok = csr::encode_split_supported(a);
    if (d->algo == CSR_ENCODE_MFMA && !mfma_ok)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the MFMA encoder needs fp16 inputs, chunks of 32, 64 or 128 dimensions and N a multiple of 32 (got d/s_n=%d N=%d %s)",
                    dc, d->N, a.f16 ? "f16" : "f32");
    if (d->algo == CSR_ENCODE_SPLIT && !split_ok)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the split encoder needs fp16 inputs, chunks of 64 or 128 dimensions, N a multiple of 32 "
                    "and at most 128 vectors per dictionary (got d/s_n=%d N=%d %s, %lld vectors per dictionary)",
                    dc, d->N, a.f16 ? "f16" : "f32", (long long)(a.dict_count ? (int64_t)(a.H / a.dict_count) * a.T : 0));
    const bool resident_ok = csr::encode_resident_supported(a);
    if (d->algo == CSR_ENCODE_RESIDENT && !resident_ok)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the LDS-resident encoder needs fp16 inputs, chunks of 64 or 128 dimensions, N a multiple "
                    "of 32 and a dictionary of at most 128 KB (got d/s_n=%d N=%d %s)", dc, d->N, a.f16 ? "f16" : "f32");
    a.gram = d->gram;
    a.closed_loop = closed;
    if (closed && d->algo == CSR_ENCODE_GRAM)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the Gram encoders do not take CSR_FLAG_CLOSED_LOOP");
    const bool step_ok = !closed && d->gram != nullptr && csr::encode_gramstep_supported(a);
    if (d->algo == CSR_ENCODE_GRAM && d->gram && !step_ok)
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the Gram encoder with prepared Gram matrices needs fp16 inputs, chunks of 64 or 128 "
                    "dimensions, N a multiple of 32, at most 16384, and at most 128 vectors per dictionary (got d/s_n=%d N=%d %s, %lld "
                    "vectors per dictionary)", dc, d->N, a.f16 ? "f16" : "f32", (long long)(a.dict_count ? (int64_t)(a.H / a.dict_count) * a.T : 0));
    if (d->algo == CSR_ENCODE_GRAM && !d->gram && !csr::encode_gram_supported(a))
        return fail(CSR_ERR_UNSUPPORTED, "csr_encode: the Gram encoder needs fp16 inputs, chunks of 64 or 128 dimensions and N a multiple "
                    "of 32, at most 256 - or the descriptor's gram matrices (got d/s_n=%d N=%d %s)", dc, d->N, a.f16 ? "f16" : "f32");
    int algo = d->algo;
    if (algo == CSR_ENCODE_GRAM && d->gram) algo = kAlgoGramStep;
    if (algo == CSR_ENCODE_AUTO)
        algo = step_ok ? kAlgoGramStep : split_ok ? CSR_ENCODE_SPLIT : resident_ok ? CSR_ENCODE_RESIDENT : mfma_ok ? CSR_ENCODE_MFMA : CSR_ENCODE_VALU;
    *args = a;
    *algo_out = algo;
    return CSR_OK;
}

size_t encode_workspace(const csr::EncodeArgs &a, int algo)
{
    if (a.H == 0 || a.T == 0) return 0;
    if (algo == CSR_ENCODE_MFMA) return csr::encode_mfma_workspace_bytes(a.dict_count * a.sn, a.T, a.N, a.s);
    if (algo == CSR_ENCODE_SPLIT) return csr::encode_split_workspace_bytes(a);
    if (algo == kAlgoGramStep) return csr::encode_gramstep_workspace_bytes(a);
    return 0;
}

// Device address of `scratch` on the current device (looked up on the first call per device, then cached).
constexpr int kMaxScratchDevices = 64;
void *g_scratch_ptr[kMaxScratchDevices];
std::mutex g_scratch_mutex;

hipError_t static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxScratchDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

csr_status check_decode_desc(const csr_decode_desc *d, csr::DecodePlan *plan)
{
    if (!d) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: descriptor is NULL");
    if (d->B < 0 || d->T < 0) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: B=%d T=%lld must be >= 0", d->B, (long long)d->T);
    if (d->flags != 0) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: flags must be 0");
    if (d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0)
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: Hq=%d must be a positive multiple of Hkv=%d", d->Hq, d->Hkv);
    if (!valid_dtype(d->q_dtype) || !valid_dtype(d->dict_dtype) || !valid_dtype(d->coef_dtype) ||
        !valid_dtype(d->out_dtype) || !valid_itype(d->idx_dtype))
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: unknown dtype / index type");
    if (d->sK < 1 || d->sK > 32 || d->sV < 1 || d->sV > 32)
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: sK=%d sV=%d outside 1..32", d->sK, d->sV);
    if (d->N < 1) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: N=%d must be >= 1", d->N);
    if (d->idx_dtype == CSR_I16 && d->N > 65536)
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: N=%d does not fit unsigned 16-bit indices", d->N);
    if (!(d->scale >= 0.0f) || std::isinf(d->scale))
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: scale must be finite and >= 0 (0 selects 1/sqrt(d))");
    if (d->d != 128) return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: d=%d not supported (128)", d->d);
    if (d->Hq / d->Hkv > 8) return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: group size %d above 8", d->Hq / d->Hkv);
    if (d->Hkv > 65535 || d->B > 65535) return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: B or Hkv above 65535");
    if (d->T > (int64_t)1 << 20) return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: T above 2^20");
    const int snK = d->snK ? d->snK : 1, snV = d->snV ? d->snV : 1;
    for (int sn : {snK, snV}) {
        if (sn != 1 && sn != 2 && sn != 4 && sn != 8)
            return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: chunk counts snK=%d snV=%d must be 0, 1, 2, 4 or 8", d->snK, d->snV);
    }
    if (snK > 1 || snV > 1) {
        if (d->q_dtype != CSR_F16 || d->dict_dtype != CSR_F16)
            return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: chunked codes need fp16 queries and dictionaries");
        if (d->N % 128 != 0) return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: chunked codes need N a multiple of 128 (got %d)", d->N);
        if (snK * d->sK > 32 || snV * d->sV > 32)
            return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: more than 32 pairs per token and stream (sn * s)");
    }
    const bool rope = d->rope_base != 0.0f;
    if (rope) {
        if (!(d->rope_base > 1.0f) || std::isinf(d->rope_base))
            return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: rope_base must be 0 (off) or a finite number above 1");
        if (d->rope_layout != 0 && d->rope_layout != 1)
            return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: rope_layout=%d must be 0 or 1", d->rope_layout);
        if (d->rope_pos0 < 0 || d->rope_pos0 > (int64_t)1 << 40)
            return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: rope_pos0 outside 0 .. 2^40");
        if (d->q_dtype != CSR_F16 || d->dict_dtype != CSR_F16 || d->coef_dtype != CSR_F16 || d->idx_dtype != CSR_I16)
            return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: rotary keys need fp16 queries, dictionaries and coefficients and 16-bit indices");
        if (!csr::decode_rope_shape_supported(d->d, d->N, d->sK, snK))
            return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: rotary keys need whole-vector key codes and sK a multiple of 4 "
                                             "(N=%d, sK=%d, snK=%d)", d->N, d->sK, snK);
    } else if (d->rope_layout != 0 || d->rope_pos0 != 0) {
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: rope_layout and rope_pos0 must be 0 when rope_base is 0");
    }
    const int code_vecs = d->idx_dtype == CSR_I16 && d->coef_dtype == CSR_F16 && snK == 1 && snV == 1 && d->sK == d->sV &&
                                  (d->sK == 8 || d->sK == 16)
                              ? d->sK / 8 : 0;
    if (!csr::plan_decode(d->B, d->Hq, d->Hkv, d->T, d->d, d->N, snK, snV, rope, code_vecs, plan))
        return fail(CSR_ERR_UNSUPPORTED, "csr_decode_attn: N=%d atoms do not fit the LDS-resident score and histogram tables, or T=%lld "
                                         "exceeds what 128 token chunks hold", d->N, (long long)d->T);
    return CSR_OK;
}

}  // namespace

extern "C" {

int csr_version(void) { return CSR_VERSION; }

const char *csr_last_error(void) { return g_err; }

size_t csr_code_bytes(int32_t s, int32_t s_n, int32_t idx_dtype, int32_t coef_dtype)
{
    if (s < 1 || s_n < 1 || !valid_itype(idx_dtype) || !valid_dtype(coef_dtype)) return 0;
    const size_t ib = idx_dtype == CSR_I16 ? 2 : 4, cb = coef_dtype == CSR_F16 ? 2 : 4;
    return (size_t)s * (size_t)s_n * (ib + cb);
}

size_t csr_encode_workspace_bytes(const csr_encode_desc *desc)
{
    csr::EncodeArgs a{};
    int algo = 0;
    if (check_encode_desc(desc, &a, &algo) != CSR_OK) return (size_t)-1;
    return encode_workspace(a, algo);
}

csr_status csr_encode(const csr_encode_desc *desc, const void *X, const void *D, void *idx,
                      void *coef, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    csr::EncodeArgs a{};
    int algo = 0;
    csr_status st = check_encode_desc(desc, &a, &algo);
    if (st != CSR_OK) return st;
    if (desc->H == 0 || desc->T == 0) return CSR_OK;
    if (!X || !D || !idx || !coef) return fail(CSR_ERR_INVALID_ARG, "csr_encode: NULL data pointer");
    if (!aligned(X, 16) || !aligned(D, 16)) return fail(CSR_ERR_INVALID_ARG, "csr_encode: X and D must be 16-byte aligned");
    if (!aligned(idx, a.idx16 ? 2 : 4) || !aligned(coef, a.coef16 ? 2 : 4))
        return fail(CSR_ERR_INVALID_ARG, "csr_encode: idx and coef must be aligned to their element size");
    const size_t need = encode_workspace(a, algo);
    if (need) {
        if (!workspace || workspace_bytes < need || !aligned(workspace, 256))
            return fail(CSR_ERR_WORKSPACE, "csr_encode: workspace of %zu bytes (256-byte aligned) required, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    }
    if (desc->res_norm2 && !aligned(desc->res_norm2, 4)) return fail(CSR_ERR_INVALID_ARG, "csr_encode: res_norm2 must be 4-byte aligned");
    if (algo == kAlgoGramStep && !aligned(desc->gram, 16)) return fail(CSR_ERR_INVALID_ARG, "csr_encode: gram must be 16-byte aligned");
    a.X = X; a.D = D; a.idx = idx; a.coef = coef;
    a.res_norm2 = desc->res_norm2;
    a.workspace = workspace;
    a.stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = algo == CSR_ENCODE_MFMA ? csr::launch_encode_mfma(a)
                         : algo == CSR_ENCODE_SPLIT ? csr::launch_encode_split(a)
                         : algo == CSR_ENCODE_RESIDENT ? csr::launch_encode_resident(a)
                         : algo == CSR_ENCODE_GRAM ? csr::launch_encode_gram(a)
                         : algo == kAlgoGramStep ? csr::launch_encode_gramstep(a) : csr::launch_encode_valu(a);
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_encode: %s", hipGetErrorString(e));
    return CSR_OK;
}

csr_status csr_reconstruct(const csr_reconstruct_desc *d, const void *D, const void *idx, const void *coef,
                           void *out, void *hip_stream)
{
    if (!d) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: descriptor is NULL");
    if (d->H < 0 || d->T < 0) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: H=%d T=%lld must be >= 0", d->H, (long long)d->T);
    if (d->flags != 0) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: flags must be 0");
    if (!valid_dtype(d->dict_dtype) || !valid_dtype(d->coef_dtype) || !valid_dtype(d->out_dtype) || !valid_itype(d->idx_dtype))
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: unknown dtype / index type");
    if (d->s < 1 || d->s > 32) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: s=%d outside 1..32", d->s);
    if (d->N < 1 || d->N > (1 << 24)) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: N=%d outside 1..2^24", d->N);
    if (d->idx_dtype == CSR_I16 && d->N > 65536)
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: N=%d does not fit unsigned 16-bit indices", d->N);
    const int sn = d->s_n ? d->s_n : 1;
    if (sn < 1 || d->d < 8 || d->d > 1024 || d->d % (8 * sn) != 0)
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: d=%d must be a multiple of 8*s_n (s_n=%d) and at most 1024", d->d, sn);
    if (d->dict_count < 0 || (d->dict_count > 0 && d->H % d->dict_count != 0))
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: dict_count=%d must be 0 or divide H=%d", d->dict_count, d->H);
    const int64_t code_block = d->T * sn * d->s;
    if (d->code_stride_h < 0 || (d->code_stride_h > 0 && d->code_stride_h < code_block))
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: code_stride_h=%lld is smaller than one block's codes", (long long)d->code_stride_h);
    const int64_t st = d->out_stride_t ? d->out_stride_t : d->d;
    const int64_t sh = d->out_stride_h ? d->out_stride_h : d->T * st;
    if (st < d->d || st % 8 != 0 || sh % 8 != 0 || (d->T > 0 && d->H > 1 && sh < (d->T - 1) * st + d->d))
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: output strides (h=%lld, t=%lld) must be multiples of 8, >= d and not overlap",
                    (long long)sh, (long long)st);
    if (d->H == 0 || d->T == 0) return CSR_OK;
    if (!D || !idx || !coef || !out) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: NULL data pointer");
    if (!aligned(D, 16) || !aligned(out, 16)) return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: D and out must be 16-byte aligned");
    if (!aligned(idx, d->idx_dtype == CSR_I16 ? 2 : 4) || !aligned(coef, d->coef_dtype == CSR_F16 ? 2 : 4))
        return fail(CSR_ERR_INVALID_ARG, "csr_reconstruct: idx and coef must be aligned to their element size");
    csr::ReconstructArgs a{};
    a.D = D; a.idx = idx; a.coef = coef; a.out = out;
    a.H = d->H; a.T = d->T; a.d = d->d; a.N = d->N; a.s = d->s; a.sn = sn;
    a.dict_count = d->dict_count ? d->dict_count : d->H;
    a.code_stride_h = d->code_stride_h ? d->code_stride_h : code_block;
    a.out_stride_h = sh; a.out_stride_t = st;
    a.dict16 = d->dict_dtype == CSR_F16; a.coef16 = d->coef_dtype == CSR_F16;
    a.idx16 = d->idx_dtype == CSR_I16; a.out16 = d->out_dtype == CSR_F16;
    a.stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = csr::launch_reconstruct(a);
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_reconstruct: %s", hipGetErrorString(e));
    return CSR_OK;
}

size_t csr_gram_bytes(int32_t n_dicts, int32_t N)
{
    if (n_dicts < 0 || N < 0) return (size_t)-1;
    return (size_t)n_dicts * (size_t)N * (size_t)N * 2;
}

csr_status csr_gram_build(const void *D, int32_t n_dicts, int32_t N, int32_t d, void *gram, void *hip_stream)
{
    if (n_dicts < 0 || n_dicts > 65535) return fail(CSR_ERR_INVALID_ARG, "csr_gram_build: n_dicts=%d outside 0..65535", n_dicts);
    if (!csr::gram_build_supported(N, d))
        return fail(CSR_ERR_UNSUPPORTED, "csr_gram_build: needs rows of 64 or 128 elements and N a multiple of 32, at most 16384 (got d=%d N=%d)", d, N);
    if (n_dicts == 0) return CSR_OK;
    if (!D || !gram) return fail(CSR_ERR_INVALID_ARG, "csr_gram_build: NULL pointer");
    if (!aligned(D, 16) || !aligned(gram, 16)) return fail(CSR_ERR_INVALID_ARG, "csr_gram_build: D and gram must be 16-byte aligned");
    const hipError_t e = csr::launch_gram_build(D, n_dicts, N, d, gram, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_gram_build: %s", hipGetErrorString(e));
    return CSR_OK;
}

csr_status csr_atom_norms2(const void *D, int32_t dict_dtype, int64_t n_atoms, int32_t d, float *norms2, void *hip_stream)
{
    if (!valid_dtype(dict_dtype)) return fail(CSR_ERR_INVALID_ARG, "csr_atom_norms2: unknown dtype %d", dict_dtype);
    if (n_atoms < 0 || d < 1 || d > 65536)
        return fail(CSR_ERR_INVALID_ARG, "csr_atom_norms2: n_atoms=%lld must be >= 0 and d=%d in 1..65536", (long long)n_atoms, d);
    if (n_atoms == 0) return CSR_OK;
    if (!D || !norms2) return fail(CSR_ERR_INVALID_ARG, "csr_atom_norms2: NULL pointer");
    if (!aligned(D, dict_dtype == CSR_F16 ? 2 : 4) || !aligned(norms2, 4))
        return fail(CSR_ERR_INVALID_ARG, "csr_atom_norms2: misaligned pointer");
    const hipError_t e = csr::launch_atom_norms2(D, dict_dtype == CSR_F16, n_atoms, d, norms2, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_atom_norms2: %s", hipGetErrorString(e));
    return CSR_OK;
}

csr_status csr_check_codes(const void *idx, int32_t idx_dtype, int64_t count, int32_t N, int64_t *bad, void *hip_stream)
{
    if (!valid_itype(idx_dtype)) return fail(CSR_ERR_INVALID_ARG, "csr_check_codes: unknown index type %d", idx_dtype);
    if (count < 0 || N < 1) return fail(CSR_ERR_INVALID_ARG, "csr_check_codes: count=%lld must be >= 0 and N=%d >= 1", (long long)count, N);
    if (!bad || (count > 0 && !idx)) return fail(CSR_ERR_INVALID_ARG, "csr_check_codes: NULL pointer");
    if (!aligned(idx, idx_dtype == CSR_I16 ? 2 : 4) || !aligned(bad, 8)) return fail(CSR_ERR_INVALID_ARG, "csr_check_codes: misaligned pointer");
    const hipError_t e = csr::launch_check_codes(idx, idx_dtype == CSR_I16, count, N, bad, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_check_codes: %s", hipGetErrorString(e));
    return CSR_OK;
}

size_t csr_decode_workspace_bytes(const csr_decode_desc *desc)
{
    csr::DecodePlan p{};
    if (check_decode_desc(desc, &p) != CSR_OK) return (size_t)-1;
    return p.total_bytes;
}

// Argument checks and launch shared by csr_decode_attn and csr_decode_attn_static; `workspace` is checked by the caller.
static csr_status decode_run(const csr_decode_desc *desc, const csr::DecodePlan &p, const void *q, const void *DK,
                             const void *idxK, const void *coefK, const void *DV, const void *idxV,
                             const void *coefV, const int32_t *seq_lens, void *out, void *workspace, void *hip_stream)
{
    if (!q || !out || !DK || !DV) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: NULL data pointer");
    if (desc->T > 0 && (!idxK || !coefK || !idxV || !coefV))
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: NULL code pointer with T > 0");
    if (!aligned(q, 16) || !aligned(DK, 16) || !aligned(DV, 16) || !aligned(out, 16))
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: q, DK, DV and out must be 16-byte aligned");
    if (!aligned(idxK, 16) || !aligned(coefK, 16) || !aligned(idxV, 16) || !aligned(coefV, 16))
        return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: code streams must be 16-byte aligned");
    if (seq_lens && !aligned(seq_lens, 4)) return fail(CSR_ERR_INVALID_ARG, "csr_decode_attn: seq_lens misaligned");
    csr::DecodeArgs a{};
    a.q = q; a.DK = DK; a.idxK = idxK; a.coefK = coefK; a.DV = DV; a.idxV = idxV; a.coefV = coefV;
    a.seq_lens = seq_lens; a.out = out;
    a.B = desc->B; a.Hq = desc->Hq; a.Hkv = desc->Hkv; a.G = desc->Hq / desc->Hkv;
    a.T = desc->T; a.d = desc->d; a.N = desc->N; a.sK = desc->sK; a.sV = desc->sV;
    a.snK = desc->snK ? desc->snK : 1; a.snV = desc->snV ? desc->snV : 1;
    a.scale = desc->scale > 0.0f ? desc->scale : 1.0f / std::sqrt((float)desc->d);
    a.rope_base = desc->rope_base; a.rope_layout = desc->rope_layout; a.rope_pos0 = desc->rope_pos0;
    a.q16 = desc->q_dtype == CSR_F16;
    a.dict16 = desc->dict_dtype == CSR_F16;
    a.coef16 = desc->coef_dtype == CSR_F16;
    a.idx16 = desc->idx_dtype == CSR_I16;
    a.out16 = desc->out_dtype == CSR_F16;
    a.workspace = workspace;
    a.stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = csr::launch_decode(a, p);
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_decode_attn: %s", hipGetErrorString(e));
    return CSR_OK;
}

csr_status csr_decode_attn(const csr_decode_desc *desc, const void *q, const void *DK,
                           const void *idxK, const void *coefK, const void *DV, const void *idxV,
                           const void *coefV, const int32_t *seq_lens, void *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    csr::DecodePlan p{};
    csr_status st = check_decode_desc(desc, &p);
    if (st != CSR_OK) return st;
    if (desc->B == 0) return CSR_OK;
    if (!workspace || workspace_bytes < p.total_bytes || !aligned(workspace, 256))
        return fail(CSR_ERR_WORKSPACE, "csr_decode_attn: workspace of %zu bytes (256-byte aligned) required, got %zu",
                    p.total_bytes, workspace ? workspace_bytes : (size_t)0);
    return decode_run(desc, p, q, DK, idxK, coefK, DV, idxV, coefV, seq_lens, out, workspace, hip_stream);
}

csr_status csr_decode_attn_static(const csr_decode_desc *desc, const void *q, const void *DK,
                                  const void *idxK, const void *coefK, const void *DV, const void *idxV,
                                  const void *coefV, const int32_t *seq_lens, void *out, void *hip_stream)
{
    csr::DecodePlan p{};
    csr_status st = check_decode_desc(desc, &p);
    if (st != CSR_OK) return st;
    if (desc->B == 0) return CSR_OK;
    if (p.total_bytes > kStaticScratchBytes)
        return fail(CSR_ERR_WORKSPACE, "csr_decode_attn_static: this shape needs %zu bytes of scratch, the library's static "
                    "scratch holds %zu; use csr_decode_attn with a workspace", p.total_bytes, kStaticScratchBytes);
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return fail(CSR_ERR_DEVICE, "csr_decode_attn_static: static scratch: %s", hipGetErrorString(e));
    // Nothing in the scratch has to start at zero: every launch writes what the next one reads (chunk histograms
    // of chunks without tokens are never read), so the previous call's contents are simply overwritten.
    return decode_run(desc, p, q, DK, idxK, coefK, DV, idxV, coefV, seq_lens, out, ws, hip_stream);
}

}  // extern "C"
