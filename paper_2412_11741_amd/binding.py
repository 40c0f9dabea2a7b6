"""Thin ctypes binding of libcsr_hip.so (the C ABI of include/csr.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels.  PyTorch is
used for device memory and the current stream.  There is no CPU fallback: if the library is
missing, or a tensor is not on the GPU, the call raises.
"""
import ctypes
import os

import torch  # must precede loading the library: it brings the HIP runtime the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcsr_hip.so")

CSR_OK, CSR_ERR_INVALID_ARG, CSR_ERR_UNSUPPORTED, CSR_ERR_WORKSPACE, CSR_ERR_DEVICE = range(5)
CSR_F32, CSR_F16 = 0, 1
CSR_I32, CSR_I16 = 0, 1
CSR_ENCODE_AUTO, CSR_ENCODE_VALU, CSR_ENCODE_MFMA, CSR_ENCODE_SPLIT, CSR_ENCODE_RESIDENT, CSR_ENCODE_GRAM = 0, 1, 2, 3, 4, 5
CSR_FLAG_CLOSED_LOOP = 1

EXPORTS = ("csr_version", "csr_last_error", "csr_code_bytes", "csr_encode_workspace_bytes",
           "csr_encode", "csr_decode_workspace_bytes", "csr_decode_attn", "csr_reconstruct", "csr_atom_norms2",
           "csr_gram_bytes", "csr_gram_build", "csr_decode_attn_static", "csr_check_codes")
STATIC_SCRATCH_BYTES = 16 << 20   # CSR_STATIC_SCRATCH_BYTES of include/csr.h


class EncodeDesc(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int32), ("T", ctypes.c_int64), ("d", ctypes.c_int32),
                ("N", ctypes.c_int32), ("s", ctypes.c_int32), ("s_n", ctypes.c_int32),
                ("x_dtype", ctypes.c_int32),
                ("dict_dtype", ctypes.c_int32), ("coef_dtype", ctypes.c_int32),
                ("idx_dtype", ctypes.c_int32), ("x_stride_h", ctypes.c_int64),
                ("x_stride_t", ctypes.c_int64), ("dict_count", ctypes.c_int32),
                ("code_stride_h", ctypes.c_int64), ("algo", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("res_norm2", ctypes.c_void_p), ("gram", ctypes.c_void_p)]


class ReconstructDesc(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int32), ("T", ctypes.c_int64), ("d", ctypes.c_int32), ("N", ctypes.c_int32),
                ("s", ctypes.c_int32), ("s_n", ctypes.c_int32), ("dict_dtype", ctypes.c_int32),
                ("coef_dtype", ctypes.c_int32), ("idx_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("dict_count", ctypes.c_int32), ("code_stride_h", ctypes.c_int64),
                ("out_stride_h", ctypes.c_int64), ("out_stride_t", ctypes.c_int64), ("flags", ctypes.c_uint32)]


class DecodeDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("T", ctypes.c_int64), ("d", ctypes.c_int32), ("N", ctypes.c_int32),
                ("sK", ctypes.c_int32), ("sV", ctypes.c_int32), ("snK", ctypes.c_int32),
                ("snV", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_dtype", ctypes.c_int32), ("dict_dtype", ctypes.c_int32),
                ("coef_dtype", ctypes.c_int32), ("idx_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("rope_base", ctypes.c_float), ("rope_layout", ctypes.c_int32), ("rope_pos0", ctypes.c_int64)]


class CsrError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"csr status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2412_11741_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2412_11741_amd.build` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.csr_version.restype = ctypes.c_int
        L.csr_last_error.restype = ctypes.c_char_p
        L.csr_code_bytes.restype = sz
        L.csr_code_bytes.argtypes = [ctypes.c_int32] * 4
        L.csr_encode_workspace_bytes.restype = sz
        L.csr_encode_workspace_bytes.argtypes = [ctypes.POINTER(EncodeDesc)]
        L.csr_encode.restype = ctypes.c_int
        L.csr_encode.argtypes = [ctypes.POINTER(EncodeDesc), vp, vp, vp, vp, vp, sz, vp]
        L.csr_reconstruct.restype = ctypes.c_int
        L.csr_reconstruct.argtypes = [ctypes.POINTER(ReconstructDesc), vp, vp, vp, vp, vp]
        L.csr_gram_bytes.restype = sz
        L.csr_gram_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
        L.csr_gram_build.restype = ctypes.c_int
        L.csr_gram_build.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
        L.csr_atom_norms2.restype = ctypes.c_int
        L.csr_atom_norms2.argtypes = [vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp, vp]
        L.csr_check_codes.restype = ctypes.c_int
        L.csr_check_codes.argtypes = [vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp, vp]
        L.csr_decode_workspace_bytes.restype = sz
        L.csr_decode_workspace_bytes.argtypes = [ctypes.POINTER(DecodeDesc)]
        L.csr_decode_attn.restype = ctypes.c_int
        L.csr_decode_attn.argtypes = [ctypes.POINTER(DecodeDesc)] + [vp] * 10 + [sz, vp]
        L.csr_decode_attn_static.restype = ctypes.c_int
        L.csr_decode_attn_static.argtypes = [ctypes.POINTER(DecodeDesc)] + [vp] * 9 + [vp]
        _lib = L
    return _lib


def last_error():
    return lib().csr_last_error().decode()


def _check(status):
    if status != CSR_OK:
        raise CsrError(status, last_error())


_DT = {torch.float32: CSR_F32, torch.float16: CSR_F16}
_IT = {torch.int32: CSR_I32, torch.int16: CSR_I16}


def _dev(t, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor (no CPU path exists)")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def csr_code_bytes(s, s_n=1, idx_dtype=torch.int16, coef_dtype=torch.float16):
    return int(lib().csr_code_bytes(s, s_n, _IT[idx_dtype], _DT[coef_dtype]))


def encode_desc(X, D, s, coef_dtype, idx_dtype, algo=CSR_ENCODE_AUTO, code_stride_h=0, flags=0):
    """Descriptor from tensor shapes.  D may hold fewer dictionaries than X has blocks (D.shape[0] divides
    X.shape[0]): block h then uses dictionary h % D.shape[0]."""
    H, T, d = X.shape
    if X.stride(2) != 1:
        raise ValueError("X must be contiguous along d")
    return EncodeDesc(H=H, T=T, d=d, N=D.shape[-2], s=s, s_n=D.shape[1] if D.dim() == 4 else 1, x_dtype=_DT[X.dtype], dict_dtype=_DT[D.dtype],
                      coef_dtype=_DT[coef_dtype], idx_dtype=_IT[idx_dtype],
                      x_stride_h=X.stride(0) if H > 1 and T > 0 else 0,
                      x_stride_t=X.stride(1) if T > 1 else 0, dict_count=D.shape[0] if D.shape[0] != H else 0,
                      code_stride_h=code_stride_h, algo=algo, flags=flags)


def csr_encode_workspace_bytes(desc):
    n = lib().csr_encode_workspace_bytes(ctypes.byref(desc))
    if n == ctypes.c_size_t(-1).value:
        raise CsrError(CSR_ERR_INVALID_ARG, last_error())
    return int(n)


def csr_gram_build(D, out=None):
    """Gram matrices of fp16 dictionaries D [H', N, d] (or chunked [H', s_n, N, d / s_n]) -> fp16 [H', N, N]
    ([H', s_n, N, N]), for csr_encode(..., gram=...): C - c G[i, :], the Gram form of Eq.2-4's correlations."""
    _dev(D, "D")
    if D.dim() not in (3, 4) or D.dtype != torch.float16:
        raise ValueError("D must be an fp16 tensor [H', N, d] or [H', s_n, N, d / s_n]")
    D = D.contiguous()
    N, d = D.shape[-2], D.shape[-1]
    shape = tuple(D.shape[:-1]) + (N,)
    n_dicts = D.numel() // (N * d) if N * d else 0
    if out is None:
        out = torch.empty(shape, dtype=torch.float16, device=D.device)
    _dev(out, "out")
    if tuple(out.shape) != shape or out.dtype != torch.float16 or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous fp16 tensor of shape {shape}")
    _check(lib().csr_gram_build(_ptr(D), n_dicts, N, d, _ptr(out), _stream()))
    return out


def csr_encode(X, D, s, coef_dtype=None, idx_dtype=None, algo=CSR_ENCODE_AUTO, idx=None, coef=None,
               workspace=None, res_norm2=None, gram=None, closed_loop=False):
    """Matching Pursuit encode.  X [H, T, d], D [H, N, d] on the GPU -> (idx, coef) [H, T, s].
    Chunked: D [H, s_n, N, d / s_n] -> (idx, coef) [H, T, s_n, s], every chunk encoded on its own dictionary.
    D may hold H' < H dictionaries (H' divides H): block h uses dictionary h % H' (blocks ordered sequence-major,
    head-minor).  `idx` / `coef` may be views into a larger cache whose blocks are further apart (stride(0) larger
    than one block's codes, the rest contiguous): the codes are then written in place, e.g. appended at a token
    position.  `res_norm2` (fp32, [H, T] or [H, T, s_n], contiguous) receives the squared norm of each vector's
    final residual, i.e. its squared reconstruction error.  `gram` (csr_gram_build(D)) lets a few vectors per
    dictionary - one decoding step's - be encoded with one sweep of each dictionary instead of s.
    closed_loop: CSR_FLAG_CLOSED_LOOP - Eq.4 subtracts the coefficient as it is stored (rounded to coef_dtype)."""
    _dev(X, "X"); _dev(D, "D")
    if X.dim() != 3 or D.dim() not in (3, 4) or D.shape[0] < 1 or X.shape[0] % D.shape[0] != 0 or \
            D.shape[-1] * (D.shape[1] if D.dim() == 4 else 1) != X.shape[2]:
        raise ValueError("expected X [H, T, d] and D [H', N, d] or [H', s_n, N, d / s_n] with H' dividing H")
    D = D.contiguous()
    coef_dtype = coef_dtype or X.dtype
    idx_dtype = idx_dtype or (torch.int16 if X.dtype == torch.float16 else torch.int32)
    H, T, _ = X.shape
    shape = (H, T, s) if D.dim() == 3 else (H, T, D.shape[1], s)
    if idx is None:
        idx = torch.empty(shape, dtype=idx_dtype, device=X.device)
    if coef is None:
        coef = torch.empty(shape, dtype=coef_dtype, device=X.device)
    code_stride_h = 0
    for name, t, dt in (("idx", idx, idx_dtype), ("coef", coef, coef_dtype)):
        _dev(t, name)
        if tuple(t.shape) != shape or t.dtype != dt or (T > 0 and H > 0 and not t[0].is_contiguous()):
            raise ValueError(f"{name} must have shape {shape}, dtype {dt} and contiguous blocks")
    if H > 1 and T > 0:
        if idx.stride(0) != coef.stride(0):
            raise ValueError("idx and coef must have the same distance between blocks")
        code_stride_h = idx.stride(0)
    desc = encode_desc(X, D, s, coef_dtype, idx_dtype, algo, code_stride_h, CSR_FLAG_CLOSED_LOOP if closed_loop else 0)
    if res_norm2 is not None:
        _dev(res_norm2, "res_norm2")
        want = (H, T) if D.dim() == 3 else (H, T, D.shape[1])
        if tuple(res_norm2.shape) != want or res_norm2.dtype != torch.float32 or not res_norm2.is_contiguous():
            raise ValueError(f"res_norm2 must be a contiguous float32 tensor of shape {want}")
        desc.res_norm2 = res_norm2.data_ptr()
    if gram is not None:
        _dev(gram, "gram")
        want = tuple(D.shape[:-1]) + (D.shape[-2],)
        if tuple(gram.shape) != want or gram.dtype != torch.float16 or not gram.is_contiguous():
            raise ValueError(f"gram must be a contiguous fp16 tensor of shape {want} (csr_gram_build(D))")
        desc.gram = gram.data_ptr()
    need = csr_encode_workspace_bytes(desc)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().csr_encode(ctypes.byref(desc), _ptr(X), _ptr(D), _ptr(idx), _ptr(coef),
                            _ptr(workspace), wsb, _stream()))
    return idx, coef


def csr_reconstruct(D, idx, coef, out=None, out_dtype=None):
    """Eq.12, X~ = D r.  D [H', N, d] with codes [H, T, s], or chunked D [H', s_n, N, d / s_n] with codes
    [H, T, s_n, s] (H' divides H: block h uses dictionary h % H') -> out [H, T, d].  `idx` / `coef` may be views
    into a larger cache (blocks further apart); `out` may be a strided view with contiguous vectors."""
    for name, t in (("D", D), ("idx", idx), ("coef", coef)):
        _dev(t, name)
    chunked = D.dim() == 4
    if D.dim() not in (3, 4) or idx.dim() != D.dim() or coef.shape != idx.shape or idx.shape[0] % D.shape[0] != 0 or \
            (chunked and idx.shape[2] != D.shape[1]):
        raise ValueError("expected D [H', N, d] with codes [H, T, s] or D [H', s_n, N, d/s_n] with codes [H, T, s_n, s]")
    D = D.contiguous()
    H, T, s = idx.shape[0], idx.shape[1], idx.shape[-1]
    sn = D.shape[1] if chunked else 1
    d = D.shape[-1] * sn
    out_dtype = out_dtype or D.dtype
    if out is None:
        out = torch.empty((H, T, d), dtype=out_dtype, device=D.device)
    _dev(out, "out")
    if tuple(out.shape) != (H, T, d) or out.dtype != out_dtype or out.stride(2) != 1:
        raise ValueError(f"out must have shape {(H, T, d)}, dtype {out_dtype} and contiguous vectors")
    if H > 0 and T > 0 and (not idx[0].is_contiguous() or not coef[0].is_contiguous() or
                            (H > 1 and idx.stride(0) != coef.stride(0))):
        raise ValueError("idx and coef must have contiguous blocks, equally far apart")
    desc = ReconstructDesc(H=H, T=T, d=d, N=D.shape[-2], s=s, s_n=sn, dict_dtype=_DT[D.dtype],
                           coef_dtype=_DT[coef.dtype], idx_dtype=_IT[idx.dtype], out_dtype=_DT[out_dtype],
                           dict_count=D.shape[0] if D.shape[0] != H else 0,
                           code_stride_h=idx.stride(0) if H > 1 and T > 0 else 0,
                           out_stride_h=out.stride(0) if H > 1 and T > 0 else 0,
                           out_stride_t=out.stride(1) if T > 1 else 0, flags=0)
    _check(lib().csr_reconstruct(ctypes.byref(desc), _ptr(D), _ptr(idx), _ptr(coef), _ptr(out), _stream()))
    return out


def csr_atom_norms2(D, out=None):
    """Squared norms of the atoms of D [..., N, d] (fp16 or fp32) -> fp32 [..., N]; Section "Sparse representation"
    takes them to be 1."""
    _dev(D, "D")
    if D.dim() < 2 or D.dtype not in _DT:
        raise ValueError("D must be [..., N, d] in fp16 or fp32")
    D = D.contiguous()
    shape = tuple(D.shape[:-1])
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=D.device)
    _dev(out, "out")
    if tuple(out.shape) != shape or out.dtype != torch.float32 or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous fp32 tensor of shape {shape}")
    _check(lib().csr_atom_norms2(_ptr(D), _DT[D.dtype], out.numel(), D.shape[-1], _ptr(out), _stream()))
    return out


def csr_check_codes(idx, N, out=None):
    """Number of atom indices of `idx` (int16 read unsigned, or int32; contiguous) outside [0, N), as a one-element
    int64 GPU tensor (`out`, or a new one)."""
    _dev(idx, "idx")
    if idx.dtype not in _IT or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int16 or int32 tensor")
    if out is None:
        out = torch.empty(1, dtype=torch.int64, device=idx.device)
    _dev(out, "out")
    if out.dtype != torch.int64 or out.numel() != 1:
        raise ValueError("out must be one int64")
    _check(lib().csr_check_codes(_ptr(idx), _IT[idx.dtype], idx.numel(), int(N), _ptr(out), _stream()))
    return out


def decode_desc(q, DK, idxK, coefK, idxV, sV=None, scale=0.0, out_dtype=None, rope_base=0.0, rope_layout=0,
                rope_pos0=0):
    """Descriptor from tensor shapes.  Whole-vector codes: DK [Hkv, N, d], idx [B, Hkv, T, s].  Chunked codes:
    DK [Hkv, sn, N, d/sn], idx [B, Hkv, T, sn, s] (keys and values may differ in sn and s)."""
    B, Hq, d = q.shape
    Hkv, N = DK.shape[0], DK.shape[-2]
    T, sK = idxK.shape[2], idxK.shape[-1]
    snK = idxK.shape[3] if idxK.dim() == 5 else 1
    snV = idxV.shape[3] if idxV.dim() == 5 else 1
    return DecodeDesc(B=B, Hq=Hq, Hkv=Hkv, T=T, d=d, N=N, sK=sK, sV=idxV.shape[-1], snK=snK, snV=snV,
                      scale=float(scale),
                      q_dtype=_DT[q.dtype], dict_dtype=_DT[DK.dtype], coef_dtype=_DT[coefK.dtype],
                      idx_dtype=_IT[idxK.dtype], out_dtype=_DT[out_dtype or q.dtype], flags=0,
                      rope_base=float(rope_base), rope_layout=int(rope_layout), rope_pos0=int(rope_pos0))


def csr_decode_workspace_bytes(desc):
    n = lib().csr_decode_workspace_bytes(ctypes.byref(desc))
    if n == ctypes.c_size_t(-1).value:
        raise CsrError(CSR_ERR_INVALID_ARG, last_error())
    return int(n)


def csr_decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, scale=0.0, seq_lens=None, out=None,
                    out_dtype=None, workspace=None, rope_base=0.0, rope_layout=0, rope_pos0=0, static_scratch=False):
    """Decode attention on codes.  q [B, Hq, d]; DK/DV [Hkv, N, d]; codes [B, Hkv, T, s*] -> out [B, Hq, d].
    Chunked codes: DK [Hkv, sn, N, d/sn] with codes [B, Hkv, T, sn, s] (keys and values independently).
    rope_base > 1: the keys were coded before the rotary embedding; cache token t sits at position rope_pos0 + t.
    static_scratch: call csr_decode_attn_static (the library's own static device scratch, no workspace; `out` must
    then be given, so that nothing at all is allocated)."""
    for name, t in (("q", q), ("DK", DK), ("idxK", idxK), ("coefK", coefK), ("DV", DV), ("idxV", idxV),
                    ("coefV", coefV)):
        _dev(t, name)
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if (DV.shape[0] != DK.shape[0] or DV.shape[-2] != DK.shape[-2] or DV.dtype != DK.dtype or
            coefV.dtype != coefK.dtype or idxV.dtype != idxK.dtype):
        raise ValueError("key and value dictionaries / codes must share KV heads, atoms per dictionary and dtypes")
    for D_, i_, what in ((DK, idxK, "key"), (DV, idxV, "value")):
        sn = i_.shape[3] if i_.dim() == 5 else 1
        want = (DK.shape[0], sn, D_.shape[-2], q.shape[2] // sn) if i_.dim() == 5 else (DK.shape[0], D_.shape[-2], q.shape[2])
        if tuple(D_.shape) != want:
            raise ValueError(f"{what} dictionary shape {tuple(D_.shape)} does not match its codes (expected {want})")
    if idxV.shape[:3] != idxK.shape[:3] or coefK.shape != idxK.shape or coefV.shape != idxV.shape:
        raise ValueError("code tensors disagree in shape")
    desc = decode_desc(q, DK, idxK, coefK, idxV, scale=scale, out_dtype=out_dtype, rope_base=rope_base,
                       rope_layout=rope_layout, rope_pos0=rope_pos0)
    if out is None:
        if static_scratch:
            raise ValueError("static_scratch: pass `out` (the call itself allocates nothing)")
        out = torch.empty(q.shape, dtype=out_dtype or q.dtype, device=q.device)
    if seq_lens is not None:
        _dev(seq_lens, "seq_lens")
        if seq_lens.dtype != torch.int32 or seq_lens.numel() != q.shape[0]:
            raise ValueError("seq_lens must be int32 [B]")
    if static_scratch:
        if workspace is not None:
            raise ValueError("static_scratch takes no workspace")
        _check(lib().csr_decode_attn_static(ctypes.byref(desc), _ptr(q), _ptr(DK), _ptr(idxK), _ptr(coefK), _ptr(DV),
                                            _ptr(idxV), _ptr(coefV), _ptr(seq_lens), _ptr(out), _stream()))
        return out
    need = csr_decode_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().csr_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(DK), _ptr(idxK), _ptr(coefK), _ptr(DV),
                                 _ptr(idxV), _ptr(coefV), _ptr(seq_lens), _ptr(out), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()))
    return out


def csr_decode_attn_static(q, DK, idxK, coefK, DV, idxV, coefV, out, scale=0.0, seq_lens=None, out_dtype=None,
                           rope_base=0.0, rope_layout=0, rope_pos0=0):
    """csr_decode_attn on the library's static device scratch (at most STATIC_SCRATCH_BYTES of it): no workspace, and
    nothing is allocated - `out` is the caller's.  Calls that overlap on one GPU race on the scratch."""
    return csr_decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, scale=scale, seq_lens=seq_lens, out=out,
                           out_dtype=out_dtype or out.dtype, rope_base=rope_base, rope_layout=rope_layout,
                           rope_pos0=rope_pos0, static_scratch=True)
