"""ctypes binding of libawq_mi355x.so (see include/awq_mi355x.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the
shared library.  PyTorch is used for device memory (``tensor.data_ptr()``) and
streams (``torch.cuda.current_stream()``).  There is no CPU fallback: if the
library has not been built, importing a function from it raises.

Function names and argument order mirror the C ABI:
    awq_act_scale, awq_apply_inv_scale            (AWQ Sec. 3.2, Eq. 4-5)
    awq_rmsnorm_inv_scale                         (Sec. 4.2 fused normalisation with the 1/s of Eq. 4)
    awq_quantize_pack, awq_unpack                 (Sec. 3.2, Eq. 1-2; Sec. 4.2 packing)
    awq_w4a16_linear, awq_w4a16_linear_multi      (Sec. 4.2 fused dequantization, kernel fusion)
    awq_search_scale                              (Sec. 3.2, the search for the scale, Eq. 4-5)
    awq_quantize_pack_clip                        (Sec. 3.2 weight clipping)
    awq_decode_attention                          (Sec. 4.2 fused attention: rotary embedding, cache update)
    awq_*_w3                                      (Sec. 5, INT3-g128 variant: quantize, unpack, decode)
    awq_*_w2                                      (Sec. 5, INT2-g64 variant: quantize, unpack, decode)
"""
from __future__ import annotations

import ctypes
import os

import torch  # first: its HIP runtime must be the one this process uses

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libawq_mi355x.so")
GROUP = 128

EXPORTS = [
    "awq_version", "awq_status_string", "awq_packed_sizes", "awq_act_scale",
    "awq_apply_inv_scale", "awq_quantize_pack", "awq_unpack", "awq_linear_workspace_bytes",
    "awq_w4a16_linear", "awq_w4a16_linear_multi",
    "awq_search_scale_workspace_bytes", "awq_search_scale", "awq_quantize_pack_clip",
    "awq_packed_sizes_w3", "awq_quantize_pack_w3", "awq_unpack_w3", "awq_w3a16_linear",
    "awq_w3a16_linear_multi", "awq_rmsnorm_inv_scale", "awq_read_probe",
    "awq_decode_attention_workspace_bytes", "awq_decode_attention", "awq_silu_mul",
    "awq_w4a16_linear_fused_multi", "awq_w4a16_linear_fused_fits",
    "awq_repack_w3_to_w4", "awq_w3a16_prefill_workspace_bytes", "awq_w3a16_linear_prefill",
    "awq_packed_sizes_w2", "awq_quantize_pack_w2", "awq_unpack_w2", "awq_w2a16_linear",
    "awq_w2a16_linear_multi",
    "awq_last_grouped_plan", "awq_static_scratch_bytes", "awq_w4a16_linear_static",
    "awq_quantize_pack_multi", "awq_w4a16_linear_chain", "awq_blob_header_init", "awq_blob_header_check",
    "awq_act_scale_multi",
]
MULTI_MAX = 56


class LinearDesc(ctypes.Structure):
    """awq_linear_desc of the C ABI."""
    _fields_ = [("x_f16", ctypes.c_void_p), ("qweight", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p),
                ("y_f16", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64)]

_lib = None


class BlobHeader(ctypes.Structure):
    """awq_blob_header of the C ABI (64 bytes)."""
    _fields_ = [("magic", ctypes.c_char * 8), ("layout_version", ctypes.c_uint32), ("bits", ctypes.c_uint32),
                ("group", ctypes.c_uint32), ("reserved", ctypes.c_uint32), ("N", ctypes.c_int64),
                ("K", ctypes.c_int64), ("qweight_bytes", ctypes.c_uint64), ("scales_bytes", ctypes.c_uint64),
                ("zeros_bytes", ctypes.c_uint64)]


def awq_blob_header(bits: int, N: int, K: int, group: int | None = None) -> BlobHeader:
    """Header for a file holding the packed arrays of an [N,K] weight in the `bits`-bit layout."""
    h = BlobHeader()
    _check(load().awq_blob_header_init(ctypes.byref(h), bits, N, K, group or (64 if bits == 2 else GROUP)),
           "awq_blob_header_init")
    return h


def awq_blob_header_check(h: BlobHeader) -> None:
    _check(load().awq_blob_header_check(ctypes.byref(h)), "awq_blob_header_check")


class QuantizeDesc(ctypes.Structure):
    """awq_quantize_desc of the C ABI."""
    _fields_ = [("W_f16", ctypes.c_void_p), ("s", ctypes.c_void_p), ("N", ctypes.c_int64),
                ("K", ctypes.c_int64), ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("zeros", ctypes.c_void_p)]


QUANTIZE_MULTI_MAX = 64


class ActScaleDesc(ctypes.Structure):
    """awq_act_scale_desc of the C ABI."""
    _fields_ = [("X_f16", ctypes.c_void_p), ("T", ctypes.c_int64), ("K", ctypes.c_int64), ("s", ctypes.c_void_p)]


ACT_SCALE_MULTI_MAX = 64


class FusedDesc(ctypes.Structure):
    _fields_ = [("linear", LinearDesc), ("pre_f16", ctypes.c_void_p), ("residual_f16", ctypes.c_void_p),
                ("eps", ctypes.c_float), ("pre_op", ctypes.c_int)]


PRE_NONE, PRE_RMSNORM, PRE_SCALE, FUSED_MAX = 0, 1, 2, 24


class AwqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def load() -> ctypes.CDLL:
    """Load the shared library (built by ``paper_2306_00978_amd.build``); no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    # AWQ_MI355X_LIBRARY names another build of the same library (the host-sanitized one of the tests)
    path = os.environ.get("AWQ_MI355X_LIBRARY") or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2306_00978_amd.build` "
            "(there is no CPU or PyTorch fallback for this library)")
    lib = ctypes.CDLL(path)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.awq_version.restype = i32
    lib.awq_version.argtypes = []
    lib.awq_status_string.restype = ctypes.c_char_p
    lib.awq_status_string.argtypes = [i32]
    lib.awq_packed_sizes.restype = i32
    lib.awq_packed_sizes.argtypes = [i64, i64, i32, szp, szp, szp]
    lib.awq_act_scale.restype = i32
    lib.awq_act_scale.argtypes = [vp, i64, i64, ctypes.c_float, vp, vp]
    lib.awq_apply_inv_scale.restype = i32
    lib.awq_apply_inv_scale.argtypes = [vp, vp, i64, i64, vp, vp]
    lib.awq_quantize_pack.restype = i32
    lib.awq_quantize_pack.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_unpack.restype = i32
    lib.awq_unpack.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_linear_workspace_bytes.restype = sz
    lib.awq_linear_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.awq_w4a16_linear.restype = i32
    lib.awq_w4a16_linear.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, sz, vp]
    lib.awq_w4a16_linear_multi.restype = i32
    lib.awq_w4a16_linear_multi.argtypes = [ctypes.POINTER(LinearDesc), i32, i64, i32, vp, sz, vp]
    lib.awq_quantize_pack_clip.restype = i32
    lib.awq_quantize_pack_clip.argtypes = [vp, vp, i64, i64, i32, ctypes.POINTER(ctypes.c_float), i32,
                                           vp, i64, vp, vp, vp, vp, vp]
    lib.awq_packed_sizes_w3.restype = i32
    lib.awq_packed_sizes_w3.argtypes = [i64, i64, i32, szp, szp, szp]
    lib.awq_quantize_pack_w3.restype = i32
    lib.awq_quantize_pack_w3.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_unpack_w3.restype = i32
    lib.awq_unpack_w3.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_w3a16_linear.restype = i32
    lib.awq_w3a16_linear.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
    lib.awq_decode_attention_workspace_bytes.restype = sz
    lib.awq_decode_attention_workspace_bytes.argtypes = [i64, i64, i64]
    lib.awq_decode_attention.restype = i32
    lib.awq_decode_attention.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ctypes.c_float,
                                         vp, vp, sz, vp]
    lib.awq_w4a16_linear_fused_multi.restype = i32
    lib.awq_w4a16_linear_fused_multi.argtypes = [ctypes.POINTER(FusedDesc), i32, i64, i32, vp]
    lib.awq_w4a16_linear_fused_fits.restype = i32
    lib.awq_w4a16_linear_fused_fits.argtypes = [i64, i64, i64, i32]
    lib.awq_repack_w3_to_w4.restype = i32
    lib.awq_repack_w3_to_w4.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.awq_w3a16_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.awq_w3a16_prefill_workspace_bytes.argtypes = [i64, i64, i32]
    lib.awq_w3a16_linear_prefill.restype = i32
    lib.awq_w3a16_linear_prefill.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, ctypes.c_size_t, vp]
    lib.awq_last_grouped_plan.restype = i32
    lib.awq_last_grouped_plan.argtypes = []
    lib.awq_act_scale_multi.restype = i32
    lib.awq_act_scale_multi.argtypes = [ctypes.POINTER(ActScaleDesc), i32, ctypes.c_float, vp]
    lib.awq_quantize_pack_multi.restype = i32
    lib.awq_quantize_pack_multi.argtypes = [ctypes.POINTER(QuantizeDesc), i32, i32, vp]
    lib.awq_blob_header_init.restype = i32
    lib.awq_blob_header_init.argtypes = [ctypes.c_void_p, i32, i64, i64, i32]
    lib.awq_blob_header_check.restype = i32
    lib.awq_blob_header_check.argtypes = [ctypes.c_void_p]
    lib.awq_w4a16_linear_chain.restype = i32
    lib.awq_w4a16_linear_chain.argtypes = [ctypes.c_void_p, i32, i64, i32, vp, i32, vp]
    lib.awq_static_scratch_bytes.restype = sz
    lib.awq_static_scratch_bytes.argtypes = []
    lib.awq_w4a16_linear_static.restype = i32
    lib.awq_w4a16_linear_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
    lib.awq_silu_mul.restype = i32
    lib.awq_silu_mul.argtypes = [vp, vp, i64, vp, vp]
    lib.awq_read_probe.restype = i32
    lib.awq_read_probe.argtypes = [vp, sz, vp, vp]
    lib.awq_rmsnorm_inv_scale.restype = i32
    lib.awq_rmsnorm_inv_scale.argtypes = [vp, vp, vp, i64, i64, ctypes.c_float, vp, vp]
    lib.awq_packed_sizes_w2.restype = i32
    lib.awq_packed_sizes_w2.argtypes = [i64, i64, i32, szp, szp, szp]
    lib.awq_quantize_pack_w2.restype = i32
    lib.awq_quantize_pack_w2.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_unpack_w2.restype = i32
    lib.awq_unpack_w2.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.awq_w2a16_linear.restype = i32
    lib.awq_w2a16_linear.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
    lib.awq_w2a16_linear_multi.restype = i32
    lib.awq_w2a16_linear_multi.argtypes = [ctypes.POINTER(LinearDesc), i32, i64, i32, vp]
    lib.awq_w3a16_linear_multi.restype = i32
    lib.awq_w3a16_linear_multi.argtypes = [ctypes.POINTER(LinearDesc), i32, i64, i32, vp]
    lib.awq_search_scale_workspace_bytes.restype = sz
    lib.awq_search_scale_workspace_bytes.argtypes = [i64, i64, i64, i32, i32]
    lib.awq_search_scale.restype = i32
    lib.awq_search_scale.argtypes = [vp, vp, i64, i64, i64, ctypes.POINTER(ctypes.c_float), i32, i32,
                                     vp, sz, vp, vp, vp, vp]
    _lib = lib
    return lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise AwqError(status, what)


def _dev(t: torch.Tensor, dtype, what: str) -> torch.Tensor:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{what}: expected a contiguous {dtype} tensor on the GPU")
    return t


def awq_version() -> int:
    return load().awq_version()


def status_string(status: int) -> str:
    return load().awq_status_string(int(status)).decode()


def awq_packed_sizes(N: int, K: int, group: int = GROUP):
    q, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().awq_packed_sizes(N, K, group, ctypes.byref(q), ctypes.byref(s), ctypes.byref(z)),
           "awq_packed_sizes")
    return q.value, s.value, z.value


def awq_act_scale(X: torch.Tensor, alpha: float = 0.5, out: torch.Tensor | None = None):
    """s[k] = max(mean_t |X[t,k]|, 1e-4)^alpha; X [T,K] fp16 -> s [K] fp32."""
    _dev(X, torch.float16, "X")
    T, K = X.shape
    s = out if out is not None else torch.empty(K, dtype=torch.float32, device=X.device)
    _dev(s, torch.float32, "s")
    _check(load().awq_act_scale(_ptr(X), T, K, float(alpha), _ptr(s), _stream()), "awq_act_scale")
    return s


def prepare_act_scale_multi(matrices, alpha: float = 0.5):
    """Marshal one awq_act_scale_multi call.  `matrices` is a list of (X [T,K] fp16, s [K] fp32);
    returns a zero-argument callable that enqueues the call on the then-current stream."""
    if not 1 <= len(matrices) <= ACT_SCALE_MULTI_MAX:
        raise ValueError(f"1..{ACT_SCALE_MULTI_MAX} matrices per call")
    descs = (ActScaleDesc * len(matrices))()
    for i, (X, s) in enumerate(matrices):
        _dev(X, torch.float16, "X")
        _dev(s, torch.float32, "s")
        T, K = X.shape
        if s.numel() != K:
            raise ValueError("s must have K elements")
        descs[i] = ActScaleDesc(X.data_ptr(), T, K, s.data_ptr())
    fn = load().awq_act_scale_multi
    count = len(matrices)
    keep = list(matrices)

    def call(_keep=keep):
        st = fn(descs, count, float(alpha), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != 0:
            raise AwqError(st, "awq_act_scale_multi")
    return call


def awq_act_scale_multi(Xs, alpha: float = 0.5):
    """[X, ...] -> [s, ...]: awq_act_scale of every matrix in one call of the library."""
    full = [(X, torch.empty(X.shape[1], dtype=torch.float32, device=X.device)) for X in Xs]
    prepare_act_scale_multi(full, alpha)()
    return [m[1] for m in full]


def awq_apply_inv_scale(x: torch.Tensor, s: torch.Tensor, out: torch.Tensor | None = None):
    """xs = fp16(fp32(x) / s); x [M,K] fp16, s [K] fp32."""
    _dev(x, torch.float16, "x")
    _dev(s, torch.float32, "s")
    M, K = x.shape
    if s.numel() != K:
        raise ValueError("s must have K elements")
    xs = out if out is not None else torch.empty_like(x)
    _dev(xs, torch.float16, "xs")
    _check(load().awq_apply_inv_scale(_ptr(x), _ptr(s), M, K, _ptr(xs), _stream()),
           "awq_apply_inv_scale")
    return xs


def awq_quantize_pack(W: torch.Tensor, s: torch.Tensor | None = None, group: int = GROUP,
                      out=None):
    """W [N,K] fp16, s [K] fp32 or None -> (qweight u8[N*K/2], scales f16[N*K/128],
    zeros u8[N*K/256]) in the packed layout."""
    _dev(W, torch.float16, "W")
    N, K = W.shape
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if out is None:
        qweight = torch.empty(qb, dtype=torch.uint8, device=W.device)
        scales = torch.empty(sb // 2, dtype=torch.float16, device=W.device)
        zeros = torch.empty(zb, dtype=torch.uint8, device=W.device)
    else:
        qweight, scales, zeros = out
        if qweight.numel() * qweight.element_size() < qb or scales.numel() * 2 < sb \
                or zeros.numel() * zeros.element_size() < zb:
            raise ValueError("output buffers are too small")
    _check(load().awq_quantize_pack(_ptr(W), _ptr(s), N, K, group, _ptr(qweight), _ptr(scales),
                                    _ptr(zeros), _stream()), "awq_quantize_pack")
    return qweight, scales, zeros


def prepare_quantize_pack(W: torch.Tensor, s: torch.Tensor | None, out, group: int = GROUP):
    """Marshal the arguments of awq_quantize_pack once and return a zero-argument callable that
    enqueues it on the then-current stream (a pass over many matrices costs one C call each).
    out = (qweight, scales, zeros) buffers; every tensor must stay alive and in place."""
    _dev(W, torch.float16, "W")
    N, K = W.shape
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    qb, sb, zb = awq_packed_sizes(N, K, group)
    qweight, scales, zeros = out
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("output buffers are too small")
    fn = load().awq_quantize_pack
    c = ctypes
    fixed = (c.c_void_p(W.data_ptr()), c.c_void_p(_ptr(s)), c.c_int64(N), c.c_int64(K), c.c_int(group),
             c.c_void_p(qweight.data_ptr()), c.c_void_p(scales.data_ptr()), c.c_void_p(zeros.data_ptr()))
    keep = (W, s, qweight, scales, zeros)

    def call(_keep=keep):
        st = fn(*fixed, c.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != 0:
            raise AwqError(st, "awq_quantize_pack")
    return call


def prepare_quantize_pack_multi(matrices, group: int = GROUP):
    """Marshal one awq_quantize_pack_multi call.  `matrices` is a list of (W, s or None,
    (qweight, scales, zeros)); returns a zero-argument callable that enqueues the call on the
    then-current stream.  Every tensor must stay alive and in place."""
    if not 1 <= len(matrices) <= QUANTIZE_MULTI_MAX:
        raise ValueError(f"1..{QUANTIZE_MULTI_MAX} matrices per call")
    descs = (QuantizeDesc * len(matrices))()
    for i, (W, s, out) in enumerate(matrices):
        _dev(W, torch.float16, "W")
        N, K = W.shape
        if s is not None:
            _dev(s, torch.float32, "s")
            if s.numel() != K:
                raise ValueError("s must have K elements")
        qb, sb, zb = awq_packed_sizes(N, K, group)
        qweight, scales, zeros = out
        if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
                or zeros.numel() * zeros.element_size() < zb:
            raise ValueError("output buffers are too small")
        descs[i] = QuantizeDesc(W.data_ptr(), _ptr(s), N, K, qweight.data_ptr(), scales.data_ptr(),
                                zeros.data_ptr())
    fn = load().awq_quantize_pack_multi
    count = len(matrices)
    keep = list(matrices)

    def call(_keep=keep):
        st = fn(descs, count, group, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != 0:
            raise AwqError(st, "awq_quantize_pack_multi")
    return call


def awq_quantize_pack_multi(matrices, group: int = GROUP):
    """[(W, s or None), ...] -> [(qweight, scales, zeros), ...], all in one call of the library."""
    full = []
    for W, s in matrices:
        N, K = W.shape
        qb, sb, zb = awq_packed_sizes(N, K, group)
        full.append((W, s, (torch.empty(qb, dtype=torch.uint8, device=W.device),
                            torch.empty(sb // 2, dtype=torch.float16, device=W.device),
                            torch.empty(zb, dtype=torch.uint8, device=W.device))))
    prepare_quantize_pack_multi(full, group)()
    return [m[2] for m in full]


def awq_unpack(qweight, scales, zeros, N: int, K: int, group: int = GROUP):
    """Packed arrays -> (codes u8[N,K], scales f16[N,G], zeros u8[N,G])."""
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("packed buffers are too small for this shape")
    G = K // group
    dev = qweight.device
    codes = torch.empty((N, K), dtype=torch.uint8, device=dev)
    sc = torch.empty((N, G), dtype=torch.float16, device=dev)
    zr = torch.empty((N, G), dtype=torch.uint8, device=dev)
    _check(load().awq_unpack(_ptr(qweight), _ptr(scales), _ptr(zeros), N, K, group, _ptr(codes),
                             _ptr(sc), _ptr(zr), _stream()), "awq_unpack")
    return codes, sc, zr


def prepare_linear(x: torch.Tensor, qweight, scales, zeros, y: torch.Tensor, N: int,
                   group: int = GROUP, workspace: torch.Tensor | None = None):
    """Marshal the arguments of awq_w4a16_linear once and return a callable that enqueues the
    layer on the then-current stream, or on the raw stream handle passed to it (tight decode
    loops, graph capture).
    The tensors must stay alive and in place for as long as the callable is used."""
    _dev(x, torch.float16, "x")
    _dev(y, torch.float16, "y")
    M, K = x.shape
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb or y.numel() != M * N:
        raise ValueError("buffer sizes do not match the shape")
    # the workspace is optional, as in the C ABI: without one the call runs without the K split
    need = awq_linear_workspace_bytes(M, N, K, group)
    use_ws = bool(need) and workspace is not None
    if use_ws and workspace.numel() * workspace.element_size() < need:
        raise ValueError(f"the workspace of this shape is {need} bytes")
    fn = load().awq_w4a16_linear
    c = ctypes
    fixed = (c.c_void_p(x.data_ptr()), c.c_void_p(qweight.data_ptr()), c.c_void_p(scales.data_ptr()),
             c.c_void_p(zeros.data_ptr()), c.c_void_p(y.data_ptr()), c.c_int64(M), c.c_int64(N),
             c.c_int64(K), c.c_int(group), c.c_void_p(workspace.data_ptr() if use_ws else None),
             c.c_size_t(workspace.numel() * workspace.element_size() if use_ws else 0))
    keep = (x, qweight, scales, zeros, y, workspace)

    def call(stream=None, _keep=keep):
        st = fn(*fixed, c.c_void_p(torch.cuda.current_stream().cuda_stream if stream is None else stream))
        if st != 0:
            raise AwqError(st, "awq_w4a16_linear")
    return call


def awq_linear_workspace_bytes(M: int, N: int, K: int, group: int = GROUP) -> int:
    return int(load().awq_linear_workspace_bytes(M, N, K, group))


def awq_w4a16_linear(x: torch.Tensor, qweight, scales, zeros, N: int, group: int = GROUP,
                     out: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """y[M,N] = x[M,K] . dequant(qweight, scales, zeros)^T (fp16 in, fp32 accumulate, fp16 out).
    x must already be divided by the activation-aware scale s.  `workspace`: a uint8 tensor of
    awq_linear_workspace_bytes() bytes, None (allocated here when the shape uses one) or False
    (run without it)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("packed buffers are too small for this shape")
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    if y.numel() != M * N:
        raise ValueError("y must have M*N elements")
    need = awq_linear_workspace_bytes(M, N, K, group)
    ws_bytes = 0
    if workspace is False or not need:
        workspace = None                              # False: run without the K split
    else:
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
        ws_bytes = workspace.numel() * workspace.element_size()
    _check(load().awq_w4a16_linear(_ptr(x), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(y),
                                   M, N, K, group, _ptr(workspace), ws_bytes,
                                   _stream()), "awq_w4a16_linear")
    return y


def awq_static_scratch_bytes() -> int:
    return int(load().awq_static_scratch_bytes())


def awq_w4a16_linear_static(x: torch.Tensor, qweight, scales, zeros, N: int, y: torch.Tensor,
                            group: int = GROUP):
    """awq_w4a16_linear for callers that cannot allocate: the scratch of the K-range prefill form
    comes from the array built into the library (one per GPU, shared by all calls on it: do not
    overlap calls).  The caller brings y; nothing is allocated here or in the library."""
    _dev(x, torch.float16, "x")
    _dev(y, torch.float16, "y")
    M, K = x.shape
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb or y.numel() != M * N:
        raise ValueError("buffer sizes do not match the shape")
    _check(load().awq_w4a16_linear_static(_ptr(x), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(y),
                                          M, N, K, group, _stream()), "awq_w4a16_linear_static")
    return y


def _prepare_multi(linears, group, sizes, name, with_workspace):
    """Marshalling shared by the grouped decode calls of the 4-, 3- and 2-bit layouts: `sizes` gives
    the packed sizes of the layout, `name` the C entry point."""
    if not 1 <= len(linears) <= MULTI_MAX:
        raise ValueError(f"1..{MULTI_MAX} linears per grouped call")
    descs = (LinearDesc * len(linears))()
    M = None
    for i, (x, qweight, scales, zeros, y, N) in enumerate(linears):
        _dev(x, torch.float16, "x")
        _dev(y, torch.float16, "y")
        m, K = x.shape
        if M is None:
            M = m
        if m != M:
            raise ValueError("all linears of a grouped call share M")
        qb, sb, zb = sizes(N, K, group)
        if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
                or zeros.numel() * zeros.element_size() < zb or y.numel() != M * N:
            raise ValueError("buffer sizes do not match the shape")
        descs[i] = LinearDesc(x.data_ptr(), qweight.data_ptr(), scales.data_ptr(), zeros.data_ptr(),
                              y.data_ptr(), N, K)
    fn = getattr(load(), name)
    count = len(linears)
    keep = list(linears)
    extra = (None, 0) if with_workspace else ()

    def call(stream=None, _keep=keep):
        """stream: a raw hipStream_t handle (torch.cuda.Stream().cuda_stream); None = torch's current one"""
        st = fn(descs, count, M, group, *extra,
                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream if stream is None else stream))
        if st != 0:
            raise AwqError(st, name)
    return call


def prepare_linear_multi(linears, group: int = GROUP):
    """Marshal one grouped decode call.  `linears` is a list of (x, qweight, scales, zeros, y, N)
    with the same M <= 16 everywhere.  Returns a callable that enqueues ONE
    awq_w4a16_linear_multi on the then-current stream (or on the raw stream handle passed to it);
    the tensors must stay alive."""
    return _prepare_multi(linears, group, awq_packed_sizes, "awq_w4a16_linear_multi", True)


def awq_w4a16_linear_multi(linears, group: int = GROUP):
    """The linears of `linears` = [(x, qweight, scales, zeros, y, N), ...] in one kernel launch."""
    prepare_linear_multi(linears, group)()
    return [l[4] for l in linears]


def awq_search_scale(W: torch.Tensor, X: torch.Tensor, alphas, group: int = GROUP,
                     workspace: torch.Tensor | None = None):
    """Grid search of Eq. 5 for one linear: W [N,K] fp16, X [T,K] fp16 calibration rows,
    `alphas` a sequence of values in [0,1].  Returns device tensors
    (best [1] int32, losses [len(alphas)] fp64, s_best [K] fp32); nothing is synchronised."""
    _dev(W, torch.float16, "W")
    _dev(X, torch.float16, "X")
    N, K = W.shape
    T, K2 = X.shape
    if K2 != K:
        raise ValueError("W and X disagree on K")
    n = len(alphas)
    arr = (ctypes.c_float * max(n, 1))(*[float(a) for a in alphas])
    need = load().awq_search_scale_workspace_bytes(T, N, K, n, group)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=W.device)
    losses = torch.empty(max(n, 1), dtype=torch.float64, device=W.device)
    best = torch.empty(1, dtype=torch.int32, device=W.device)
    s_best = torch.empty(K, dtype=torch.float32, device=W.device)
    _check(load().awq_search_scale(W.data_ptr(), X.data_ptr(), T, N, K, arr, n, group,
                                   workspace.data_ptr(), workspace.numel(), losses.data_ptr(),
                                   best.data_ptr(), s_best.data_ptr(), _stream()), "awq_search_scale")
    return best, losses[:n], s_best


def awq_quantize_pack_clip(W: torch.Tensor, s: torch.Tensor | None, ratios, group: int = GROUP,
                           out=None, want_choice: bool = False, xs: torch.Tensor | None = None):
    """awq_quantize_pack with the per-group clipping search over `ratios` (values in (0, 1]);
    with `xs` ([T,K] fp16 rows of x/s, T <= 64) the error is measured on the layer output.
    Returns (qweight, scales, zeros) and, if asked for, choice [N, K/128] u8."""
    _dev(W, torch.float16, "W")
    N, K = W.shape
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    qb, sb, zb = awq_packed_sizes(N, K, group)
    if out is None:
        out = (torch.empty(qb, dtype=torch.uint8, device=W.device),
               torch.empty(sb // 2, dtype=torch.float16, device=W.device),
               torch.empty(zb, dtype=torch.uint8, device=W.device))
    qweight, scales, zeros = out
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * 2 < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("output buffers are too small")
    n = len(ratios)
    arr = (ctypes.c_float * max(n, 1))(*[float(r) for r in ratios])
    choice = torch.empty((N, K // group), dtype=torch.uint8, device=W.device) if want_choice else None
    T = 0
    if xs is not None:
        _dev(xs, torch.float16, "xs")
        T, K2 = xs.shape
        if K2 != K:
            raise ValueError("xs and W disagree on K")
    _check(load().awq_quantize_pack_clip(_ptr(W), _ptr(s), N, K, group, arr, n, _ptr(xs), T,
                                         _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(choice),
                                         _stream()),
           "awq_quantize_pack_clip")
    return (qweight, scales, zeros, choice) if want_choice else (qweight, scales, zeros)


# ---------------------------------------------------------------- INT3-g128 variant

def awq_packed_sizes_w3(N: int, K: int, group: int = GROUP):
    q, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().awq_packed_sizes_w3(N, K, group, ctypes.byref(q), ctypes.byref(s), ctypes.byref(z)),
           "awq_packed_sizes_w3")
    return q.value, s.value, z.value


def awq_quantize_pack_w3(W: torch.Tensor, s: torch.Tensor | None = None, group: int = GROUP, out=None):
    """W [N,K] fp16, s [K] fp32 or None -> (qweight u8[N*K*3/8], scales f16, zeros u8), 3-bit layout."""
    _dev(W, torch.float16, "W")
    N, K = W.shape
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    qb, sb, zb = awq_packed_sizes_w3(N, K, group)
    if out is None:
        out = (torch.empty(qb, dtype=torch.uint8, device=W.device),
               torch.empty(sb // 2, dtype=torch.float16, device=W.device),
               torch.empty(zb, dtype=torch.uint8, device=W.device))
    qweight, scales, zeros = out
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * 2 < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("output buffers are too small")
    _check(load().awq_quantize_pack_w3(_ptr(W), _ptr(s), N, K, group, _ptr(qweight), _ptr(scales),
                                       _ptr(zeros), _stream()), "awq_quantize_pack_w3")
    return qweight, scales, zeros


def awq_unpack_w3(qweight, scales, zeros, N: int, K: int, group: int = GROUP):
    """Canonical arrays of the 3-bit layout: codes u8[N,K], scales f16[N,K/128], zeros u8[N,K/128]."""
    dev = qweight.device
    codes = torch.empty((N, K), dtype=torch.uint8, device=dev)
    sc = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    zp = torch.empty((N, K // group), dtype=torch.uint8, device=dev)
    _check(load().awq_unpack_w3(_ptr(qweight), _ptr(scales), _ptr(zeros), N, K, group, _ptr(codes),
                                _ptr(sc), _ptr(zp), _stream()), "awq_unpack_w3")
    return codes, sc, zp


def awq_repack_w3_to_w4(qweight, N: int, K: int, group: int = GROUP, out=None):
    """The codes of a 3-bit packed weight in the 4-bit layout (N*K/2 bytes); scales and zeros are
    shared between the two layouts."""
    if out is None:
        out = torch.empty(N * K // 2, dtype=torch.uint8, device=qweight.device)
    _check(load().awq_repack_w3_to_w4(_ptr(qweight), N, K, group, _ptr(out), _stream()), "awq_repack_w3_to_w4")
    return out


def awq_w3a16_linear(x: torch.Tensor, qweight, scales, zeros, N: int, group: int = GROUP, out=None,
                     workspace=None):
    """y [M,N] fp16 = x [M,K] fp16 (already divided by s) times the 3-bit packed weight.  M <= 16:
    the decode kernel; larger M: awq_w3a16_linear_prefill (workspace of N*K/2 bytes, allocated
    here if not given)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _dev(out, torch.float16, "y")
    if M > 16:
        need = int(load().awq_w3a16_prefill_workspace_bytes(N, K, group))
        if workspace is None:
            # re-packed codes, then the fp32 partial tiles of the K ranges (if the shape uses them)
            need = (need + 255) // 256 * 256 + awq_linear_workspace_bytes(M, N, K, group)
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
        _check(load().awq_w3a16_linear_prefill(_ptr(x), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(out),
                                               M, N, K, group, _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream()),
               "awq_w3a16_linear_prefill")
        return out
    _check(load().awq_w3a16_linear(_ptr(x), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(out), M, N, K,
                                   group, _stream()), "awq_w3a16_linear")
    return out


# ---------------------------------------------------------------- INT2-g64 variant

GROUP_W2 = 64


def awq_packed_sizes_w2(N: int, K: int, group: int = GROUP_W2):
    q, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().awq_packed_sizes_w2(N, K, group, ctypes.byref(q), ctypes.byref(s), ctypes.byref(z)),
           "awq_packed_sizes_w2")
    return q.value, s.value, z.value


def awq_quantize_pack_w2(W: torch.Tensor, s: torch.Tensor | None = None, group: int = GROUP_W2, out=None):
    """W [N,K] fp16, s [K] fp32 or None -> (qweight u8[N*K/4], scales f16, zeros u8), 2-bit layout."""
    _dev(W, torch.float16, "W")
    N, K = W.shape
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    qb, sb, zb = awq_packed_sizes_w2(N, K, group)
    if out is None:
        out = (torch.empty(qb, dtype=torch.uint8, device=W.device),
               torch.empty(sb // 2, dtype=torch.float16, device=W.device),
               torch.empty(max(zb, 16), dtype=torch.uint8, device=W.device)[:zb])
    qweight, scales, zeros = out
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * 2 < sb \
            or zeros.numel() * zeros.element_size() < zb:
        raise ValueError("output buffers are too small")
    _check(load().awq_quantize_pack_w2(_ptr(W), _ptr(s), N, K, group, _ptr(qweight), _ptr(scales),
                                       _ptr(zeros), _stream()), "awq_quantize_pack_w2")
    return qweight, scales, zeros


def awq_unpack_w2(qweight, scales, zeros, N: int, K: int, group: int = GROUP_W2):
    """Canonical arrays of the 2-bit layout: codes u8[N,K], scales f16[N,K/64], zeros u8[N,K/64]."""
    dev = qweight.device
    codes = torch.empty((N, K), dtype=torch.uint8, device=dev)
    sc = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    zp = torch.empty((N, K // group), dtype=torch.uint8, device=dev)
    _check(load().awq_unpack_w2(_ptr(qweight), _ptr(scales), _ptr(zeros), N, K, group, _ptr(codes),
                                _ptr(sc), _ptr(zp), _stream()), "awq_unpack_w2")
    return codes, sc, zp


def awq_w2a16_linear(x: torch.Tensor, qweight, scales, zeros, N: int, group: int = GROUP_W2, out=None):
    """y [M,N] fp16 = x [M,K] fp16 (already divided by s) times the 2-bit packed weight (any M; the
    decode kernel, 128 rows per launch)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _dev(out, torch.float16, "y")
    qb, sb, zb = awq_packed_sizes_w2(N, K, group)
    if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
            or zeros.numel() * zeros.element_size() < zb or out.numel() != M * N:
        raise ValueError("buffer sizes do not match the shape")
    _check(load().awq_w2a16_linear(_ptr(x), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(out), M, N, K,
                                   group, _stream()), "awq_w2a16_linear")
    return out


def prepare_linear_multi_w2(linears, group: int = GROUP_W2):
    """As prepare_linear_multi for linears in the 2-bit layout."""
    return _prepare_multi(linears, group, awq_packed_sizes_w2, "awq_w2a16_linear_multi", False)


def awq_w2a16_linear_multi(linears, group: int = GROUP_W2):
    prepare_linear_multi_w2(linears, group)()
    return [l[4] for l in linears]


def prepare_linear_multi_w3(linears, group: int = GROUP):
    """As prepare_linear_multi for linears in the 3-bit layout."""
    return _prepare_multi(linears, group, awq_packed_sizes_w3, "awq_w3a16_linear_multi", False)


def awq_w3a16_linear_multi(linears, group: int = GROUP):
    prepare_linear_multi_w3(linears, group)()
    return [l[4] for l in linears]


def awq_rmsnorm_inv_scale(x: torch.Tensor, gamma: torch.Tensor, s: torch.Tensor | None = None,
                          eps: float = 1e-5, out: torch.Tensor | None = None):
    """x' = fp16(x / sqrt(mean x^2 + eps) * gamma / s); x [M,K] fp16, gamma [K] fp16, s [K] fp32 or None."""
    _dev(x, torch.float16, "x")
    _dev(gamma, torch.float16, "gamma")
    M, K = x.shape
    if gamma.numel() != K:
        raise ValueError("gamma must have K elements")
    if s is not None:
        _dev(s, torch.float32, "s")
        if s.numel() != K:
            raise ValueError("s must have K elements")
    if out is None:
        out = torch.empty_like(x)
    _dev(out, torch.float16, "out")
    _check(load().awq_rmsnorm_inv_scale(_ptr(x), _ptr(gamma), _ptr(s), M, K, float(eps), _ptr(out),
                                        _stream()), "awq_rmsnorm_inv_scale")
    return out


def awq_read_probe(buffer: torch.Tensor, sink: torch.Tensor, nbytes: int | None = None):
    """Read-only streaming pass over `buffer` (measurement aid of the benchmark)."""
    n = buffer.numel() * buffer.element_size() if nbytes is None else nbytes
    _check(load().awq_read_probe(_ptr(buffer), n, _ptr(sink), _stream()), "awq_read_probe")


def awq_decode_attention(q, k, v, k_cache, v_cache, pos: int, rope_theta: float = 10000.0,
                         out=None, workspace=None):
    """One decode step of the attention layer: q [H,D], k, v [Hkv,D] fp16 of the token at `pos`;
    k_cache, v_cache [Hkv,Lmax,D] fp16 are updated in place; returns out [H,D] fp16."""
    for t, name in ((q, "q"), (k, "k"), (v, "v"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _dev(t, torch.float16, name)
    H, D = q.shape
    Hkv, Lmax, D2 = k_cache.shape
    if k.shape != (Hkv, D) or v.shape != (Hkv, D) or v_cache.shape != k_cache.shape or D2 != D:
        raise ValueError("shapes of q, k, v and the caches do not agree")
    if out is None:
        out = torch.empty((H, D), dtype=torch.float16, device=q.device)
    need = load().awq_decode_attention_workspace_bytes(H, D, pos + 1)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(load().awq_decode_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache), H, Hkv, D,
                                       Lmax, pos, float(rope_theta), _ptr(out), _ptr(workspace),
                                       workspace.numel(), _stream()), "awq_decode_attention")
    return out


def awq_silu_mul(gate: torch.Tensor, up: torch.Tensor, out: torch.Tensor | None = None):
    """out = fp16(silu(gate) * up), element-wise; gate, up fp16 of the same shape."""
    _dev(gate, torch.float16, "gate")
    _dev(up, torch.float16, "up")
    if gate.shape != up.shape:
        raise ValueError("gate and up must have the same shape")
    if out is None:
        out = torch.empty_like(gate)
    _dev(out, torch.float16, "out")
    _check(load().awq_silu_mul(_ptr(gate), _ptr(up), gate.numel(), _ptr(out), _stream()), "awq_silu_mul")
    return out


def _fused_descs(linears, group, M=None):
    """FusedDesc array of a list of dicts (see prepare_linear_fused_multi); returns (descs, M)."""
    descs = (FusedDesc * len(linears))()
    for i, l in enumerate(linears):
        x, y, N = l["x"], l["y"], l["N"]
        _dev(x, torch.float16, "x")
        _dev(y, torch.float16, "y")
        m, K = x.shape
        if M is None:
            M = m
        if m != M:
            raise ValueError("all linears of a grouped call share M")
        qb, sb, zb = awq_packed_sizes(N, K, group)
        qweight, scales, zeros = l["qweight"], l["scales"], l["zeros"]
        if qweight.numel() * qweight.element_size() < qb or scales.numel() * scales.element_size() < sb \
                or zeros.numel() * zeros.element_size() < zb or y.numel() != M * N:
            raise ValueError("buffer sizes do not match the shape")
        norm, res, scale = l.get("norm"), l.get("residual"), l.get("scale")
        if norm is not None and scale is not None:
            raise ValueError("a linear takes a normalisation or a column scale, not both")
        pre = norm if norm is not None else scale
        if pre is not None:
            _dev(pre, torch.float16, "norm/scale")
            if pre.numel() != K:
                raise ValueError("norm / scale must have K elements")
        if res is not None:
            _dev(res, torch.float16, "residual")
            if res.numel() != M * N:
                raise ValueError("residual must be [M,N]")
        descs[i] = FusedDesc(LinearDesc(x.data_ptr(), qweight.data_ptr(), scales.data_ptr(), zeros.data_ptr(),
                                        y.data_ptr(), N, K),
                             pre.data_ptr() if pre is not None else None,
                             res.data_ptr() if res is not None else None,
                             float(l.get("eps", 1e-5)),
                             PRE_RMSNORM if norm is not None else (PRE_SCALE if scale is not None else PRE_NONE))
    return descs, M


def prepare_linear_fused_multi(linears, group: int = GROUP):
    """Marshal one fused grouped decode call.  `linears` is a list of dicts with the keys
    x, qweight, scales, zeros, y, N and optionally norm (fp16 [K] factors: the linear then runs on
    the RMS-normalised x times these) with eps, or scale (fp16 [K]: the linear runs on x times
    these), and residual (fp16 [M,N], added to the output; may be y).
    Returns a zero-argument callable that enqueues ONE awq_w4a16_linear_fused_multi."""
    if not 1 <= len(linears) <= FUSED_MAX:
        raise ValueError(f"1..{FUSED_MAX} linears per fused call")
    descs, M = _fused_descs(linears, group)
    fn = load().awq_w4a16_linear_fused_multi
    count = len(linears)
    keep = list(linears)

    def call(_keep=keep):
        st = fn(descs, count, M, group, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != 0:
            raise AwqError(st, "awq_w4a16_linear_fused_multi")
    return call


class ChainStage(ctypes.Structure):
    """awq_chain_stage of the C ABI."""
    _fields_ = [("descs", ctypes.POINTER(FusedDesc)), ("count", ctypes.c_int)]


CHAIN_MAX_STAGES, CHAIN_MAX_LINEARS, CHAIN_SYNC_BYTES = 4, 10, 8192


def chain_sync(device="cuda") -> torch.Tensor:
    """A zeroed sync area for awq_w4a16_linear_chain."""
    return torch.zeros(CHAIN_SYNC_BYTES // 4, dtype=torch.int32, device=device)


def prepare_linear_chain(stages, sync: torch.Tensor, group: int = GROUP, spin_limit: int = 0):
    """Marshal one awq_w4a16_linear_chain call.  `stages` is a list of stages, each a list of dicts
    as for prepare_linear_fused_multi; a linear may read (as x or residual) what a linear of an
    earlier stage writes.  `sync`: chain_sync() (zeroed, CHAIN_SYNC_BYTES); it is zero again after every
    call that ends normally, and sync[0] != 0 afterwards means a wait ran out (outputs invalid).
    Returns a zero-argument callable that enqueues the ONE launch on the then-current stream."""
    if not 1 <= len(stages) <= CHAIN_MAX_STAGES:
        raise ValueError(f"1..{CHAIN_MAX_STAGES} stages per chain")
    if not (sync.is_cuda and sync.is_contiguous() and sync.numel() * sync.element_size() >= CHAIN_SYNC_BYTES):
        raise TypeError(f"sync: a contiguous GPU tensor of at least {CHAIN_SYNC_BYTES} bytes")
    arr = (ChainStage * len(stages))()
    keep, M = [sync], None
    for s, linears in enumerate(stages):
        if not 1 <= len(linears) <= CHAIN_MAX_LINEARS:
            raise ValueError(f"1..{CHAIN_MAX_LINEARS} linears per stage")
        descs, M = _fused_descs(linears, group, M)
        arr[s] = ChainStage(ctypes.cast(descs, ctypes.POINTER(FusedDesc)), len(linears))
        keep += [descs, list(linears)]
    fn = load().awq_w4a16_linear_chain
    n = len(stages)
    sync_ptr = ctypes.c_void_p(sync.data_ptr())

    def call(_keep=keep):
        st = fn(arr, n, M, group, sync_ptr, spin_limit, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != 0:
            raise AwqError(st, "awq_w4a16_linear_chain")
    return call


def awq_w4a16_linear_fused_multi(linears, group: int = GROUP):
    """The linears of `linears` (see prepare_linear_fused_multi) in one kernel launch."""
    prepare_linear_fused_multi(linears, group)()
    return [l["y"] for l in linears]


def awq_w4a16_linear_fused_fits(N: int, K: int, M: int, group: int = GROUP) -> bool:
    """Whether a linear of this shape can be part of a fused grouped call at this M."""
    return bool(load().awq_w4a16_linear_fused_fits(N, K, M, group))


def awq_last_grouped_plan() -> int:
    """Diagnostic: 1 if the last grouped decode launch used one size of workgroup per linear, 2 if
    it used the paired plan, 0 if there was none yet."""
    return int(load().awq_last_grouped_plan())
