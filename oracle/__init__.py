"""CPU oracle for the AWQ W4A16 linear path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``awq_oracle.c`` (plain C, built with gcc).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product never does, and this package
never imports the product.

Every function follows the passage of AWQ (arXiv 2306.00978) named in its
docstring; the arithmetic itself lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "awq_oracle.c")
_LIB = os.path.join(_HERE, "libawq_oracle.so")
GROUP = 128

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc. No FMA contraction, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized(out_dir: str) -> str:
    """The same source under AddressSanitizer + UndefinedBehaviorSanitizer (gcc), for a process
    that has gcc's libasan preloaded; AWQ_ORACLE_LIBRARY then names the result."""
    out = os.path.join(out_dir, "libawq_oracle_san.so")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-shared", "-fPIC", "-o", out, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return out


def _load():
    global _lib
    if _lib is None:
        other = os.environ.get("AWQ_ORACLE_LIBRARY")
        if not other:
            build()
        lib = ctypes.CDLL(other or _LIB)
        lib.awq_oracle_f16_to_f32.restype = ctypes.c_float
        lib.awq_oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.awq_oracle_f32_to_f16.restype = ctypes.c_uint16
        lib.awq_oracle_f32_to_f16.argtypes = [ctypes.c_float]
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (rc={rc})")


def _as_f16_bits(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError("expected float16 (or its uint16 bit pattern)")


def f16_to_f32_scalar(bits: int) -> float:
    return float(_load().awq_oracle_f16_to_f32(int(bits)))


def f32_to_f16_scalar(v: float) -> int:
    return int(_load().awq_oracle_f32_to_f16(float(np.float32(v))))


def act_scale(X, alpha: float = 0.5, floor: float = 1e-4) -> np.ndarray:
    """Sec. 3.2, Eq. 5: s = s_X^alpha, s_X = per-input-channel mean |X| (fp64)."""
    Xb = _as_f16_bits(X)
    T, K = Xb.shape
    s = np.empty(K, dtype=np.float64)
    _chk(_load().awq_oracle_act_scale(_p(Xb), _i64(T), _i64(K), ctypes.c_double(alpha),
                                      ctypes.c_double(floor), _p(s)), "act_scale")
    return s


def apply_inv_scale(x, s) -> np.ndarray:
    """Sec. 3.2, Eq. 4: the diag(s)^-1 X factor; x' = fp16(fp32(x) / s)."""
    xb = _as_f16_bits(x)
    M, K = xb.shape
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.shape == (K,)
    out = np.empty((M, K), dtype=np.uint16)
    _chk(_load().awq_oracle_apply_inv_scale(_p(xb), _p(s), _i64(M), _i64(K), _p(out)),
         "apply_inv_scale")
    return out.view(np.float16)


def rmsnorm_inv_scale(x, gamma, s=None, eps: float = 1e-5) -> np.ndarray:
    """Sec. 4.2 kernel fusion + Sec. 3.2 Eq. 4: RMS normalisation with the 1/s factor folded in,
    x' = fp16(x / sqrt(mean x^2 + eps) * gamma / s), fp64 inside."""
    xb = _as_f16_bits(x)
    M, K = xb.shape
    gb = _as_f16_bits(gamma)
    assert gb.shape == (K,)
    sp = None
    if s is not None:
        s = np.ascontiguousarray(s, dtype=np.float32)
        assert s.shape == (K,)
        sp = _p(s)
    out = np.empty((M, K), dtype=np.uint16)
    _chk(_load().awq_oracle_rmsnorm_inv_scale(_p(xb), _p(gb), sp, _i64(M), _i64(K),
                                              ctypes.c_double(eps), _p(out)), "rmsnorm_inv_scale")
    return out.view(np.float16)


def quantize(W, s=None, group: int = GROUP):
    """Sec. 3.2, Eq. 1-2: Q(w*s) per group of 128 input channels (asymmetric
    16-level min/max form).  Returns codes[N,K] u8, scales[N,G] f16, zeros[N,G] u8."""
    Wb = _as_f16_bits(W)
    N, K = Wb.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    G = K // group
    sp = None
    if s is not None:
        s = np.ascontiguousarray(s, dtype=np.float32)
        assert s.shape == (K,)
        sp = _p(s)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_quantize(_p(Wb), sp, _i64(N), _i64(K), ctypes.c_int(group),
                                     _p(codes), _p(scales), _p(zeros)), "quantize")
    return codes, scales.view(np.float16), zeros


def quantize_clip(W, s, ratios, xs=None, group: int = GROUP):
    """Sec. 3.2, weight clipping (one sentence in the paper; the reading is stated in the C
    file): per group the range of w*s is shrunk by each ratio of the grid and the ratio with
    the smallest squared quantization error wins -- the error of the weights themselves, or,
    with rows xs = x/s [T,K] given, of the group's contribution to the layer output on those
    rows.  Returns codes, scales, zeros as `quantize` and choice[N,G] u8, the index of the
    winning ratio."""
    Wb = _as_f16_bits(W)
    N, K = Wb.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    G = K // group
    sp = None
    if s is not None:
        s = np.ascontiguousarray(s, dtype=np.float32)
        assert s.shape == (K,)
        sp = _p(s)
    ratios = np.ascontiguousarray(ratios, dtype=np.float32)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    choice = np.empty((N, G), dtype=np.uint8)
    xp, T = None, 0
    if xs is not None:
        xb = _as_f16_bits(xs)
        T = xb.shape[0]
        assert xb.shape == (T, K)
        xp = _p(xb)
    _chk(_load().awq_oracle_quantize_clip(_p(Wb), sp, _i64(N), _i64(K), ctypes.c_int(group),
                                          _p(ratios), ctypes.c_int(ratios.size), xp, _i64(T),
                                          _p(codes), _p(scales), _p(zeros), _p(choice)),
         "quantize_clip")
    return codes, scales.view(np.float16), zeros, choice


def packed_sizes(N: int, K: int, group: int = GROUP):
    G = K // group
    return N * K // 2, N * G * 2, N * G // 2


def pack(codes, scales, zeros, group: int = GROUP):
    """Sec. 4.2 weight packing, in the byte layout of this library (see C file)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    G = K // group
    sb = _as_f16_bits(scales)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    assert sb.shape == (N, G) and zeros.shape == (N, G)
    qb, sbytes, zb = packed_sizes(N, K, group)
    qweight = np.empty(qb, dtype=np.uint8)
    scales_p = np.empty(sbytes // 2, dtype=np.uint16)
    zeros_p = np.empty(zb, dtype=np.uint8)
    _chk(_load().awq_oracle_pack(_p(codes), _p(sb), _p(zeros), _i64(N), _i64(K),
                                 ctypes.c_int(group), _p(qweight), _p(scales_p), _p(zeros_p)),
         "pack")
    return qweight, scales_p, zeros_p


def unpack(qweight, scales_p, zeros_p, N: int, K: int, group: int = GROUP):
    qweight = np.ascontiguousarray(qweight, dtype=np.uint8)
    scales_p = _as_f16_bits(scales_p).reshape(-1)
    zeros_p = np.ascontiguousarray(zeros_p, dtype=np.uint8)
    G = K // group
    qb, sbytes, zb = packed_sizes(N, K, group)
    assert qweight.size == qb and scales_p.size * 2 == sbytes and zeros_p.size == zb
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_unpack(_p(qweight), _p(scales_p), _p(zeros_p), _i64(N), _i64(K),
                                   ctypes.c_int(group), _p(codes), _p(scales), _p(zeros)),
         "unpack")
    return codes, scales.view(np.float16), zeros


def dequant(codes, scales, zeros, group: int = GROUP) -> np.ndarray:
    """Sec. 4.2 on-the-fly dequantization: Wdq = (q - zero) * scale, fp32 (exact)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    sb = _as_f16_bits(scales)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    Wdq = np.empty((N, K), dtype=np.float32)
    _chk(_load().awq_oracle_dequant(_p(codes), _p(sb), _p(zeros), _i64(N), _i64(K),
                                    ctypes.c_int(group), _p(Wdq)), "dequant")
    return Wdq


def matmul(x, Wdq, acc32: bool = False) -> np.ndarray:
    """y[m,n] = sum_k x[m,k] * Wdq[n,k]; fp64 accumulation (fp32 sequential if acc32)."""
    xb = _as_f16_bits(x)
    M, K = xb.shape
    Wdq = np.ascontiguousarray(Wdq, dtype=np.float32)
    N = Wdq.shape[0]
    assert Wdq.shape == (N, K)
    y = np.empty((M, N), dtype=np.float64)
    _chk(_load().awq_oracle_matmul(_p(xb), _p(Wdq), _i64(M), _i64(N), _i64(K),
                                   ctypes.c_int(1 if acc32 else 0), _p(y)), "matmul")
    return y


def norm_error(y_gpu, y_ref, x, Wdq) -> np.ndarray:
    """Acceptance metric: |y_gpu - y_ref| / (||x_row||_2 * max|Wdq| + 1e-6), per element."""
    yb = _as_f16_bits(y_gpu)
    xb = _as_f16_bits(x)
    M, K = xb.shape
    Wdq = np.ascontiguousarray(Wdq, dtype=np.float32)
    N = Wdq.shape[0]
    y_ref = np.ascontiguousarray(y_ref, dtype=np.float64)
    assert yb.shape == (M, N) and y_ref.shape == (M, N)
    err = np.empty((M, N), dtype=np.float64)
    _chk(_load().awq_oracle_norm_error(_p(yb), _p(y_ref), _p(xb), _p(Wdq), _i64(M), _i64(N),
                                       _i64(K), _p(err)), "norm_error")
    return err


def linear(x, codes, scales, zeros, group: int = GROUP) -> np.ndarray:
    """The whole layer as the paper states it: dequantize, then matmul (fp64 acc)."""
    return matmul(x, dequant(codes, scales, zeros, group))


def scale_search_loss(W, X, s) -> float:
    """Sec. 3.2, Eq. 4: L(s) = || Q(W diag(s)) (diag(s)^-1 X) - W X ||^2 for one linear layer,
    the norm taken over all entries (Frobenius) and returned squared.  Q is `quantize`, the
    diag(s)^-1 X factor is the fp16 array the layer is really fed (`apply_inv_scale`), both
    products are accumulated in fp64.  W [N,K] fp16, X [T,K] fp16 (rows = tokens), s [K]."""
    W = np.ascontiguousarray(W)
    if W.dtype != np.float16:
        raise TypeError("W must be float16")
    s = np.ascontiguousarray(s, dtype=np.float32)
    codes, scales, zeros = quantize(W, s)
    yq = matmul(apply_inv_scale(X, s), dequant(codes, scales, zeros))
    y = matmul(X, W.astype(np.float32))
    d = yq - y
    return float(np.sum(d * d))


def search_scale(W, X, alphas):
    """Sec. 3.2, Eq. 5: s = s_X^alpha with s_X the per-channel mean |X|; alpha* minimises the
    loss of Eq. 4 over the given grid (first minimum on ties).
    Returns (index of alpha*, losses[len(alphas)] fp64, s* [K] fp32)."""
    losses = np.array([scale_search_loss(W, X, act_scale(X, float(a)).astype(np.float32))
                       for a in alphas], dtype=np.float64)
    best = int(np.argmin(losses))
    return best, losses, act_scale(X, float(alphas[best])).astype(np.float32)


# ---------------------------------------------------------------- INT3-g128 variant

def quantize_w3(W, s=None, group: int = GROUP):
    """Sec. 5 (INT3-g128): the 8-level form of `quantize`.  Returns codes[N,K] u8 in 0..7,
    scales[N,G] f16, zeros[N,G] u8 in 0..7."""
    Wb = _as_f16_bits(W)
    N, K = Wb.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    G = K // group
    sp = None
    if s is not None:
        s = np.ascontiguousarray(s, dtype=np.float32)
        assert s.shape == (K,)
        sp = _p(s)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_quantize_w3(_p(Wb), sp, _i64(N), _i64(K), ctypes.c_int(group),
                                        _p(codes), _p(scales), _p(zeros)), "quantize_w3")
    return codes, scales.view(np.float16), zeros


def packed_sizes_w3(N: int, K: int, group: int = GROUP):
    G = K // group
    return N * K * 3 // 8, N * G * 2, N * G // 2


def pack_w3(codes, scales, zeros, group: int = GROUP):
    """The 3-bit packed layout of this library (see the C file)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    G = K // group
    sb = _as_f16_bits(scales)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    assert sb.shape == (N, G) and zeros.shape == (N, G)
    qb, sbytes, zb = packed_sizes_w3(N, K, group)
    qweight = np.empty(qb, dtype=np.uint8)
    scales_p = np.empty(sbytes // 2, dtype=np.uint16)
    zeros_p = np.empty(zb, dtype=np.uint8)
    _chk(_load().awq_oracle_pack_w3(_p(codes), _p(sb), _p(zeros), _i64(N), _i64(K),
                                    ctypes.c_int(group), _p(qweight), _p(scales_p), _p(zeros_p)),
         "pack_w3")
    return qweight, scales_p, zeros_p


def unpack_w3(qweight, scales_p, zeros_p, N: int, K: int, group: int = GROUP):
    qweight = np.ascontiguousarray(qweight, dtype=np.uint8)
    scales_p = _as_f16_bits(scales_p).reshape(-1)
    zeros_p = np.ascontiguousarray(zeros_p, dtype=np.uint8)
    G = K // group
    qb, sbytes, zb = packed_sizes_w3(N, K, group)
    assert qweight.size == qb and scales_p.size * 2 == sbytes and zeros_p.size == zb
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_unpack_w3(_p(qweight), _p(scales_p), _p(zeros_p), _i64(N), _i64(K),
                                      ctypes.c_int(group), _p(codes), _p(scales), _p(zeros)),
         "unpack_w3")
    return codes, scales.view(np.float16), zeros


# ---------------------------------------------------------------- INT2-g64 variant

GROUP_W2 = 64


def quantize_w2(W, s=None, group: int = GROUP_W2):
    """Sec. 5 (INT2-g64 of the extreme low-bit table): the 4-level form of `quantize` over groups
    of 64 input channels.  Returns codes[N,K] u8 in 0..3, scales[N,K/64] f16, zeros[N,K/64] u8."""
    Wb = _as_f16_bits(W)
    N, K = Wb.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    G = K // group
    sp = None
    if s is not None:
        s = np.ascontiguousarray(s, dtype=np.float32)
        assert s.shape == (K,)
        sp = _p(s)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_quantize_w2(_p(Wb), sp, _i64(N), _i64(K), ctypes.c_int(group),
                                        _p(codes), _p(scales), _p(zeros)), "quantize_w2")
    return codes, scales.view(np.float16), zeros


def packed_sizes_w2(N: int, K: int, group: int = GROUP_W2):
    G = K // group
    return N * K // 4, N * G * 2, N * G // 4


def pack_w2(codes, scales, zeros, group: int = GROUP_W2):
    """The 2-bit packed layout of this library (see the C file); K a multiple of 256."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    G = K // group
    sb = _as_f16_bits(scales)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    assert sb.shape == (N, G) and zeros.shape == (N, G)
    qb, sbytes, zb = packed_sizes_w2(N, K, group)
    qweight = np.empty(qb, dtype=np.uint8)
    scales_p = np.empty(sbytes // 2, dtype=np.uint16)
    zeros_p = np.empty(zb, dtype=np.uint8)
    _chk(_load().awq_oracle_pack_w2(_p(codes), _p(sb), _p(zeros), _i64(N), _i64(K),
                                    ctypes.c_int(group), _p(qweight), _p(scales_p), _p(zeros_p)),
         "pack_w2")
    return qweight, scales_p, zeros_p


def unpack_w2(qweight, scales_p, zeros_p, N: int, K: int, group: int = GROUP_W2):
    qweight = np.ascontiguousarray(qweight, dtype=np.uint8)
    scales_p = _as_f16_bits(scales_p).reshape(-1)
    zeros_p = np.ascontiguousarray(zeros_p, dtype=np.uint8)
    G = K // group
    qb, sbytes, zb = packed_sizes_w2(N, K, group)
    assert qweight.size == qb and scales_p.size * 2 == sbytes and zeros_p.size == zb
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint8)
    _chk(_load().awq_oracle_unpack_w2(_p(qweight), _p(scales_p), _p(zeros_p), _i64(N), _i64(K),
                                      ctypes.c_int(group), _p(codes), _p(scales), _p(zeros)),
         "unpack_w2")
    return codes, scales.view(np.float16), zeros


# ---------------------------------------------------------------- decode attention (Sec. 4.2 fusion)

def rope_rotate(x, pos: int, theta: float = 10000.0) -> np.ndarray:
    """Rotary position embedding of x [..., D] (fp64): the pairs (i, i + D/2) are rotated by the
    angle pos * theta^(-2 i / D) (the half-split pairing of Llama-style models; Sec. 4.2 only
    says that the attention kernel evaluates the position embedding itself)."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    i = np.arange(D // 2, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * i / D)
    c, s_ = np.cos(ang), np.sin(ang)
    a, b = x[..., : D // 2], x[..., D // 2:]
    return np.concatenate([a * c - b * s_, b * c + a * s_], axis=-1)


def decode_attention(q, k, v, k_cache, v_cache, pos: int, theta: float = 10000.0):
    """Sec. 4.2, kernel fusion (attention): one decode step of one sequence.  q [H,D], k, v
    [Hkv,D] fp16 are the projections of the token at position pos; k_cache, v_cache
    [Hkv,Lmax,D] fp16 hold the rotated keys and the values of positions < pos.  Rotates q and k,
    stores fp16(k_rot) and v in row pos of the caches (returned as new arrays), and returns
    out [H,D] fp16 = softmax(q_rot K^T / sqrt(D)) V over positions 0..pos, fp64 inside; query
    head h reads kv head h // (H / Hkv).  The current token's key enters the scores unrounded
    (it never left the chip), the cached ones as stored."""
    q = np.asarray(q); k = np.asarray(k); v = np.asarray(v)
    H, D = q.shape
    Hkv = k.shape[0]
    rep = H // Hkv
    kc = np.array(k_cache, copy=True)
    vc = np.array(v_cache, copy=True)
    k_rot = rope_rotate(k.astype(np.float64), pos, theta)
    q_rot = rope_rotate(q.astype(np.float64), pos, theta)
    kc[:, pos, :] = k_rot.astype(np.float32).astype(np.float16)
    vc[:, pos, :] = v
    out = np.empty((H, D), dtype=np.float64)
    for h in range(H):
        g = h // rep
        keys = kc[g, : pos + 1].astype(np.float64)
        keys[pos] = k_rot[g]
        vals = vc[g, : pos + 1].astype(np.float64)
        sc = keys @ q_rot[h] / np.sqrt(D)
        p = np.exp(sc - sc.max())
        out[h] = (p / p.sum()) @ vals
    return out.astype(np.float32).astype(np.float16), kc, vc


def silu_mul(gate, up) -> np.ndarray:
    """The gated activation between the gate/up and the down projection of a Llama-style MLP,
    one of the element-wise operators Sec. 4.2 fuses: fp16(silu(gate) * up), fp64 inside."""
    g = np.asarray(gate, dtype=np.float16).astype(np.float64)
    u = np.asarray(up, dtype=np.float16).astype(np.float64)
    return (g / (1.0 + np.exp(-g)) * u).astype(np.float32).astype(np.float16)


def scale_columns(x, w) -> np.ndarray:
    """Sec. 3.2, Eq. 4, the diag(s)^-1 factor applied as a multiplication by w = 1/s given in
    fp16: x'[m,k] = fp16(x[m,k] * w[k]), the product formed exactly (fp64) and rounded once."""
    x = np.asarray(x, dtype=np.float16).astype(np.float64)
    w = np.asarray(w, dtype=np.float16).astype(np.float64)
    return (x * w[None, :]).astype(np.float16)
