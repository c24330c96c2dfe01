"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU (so these run on a box without one)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "awq_mi355x.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2306_00978_amd as awq
    if not os.path.exists(awq.LIB_PATH):
        from paper_2306_00978_amd import build
        build.build()
    return awq.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(awq_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    import paper_2306_00978_amd as awq
    assert declared_functions() == sorted(awq.EXPORTS)


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert lib.awq_version() == 1
    seen = set()
    for st in range(0, -8, -1):
        s = lib.awq_status_string(st).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.awq_status_string(-99).decode() == "unknown status"


def test_packed_sizes(lib):
    q, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.awq_packed_sizes(4096, 11008, 128, ctypes.byref(q), ctypes.byref(s), ctypes.byref(z)) == 0
    assert (q.value, s.value, z.value) == (4096 * 11008 // 2, 4096 * 86 * 2, 4096 * 86 // 2)
    # 0.51953125 bytes per weight
    assert (q.value + s.value + z.value) * 128 * 4 == 4096 * 11008 * 266
    assert lib.awq_packed_sizes(4096, 4096, 64, None, None, None) == -3
    assert lib.awq_packed_sizes(4096, 4000, 128, None, None, None) == -2
    assert lib.awq_packed_sizes(4090, 4096, 128, None, None, None) == -2
    assert lib.awq_packed_sizes(0, 4096, 128, None, None, None) == -2
    assert lib.awq_packed_sizes(16, 128, 128, None, None, None) == 0


def test_argument_validation_happens_before_any_launch(lib):
    P = ctypes.c_void_p
    ok = P(0x1000)          # non-null, 16-byte aligned, never dereferenced on these paths
    odd = P(0x1008)
    # null pointers
    assert lib.awq_quantize_pack(None, None, 16, 128, 128, ok, ok, ok, None) == -1
    assert lib.awq_w4a16_linear(ok, None, ok, ok, ok, 1, 16, 128, 128, None, 0, None) == -1
    assert lib.awq_unpack(ok, ok, None, 16, 128, 128, ok, ok, ok, None) == -1
    assert lib.awq_act_scale(None, 4, 128, 0.5, ok, None) == -1
    assert lib.awq_apply_inv_scale(ok, None, 1, 128, ok, None) == -1
    # shapes / group
    assert lib.awq_quantize_pack(ok, None, 16, 100, 128, ok, ok, ok, None) == -2
    assert lib.awq_quantize_pack(ok, None, 8, 128, 128, ok, ok, ok, None) == -2
    assert lib.awq_quantize_pack(ok, None, 16, 128, 32, ok, ok, ok, None) == -3
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, ok, 0, 16, 128, 128, None, 0, None) == -2
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, ok, -3, 16, 128, 128, None, 0, None) == -2
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, ok, 1, 16, 128, 64, None, 0, None) == -3
    assert lib.awq_act_scale(ok, 0, 128, 0.5, ok, None) == -2
    assert lib.awq_act_scale(ok, 4, 100, 0.5, ok, None) == -2
    assert lib.awq_apply_inv_scale(ok, ok, 1, 12, ok, None) == -2
    # scalar range
    assert lib.awq_act_scale(ok, 4, 128, 1.5, ok, None) == -7
    assert lib.awq_act_scale(ok, 4, 128, float("nan"), ok, None) == -7
    # alignment
    assert lib.awq_quantize_pack(odd, None, 16, 128, 128, ok, ok, ok, None) == -4
    assert lib.awq_quantize_pack(ok, odd, 16, 128, 128, ok, ok, ok, None) == -4
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, odd, 1, 16, 128, 128, None, 0, None) == -4
    # a workspace that would be used has to be aligned
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, ok, 200, 4096, 4096, 128, odd, 1 << 30, None) == -4
    assert lib.awq_w4a16_linear(ok, ok, ok, ok, ok, 200, 4096, 4096, 128, ok, 7 * 200 * 4096 * 4 - 1, None) == -5
    assert lib.awq_unpack(ok, ok, ok, 16, 128, 128, odd, None, None, None) == -4
    # workspace query never fails
    assert lib.awq_linear_workspace_bytes(1, 4096, 4096, 128) >= 0
    assert lib.awq_linear_workspace_bytes(-1, 0, 7, 3) == 0
    # K is cut into ranges only where the prefill kernel has too few tiles for the chip
    wsb = lib.awq_linear_workspace_bytes
    assert wsb(16, 4096, 4096, 128) == 0 and wsb(48, 4096, 11008, 128) == 0
    assert wsb(2048, 4096, 4096, 128) == 0 and wsb(2048, 11008, 4096, 128) == 0
    assert wsb(200, 4096, 4096, 128) == 7 * 200 * 4096 * 4          # 32 tiles of 32 groups: seven ranges
    assert wsb(512, 4096, 4096, 128) == 4 * 512 * 4096 * 4
    assert wsb(128, 4096, 4096, 128) == 0                           # blocks of 16 through the decode kernels
    assert wsb(128, 4096, 11008, 128) == 8 * 128 * 4096 * 4         # does not fit their grouped launch
    assert wsb(300, 176, 1408, 128) == 2 * 300 * 176 * 4            # 11 groups: two ranges at most


def test_grouped_and_search_calls_validate_before_any_launch(lib):
    import paper_2306_00978_amd as awq
    ok, odd = 0x1000, 0x1008
    def descs(n, **kw):
        arr = (awq.LinearDesc * max(n, 1))()
        for i in range(n):
            d = dict(x_f16=ok, qweight=ok, scales=ok, zeros=ok, y_f16=ok, N=16, K=128)
            d.update(kw)
            arr[i] = awq.LinearDesc(**d)
        return arr
    f = lib.awq_w4a16_linear_multi
    assert f(None, 1, 1, 128, None, 0, None) == -1
    assert f(descs(1), 0, 1, 128, None, 0, None) == -7
    assert f(descs(1), awq.MULTI_MAX + 1, 1, 128, None, 0, None) == -7
    assert f(descs(2), 2, 17, 128, None, 0, None) == -2          # not a decode call
    assert f(descs(2), 2, 0, 128, None, 0, None) == -2
    assert f(descs(2, y_f16=None), 2, 1, 128, None, 0, None) == -1
    assert f(descs(2, K=100), 2, 1, 128, None, 0, None) == -2
    assert f(descs(2, N=8), 2, 1, 128, None, 0, None) == -2
    assert f(descs(2), 2, 1, 64, None, 0, None) == -3
    assert f(descs(2, x_f16=odd), 2, 1, 128, None, 0, None) == -4

    def qdescs(n, **kw):
        arr = (awq.QuantizeDesc * max(n, 1))()
        for i in range(n):
            d = dict(W_f16=ok, s=None, N=16, K=128, qweight=ok, scales=ok, zeros=ok)
            d.update(kw)
            arr[i] = awq.QuantizeDesc(**d)
        return arr
    qm = lib.awq_quantize_pack_multi
    assert qm(None, 1, 128, None) == -1
    assert qm(qdescs(1), 0, 128, None) == -7
    assert qm(qdescs(1), awq.QUANTIZE_MULTI_MAX + 1, 128, None) == -7
    assert qm(qdescs(3, zeros=None), 3, 128, None) == -1
    assert qm(qdescs(3, K=192), 3, 128, None) == -2
    assert qm(qdescs(3, N=24), 3, 128, None) == -2
    assert qm(qdescs(3), 3, 64, None) == -3
    assert qm(qdescs(3, s=odd), 3, 128, None) == -4
    assert qm(qdescs(3, W_f16=odd), 3, 128, None) == -4

    def adescs(n, **kw):
        arr = (awq.ActScaleDesc * max(n, 1))()
        for i in range(n):
            d = dict(X_f16=ok, T=64, K=128, s=ok)
            d.update(kw)
            arr[i] = awq.ActScaleDesc(**d)
        return arr
    am = lib.awq_act_scale_multi
    assert am(None, 1, 0.5, None) == -1
    assert am(adescs(1), 0, 0.5, None) == -7
    assert am(adescs(1), awq.ACT_SCALE_MULTI_MAX + 1, 0.5, None) == -7
    assert am(adescs(2), 2, 1.5, None) == -7
    assert am(adescs(2, s=None), 2, 0.5, None) == -1
    assert am(adescs(2, K=100), 2, 0.5, None) == -2
    assert am(adescs(2, T=0), 2, 0.5, None) == -2
    assert am(adescs(2, X_f16=odd), 2, 0.5, None) == -4

    def fdescs(n, **kw):
        arr = (awq.FusedDesc * max(n, 1))()
        for i in range(n):
            d = dict(x_f16=ok, qweight=ok, scales=ok, zeros=ok, y_f16=ok, N=16, K=128)
            d.update(kw)
            arr[i] = awq.FusedDesc(awq.LinearDesc(**d), None, None, 1e-5, 0)
        return arr
    def stages(n, per=1, **kw):
        arr = (awq.ChainStage * max(n, 1))()
        keep = []
        for i in range(n):
            fd = fdescs(per, **kw)
            keep.append(fd)
            arr[i] = awq.ChainStage(ctypes.cast(fd, ctypes.POINTER(awq.FusedDesc)), per)
        return arr, keep
    ch = lib.awq_w4a16_linear_chain
    Pv = ctypes.c_void_p
    st2, k2 = stages(2)
    assert ch(None, 2, 1, 128, Pv(ok), 0, None) == -1
    assert ch(st2, 2, 1, 128, None, 0, None) == -1
    assert ch(st2, 0, 1, 128, Pv(ok), 0, None) == -7
    assert ch(st2, 5, 1, 128, Pv(ok), 0, None) == -7
    assert ch(st2, 2, 1, 128, Pv(ok), -1, None) == -7
    assert ch(st2, 2, 17, 128, Pv(ok), 0, None) == -2
    assert ch(st2, 2, 1, 128, Pv(odd), 0, None) == -4
    assert ch(st2, 2, 1, 64, Pv(ok), 0, None) == -3
    bad, kb = stages(2, per=1, K=100)
    assert ch(bad, 2, 1, 128, Pv(ok), 0, None) == -2
    bad, kb = stages(2, per=1, y_f16=None)
    assert ch(bad, 2, 1, 128, Pv(ok), 0, None) == -1
    many, km = stages(1, per=11)
    assert ch(many, 1, 1, 128, Pv(ok), 0, None) == -7

    c = lib.awq_quantize_pack_clip
    rat = (ctypes.c_float * 3)(1.0, 0.9, 0.8)
    Pq = ctypes.c_void_p
    assert c(Pq(ok), None, 16, 128, 128, None, 3, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -1
    assert c(None, None, 16, 128, 128, rat, 3, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -1
    assert c(Pq(ok), None, 16, 128, 128, rat, 0, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -7
    assert c(Pq(ok), None, 16, 128, 128, rat, 33, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -7
    assert c(Pq(ok), None, 16, 128, 128, (ctypes.c_float * 1)(0.0), 1, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -7
    assert c(Pq(ok), None, 16, 100, 128, rat, 3, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -2
    assert c(Pq(odd), None, 16, 128, 128, rat, 3, None, 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -4
    assert c(Pq(ok), None, 16, 128, 128, rat, 3, Pq(ok), 0, Pq(ok), Pq(ok), Pq(ok), None, None) == -2
    assert c(Pq(ok), None, 16, 128, 128, rat, 3, Pq(ok), 65, Pq(ok), Pq(ok), Pq(ok), None, None) == -2
    assert c(Pq(ok), None, 16, 128, 128, rat, 3, Pq(odd), 8, Pq(ok), Pq(ok), Pq(ok), None, None) == -4

    rn = lib.awq_rmsnorm_inv_scale
    rn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                   ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]
    assert rn(None, ok, None, 1, 128, 1e-5, ok, None) == -1
    assert rn(ok, ok, None, 0, 128, 1e-5, ok, None) == -2
    assert rn(ok, ok, None, 1, 100, 1e-5, ok, None) == -2
    assert rn(ok, ok, None, 1, 128, -1.0, ok, None) == -7
    assert rn(ok, odd, None, 1, 128, 1e-5, ok, None) == -4
    assert rn(ok, ok, odd, 1, 128, 1e-5, ok, None) == -4

    fm = lib.awq_w4a16_linear_fused_multi
    ff = lib.awq_w4a16_linear_fused_fits
    ff.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int]
    assert ff(4096, 4096, 1, 128) == 1 and ff(4096, 11008, 4, 128) == 1 and ff(4096, 11008, 16, 128) == 0
    assert ff(4096, 4096, 17, 128) == 0 and ff(4096, 4100, 1, 128) == 0 and ff(4096, 4096, 1, 64) == 0
    fd = (awq.FusedDesc * 1)()
    fd[0] = awq.FusedDesc(awq.LinearDesc(ok, ok, ok, ok, ok, 4096, 4096), None, None, 1e-5, 0)
    fm.argtypes = [ctypes.POINTER(awq.FusedDesc), ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    assert fm(None, 1, 1, 128, None) == -1 and fm(fd, 0, 1, 128, None) == -7 and fm(fd, 25, 1, 128, None) == -7
    assert fm(fd, 1, 17, 128, None) == -2 and fm(fd, 1, 1, 64, None) != 0
    fd[0].pre_op = 1                                       # normalisation without factors
    assert fm(fd, 1, 1, 128, None) == -1
    fd[0].pre_f16 = odd
    assert fm(fd, 1, 1, 128, None) == -4
    fd[0].pre_f16, fd[0].eps = ok, -1.0
    assert fm(fd, 1, 1, 128, None) == -7
    fd[0].eps, fd[0].pre_op = 1e-5, 5
    assert fm(fd, 1, 1, 128, None) == -7
    fd[0] = awq.FusedDesc(awq.LinearDesc(ok, ok, ok, ok, ok, 4096, 11008), ok, None, 1e-5, 1)
    assert fm(fd, 1, 16, 128, None) == -2                  # with a normalisation: does not fit at M = 16

    rp = lib.awq_repack_w3_to_w4
    rp.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert rp(None, 16, 128, 128, ok, None) == -1 and rp(ok, 16, 100, 128, ok, None) == -2
    assert rp(ok, 16, 128, 128, odd, None) == -4 and rp(ok, 16, 128, 64, ok, None) == -3
    wb = lib.awq_w3a16_prefill_workspace_bytes
    wb.restype = ctypes.c_size_t
    wb.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    assert wb(4096, 4096, 128) == 4096 * 4096 // 2 and wb(4096, 100, 128) == 0
    pf = lib.awq_w3a16_linear_prefill
    pf.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int64] * 3 + [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                                 ctypes.c_void_p]
    assert pf(ok, ok, ok, ok, ok, 64, 16, 128, 128, None, 1 << 20, None) == -1
    assert pf(ok, ok, ok, ok, ok, 16, 16, 128, 128, ok, 1 << 20, None) == -2      # decode sizes: the other call
    assert pf(ok, ok, ok, ok, ok, 64, 16, 128, 128, odd, 1 << 20, None) == -4
    assert pf(ok, ok, ok, ok, ok, 64, 16, 128, 128, ok, 1023, None) == -5

    sm = lib.awq_silu_mul
    sm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    assert sm(None, ok, 8, ok, None) == -1 and sm(ok, ok, 8, None, None) == -1
    assert sm(ok, ok, 0, ok, None) == -2 and sm(ok, ok, 12, ok, None) == -2
    assert sm(ok, odd, 8, ok, None) == -4

    at = lib.awq_decode_attention
    wsa = lib.awq_decode_attention_workspace_bytes
    assert wsa(32, 128, 2048) == 32 * 16 * 130 * 4 and wsa(32, 64, 10) == 0 and wsa(32, 128, 0) == 0
    okp = ctypes.c_void_p(ok)
    base = [okp, okp, okp, okp, okp, 32, 32, 128, 64, 5, 10000.0, okp, okp, 1 << 20, None]
    def att(**kw):
        a = list(base)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return at(*a)
    assert att(_0=None) == -1 and att(_12=None) == -1
    assert att(_7=64) == -2 and att(_6=5) == -2 and att(_9=64) == -2 and att(_9=-1) == -2
    assert att(_10=1.0) == -7
    assert att(_3=ctypes.c_void_p(odd)) == -4
    assert att(_13=16) == -5

    # INT3-g128 variant
    q3, s3, z3 = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.awq_packed_sizes_w3(4096, 4096, 128, ctypes.byref(q3), ctypes.byref(s3), ctypes.byref(z3)) == 0
    assert (q3.value, s3.value, z3.value) == (4096 * 4096 * 3 // 8, 4096 * 32 * 2, 4096 * 32 // 2)
    assert (q3.value + s3.value + z3.value) * 256 == 4096 * 4096 * 101          # 0.39453125 B per weight
    assert lib.awq_packed_sizes_w3(4096, 4000, 128, None, None, None) == -2
    assert lib.awq_quantize_pack_w3(None, None, 16, 128, 128, Pq(ok), Pq(ok), Pq(ok), None) == -1
    assert lib.awq_quantize_pack_w3(Pq(ok), None, 16, 128, 64, Pq(ok), Pq(ok), Pq(ok), None) == -3
    assert lib.awq_quantize_pack_w3(Pq(odd), None, 16, 128, 128, Pq(ok), Pq(ok), Pq(ok), None) == -4
    assert lib.awq_unpack_w3(Pq(ok), None, Pq(ok), 16, 128, 128, Pq(ok), Pq(ok), Pq(ok), None) == -1
    assert lib.awq_w3a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), None, 1, 16, 128, 128, None) == -1
    assert lib.awq_w3a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(ok), 17, 16, 128, 128, None) == -2
    assert lib.awq_w3a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(ok), 0, 16, 128, 128, None) == -2
    assert lib.awq_w3a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(odd), 1, 16, 128, 128, None) == -4

    # INT2-g64 variant
    q2, s2, z2 = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.awq_packed_sizes_w2(4096, 4096, 64, ctypes.byref(q2), ctypes.byref(s2), ctypes.byref(z2)) == 0
    assert (q2.value, s2.value, z2.value) == (4096 * 4096 // 4, 4096 * 64 * 2, 4096 * 64 // 4)
    assert (q2.value + s2.value + z2.value) * 256 == 4096 * 4096 * 73          # 0.28515625 B per weight
    assert lib.awq_packed_sizes_w2(4096, 4096 + 128, 64, None, None, None) == -2      # K % 256
    assert lib.awq_packed_sizes_w2(4096, 4096, 128, None, None, None) == -3
    assert lib.awq_quantize_pack_w2(None, None, 16, 256, 64, Pq(ok), Pq(ok), Pq(ok), None) == -1
    assert lib.awq_quantize_pack_w2(Pq(ok), None, 16, 256, 128, Pq(ok), Pq(ok), Pq(ok), None) == -3
    assert lib.awq_quantize_pack_w2(Pq(odd), None, 16, 256, 64, Pq(ok), Pq(ok), Pq(ok), None) == -4
    assert lib.awq_unpack_w2(Pq(ok), None, Pq(ok), 16, 256, 64, Pq(ok), Pq(ok), Pq(ok), None) == -1
    assert lib.awq_w2a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), None, 1, 16, 256, 64, None) == -1
    assert lib.awq_w2a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(ok), 1 << 31, 16, 256, 64, None) == -2
    assert lib.awq_w2a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(ok), 0, 16, 256, 64, None) == -2
    assert lib.awq_w2a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(ok), 1, 16, 384, 64, None) == -2
    assert lib.awq_w2a16_linear(Pq(ok), Pq(ok), Pq(ok), Pq(ok), Pq(odd), 1, 16, 256, 64, None) == -4
    assert lib.awq_w2a16_linear_multi(None, 1, 1, 64, None) == -1

    g = lib.awq_search_scale
    wsb = lib.awq_search_scale_workspace_bytes
    al = (ctypes.c_float * 3)(0.0, 0.5, 1.0)
    need = wsb(64, 4096, 4096, 3, 128)
    # packed candidate + x/s + two [T,N] outputs + means, s and partial sums
    assert need >= 4096 * 4096 // 2 + 64 * 4096 * 2 * 3 + 3 * 1024 * 8
    assert wsb(64, 4096, 4000, 3, 128) == 0 and wsb(0, 4096, 4096, 3, 128) == 0
    assert wsb(64, 4096, 4096, 65, 128) == 0 and wsb(64, 4096, 4096, 3, 64) == 0
    P = ctypes.c_void_p
    args = lambda **kw: [kw.get("W", P(ok)), kw.get("X", P(ok)), kw.get("T", 64), 4096, kw.get("K", 4096),
                         kw.get("al", al), kw.get("n", 3), kw.get("group", 128), kw.get("ws", P(ok)),
                         kw.get("wsb", need), kw.get("losses", P(ok)), kw.get("best", P(ok)),
                         kw.get("s", P(ok)), None]
    assert g(*args(W=None)) == -1
    assert g(*args(al=None)) == -1
    assert g(*args(ws=None)) == -1
    assert g(*args(K=4000)) == -2
    assert g(*args(T=0)) == -2
    assert g(*args(group=32)) == -3
    assert g(*args(n=0)) == -7
    assert g(*args(n=65)) == -7
    assert g(*args(al=(ctypes.c_float * 3)(0.0, 1.5, 1.0))) == -7
    assert g(*args(X=P(odd))) == -4
    assert g(*args(ws=P(0x1010))) == -4                           # workspace wants 256-byte alignment
    assert g(*args(wsb=need - 1)) == -5


def test_blob_header_round_trip_and_refusals(lib):
    import paper_2306_00978_amd as awq
    assert ctypes.sizeof(awq.BlobHeader) == 64
    for bits, N, K in ((4, 4096, 11008), (3, 176, 1408), (2, 64, 512)):
        h = awq.awq_blob_header(bits, N, K)
        assert h.magic == b"AWQgfx95" and h.layout_version == awq.awq_version() and h.bits == bits
        sizes = {4: awq.awq_packed_sizes, 3: awq.awq_packed_sizes_w3, 2: awq.awq_packed_sizes_w2}[bits](N, K)
        assert (h.qweight_bytes, h.scales_bytes, h.zeros_bytes) == tuple(sizes)
        awq.awq_blob_header_check(h)
        raw = bytes(h)
        assert awq.awq_blob_header_check(awq.BlobHeader.from_buffer_copy(raw)) is None
        for field, value in (("layout_version", 2), ("bits", 5), ("K", K + 1), ("qweight_bytes", 1), ("reserved", 7),
                             ("magic", b"AWQgfx94")):
            bad = awq.BlobHeader.from_buffer_copy(raw)
            setattr(bad, field, value)
            assert lib.awq_blob_header_check(ctypes.byref(bad)) < 0, field
    h = awq.BlobHeader()
    assert lib.awq_blob_header_init(ctypes.byref(h), 4, 100, 128, 128) == -2
    assert lib.awq_blob_header_init(ctypes.byref(h), 5, 16, 128, 128) == -7
    assert lib.awq_blob_header_init(None, 4, 16, 128, 128) == -1
    assert lib.awq_blob_header_check(None) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2306_00978_amd as awq
    with pytest.raises(TypeError):
        awq.awq_quantize_pack(torch.zeros(16, 128, dtype=torch.float16))
    with pytest.raises(TypeError):
        awq.awq_w4a16_linear(torch.zeros(1, 128, dtype=torch.float16), None, None, None, 16)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2306_00978_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "awq_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2306_00978_amd" not in text and "awq_mi355x" not in text, f
