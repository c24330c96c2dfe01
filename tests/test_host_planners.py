"""The host side of every launch bench.py and the GPU tests make -- validation, planners, launch
tables, argument marshalling -- run on the CPU, without a GPU: the entry points are called with
made-up (aligned, non-null) device addresses.  Everything up to the launch itself executes, the
launch fails for want of a device and the call returns AWQ_ERR_HIP.  tests/test_sanitizers.py runs
this file against the build whose host code is under AddressSanitizer and
UndefinedBehaviorSanitizer, so an out-of-bounds write into a launch table, an overflow in a plan or
a misuse of a descriptor array would end that run.

On a machine WITH a GPU the made-up addresses would reach real kernels: the whole file is skipped
there."""
import ctypes
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def _gpu_present():
    import torch
    return torch.cuda.device_count() > 0


pytestmark = pytest.mark.skipif(_gpu_present(), reason="made-up device addresses: only where no GPU can run them")

AWQ_ERR_HIP = -6
SHAPES_7B = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
SHAPES_70B = [(8192, 8192), (1024, 8192), (1024, 8192), (8192, 8192), (28672, 8192), (28672, 8192), (8192, 28672)]
RAGGED = [(4112, 4096), (2064, 4096), (8208, 2048), (1040, 8192), (4112, 1408), (6160, 4096), (3088, 11008),
          (272, 28672), (16, 4096), (32, 512), (80, 384), (16400, 640)]


@pytest.fixture(scope="module")
def awq():
    import paper_2306_00978_amd as m
    m.load()
    return m


class Addresses:
    """Distinct 256-byte-aligned made-up addresses."""
    def __init__(self):
        self.next = 0x7E0000000000

    def take(self, nbytes):
        a = self.next
        self.next += (int(nbytes) + 255) // 256 * 256 + 256
        return a


def linear_descs(awq, addr, shapes, M, bits=4):
    arr = (awq.LinearDesc * len(shapes))()
    per_weight = {4: 0.5, 3: 0.375, 2: 0.25}[bits]
    for i, (N, K) in enumerate(shapes):
        arr[i] = awq.LinearDesc(addr.take(2 * M * K), addr.take(N * K * per_weight), addr.take(N * K // 32),
                                addr.take(N * K // 128), addr.take(2 * M * N), N, K)
    return arr


def test_grouped_decode_plans(awq):
    lib = awq.load()
    addr = Addresses()
    seen = set()
    for shapes in (SHAPES_7B, SHAPES_70B, SHAPES_7B * 8, RAGGED, RAGGED[-1:], SHAPES_7B[:1], SHAPES_7B[6:]):
        for M in (1, 2, 3, 4, 5, 8, 9, 16):
            arr = linear_descs(awq, addr, shapes, M)
            st = lib.awq_w4a16_linear_multi(arr, len(shapes), ctypes.c_int64(M), 128, None, ctypes.c_size_t(0), None)
            assert st == AWQ_ERR_HIP, (len(shapes), M, st)
            seen.add(lib.awq_last_grouped_plan())
    assert {1, 2} <= seen                      # both plans of the streaming kernel were built
    for shapes in (SHAPES_7B, RAGGED[:6]):
        for M in (1, 4, 16):
            arr = linear_descs(awq, addr, shapes, M, bits=3)
            assert lib.awq_w3a16_linear_multi(arr, len(shapes), ctypes.c_int64(M), 128, None) == AWQ_ERR_HIP
    w2 = [(N, K) for N, K in SHAPES_7B]
    for M in (1, 8, 16):
        arr = linear_descs(awq, addr, w2, M, bits=2)
        assert lib.awq_w2a16_linear_multi(arr, len(w2), ctypes.c_int64(M), 64, None) == AWQ_ERR_HIP


def test_single_linear_every_route(awq):
    """Decode, token blocks of 16, K-range prefill with and without workspace, the static entry."""
    lib = awq.load()
    addr = Addresses()
    for N, K in [(4096, 4096), (11008, 4096), (4096, 11008), (32000, 4096), (176, 1408), (28672, 8192)]:
        for M in (1, 7, 16, 17, 24, 100, 128, 200, 512, 2048):
            x, q, s, z, y = (addr.take(2 * M * K), addr.take(N * K // 2), addr.take(N * K // 32),
                             addr.take(N * K // 128), addr.take(2 * M * N))
            need = lib.awq_linear_workspace_bytes(ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), 128)
            for ws in ((None, 0), (addr.take(need), need)) if need else ((None, 0),):
                st = lib.awq_w4a16_linear(x, q, s, z, y, ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), 128,
                                          ws[0], ctypes.c_size_t(ws[1]), None)
                assert st == AWQ_ERR_HIP, (N, K, M, st)
            st = lib.awq_w4a16_linear_static(x, q, s, z, y, ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K),
                                             128, None)
            assert st in (AWQ_ERR_HIP, -8), (N, K, M, st)     # -8: beyond the static scratch


def test_fused_chain_and_quantize_tables(awq):
    lib = awq.load()
    addr = Addresses()
    M = 1

    def fused(shapes, pre_op, with_residual):
        arr = (awq.FusedDesc * len(shapes))()
        for i, (N, K) in enumerate(shapes):
            lin = awq.LinearDesc(addr.take(2 * M * K), addr.take(N * K // 2), addr.take(N * K // 32),
                                 addr.take(N * K // 128), addr.take(2 * M * N), N, K)
            arr[i] = awq.FusedDesc(lin, addr.take(2 * K) if pre_op else None,
                                   addr.take(2 * M * N) if with_residual else None, 1e-5, pre_op)
        return arr

    qkv = fused([(4096, 4096)] * 3, 1, False)
    o = fused([(4096, 4096)], 0, True)
    gate_up = fused([(11008, 4096)] * 2, 1, False)
    down = fused([(4096, 11008)], 0, True)
    for arr in (qkv, o, gate_up, down):
        st = lib.awq_w4a16_linear_fused_multi(arr, len(arr), ctypes.c_int64(M), 128, None)
        assert st == AWQ_ERR_HIP, st
    stages = (awq.ChainStage * 4)()
    for i, arr in enumerate((qkv, o, gate_up, down)):
        stages[i] = awq.ChainStage(ctypes.cast(arr, ctypes.POINTER(awq.FusedDesc)), len(arr))
    st = lib.awq_w4a16_linear_chain(stages, 4, ctypes.c_int64(M), 128, addr.take(8192), 0, None)
    assert st == AWQ_ERR_HIP, st

    ad = (awq.ActScaleDesc * 64)()
    for i in range(64):
        T, K = [(65536, 4096), (64, 11008), (5, 136), (1, 8)][i % 4]
        ad[i] = awq.ActScaleDesc(addr.take(2 * T * K), T, K, addr.take(4 * K))
    for count in (1, 4, 16, 17, 64):
        assert lib.awq_act_scale_multi(ad, count, 0.5, None) == AWQ_ERR_HIP

    qd = (awq.QuantizeDesc * 64)()
    for i in range(64):
        N, K = (SHAPES_7B + RAGGED)[i % 19]
        qd[i] = awq.QuantizeDesc(addr.take(2 * N * K), addr.take(4 * K) if i % 2 else None, N, K,
                                 addr.take(N * K // 2), addr.take(N * K // 32), addr.take(N * K // 128))
    for count in (1, 7, 16, 17, 64):
        assert lib.awq_quantize_pack_multi(qd, count, 128, None) == AWQ_ERR_HIP
