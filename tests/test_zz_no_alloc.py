"""awq_w4a16_linear_static (the entry point for callers that cannot allocate) against
awq_w4a16_linear with a caller's workspace: same kernels, same K ranges, so the outputs must be
equal bit for bit -- on two calls in a row, the second with a smaller input (the built-in scratch
keeps the first call's contents), and against the oracle at the tolerance of the linear.  Shapes
that need no scratch, and a shape beyond the limit, are covered as well."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2306_00978_amd as awq

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _case(N, K, M, proj):
    case = workloads.linear_case("static", N, K, M, workloads.SIGMA_7B, cfg=2, layer=7, proj=proj)
    s = oracle.act_scale(case.calib, 0.5).astype(np.float32)
    xs = oracle.apply_inv_scale(case.x, s)
    codes, scales, zeros = oracle.quantize(case.W, s)
    packed = [torch.from_numpy(a).cuda() for a in oracle.pack(codes, scales, zeros)]
    packed[1] = packed[1].view(torch.float16)
    return xs, torch.from_numpy(xs).cuda(), packed, oracle.dequant(codes, scales, zeros)


def test_static_scratch_entry_point_equals_the_workspace_call_twice_in_a_row():
    assert torch.cuda.is_available()
    limit = awq.awq_static_scratch_bytes()
    assert limit == 32 << 20
    # first call: 512 tokens on 1024 x 4096 (8 K ranges); second: 200 tokens on 512 x 2048 -- smaller
    # in every dimension, so it runs on scratch the first call left filled
    for (N, K, M, proj) in ((1024, 4096, 512, 0), (512, 2048, 200, 1)):
        xs, x, (q, sc, zp), Wdq = _case(N, K, M, proj)
        need = awq.awq_linear_workspace_bytes(M, N, K)
        assert 0 < need <= limit, (N, K, M, need)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        y_ref = awq.awq_w4a16_linear(x, q, sc, zp, N, workspace=ws)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        awq.awq_w4a16_linear_static(x, q, sc, zp, N, y)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (N, K, M)
        rows = np.linspace(0, M - 1, 24).astype(int)
        err = oracle.norm_error(y.cpu().numpy()[rows], oracle.matmul(xs[rows], Wdq), xs[rows], Wdq)
        assert err.max() <= TOL, (N, K, M, err.max())


def test_static_entry_point_without_scratch_and_beyond_the_limit():
    # decode and M = 160 on a shape whose prefill needs no K ranges: the scratch is not touched
    for (N, K, M, proj) in ((256, 1024, 4, 2), (512, 512, 1000, 3)):
        xs, x, (q, sc, zp), Wdq = _case(N, K, M, proj)
        y_ref = awq.awq_w4a16_linear(x, q, sc, zp, N, workspace=False)
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        awq.awq_w4a16_linear_static(x, q, sc, zp, N, y)
        torch.cuda.synchronize()
        assert awq.awq_linear_workspace_bytes(M, N, K) == 0
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
        err = oracle.norm_error(y.cpu().numpy(), oracle.matmul(xs, Wdq), xs, Wdq)
        assert err.max() <= TOL
    # beyond the limit: refused before anything is launched, y untouched
    N, K, M = 4096, 8192, 1025
    need = awq.awq_linear_workspace_bytes(M, N, K)
    assert need > awq.awq_static_scratch_bytes()
    q = torch.zeros(N * K // 2, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(N * K // 128, dtype=torch.float16, device="cuda")
    zp = torch.zeros(N * K // 256, dtype=torch.uint8, device="cuda")
    x = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    y = torch.full((M, N), 3.0, dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.awq_w4a16_linear_static(x, q, sc, zp, N, y)
    assert e.value.status == -8
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())
