"""Parity of the INT2-g64 variant (AWQ Sec. 5, extreme low-bit table) of the HIP path against
the CPU oracle, through the C ABI.  Bars as for the 4-bit path: packed bytes, steps and zero
points bit-exact; outputs within 2e-3 of the normalised error."""
import numpy as np
import pytest

from test_gpu_parity import TOL, awq, dev, guarded, host, make_case  # noqa: F401  (awq is a fixture)

pytestmark = pytest.mark.gpu


def quantize_w2_bit_exact(awq, W, s):
    import torch
    import oracle
    N, K = W.shape
    codes, scales, zeros = oracle.quantize_w2(W, s)
    q_ref, s_ref, z_ref = oracle.pack_w2(codes, scales, zeros)
    qb, sb, zb = awq.awq_packed_sizes_w2(N, K)
    assert (qb, sb, zb) == oracle.packed_sizes_w2(N, K)
    q_gpu, cq = guarded(qb, torch.uint8)
    s_gpu, cs = guarded(sb, torch.float16)
    z_gpu, cz = guarded(zb, torch.uint8)
    awq.awq_quantize_pack_w2(dev(W), None if s is None else dev(s), out=(q_gpu, s_gpu, z_gpu))
    cq(); cs(); cz()
    assert np.array_equal(host(s_gpu).view(np.uint16), s_ref), "steps differ"
    assert np.array_equal(host(z_gpu), z_ref), "zero points differ"
    assert np.array_equal(host(q_gpu), q_ref), "packed codes differ"
    c_u, s_u, z_u = awq.awq_unpack_w2(q_gpu, s_gpu, z_gpu, N, K)
    assert np.array_equal(host(c_u), codes)
    assert np.array_equal(host(s_u).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(host(z_u), zeros)
    return (codes, scales, zeros), (q_gpu, s_gpu, z_gpu)


def check_linear_w2(awq, xs, Wdq, gpu_packed, N):
    import torch
    import oracle
    M, K = xs.shape
    y_gpu, cy = guarded(M * N * 2, torch.float16)
    y_gpu = y_gpu.view(M, N)
    awq.awq_w2a16_linear(dev(xs), *gpu_packed, N, out=y_gpu)
    cy()
    yh = host(y_gpu)
    assert np.all(np.isfinite(yh.astype(np.float32)))
    err = oracle.norm_error(yh, oracle.matmul(xs, Wdq), xs, Wdq)
    assert err.max() <= TOL, f"max normalised error {err.max():.3e} (M={M})"


@pytest.mark.parametrize("N,K", [(16, 256), (48, 768), (176, 1280), (272, 2304), (32, 8192)])
def test_w2_small_shapes_every_m(awq, N, K):
    """One block per row (three of a workgroup's four waves idle), odd block counts, K cut into four
    slices with ragged batches, long rows (K = 8192: eight blocks per wave)."""
    import oracle
    case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=40)
    ref, gpu = quantize_w2_bit_exact(awq, case.W, s)
    quantize_w2_bit_exact(awq, case.W, None)
    Wdq = oracle.dequant(*ref, group=64)
    for M in range(1, 17):
        check_linear_w2(awq, xs[:M], Wdq, gpu, N)
    check_linear_w2(awq, np.tile(xs, (3, 1))[:37], Wdq, gpu, N)       # blocks of 16 rows, last moved back
    check_linear_w2(awq, np.tile(xs, (8, 1)), Wdq, gpu, N)            # 128 rows: eight blocks
    if K <= 1280:
        big = np.tile(xs, (19, 1))
        check_linear_w2(awq, big[:300], Wdq, gpu, N)                  # 128 + 128 + 44 rows
        check_linear_w2(awq, big[:261], Wdq, gpu, N)                  # 128 + 128 + 5 rows (a plain launch)


def test_w2_edge_groups_and_exactness_on_integer_data(awq):
    import oracle
    g = np.random.default_rng(81)
    N, K = 64, 512
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0, :64] = 0
    W[1, :64] = np.float16(0.37)
    W[2, 64:128] = np.abs(W[2, 64:128])
    W[3, 64:128] = -np.abs(W[3, 64:128])
    W[4, 256:320] *= 1000
    W[5, 0], W[5, 1] = 65504.0, -65504.0
    W[6, :] = np.float16(6e-8)
    quantize_w2_bit_exact(awq, W, None)
    quantize_w2_bit_exact(awq, W, (10.0 ** g.uniform(-3, 3, size=K)).astype(np.float32))
    # small integers: every product and sum is exact, the kernel must reproduce the oracle
    codes = g.integers(0, 4, size=(N, K), dtype=np.uint8)
    scales = (2.0 ** g.integers(-3, 2, size=(N, K // 64))).astype(np.float16)
    zeros = g.integers(0, 4, size=(N, K // 64), dtype=np.uint8)
    q, sp, zp = oracle.pack_w2(codes, scales, zeros)
    gpu = (dev(q), dev(sp.view(np.float16)), dev(zp))
    Wdq = oracle.dequant(codes, scales, zeros, group=64)
    for M in (1, 5, 16, 40):
        x = g.integers(-4, 5, size=(M, K)).astype(np.float16)
        y_ref = oracle.matmul(x, Wdq)
        y1 = host(awq.awq_w2a16_linear(dev(x), *gpu, N))
        y2 = host(awq.awq_w2a16_linear(dev(x), *gpu, N))
        assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
        assert np.array_equal(y1.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))


def test_w2_rejects_what_it_cannot_run(awq):
    import torch
    x = torch.zeros((1, 384), dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.awq_packed_sizes_w2(16, 384)                      # K not a multiple of 256
    assert e.value.status == -2
    with pytest.raises(awq.AwqError) as e:
        awq.awq_packed_sizes_w2(16, 256, group=128)
    assert e.value.status == -3
    q = torch.zeros(16 * 256 // 4, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(16 * 4, dtype=torch.float16, device="cuda")
    zp = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        awq.awq_w2a16_linear(torch.zeros((1, 256), dtype=torch.float16, device="cuda"), q[:512], sc, zp, 16)
    del x


def check_multi_w2(awq, problems, M):
    import torch
    import oracle
    linears, checks, outs = [], [], []
    for xs, Wdq, gpu_packed, N in problems:
        y, cy = guarded(M * N * 2, torch.float16)
        y = y.view(M, N)
        linears.append((dev(xs[:M]), *gpu_packed, y, N))
        checks.append(cy)
        outs.append(y)
    awq.awq_w2a16_linear_multi(linears)
    for (xs, Wdq, gpu_packed, N), y, cy in zip(problems, outs, checks):
        cy()
        yh = host(y)
        assert np.all(np.isfinite(yh.astype(np.float32)))
        err = oracle.norm_error(yh, oracle.matmul(xs[:M], Wdq), xs[:M], Wdq)
        assert err.max() <= TOL, f"max normalised error {err.max():.3e} (N={N}, M={M})"


def test_w2_grouped_small_every_m(awq):
    """Linears of different K in one launch (each with its own number of K slices), more than
    eight linears (several launches)."""
    import oracle
    probs = []
    for i, (N, K) in enumerate([(176, 1280), (64, 256), (48, 2048), (320, 512), (32, 8192)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=45 + i)
        ref, gpu = quantize_w2_bit_exact(awq, case.W, s)
        probs.append((xs, oracle.dequant(*ref, group=64), gpu, N))
    for M in range(1, 17):
        check_multi_w2(awq, probs, M)
    check_multi_w2(awq, probs[:1], 3)
    check_multi_w2(awq, probs[:4] * 5, 2)                     # 20 entries: three launches


def test_w2_grouped_many_rows_ragged_row_block_counts(awq):
    """More than 1024 row blocks in the launch: K is cut by the length of the rows (5 blocks: one
    slice, four row blocks per workgroup; 9 blocks: two slices, two row blocks; 17 blocks: four
    slices), and no linear has a multiple of four row blocks, so the last workgroup of each has
    waves without a row block."""
    import oracle
    probs = []
    for i, (N, K) in enumerate([(6000, 1280), (5008, 2304), (5520, 256), (2000, 4352)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=60 + i)
        ref, gpu = quantize_w2_bit_exact(awq, case.W, s)
        probs.append((xs, oracle.dequant(*ref, group=64), gpu, N))
    for M in (1, 3, 8, 16):
        check_multi_w2(awq, probs, M)


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 11008)])
def test_w2_llama7b_shapes_full_size(awq, N, K):
    import oracle
    case, s, xs = make_case(N, K, 16, 0.02, cfg=1, proj=50)
    ref, gpu = quantize_w2_bit_exact(awq, case.W, s)
    Wdq = oracle.dequant(*ref, group=64)
    for M in (1, 4, 16):
        check_linear_w2(awq, xs[:M], Wdq, gpu, N)
    check_linear_w2(awq, np.tile(xs, (3, 1))[:40], Wdq, gpu, N)


def test_w2_grouped_llama7b_layer_full_size(awq):
    import oracle
    probs = []
    for i, (N, K) in enumerate([(4096, 4096), (11008, 4096), (4096, 11008)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=1, proj=52 + i)
        ref, gpu = quantize_w2_bit_exact(awq, case.W, s)
        probs.append((xs, oracle.dequant(*ref, group=64), gpu, N))
    layer = [probs[0]] * 4 + [probs[1]] * 2 + [probs[2]]
    for M in (1, 4, 16):
        check_multi_w2(awq, layer, M)
