"""Parity of the HIP path (through the C ABI) against the CPU oracle.

Bars: codes / steps / zero points / packed bytes bit-exact; outputs within
|y_gpu - y_ref| / (||x_row||_2 * max|Wdq| + 1e-6) <= 2e-3 for every element.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def awq():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2306_00978_amd as awq
    awq.load()          # raises if the HIP library is missing: no fallback
    return awq


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def guarded(nbytes, dtype, fill=0xA5, pad=4096):
    """A device buffer with canary bytes on both sides; returns (view, check)."""
    import torch
    raw = torch.full((nbytes + 2 * pad,), fill, dtype=torch.uint8, device="cuda")
    view = raw[pad:pad + nbytes].view(dtype)

    def check():
        torch.cuda.synchronize()
        assert bool((raw[:pad] == fill).all()) and bool((raw[pad + nbytes:] == fill).all()), \
            "kernel wrote outside its output buffer"
    return view, check


# ----------------------------------------------------------------------------- quantize

def quantize_both(awq, W, s):
    import torch
    import oracle
    N, K = W.shape
    codes, scales, zeros = oracle.quantize(W, s)
    q_ref, s_ref, z_ref = oracle.pack(codes, scales, zeros)
    qb, sb, zb = awq.awq_packed_sizes(N, K)
    q_gpu, cq = guarded(qb, torch.uint8)
    s_gpu, cs = guarded(sb, torch.float16)
    z_gpu, cz = guarded(zb, torch.uint8)
    awq.awq_quantize_pack(dev(W), None if s is None else dev(s), out=(q_gpu, s_gpu, z_gpu))
    cq(); cs(); cz()
    return (codes, scales, zeros), (q_ref, s_ref, z_ref), (q_gpu, s_gpu, z_gpu)


def assert_quantize_bit_exact(awq, W, s):
    import oracle
    N, K = W.shape
    (codes, scales, zeros), (q_ref, s_ref, z_ref), (q_gpu, s_gpu, z_gpu) = quantize_both(awq, W, s)
    assert np.array_equal(host(s_gpu).view(np.uint16), s_ref), "steps differ"
    assert np.array_equal(host(z_gpu), z_ref), "zero points differ"
    qg = host(q_gpu)
    if not np.array_equal(qg, q_ref):
        c_gpu, _, _ = oracle.unpack(qg, s_ref, z_ref, N, K)
        bad = np.argwhere(c_gpu != codes)
        raise AssertionError(f"{len(bad)} codes differ, first at {bad[:5].tolist()}")
    # the export path returns the canonical arrays
    c_u, s_u, z_u = awq.awq_unpack(q_gpu, s_gpu, z_gpu, N, K)
    assert np.array_equal(host(c_u), codes)
    assert np.array_equal(host(s_u).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(host(z_u), zeros)
    return (codes, scales, zeros), (q_gpu, s_gpu, z_gpu)


def make_case(N, K, M, sigma, cfg, proj=0):
    """Raw inputs from the seeded generator; s and x' through the oracle."""
    import oracle
    import workloads
    case = workloads.linear_case(f"{N}x{K}", N, K, M, sigma, cfg, layer=0, proj=proj)
    s = oracle.act_scale(case.calib, 0.5).astype(np.float32)
    xs = oracle.apply_inv_scale(case.x, s)
    return case, s, xs


@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (80, 1408), (272, 256)])
def test_quantize_pack_small_shapes(awq, N, K):
    g = np.random.default_rng(100 + N)
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    s = g.uniform(0.3, 5.0, size=K).astype(np.float32)
    assert_quantize_bit_exact(awq, W, s)
    assert_quantize_bit_exact(awq, W, None)


def test_quantize_pack_edge_groups(awq):
    K = 512
    W = np.zeros((32, K), dtype=np.float16)
    W[1, :] = 0.5
    W[2, :] = -0.25
    W[3, :128] = np.linspace(1.0, 2.5, 128)
    W[4, :128] = -np.linspace(1.0, 2.5, 128)
    W[5, 0], W[5, 1] = 65504.0, -65504.0                 # step clamps at the fp16 maximum
    W[6, :] = np.float16(6e-8)                            # subnormal halves
    g = np.random.default_rng(7)
    W[7, :] = (g.standard_normal(K) * 1e-6).astype(np.float16)
    W[8, :] = (g.standard_normal(K) * 100).astype(np.float16)
    # exact ties: w/scale lands on .5 -> round-half-even must agree
    W[9, :128] = (np.arange(128) % 31) * 0.25
    W[10:, :] = (g.standard_normal((22, K)) * 0.02).astype(np.float16)
    s = np.full(K, 16.0, dtype=np.float32)
    assert_quantize_bit_exact(awq, W, s)
    assert_quantize_bit_exact(awq, W, None)
    s2 = g.uniform(1e-3, 1e3, size=K).astype(np.float32)
    assert_quantize_bit_exact(awq, W, s2)


def test_quantize_near_ties_and_wide_ranges(awq):
    """Groups built so that w/step lands on or next to half-integers, over the whole range of
    step magnitudes (2^-14 .. 6e4) and with s spread over six decades: the kernel's division by
    the group's step must reproduce the IEEE quotient the oracle uses, bit for bit."""
    g = np.random.default_rng(99)
    N, K = 512, 1024
    W = np.zeros((N, K), dtype=np.float32)
    for n in range(N):
        for grp in range(K // 128):
            step = 2.0 ** g.uniform(-13, 11)
            k = g.integers(0, 16, size=128).astype(np.float64)
            frac = g.choice([0.0, 0.5, 0.5 - 2e-4, 0.5 + 2e-4, 0.25, 0.4999, 0.5001], size=128)
            v = (k + frac) * step - g.integers(0, 9) * step
            v[0], v[1] = v.min() - 0.0, v.max() + 0.0
            W[n, grp * 128:(grp + 1) * 128] = v
    W = np.clip(W, -60000, 60000).astype(np.float16)
    assert_quantize_bit_exact(awq, W, None)
    s = (10.0 ** g.uniform(-3, 3, size=K)).astype(np.float32)
    assert_quantize_bit_exact(awq, W, s)
    s_huge = np.full(K, 1e25, dtype=np.float32)            # |w s| beyond the shared-reciprocal range
    assert_quantize_bit_exact(awq, W, s_huge)


def test_quantize_pack_multi_equals_the_oracle_on_every_matrix(awq):
    """awq_quantize_pack_multi: matrices of different shapes in one call (more than one launch's
    worth: 19 matrices = 16 + 3), with and without s, ragged group counts, one matrix much larger
    than the rest -- every packed array bit for bit the oracle's, and nothing written around them."""
    import torch
    import oracle
    g = np.random.default_rng(4242)
    shapes = [(64, 512), (16, 128), (176, 1408), (1024, 4096), (48, 384), (320, 256), (16, 4096)] * 3
    shapes = shapes[:19]
    mats, refs, outs, guards = [], [], [], []
    for i, (N, K) in enumerate(shapes):
        W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
        s = None if i % 3 == 2 else g.uniform(0.3, 5.0, size=K).astype(np.float32)
        codes, scales, zeros = oracle.quantize(W, s)
        refs.append(oracle.pack(codes, scales, zeros))
        bufs = []
        for nb, dt in zip(awq.awq_packed_sizes(N, K), (torch.uint8, torch.float16, torch.uint8)):
            pad = 256 // (2 if dt == torch.float16 else 1)
            whole = torch.full((nb // (2 if dt == torch.float16 else 1) + 2 * pad,), 7, dtype=dt, device="cuda")
            guards.append((whole, pad))
            bufs.append(whole[pad:whole.numel() - pad])
        outs.append(tuple(bufs))
        mats.append((dev(W), None if s is None else dev(s), outs[-1]))
    awq.prepare_quantize_pack_multi(mats)()
    torch.cuda.synchronize()
    for i, ((q, sc, zp), (q_ref, s_ref, z_ref)) in enumerate(zip(outs, refs)):
        assert np.array_equal(host(q), q_ref), f"matrix {i}: codes"
        assert np.array_equal(host(sc).view(np.uint16), s_ref), f"matrix {i}: steps"
        assert np.array_equal(host(zp), z_ref), f"matrix {i}: zero points"
    for whole, pad in guards:
        assert bool((whole[:pad] == 7).all()) and bool((whole[whole.numel() - pad:] == 7).all())
    # the single call is the one-matrix case of the same launch
    W, s, _ = mats[3]
    q1, s1, z1 = awq.awq_quantize_pack(W, s)
    assert torch.equal(q1, outs[3][0]) and torch.equal(s1.view(torch.int16), outs[3][1].view(torch.int16))


CONFIG_SHAPES = [
    # (N, K, sigma, cfg)
    (4096, 4096, 0.02, 1), (11008, 4096, 0.02, 1), (4096, 11008, 0.02, 1),
    (8192, 8192, 0.015, 3), (1024, 8192, 0.015, 3), (28672, 8192, 0.015, 3),
    (8192, 28672, 0.015, 3),
]
_cache = {}


def config_case(awq, N, K, sigma, cfg):
    """Quantize once per distinct shape (bit-exact check included) and reuse."""
    key = (N, K, cfg)
    if key not in _cache:
        while len(_cache) >= 3:                          # keep host memory bounded
            _cache.pop(next(iter(_cache)))
        proj = [c[:2] for c in CONFIG_SHAPES].index((N, K))
        case, s, xs16 = make_case(N, K, 16, sigma, cfg, proj=proj)
        ref, gpu = assert_quantize_bit_exact(awq, case.W, s)
        import oracle
        Wdq = oracle.dequant(*ref)
        _cache[key] = (case, s, xs16, ref, gpu, Wdq)
    return _cache[key]


def check_linear(awq, xs, Wdq, gpu_packed, N, rows=None):
    """Run the GPU layer on xs[M,K]; compare rows (all if None) with the oracle."""
    import torch
    import oracle
    M, K = xs.shape
    y_gpu, cy = guarded(M * N * 2, torch.float16)
    y_gpu = y_gpu.view(M, N)
    awq.awq_w4a16_linear(dev(xs), *gpu_packed, N, out=y_gpu)
    cy()
    yh = host(y_gpu)
    sel = np.arange(M) if rows is None else np.asarray(rows)
    y_ref = oracle.matmul(xs[sel], Wdq)
    err = oracle.norm_error(yh[sel], y_ref, xs[sel], Wdq)
    assert np.all(np.isfinite(yh.astype(np.float32)))
    assert err.max() <= TOL, f"max normalised error {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"
    return err.max()


@pytest.mark.parametrize("N,K,sigma,cfg", CONFIG_SHAPES)
def test_config_shapes_quantize_and_decode(awq, N, K, sigma, cfg):
    """Every distinct (N,K) of the five configs: bit-exact quantize/pack at full size, then
    the decode path at the M values the configs name (1, 4, 8, 16)."""
    case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, sigma, cfg)
    for M in ((1, 4, 16) if cfg == 1 else (1, 8)):
        check_linear(awq, xs16[:M], Wdq, gpu, N)


@pytest.mark.parametrize("N,K", [(4096, 4096), (11008, 4096), (4096, 11008)])
def test_config2_prefill_full_size_sampled_rows(awq, N, K):
    """M = 2048 prefill at full size; 64 seeded rows are checked against the oracle
    (every output column of those rows)."""
    import oracle
    import workloads
    case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.02, 1)
    X = workloads.activations(2048, K, 2, 0, 0, workloads.ROLE_X, case.outliers)
    xs = oracle.apply_inv_scale(X, s)
    rows = np.sort(np.random.default_rng(5).choice(2048, size=64, replace=False))
    check_linear(awq, xs, Wdq, gpu, N, rows=rows)


# ------------------------------------------------------------------- decode / prefill, small

@pytest.fixture(scope="module")
def small(awq):
    N, K = 176, 1408          # 11 row blocks (not a multiple of 8), 11 groups
    case, s, xs = make_case(N, K, 300, 0.02, cfg=0)
    ref, gpu = assert_quantize_bit_exact(awq, case.W, s)
    import oracle
    return N, K, xs, oracle.dequant(*ref), gpu


@pytest.mark.parametrize("M", list(range(1, 17)))
def test_decode_every_m(awq, small, M):
    N, K, xs, Wdq, gpu = small
    check_linear(awq, xs[:M], Wdq, gpu, N)


@pytest.mark.parametrize("M", [24, 100])
def test_small_prefill_full_size_blocks_of_16(awq, M):
    """17..128 tokens run through the decode kernels in blocks of 16 (the last block moved back):
    full-size shapes (4096 x 4096 through the register-resident kernel, the two larger ones through
    the kernel that stages the activations in LDS, where the rows the last block shares with its
    neighbour are written by the neighbour alone), every row against the oracle, twice bit for bit
    alike."""
    for N, K in [(4096, 4096), (4096, 11008), (11008, 4096)]:
        case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.02, 1)
        g = np.random.default_rng(M)
        xs = (np.tile(xs16, ((M + 15) // 16, 1))[:M].astype(np.float32)
              * g.uniform(0.5, 1.5, size=(M, 1)).astype(np.float32)).astype(np.float16)
        check_linear(awq, xs, Wdq, gpu, N)
        a = host(awq.awq_w4a16_linear(dev(xs), *gpu, N)).copy()
        b = host(awq.awq_w4a16_linear(dev(xs), *gpu, N)).copy()
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


@pytest.mark.parametrize("M,ksplit", [(200, None), (512, 4), (2048, 1)])
def test_mid_prefill_split_k_full_size(awq, M, ksplit):
    """A few hundred tokens: with the workspace the prefill kernel cuts K into ranges (one
    workgroup per tile and range, fp32 partial tiles summed by a second kernel).  Full-size
    shapes, sampled rows against the oracle, the workspace between canaries, and the result
    next to that of the unsplit kernel."""
    import torch
    for N, K in [(4096, 4096), (4096, 11008)]:
        case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.02, 1)
        g = np.random.default_rng(M)
        xs = (np.tile(xs16, ((M + 15) // 16, 1))[:M].astype(np.float32)
              * g.uniform(0.5, 1.5, size=(M, 1)).astype(np.float32)).astype(np.float16)
        need = awq.awq_linear_workspace_bytes(M, N, K)
        ks = ksplit
        if ks is None:                                       # chosen by the library's estimate
            ks = need // (M * N * 4)
            assert 2 <= ks <= 8
        assert need == (ks * M * N * 4 if ks > 1 else 0)
        rows = np.sort(g.choice(M, size=40, replace=False))
        check_linear(awq, xs, Wdq, gpu, N, rows=rows)            # the binding brings the workspace
        ws, cw = guarded(max(need, 16), torch.uint8)
        y_split = host(awq.awq_w4a16_linear(dev(xs), *gpu, N, workspace=ws)).copy()
        cw()
        y_plain = host(awq.awq_w4a16_linear(dev(xs), *gpu, N, workspace=False)).copy()
        if need:
            with pytest.raises(awq.AwqError) as e:
                awq.awq_w4a16_linear(dev(xs), *gpu, N, workspace=ws[:need - 16])
            assert e.value.status == -5
        import oracle
        for y in (y_split, y_plain):
            err = oracle.norm_error(y[rows], oracle.matmul(xs[rows], Wdq), xs[rows], Wdq)
            assert err.max() <= TOL
        # the two differ by the order of the fp32 sums only: a rounding of the fp16 result at most
        d = np.abs(y_split.astype(np.float32) - y_plain.astype(np.float32))
        assert d.max() <= 2.0 ** -9 * max(1.0, float(np.abs(y_plain.astype(np.float32)).max()))
        if ks == 1:
            assert np.array_equal(y_split.view(np.uint16), y_plain.view(np.uint16))


@pytest.mark.parametrize("M", [17, 64, 127, 128, 129, 300])
def test_prefill_ragged_m(awq, small, M):
    N, K, xs, Wdq, gpu = small
    check_linear(awq, xs[:M], Wdq, gpu, N)


@pytest.mark.parametrize("N,K", [(16, 128), (16, 256), (32, 128), (128, 4096), (16, 28672)])
def test_degenerate_shapes(awq, N, K):
    case, s, xs = make_case(N, K, 40, 0.02, cfg=0, proj=1)
    ref, gpu = assert_quantize_bit_exact(awq, case.W, s)
    import oracle
    Wdq = oracle.dequant(*ref)
    for M in (1, 3, 16, 40):
        check_linear(awq, xs[:M], Wdq, gpu, N)


def test_linear_is_deterministic_and_exact_on_integer_data(awq):
    """Small integers: every product and partial sum is exact in fp32, so the GPU result
    must equal the oracle bit for bit, and twice in a row."""
    import oracle
    g = np.random.default_rng(11)
    N, K = 64, 512
    codes = g.integers(0, 16, size=(N, K), dtype=np.uint8)
    scales = (2.0 ** g.integers(-3, 2, size=(N, K // 128))).astype(np.float16)
    zeros = g.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
    q, sp, zp = oracle.pack(codes, scales, zeros)
    gpu = (dev(q), dev(sp.view(np.float16)), dev(zp))
    Wdq = oracle.dequant(codes, scales, zeros)
    for M in (1, 5, 16, 33):
        x = g.integers(-4, 5, size=(M, K)).astype(np.float16)
        y_ref = oracle.matmul(x, Wdq)
        assert np.abs(y_ref).max() < 60000          # finite in fp16; partial sums exact in fp32
        y1 = host(awq.awq_w4a16_linear(dev(x), *gpu, N))
        y2 = host(awq.awq_w4a16_linear(dev(x), *gpu, N))
        assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
        assert np.array_equal(y1.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))


# ------------------------------------------------------------------- grouped decode call

def check_multi(awq, problems, M):
    """problems: list of (xs[>=M,K], Wdq[N,K], gpu_packed, N).  One awq_w4a16_linear_multi
    call; every output is compared with the oracle, canaries around every output buffer."""
    import torch
    import oracle
    linears, checks, outs = [], [], []
    for xs, Wdq, gpu_packed, N in problems:
        y, cy = guarded(M * N * 2, torch.float16)
        y = y.view(M, N)
        linears.append((dev(xs[:M]), *gpu_packed, y, N))
        checks.append(cy)
        outs.append(y)
    awq.awq_w4a16_linear_multi(linears)
    worst = 0.0
    for (xs, Wdq, gpu_packed, N), y, cy in zip(problems, outs, checks):
        cy()
        yh = host(y)
        assert np.all(np.isfinite(yh.astype(np.float32)))
        err = oracle.norm_error(yh, oracle.matmul(xs[:M], Wdq), xs[:M], Wdq)
        assert err.max() <= TOL, f"max normalised error {err.max():.3e} (N={N}, M={M})"
        worst = max(worst, float(err.max()))
    return worst


@pytest.fixture(scope="module")
def small_group(awq):
    """Four small linears of different shapes: ragged group count (K=1408: 11 groups), a K that
    needs more than one wave along K at larger M, shared and separate inputs."""
    import oracle
    out = []
    for i, (N, K) in enumerate([(176, 1408), (64, 1408), (48, 2048), (320, 512)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=3 + i)
        ref, gpu = assert_quantize_bit_exact(awq, case.W, s)
        out.append((xs, oracle.dequant(*ref), gpu, N))
    return out


@pytest.mark.parametrize("M", list(range(1, 17)))
def test_multi_every_m(awq, small_group, M):
    check_multi(awq, small_group, M)


def test_multi_single_entry_and_limits(awq, small_group):
    import torch
    check_multi(awq, small_group[:1], 3)
    check_multi(awq, small_group * 14, 2)                    # 56 entries: the maximum
    check_multi(awq, small_group * 14, 9)                    # ... through the kernel for more than four tokens
    xs, Wdq, gpu, N = small_group[0]
    y = torch.empty((17, N), dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:                   # M > 16 is not a decode call
        awq.awq_w4a16_linear_multi([(dev(np.repeat(xs, 2, axis=0)[:17]), *gpu, y, N)])
    assert e.value.status == -2
    with pytest.raises(ValueError):
        awq.prepare_linear_multi(small_group * 15)


def test_multi_exact_and_deterministic_on_integer_data(awq):
    """Small integers: all products and sums are exact in fp32, so the grouped call must
    reproduce the oracle bit for bit, twice in a row."""
    import torch
    import oracle
    g = np.random.default_rng(12)
    probs = []
    for N, K in [(64, 512), (32, 1408), (96, 2048)]:
        codes = g.integers(0, 16, size=(N, K), dtype=np.uint8)
        scales = (2.0 ** g.integers(-3, 2, size=(N, K // 128))).astype(np.float16)
        zeros = g.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
        q, sp, zp = oracle.pack(codes, scales, zeros)
        probs.append((N, K, (dev(q), dev(sp.view(np.float16)), dev(zp)), oracle.dequant(codes, scales, zeros)))
    for M in (1, 2, 5, 16):
        linears, refs = [], []
        for N, K, gpu, Wdq in probs:
            x = g.integers(-4, 5, size=(M, K)).astype(np.float16)
            y_ref = oracle.matmul(x, Wdq)
            assert np.abs(y_ref).max() < 60000
            linears.append((dev(x), *gpu, torch.empty((M, N), dtype=torch.float16, device="cuda"), N))
            refs.append(y_ref)
        first = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
        second = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
        for y1, y2, y_ref in zip(first, second, refs):
            assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
            assert np.array_equal(y1.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))


def test_multi_llama7b_layer_full_size(awq):
    """The launch configuration bench.py times: the seven projections of one Llama-2-7B-shaped
    layer in one grouped call (M = 1, 4, 16), every output against the oracle."""
    probs = []
    for N, K in [(4096, 4096), (11008, 4096), (4096, 11008)]:
        case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.02, 1)
        probs.append((xs16, Wdq, gpu, N))
    layer = [probs[0]] * 4 + [probs[1]] * 2 + [probs[2]]
    for M in (1, 4, 16):
        check_multi(awq, layer, M)


def test_multi_llama70b_shapes_full_size(awq):
    """Llama-2-70B-shaped linears (config 3) through the grouped call at M = 1 and 8, two shapes at
    a time to bound host memory.  K = 28672 needs four waves along K at M = 1; at M = 8 the call
    runs the kernel that stages the activations through LDS (rows split over the two halves of a
    workgroup, up to eight row-block steps per workgroup): both paths are checked against the
    oracle."""
    pairs = [((8192, 8192), (1024, 8192)), ((28672, 8192), (1024, 8192)), ((8192, 28672), (1024, 8192))]
    for a, b in pairs:
        probs = []
        for N, K in (a, b):
            case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.015, 3)
            probs.append((xs16, Wdq, gpu, N))
        for M in (1, 8):
            check_multi(awq, probs + probs[1:], M)


def test_multi_paired_plan_ragged_shapes(awq):
    """Launches large enough for the plan that cuts every linear into workgroups of two sizes
    (row-block ranges of a linear as entries of their own), with row-block counts that are no
    multiple of the rows a workgroup takes per step, ragged group counts and K split over two
    or four waves: every output against the oracle, and bit-identical on a second call."""
    import oracle
    g = np.random.default_rng(31)
    sets = [
        [(4112, 4096), (2064, 4096), (8208, 2048), (1040, 8192), (4112, 1408), (6160, 4096), (6160, 4096),
         (6160, 4096), (3088, 11008)],
        [(11024, 4096), (11024, 4096), (4112, 11008), (4112, 4096), (272, 28672), (16, 4096)],
    ]
    expected_plan = [{1: 2, 2: 2}, {1: 2, 2: 1}]        # K = 28672 at M = 2 needs eight-wave workgroups
    for shapes, expected in zip(sets, expected_plan):
        probs = []
        for N, K in shapes:
            codes = g.integers(0, 16, size=(N, K), dtype=np.uint8)
            scales = g.uniform(0.002, 0.02, size=(N, K // 128)).astype(np.float16)
            zeros = g.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
            q, sp, zp = oracle.pack(codes, scales, zeros)
            xs = g.standard_normal((2, K)).astype(np.float16)
            probs.append((xs, oracle.dequant(codes, scales, zeros), (dev(q), dev(sp.view(np.float16)), dev(zp)), N))
            del codes
        for M in (1, 2):
            check_multi(awq, probs, M)
            assert awq.awq_last_grouped_plan() == expected[M]
        check_multi(awq, probs[:2], 1)
        assert awq.awq_last_grouped_plan() == 1                  # a small launch keeps the plain plan
        import torch
        linears = [(dev(xs[:1]), *gpu, torch.empty((1, N), dtype=torch.float16, device="cuda"), N)
                   for xs, Wdq, gpu, N in probs]
        first = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
        second = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
        for a, b in zip(first, second):
            assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
        del probs


# ------------------------------------------------------------------- the full stack (config 4)

def test_config4_full_stack_calibration_128x512_rows_on_layer0_one_sequence_on_the_others(awq):
    """The 32-layer Llama-2-7B-shaped stack: one awq_quantize_pack pass over all 224 matrices
    (every packed byte, step and zero point against the oracle), then 128 decode steps at M = 1
    over the 224 linears, issued as grouped launches (even steps: 32 launches of one layer's 7
    projections; odd steps: 4 launches of 8 layers = 56 linears).  Step 0 and three further
    seeded steps are compared with the oracle, every output element.

    s of layer 0's four distinct inputs comes from the full calibration set (128 sequences of
    512 rows), which also checks awq_act_scale at T = 65 536; the other layers use one sequence
    (512 rows) to bound the host time spent drawing random numbers."""
    import os
    import torch
    import oracle
    import workloads
    from concurrent.futures import ThreadPoolExecutor

    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    shapes = workloads.LLAMA2_7B_LAYER
    L, STEPS = workloads.STACK_LAYERS, workloads.STACK_STEPS
    widths = (4096, 11008)
    check_steps = [0] + sorted(int(v) for v in
                               np.random.default_rng(4).choice(np.arange(1, STEPS), size=3, replace=False))
    if all(st % 2 == 0 for st in check_steps[1:]):
        check_steps[-1] |= 1                                   # both launch groupings get checked

    # ---- s per (layer, distinct input); layer 0 from the full calibration set, also on the GPU
    s_of = {}
    for l in range(L):
        for inp in range(4):
            K = 11008 if inp == 3 else 4096
            out = workloads.outlier_channels(K, 4, l, inp)
            n_seq = workloads.CALIB_SEQUENCES if l == 0 else 1
            X = workloads.calibration_sequences(n_seq, K, 4, l, inp, out, threads=threads)
            s64 = oracle.act_scale(X, 0.5)
            s_of[(l, inp)] = s64.astype(np.float32)
            if l == 0:
                T = X.shape[0]
                s_gpu = host(awq.awq_act_scale(dev(X), 0.5)).astype(np.float64)
                # fp32 running sums of T/128 non-negative terms per partial, then a 7-level tree:
                # relative error of the mean <= (T/128 + 7) * 2^-24; the square root halves it
                assert np.abs(s_gpu / s64 - 1.0).max() <= 0.5 * (T / 128 + 7) * 2.0 ** -24 + 1e-7
            del X

    # ---- x' per step and width: fresh seeded rows, divided by layer 0's s of that width
    xs_all = {}
    for ki, K in enumerate(widths):
        out = workloads.outlier_channels(K, 4, 0, 0 if K == 4096 else 3)
        rows = np.concatenate([workloads.activations(1, K, 4, STEPS + st, ki, workloads.ROLE_X, out)
                               for st in range(STEPS)])
        xs_all[K] = oracle.apply_inv_scale(rows, s_of[(0, 0 if K == 4096 else 3)])
    x_chk = {K: np.ascontiguousarray(xs_all[K][check_steps]) for K in widths}

    # ---- quantize pass: layer by layer, bit-exact against the oracle; keep the packed arrays on
    # the GPU, and of the oracle only y_ref of the checked steps and max|Wdq| per matrix
    packed, y_ref, wmax, canaries = [], [], [], []
    for l in range(L):
        with ThreadPoolExecutor(min(threads, 7)) as ex:
            Ws = list(ex.map(lambda p: workloads.weights(shapes[p][1], shapes[p][2], workloads.SIGMA_7B,
                                                         4, l, p), range(7)))
        lp, ly, lw = [], [], []
        for p, (name, N, K) in enumerate(shapes):
            s = s_of[(l, workloads.LAYER_INPUT_OF_PROJ[p])]
            qb, sb, zb = awq.awq_packed_sizes(N, K)
            q_gpu, cq = guarded(qb, torch.uint8)
            s_gpu, cs = guarded(sb, torch.float16)
            z_gpu, cz = guarded(zb, torch.uint8)
            awq.awq_quantize_pack(dev(Ws[p]), dev(s), out=(q_gpu, s_gpu, z_gpu))
            codes, scales, zeros = oracle.quantize(Ws[p], s)
            q_ref, s_ref, z_ref = oracle.pack(codes, scales, zeros)
            cq(); cs(); cz()
            canaries += [cq, cs, cz]
            assert np.array_equal(host(s_gpu).view(np.uint16), s_ref), f"steps differ (layer {l}, {name})"
            assert np.array_equal(host(z_gpu), z_ref), f"zero points differ (layer {l}, {name})"
            assert np.array_equal(host(q_gpu), q_ref), f"packed codes differ (layer {l}, {name})"
            Wdq = oracle.dequant(codes, scales, zeros)
            ly.append(oracle.matmul(x_chk[K], Wdq))
            lw.append(float(np.abs(Wdq).max()))
            lp.append((q_gpu, s_gpu, z_gpu))
            del Wdq, codes
        packed.append(lp); y_ref.append(ly); wmax.append(lw)
        del Ws

    # ---- decode: 128 steps over the 224 linears
    x_dev = {K: dev(xs_all[K]) for K in widths}
    x_cur = {K: torch.empty((1, K), dtype=torch.float16, device="cuda") for K in widths}
    ys = [[torch.empty((1, N), dtype=torch.float16, device="cuda") for _, N, K in shapes] for l in range(L)]

    def entries(l):
        return [(x_cur[K], *packed[l][p], ys[l][p], N) for p, (_, N, K) in enumerate(shapes)]

    per_layer = [awq.prepare_linear_multi(entries(l)) for l in range(L)]
    per_eight = [awq.prepare_linear_multi(sum((entries(l) for l in range(l0, l0 + 8)), []))
                 for l0 in range(0, L, 8)]
    worst = 0.0
    for st in range(STEPS):
        for K in widths:
            x_cur[K].copy_(x_dev[K][st:st + 1])
        for call in (per_layer if st % 2 == 0 else per_eight):
            call()
        if st in check_steps:
            j = check_steps.index(st)
            for l in range(L):
                for p, (name, N, K) in enumerate(shapes):
                    y = host(ys[l][p]).astype(np.float64)[0]
                    assert np.all(np.isfinite(y))
                    xn = np.linalg.norm(x_chk[K][j].astype(np.float64))
                    err = np.abs(y - y_ref[l][p][j]) / (xn * wmax[l][p] + 1e-6)
                    assert err.max() <= TOL, f"step {st}, layer {l}, {name}: error {err.max():.3e}"
                    worst = max(worst, float(err.max()))
            for l in range(L):                                  # stale outputs cannot pass later
                for y in ys[l]:
                    y.zero_()
    for check in canaries:                                      # the decode steps wrote nothing there
        check()
    print(f"config 4: worst normalised error over steps {check_steps}: {worst:.3e}")


def test_multi_more_than_four_tokens_ragged_shapes(awq):
    """5..16 tokens: the grouped call stages the activations through LDS.  Row-block counts that
    are no multiple of the three or six a workgroup takes per step (down to a single block),
    ragged group counts, K from one chunk of 512 columns to 56 chunks (whole rows and rows split
    over the two halves of a workgroup), a lone wide linear: every output against the oracle,
    canaries around the outputs, and bit-identical on a second call."""
    import torch
    import oracle
    g = np.random.default_rng(47)
    shapes = [(4112, 4096), (2064, 4096), (1040, 8192), (4112, 1408), (3088, 11008), (272, 28672), (16, 4096),
              (32, 512), (80, 384)]
    probs = []
    for N, K in shapes + [(16400, 640)]:
        codes = g.integers(0, 16, size=(N, K), dtype=np.uint8)
        scales = g.uniform(0.002, 0.02, size=(N, K // 128)).astype(np.float16)
        zeros = g.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
        q, sp, zp = oracle.pack(codes, scales, zeros)
        xs = g.standard_normal((16, K)).astype(np.float16)
        probs.append((xs, oracle.dequant(codes, scales, zeros), (dev(q), dev(sp.view(np.float16)), dev(zp)), N))
        del codes
    wide = probs.pop()
    for M in (5, 8, 9, 16):
        check_multi(awq, probs, M)
        check_multi(awq, [wide], M)
    check_multi(awq, probs[-3:], 13)                              # a launch of a few workgroups
    linears = [(dev(xs[:11]), *gpu, torch.empty((11, N), dtype=torch.float16, device="cuda"), N)
               for xs, Wdq, gpu, N in probs]
    first = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
    second = [host(y).copy() for y in awq.awq_w4a16_linear_multi(linears)]
    for a, b in zip(first, second):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


@pytest.mark.parametrize("overrides", [
    {"AWQ_GEMV_STAGES": "3"}, {"AWQ_GEMV_STAGES": "4"}, {"AWQ_GEMV_SLOTS": "200"},
    {"AWQ_GEMV_SLOTS": "20000"}, {"AWQ_GEMV_KSL": "2"}, {"AWQ_GEMV_KSL": "3", "AWQ_GEMV_LOGW": "3"},
    {"AWQ_GEMV_ITERS": "1"}, {"AWQ_GEMV_JOBS": "3", "AWQ_GEMV_STAGES": "3"},
    {"AWQ_GEMV_WAVES": "2", "AWQ_GEMV_UNROLL": "1"}, {"AWQ_GEMV_WAVES": "16", "AWQ_GEMV_UNROLL": "2"},
    {"AWQ_GEMV_STREAM_SINGLE": "1"},
])
def test_grouped_decode_under_planner_overrides(awq, overrides):
    """In the tuning build of the library (libawq_mi355x_knobs.so, -DAWQ_TUNING_KNOBS) the planner's
    constants can be overridden through the environment (read once per process); every such plan
    must give the same results.  Runs the check in a child process that loads that build."""
    import os
    import subprocess
    import sys
    from paper_2306_00978_amd import build as hip_build
    assert os.path.exists(hip_build.LIB_KNOBS), "build the tuning library first (paper_2306_00978_amd.build)"
    env = dict(os.environ)
    env.update(overrides)
    env["AWQ_MI355X_LIBRARY"] = hip_build.LIB_KNOBS
    child = os.path.join(os.path.dirname(os.path.abspath(__file__)), "child_grouped_decode.py")
    res = subprocess.run([sys.executable, child], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and res.stdout.strip().endswith("OK"), res.stdout[-2000:] + res.stderr[-2000:]


# ----------------------------------------------------------------------------- a0 / a0'

@pytest.mark.parametrize("T,K", [(64, 4096), (5, 136), (1000, 11008)])
def test_act_scale_and_inverse_scale(awq, T, K):
    import oracle
    import workloads
    out = workloads.outlier_channels(K, 0, 0, 2)
    X = workloads.activations(T, K, 0, 0, 2, workloads.ROLE_CALIB, out)
    for alpha in (0.5, 0.0, 1.0):
        s_ref = oracle.act_scale(X, alpha)
        s_gpu = host(awq.awq_act_scale(dev(X), alpha)).astype(np.float64)
        assert np.abs(s_gpu / s_ref - 1.0).max() <= 2e-6
    s = oracle.act_scale(X, 0.5).astype(np.float32)
    x = X[: min(T, 16)]
    xs_ref = oracle.apply_inv_scale(x, s)
    xs_gpu = host(awq.awq_apply_inv_scale(dev(x), dev(s)))
    assert np.array_equal(xs_gpu.view(np.uint16), xs_ref.view(np.uint16))


def test_act_scale_multi_equals_the_single_calls_and_the_oracle(awq):
    """awq_act_scale_multi: matrices of different T and K in one call (more than one launch's
    worth: 19 = 16 + 3), every result bit for bit that of awq_act_scale on the same matrix and
    within the tolerance of the oracle; nothing written around the outputs."""
    import torch
    import oracle
    g = np.random.default_rng(99)
    shapes = [(64, 4096), (5, 136), (300, 11008), (1, 8), (2048, 512), (17, 1408), (129, 64)] * 3
    shapes = shapes[:19]
    Xs, outs, guards = [], [], []
    for T, K in shapes:
        Xs.append((g.standard_normal((T, K)) * g.uniform(0.01, 30.0)).astype(np.float16))
        whole = torch.full((K + 128,), -3.0, dtype=torch.float32, device="cuda")
        guards.append(whole)
        outs.append(whole[64:64 + K])
    dX = [dev(X) for X in Xs]
    for alpha in (0.5, 0.0, 0.35):
        awq.prepare_act_scale_multi(list(zip(dX, outs)), alpha)()
        torch.cuda.synchronize()
        for X, dx, s_multi, whole in zip(Xs, dX, outs, guards):
            s_one = awq.awq_act_scale(dx, alpha)
            assert torch.equal(s_one.view(torch.int32), s_multi.view(torch.int32))
            s_ref = oracle.act_scale(X, alpha)
            assert np.abs(host(s_multi).astype(np.float64) / s_ref - 1.0).max() <= 2e-6
            assert bool((whole[:64] == -3.0).all()) and bool((whole[64 + X.shape[1]:] == -3.0).all())


# ------------------------------------------------------------------- weight clipping

CLIP_RATIOS = [1.0 - 0.05 * i for i in range(11)]


def assert_clip_bit_exact(awq, W, s, ratios=CLIP_RATIOS):
    import torch
    import oracle
    N, K = W.shape
    codes, scales, zeros, choice = oracle.quantize_clip(W, s, ratios)
    q_ref, s_ref, z_ref = oracle.pack(codes, scales, zeros)
    qb, sb, zb = awq.awq_packed_sizes(N, K)
    q_gpu, cq = guarded(qb, torch.uint8)
    s_gpu, cs = guarded(sb, torch.float16)
    z_gpu, cz = guarded(zb, torch.uint8)
    _, _, _, ch_gpu = awq.awq_quantize_pack_clip(dev(W), None if s is None else dev(s), ratios,
                                                 out=(q_gpu, s_gpu, z_gpu), want_choice=True)
    cq(); cs(); cz()
    ch = host(ch_gpu)
    assert np.array_equal(ch, choice), f"{(ch != choice).sum()} of {choice.size} groups chose another ratio"
    assert np.array_equal(host(s_gpu).view(np.uint16), s_ref), "steps differ"
    assert np.array_equal(host(z_gpu), z_ref), "zero points differ"
    assert np.array_equal(host(q_gpu), q_ref), "packed codes differ"
    # without the optional output
    q2, s2, z2 = awq.awq_quantize_pack_clip(dev(W), None if s is None else dev(s), ratios)
    assert np.array_equal(host(q2), q_ref) and np.array_equal(host(z2), z_ref)
    return choice


@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (80, 1408), (272, 256)])
def test_quantize_pack_clip_small_shapes(awq, N, K):
    case, s, xs = make_case(N, K, 1, 0.02, cfg=0, proj=7)
    choice = assert_clip_bit_exact(awq, case.W, s)
    assert choice.max() > 0                                # the search does something
    assert_clip_bit_exact(awq, case.W, None, ratios=[0.8, 1.0, 0.8, 0.9])
    # a grid of one ratio 1.0 is awq_quantize_pack
    q1, s1, z1 = awq.awq_quantize_pack_clip(dev(case.W), dev(s), [1.0])
    q0, s0, z0 = awq.awq_quantize_pack(dev(case.W), dev(s))
    assert np.array_equal(host(q1), host(q0)) and np.array_equal(host(z1), host(z0))
    assert np.array_equal(host(s1).view(np.uint16), host(s0).view(np.uint16))


def test_quantize_pack_clip_edge_groups_and_full_size(awq):
    g = np.random.default_rng(31)
    N, K = 64, 512
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0, :128] = 0                          # constant group
    W[1, :128] = np.float16(0.37)
    W[2, 128:256] = np.abs(W[2, 128:256])   # one-sided groups
    W[3, 128:256] = -np.abs(W[3, 128:256])
    W[4, 256:384] *= 1000                   # large magnitudes
    W[5, 300] = np.float16(3.0)             # a lone outlier: clipping it costs more than it gains
    assert_clip_bit_exact(awq, W, None)
    s = (10.0 ** g.uniform(-2, 2, size=K)).astype(np.float32)
    assert_clip_bit_exact(awq, W, s, ratios=[0.5, 0.75, 1.0])
    case, s, xs = make_case(4096, 4096, 1, 0.02, cfg=0)
    assert_clip_bit_exact(awq, case.W, s)


def check_clip_on_activations(awq, W, s, xs, ratios=CLIP_RATIOS):
    """Error of a trial = the group's contribution to the layer output on the rows xs.  The
    kernel forms it on the matrix cores from errors rounded to fp16, so near-equal trials may be
    ordered differently than in the fp64 oracle: the choice of every group must be the oracle's
    or a trial whose oracle error is within 5e-3 of the smallest (rounding of 2^-11 per error,
    twice through the square, with margin), and the packed result must be exactly the
    quantization by the chosen ratio."""
    import torch
    import oracle
    N, K = W.shape
    G = K // 128
    T = xs.shape[0]
    q_gpu, s_gpu, z_gpu, ch_gpu = awq.awq_quantize_pack_clip(dev(W), None if s is None else dev(s), ratios,
                                                             want_choice=True, xs=dev(xs))
    ch = host(ch_gpu)
    _, _, _, ch_ref = oracle.quantize_clip(W, s, ratios, xs=xs)
    # the oracle's errors of all trials, from one full quantization per ratio
    wp = (W.astype(np.float32) * (np.ones(K, np.float32) if s is None else s)[None, :]).astype(np.float64)
    xg = xs.astype(np.float64).reshape(T, G, 128)
    per_ratio, errs = [], []
    for r in ratios:
        c, sc, z, _ = oracle.quantize_clip(W, s, [r])
        per_ratio.append((c, sc, z))
        d = (oracle.dequant(c, sc, z).astype(np.float64) - wp).reshape(N, G, 128)
        errs.append((np.einsum("ngk,tgk->ngt", d, xg) ** 2).sum(axis=2))
    errs = np.stack(errs)
    e_min = errs.min(axis=0)
    e_got = np.take_along_axis(errs, ch[None].astype(np.int64), 0)[0]
    assert np.all(e_got <= e_min * (1 + 5e-3) + 1e-30), "a group chose a clearly worse ratio"
    agree = float((ch == ch_ref).mean())
    assert agree > 0.97, agree
    # assemble the oracle's quantization for the GPU's choices and compare bit for bit
    codes = np.empty((N, K), np.uint8)
    scales = np.empty((N, G), np.float16)
    zeros = np.empty((N, G), np.uint8)
    for i, (c, sc, z) in enumerate(per_ratio):
        m = ch == i
        scales[m], zeros[m] = sc[m], z[m]
        mk = np.repeat(m, 128, axis=1)
        codes[mk] = c[mk]
    q_ref, s_ref, z_ref = oracle.pack(codes, scales, zeros)
    assert np.array_equal(host(s_gpu).view(np.uint16), s_ref)
    assert np.array_equal(host(z_gpu), z_ref)
    assert np.array_equal(host(q_gpu), q_ref)
    return agree


@pytest.mark.parametrize("N,K,T", [(48, 640, 64), (80, 1408, 5), (272, 256, 33), (1024, 4096, 64)])
def test_quantize_pack_clip_on_activation_rows(awq, N, K, T):
    import oracle
    import workloads
    case = workloads.linear_case("clipx", N, K, 1, 0.02, 0, proj=11, calib_tokens=T)
    s = oracle.act_scale(case.calib, 0.35).astype(np.float32)
    xs = oracle.apply_inv_scale(case.calib, s)
    agree = check_clip_on_activations(awq, case.W, s, xs)
    print(f"clip on {T} rows, {N}x{K}: {100 * agree:.2f} % of the groups choose as the fp64 oracle")
    check_clip_on_activations(awq, case.W, None, case.calib, ratios=[0.7, 1.0, 0.85])


def test_quantize_pack_clip_rejects_bad_ratios(awq):
    import torch
    W = torch.zeros((16, 128), dtype=torch.float16, device="cuda")
    for ratios in ([], [1.0] * 33, [0.0], [1.5], [float("nan")], [-0.5]):
        with pytest.raises(awq.AwqError) as e:
            awq.awq_quantize_pack_clip(W, None, ratios)
        assert e.value.status == -7


# ------------------------------------------------------------------- scale search (Eq. 4-5)

def loss_rtol(count):
    """Tolerance of a loss that sums `count` squared output differences d.  The GPU's d carries
    the fp16 rounding of both outputs and of the dequantized weights: uncorrelated noise e with
    rms(e) / rms(d) = r ~ 1e-2 (2^-11 of the outputs against a quantization error of about a
    tenth of a step per weight).  sum (d + e)^2 - sum d^2 = sum e^2 + 2 sum d e: the first term
    is r^2 ~ 1e-4 of the loss, the second has standard deviation 2 r / sqrt(count) of it;
    three standard deviations: 0.06 / sqrt(count)."""
    return 2e-4 + 0.06 / np.sqrt(count)


ALPHAS = [i / 20 for i in range(20)]


def check_search(awq, W, X, alphas=ALPHAS):
    import oracle
    N, K = W.shape
    best_g, losses_g, s_g = awq.awq_search_scale(dev(W), dev(X), alphas)
    best_g, losses_g, s_g = int(host(best_g)[0]), host(losses_g), host(s_g)
    best_o, losses_o, s_o = oracle.search_scale(W, X, alphas)
    assert losses_g.shape == losses_o.shape
    assert np.all(np.isfinite(losses_g))
    LOSS_RTOL = loss_rtol(N * X.shape[0])
    assert np.abs(losses_g / losses_o - 1.0).max() <= LOSS_RTOL, (losses_g / losses_o)
    # the decision is taken on the GPU's own sums: it is the first minimum of those, and by the
    # oracle's sums it is the minimum or within the tolerance of it
    assert best_g == int(np.argmin(losses_g))
    assert losses_o[best_g] <= losses_o[best_o] * (1.0 + 2 * LOSS_RTOL)
    if len(alphas) > 1 and np.sort(losses_o)[1] > losses_o[best_o] * (1.0 + 2 * LOSS_RTOL):
        assert best_g == best_o
    print(f"search N={N} K={K} T={X.shape[0]}: alpha*={alphas[best_g]}, "
          f"max |loss_gpu/loss_oracle - 1| = {np.abs(losses_g / losses_o - 1.0).max():.2e}")
    # s* is what awq_act_scale gives for alpha*, and what the oracle gives
    s_again = host(awq.awq_act_scale(dev(X), alphas[best_g]))
    assert np.array_equal(s_g.view(np.uint32), s_again.view(np.uint32))
    s_ref = oracle.act_scale(X, alphas[best_g])
    assert np.abs(s_g.astype(np.float64) / s_ref - 1.0).max() <= 2e-6
    # and quantizing with it is bit-exact against the oracle given the same s
    assert_quantize_bit_exact(awq, W, s_g)
    return best_g, losses_g


@pytest.mark.parametrize("N,K,T", [(176, 1408, 300), (48, 256, 5), (272, 512, 129)])
def test_search_scale_small(awq, N, K, T):
    """Ragged token counts and row-block counts; T = 5 evaluates through the decode kernel."""
    import workloads
    out = workloads.outlier_channels(K, 0, 0, 5)
    W = workloads.weights(N, K, 0.02, 0, 0, 5)
    X = workloads.activations(T, K, 0, 0, 5, workloads.ROLE_CALIB, out)
    best, losses = check_search(awq, W, X)
    assert best > 0                                   # outlier channels: scaling beats plain RTN
    check_search(awq, W, X, alphas=[0.5])             # a grid of one
    check_search(awq, W, X, alphas=[1.0, 0.0, 0.5, 0.5])   # unordered, with a tie: first wins


def test_search_scale_config0_full_size(awq):
    """The 4096 x 4096 linear of config 0 with its 64 calibration rows, grid of 20."""
    import workloads
    case = workloads.linear_case("cfg0", 4096, 4096, 1, workloads.SIGMA_7B, 0)
    check_search(awq, case.W, case.calib)


def test_search_scale_rejects_bad_arguments(awq):
    import torch
    W = torch.zeros((16, 128), dtype=torch.float16, device="cuda")
    X = torch.zeros((4, 128), dtype=torch.float16, device="cuda")
    for alphas, status in (([], -7), ([0.5] * 65, -7), ([1.5], -7), ([float("nan")], -7)):
        with pytest.raises(awq.AwqError) as e:
            awq.awq_search_scale(W, X, alphas)
        assert e.value.status == status
    with pytest.raises(awq.AwqError) as e:
        awq.awq_search_scale(W, X, [0.5], workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -5
    assert awq.load().awq_search_scale_workspace_bytes(4, 16, 100, 1, 128) == 0


# ------------------------------------------------------------------- INT3-g128 variant

def quantize_w3_bit_exact(awq, W, s):
    import torch
    import oracle
    N, K = W.shape
    codes, scales, zeros = oracle.quantize_w3(W, s)
    q_ref, s_ref, z_ref = oracle.pack_w3(codes, scales, zeros)
    qb, sb, zb = awq.awq_packed_sizes_w3(N, K)
    assert (qb, sb, zb) == oracle.packed_sizes_w3(N, K)
    q_gpu, cq = guarded(qb, torch.uint8)
    s_gpu, cs = guarded(sb, torch.float16)
    z_gpu, cz = guarded(zb, torch.uint8)
    awq.awq_quantize_pack_w3(dev(W), None if s is None else dev(s), out=(q_gpu, s_gpu, z_gpu))
    cq(); cs(); cz()
    assert np.array_equal(host(s_gpu).view(np.uint16), s_ref), "steps differ"
    assert np.array_equal(host(z_gpu), z_ref), "zero points differ"
    assert np.array_equal(host(q_gpu), q_ref), "packed codes differ"
    c_u, s_u, z_u = awq.awq_unpack_w3(q_gpu, s_gpu, z_gpu, N, K)
    assert np.array_equal(host(c_u), codes)
    assert np.array_equal(host(s_u).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(host(z_u), zeros)
    return (codes, scales, zeros), (q_gpu, s_gpu, z_gpu)


def check_linear_w3(awq, xs, Wdq, gpu_packed, N):
    import torch
    import oracle
    M, K = xs.shape
    y_gpu, cy = guarded(M * N * 2, torch.float16)
    y_gpu = y_gpu.view(M, N)
    awq.awq_w3a16_linear(dev(xs), *gpu_packed, N, out=y_gpu)
    cy()
    yh = host(y_gpu)
    assert np.all(np.isfinite(yh.astype(np.float32)))
    err = oracle.norm_error(yh, oracle.matmul(xs, Wdq), xs, Wdq)
    assert err.max() <= TOL, f"max normalised error {err.max():.3e}"


@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (176, 1408), (272, 256)])
def test_w3_small_shapes_every_m(awq, N, K):
    import oracle
    case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=13)
    ref, gpu = quantize_w3_bit_exact(awq, case.W, s)
    quantize_w3_bit_exact(awq, case.W, None)
    Wdq = oracle.dequant(*ref)
    for M in range(1, 17):
        check_linear_w3(awq, xs[:M], Wdq, gpu, N)


def test_w3_edge_groups_and_exactness_on_integer_data(awq):
    import oracle
    g = np.random.default_rng(71)
    N, K = 64, 512
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0, :128] = 0
    W[1, :128] = np.float16(0.37)
    W[2, 128:256] = np.abs(W[2, 128:256])
    W[3, 128:256] = -np.abs(W[3, 128:256])
    W[4, 256:384] *= 1000
    quantize_w3_bit_exact(awq, W, None)
    quantize_w3_bit_exact(awq, W, (10.0 ** g.uniform(-3, 3, size=K)).astype(np.float32))
    # small integers: every product and sum is exact, the kernel must reproduce the oracle
    codes = g.integers(0, 8, size=(N, K), dtype=np.uint8)
    scales = (2.0 ** g.integers(-3, 2, size=(N, K // 128))).astype(np.float16)
    zeros = g.integers(0, 8, size=(N, K // 128), dtype=np.uint8)
    q, sp, zp = oracle.pack_w3(codes, scales, zeros)
    gpu = (dev(q), dev(sp.view(np.float16)), dev(zp))
    Wdq = oracle.dequant(codes, scales, zeros)
    for M in (1, 5, 16):
        x = g.integers(-4, 5, size=(M, K)).astype(np.float16)
        y_ref = oracle.matmul(x, Wdq)
        y1 = host(awq.awq_w3a16_linear(dev(x), *gpu, N))
        y2 = host(awq.awq_w3a16_linear(dev(x), *gpu, N))
        assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
        assert np.array_equal(y1.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))


@pytest.mark.parametrize("N,K", [(48, 640), (176, 1408), (272, 256)])
def test_w3_repack_and_prefill(awq, N, K):
    """The 3-bit codes re-packed into the 4-bit layout unpack to the same codes, and the prefill
    call (re-pack + the 4-bit matrix-matrix kernel) matches the oracle at ragged M."""
    import torch
    import oracle
    case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=2)
    (codes, scales, zeros), gpu = quantize_w3_bit_exact(awq, case.W, s)
    q4 = awq.awq_repack_w3_to_w4(gpu[0], N, K)
    c4, s4, z4 = awq.awq_unpack(q4, gpu[1], gpu[2], N, K)
    assert np.array_equal(host(c4), codes)
    assert np.array_equal(host(s4).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(host(z4), zeros)
    Wdq = oracle.dequant(codes, scales, zeros)
    g = np.random.default_rng(77)
    for M in (17, 64, 129, 300):
        x = np.tile(xs, ((M + 15) // 16, 1))[:M] * g.uniform(0.5, 1.5, size=(M, 1)).astype(np.float16)
        x = x.astype(np.float16)
        y, cy = guarded(M * N * 2, torch.float16)
        awq.awq_w3a16_linear(dev(x), *gpu, N, out=y.view(M, N))
        cy()
        yh = host(y.view(M, N))
        err = oracle.norm_error(yh, oracle.matmul(x, Wdq), x, Wdq)
        assert err.max() <= TOL, f"max normalised error {err.max():.3e} (M={M})"
        if M > 128:
            # the binding's workspace has room for the K ranges where the shape uses them; with
            # the re-packed codes alone the unsplit kernel runs: same result up to the order of sums
            small_ws, cws = guarded(N * K // 2, torch.uint8)
            y2 = host(awq.awq_w3a16_linear(dev(x), *gpu, N, workspace=small_ws)).copy()
            cws()
            err2 = oracle.norm_error(y2, oracle.matmul(x, Wdq), x, Wdq)
            assert err2.max() <= TOL
            full = (N * K // 2 + 255) // 256 * 256 + awq.awq_linear_workspace_bytes(M, N, K)
            big_ws, cwb = guarded(full, torch.uint8)
            y3 = host(awq.awq_w3a16_linear(dev(x), *gpu, N, workspace=big_ws)).copy()
            cwb()
            assert np.array_equal(y3.view(np.uint16), yh.view(np.uint16))
    with pytest.raises(awq.AwqError) as e:          # too small a workspace is refused
        awq.awq_w3a16_linear(dev(np.tile(xs, (2, 1))), *gpu, N, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -5


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 11008)])
def test_w3_llama7b_shapes_full_size(awq, N, K):
    import oracle
    import torch
    case, s, xs = make_case(N, K, 16, 0.02, cfg=1, proj=14)
    ref, gpu = quantize_w3_bit_exact(awq, case.W, s)
    Wdq = oracle.dequant(*ref)
    for M in (1, 4, 16):
        check_linear_w3(awq, xs[:M], Wdq, gpu, N)
    check_linear_w3(awq, np.tile(xs, (3, 1))[:40], Wdq, gpu, N)      # M = 40: re-pack + the 4-bit GEMM


def check_multi_w3(awq, problems, M):
    import torch
    import oracle
    linears, checks, outs = [], [], []
    for xs, Wdq, gpu_packed, N in problems:
        y, cy = guarded(M * N * 2, torch.float16)
        y = y.view(M, N)
        linears.append((dev(xs[:M]), *gpu_packed, y, N))
        checks.append(cy)
        outs.append(y)
    awq.awq_w3a16_linear_multi(linears)
    for (xs, Wdq, gpu_packed, N), y, cy in zip(problems, outs, checks):
        cy()
        yh = host(y)
        assert np.all(np.isfinite(yh.astype(np.float32)))
        err = oracle.norm_error(yh, oracle.matmul(xs[:M], Wdq), xs[:M], Wdq)
        assert err.max() <= TOL, f"max normalised error {err.max():.3e} (N={N}, M={M})"


def test_w3_grouped_small_every_m_and_integer_exactness(awq):
    """Ragged group counts (11 groups: the last batch of a row block has three tiles), K split
    over several waves at larger M, a linear that does not fit and falls back."""
    import torch
    import oracle
    probs = []
    for i, (N, K) in enumerate([(176, 1408), (64, 1408), (48, 2048), (320, 512), (32, 128)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=15 + i)
        ref, gpu = quantize_w3_bit_exact(awq, case.W, s)
        probs.append((xs, oracle.dequant(*ref), gpu, N))
    for M in range(1, 17):
        check_multi_w3(awq, probs, M)
    check_multi_w3(awq, probs[:1], 3)
    check_multi_w3(awq, (probs[:4] * 14), 2)                  # 56 entries
    g = np.random.default_rng(72)
    ints = []
    for N, K in [(64, 512), (32, 1408), (96, 2048)]:
        codes = g.integers(0, 8, size=(N, K), dtype=np.uint8)
        scales = (2.0 ** g.integers(-3, 2, size=(N, K // 128))).astype(np.float16)
        zeros = g.integers(0, 8, size=(N, K // 128), dtype=np.uint8)
        q, sp, zp = oracle.pack_w3(codes, scales, zeros)
        ints.append((N, K, (dev(q), dev(sp.view(np.float16)), dev(zp)), oracle.dequant(codes, scales, zeros)))
    for M in (1, 2, 5, 16):
        linears, refs = [], []
        for N, K, gpu, Wdq in ints:
            x = g.integers(-4, 5, size=(M, K)).astype(np.float16)
            linears.append((dev(x), *gpu, torch.empty((M, N), dtype=torch.float16, device="cuda"), N))
            refs.append(oracle.matmul(x, Wdq))
        first = [host(y).copy() for y in awq.awq_w3a16_linear_multi(linears)]
        second = [host(y).copy() for y in awq.awq_w3a16_linear_multi(linears)]
        for y1, y2, y_ref in zip(first, second, refs):
            assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
            assert np.array_equal(y1.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))


def test_w3_grouped_llama7b_layer_full_size(awq):
    import oracle
    probs = []
    for i, (N, K) in enumerate([(4096, 4096), (11008, 4096), (4096, 11008)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=1, proj=20 + i)
        ref, gpu = quantize_w3_bit_exact(awq, case.W, s)
        probs.append((xs, oracle.dequant(*ref), gpu, N))
    layer = [probs[0]] * 4 + [probs[1]] * 2 + [probs[2]]
    for M in (1, 4, 16):
        check_multi_w3(awq, layer, M)


# ------------------------------------------------------------------- the pieces together

def test_awq_for_one_linear_end_to_end(awq):
    """Search the scale, quantize, run the layer: every stage against the oracle on the same
    inputs, and the result is closer to the fp16 layer than plain round-to-nearest.  Both
    clipping searches are checked on top: the one on the weights' own error lowers the output
    error of plain RTN but not that of the scaled layer (the scaled-up salient weights sit at
    the ends of the range); the one that measures the error on the calibration rows lowers it
    further."""
    import oracle
    import workloads
    N, K, T, M = 1024, 4096, 64, 16
    case = workloads.linear_case("e2e", N, K, M, workloads.SIGMA_7B, 0, proj=9, calib_tokens=T)
    W, X, x = case.W, case.calib, case.x
    best, losses, s_gpu = awq.awq_search_scale(dev(W), dev(X), ALPHAS)
    best = int(host(best)[0])
    s = host(s_gpu)
    assert 0 < best < len(ALPHAS) - 1                       # an interior alpha wins on outlier data
    # quantize with that s: bit-exact with the oracle given the same s, with and without clipping
    assert_clip_bit_exact(awq, W, s)
    (codes, scales, zeros), (q, sc, zp) = assert_quantize_bit_exact(awq, W, s)
    Wdq = oracle.dequant(codes, scales, zeros)
    xs = oracle.apply_inv_scale(x, s)
    xs_gpu = awq.awq_apply_inv_scale(dev(x), dev(s))
    assert np.array_equal(host(xs_gpu).view(np.uint16), xs.view(np.uint16))
    for m in (1, M):
        y = host(awq.awq_w4a16_linear(xs_gpu[:m].contiguous(), q, sc, zp, N))
        err = oracle.norm_error(y, oracle.matmul(xs[:m], Wdq), xs[:m], Wdq)
        assert err.max() <= TOL
    # against the unquantized layer, on fresh tokens: the searched scale beats RTN clearly
    y_fp = oracle.matmul(x, W.astype(np.float32))

    def out_err(xx, triple):
        return float(np.sum((oracle.matmul(xx, oracle.dequant(*triple)) - y_fp) ** 2))

    e_awq = out_err(xs, (codes, scales, zeros))
    e_rtn = out_err(x, oracle.quantize(W, None))
    assert e_awq < 0.6 * e_rtn, (e_awq, e_rtn)
    e_rtn_clip = out_err(x, oracle.quantize_clip(W, None, CLIP_RATIOS)[:3])
    e_awq_clip = out_err(xs, oracle.quantize_clip(W, s, CLIP_RATIOS)[:3])
    assert e_rtn_clip < e_rtn
    Xs = oracle.apply_inv_scale(X, s)
    check_clip_on_activations(awq, W, s, Xs)
    qa, sa, za = awq.awq_quantize_pack_clip(dev(W), dev(s), CLIP_RATIOS, xs=dev(Xs))
    ca, sca, zca = (host(t) for t in awq.awq_unpack(qa, sa, za, N, K))
    e_awq_act = out_err(xs, (ca, sca, zca))
    assert e_awq_act < 0.95 * e_awq
    print(f"output error vs fp16 layer: RTN {e_rtn:.0f}, RTN+clip {e_rtn_clip:.0f}, "
          f"searched scale {e_awq:.0f}, +clip on weights {e_awq_clip:.0f}, "
          f"+clip on calibration rows {e_awq_act:.0f}")


@pytest.mark.parametrize("M,K", [(1, 4096), (16, 11008), (300, 1408), (3, 136), (2048, 4096)])
def test_rmsnorm_with_folded_inverse_scale(awq, M, K):
    """fp32 on the GPU against fp64 in the oracle, both rounded to fp16: at most one fp16 unit
    apart (2^-10 relative), and the result is what the linear layer is fed."""
    import oracle
    import workloads
    g = np.random.default_rng(90 + M)
    out = workloads.outlier_channels(K, 0, 0, 6) if K >= 1000 else np.array([3])
    x = workloads.activations(M, K, 0, 0, 6, workloads.ROLE_X, out)
    gamma = g.uniform(0.5, 1.5, size=K).astype(np.float16)
    s = g.uniform(0.5, 4.0, size=K).astype(np.float32)
    for sv in (s, None):
        ref = oracle.rmsnorm_inv_scale(x, gamma, sv, eps=1e-5).astype(np.float64)
        got = host(awq.awq_rmsnorm_inv_scale(dev(x), dev(gamma), None if sv is None else dev(sv), 1e-5))
        got = got.astype(np.float64)
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -10 + 1e-7)
        assert (got != ref).mean() < 0.02                      # roundings differ only rarely
    xin = dev(x)                                               # in place
    awq.awq_rmsnorm_inv_scale(xin, dev(gamma), dev(s), 1e-5, out=xin)
    assert np.all(np.abs(host(xin).astype(np.float64) - oracle.rmsnorm_inv_scale(x, gamma, s).astype(np.float64))
                  <= np.abs(oracle.rmsnorm_inv_scale(x, gamma, s).astype(np.float64)) * 2.0 ** -10 + 1e-7)


def test_silu_mul(awq):
    import oracle
    g = np.random.default_rng(400)
    for shape in ((1, 11008), (16, 11008), (300, 1408)):
        gate = (g.standard_normal(shape) * 3).astype(np.float16)
        up = g.standard_normal(shape).astype(np.float16)
        ref = oracle.silu_mul(gate, up).astype(np.float64)
        got = host(awq.awq_silu_mul(dev(gate), dev(up))).astype(np.float64)
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -10 + 1e-7)


def check_fused(awq, problems, M, norm=(), residual=(), in_place=(), scale=()):
    """One awq_w4a16_linear_fused_multi call over `problems` (as for check_multi).  Linears
    whose index is in `norm` run on the RMS-normalised input times seeded factors, those in
    `residual` add a seeded [M,N] tensor (those in `in_place` pass y itself as the residual).
    Expected values: the oracle's normalisation, then its matmul, then the addition in fp64."""
    import torch
    import oracle
    g = np.random.default_rng(500 + M)
    linears, expect = [], []
    for i, (xs, Wdq, gpu_packed, N) in enumerate(problems):
        K = xs.shape[1]
        h = xs[:M]
        y, cy = guarded(M * N * 2, torch.float16)
        y = y.view(M, N)
        d = dict(x=dev(h), qweight=gpu_packed[0], scales=gpu_packed[1], zeros=gpu_packed[2], y=y, N=N)
        x_eff = h
        if i in norm:
            w = g.uniform(0.25, 1.75, size=K).astype(np.float16)
            d["norm"], d["eps"] = dev(w), 1e-5
            x_eff = oracle.rmsnorm_inv_scale(h, w, None, 1e-5)
        elif i in scale:
            w = g.uniform(0.25, 1.75, size=K).astype(np.float16)
            d["scale"] = dev(w)
            x_eff = oracle.scale_columns(h, w)
        y_ref = oracle.matmul(x_eff, Wdq)
        if i in residual or i in in_place:
            res = (g.standard_normal((M, N)) * 2).astype(np.float16)
            if i in in_place:
                y.copy_(dev(res))
                d["residual"] = y
            else:
                d["residual"] = dev(res)
            y_ref = y_ref + res.astype(np.float64)
        linears.append(d)
        expect.append((x_eff, Wdq, y_ref, y, cy, N))
    awq.awq_w4a16_linear_fused_multi(linears)
    for x_eff, Wdq, y_ref, y, cy, N in expect:
        cy()
        yh = host(y)
        assert np.all(np.isfinite(yh.astype(np.float32)))
        err = oracle.norm_error(yh, y_ref, x_eff, Wdq)
        den = np.linalg.norm(x_eff.astype(np.float64), axis=1)[:, None] * np.abs(Wdq).max() + 1e-6
        # the output is rounded once to fp16 at the magnitude of residual + sum
        allowed = TOL + 2.0 ** -11 * np.abs(y_ref) / den
        assert np.all(err <= allowed), f"max normalised error {err.max():.3e} (N={N}, M={M})"


@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 8, 16])
def test_fused_norm_and_residual_small(awq, small_group, M):
    """K = 1408 (ragged groups), 2048 and 512: one wave or several along K depending on M."""
    fits = [awq.awq_w4a16_linear_fused_fits(N, xs.shape[1], M) for xs, Wdq, gpu, N in small_group]
    assert fits == ([True] * 4 if M < 16 else [False, False, True, True])   # 11 groups over 4 waves: no
    group = [p for p, f in zip(small_group, fits) if f]
    group = group if len(group) == 4 else group * 2
    check_fused(awq, group, M, norm=(0, 2), residual=(1, 2), in_place=(3,))
    check_fused(awq, group, M, norm=(0, 1, 2, 3))
    check_fused(awq, group, M, norm=(0,), scale=(1, 3), residual=(3,))
    check_fused(awq, group, M)                                         # nothing fused: plain grouped call
    check_fused(awq, group[:1], M, norm=(0,), in_place=(0,))


def test_fused_llama7b_layer_full_size(awq):
    """The two launches of a decoder layer that carry fused operators: Q, K, V behind the
    normalisation; gate, up behind the normalisation; o and down with the residual in place."""
    probs = {}
    for N, K in [(4096, 4096), (11008, 4096), (4096, 11008)]:
        case, s, xs16, ref, gpu, Wdq = config_case(awq, N, K, 0.02, 1)
        probs[(N, K)] = (xs16, Wdq, gpu, N)
    for M in (1, 4):
        check_fused(awq, [probs[(4096, 4096)]] * 3, M, norm=(0, 1, 2))
        check_fused(awq, [probs[(11008, 4096)]] * 2, M, norm=(0, 1))
        check_fused(awq, [probs[(4096, 4096)]], M, in_place=(0,))
        check_fused(awq, [probs[(4096, 11008)]], M, in_place=(0,))
    check_fused(awq, [probs[(4096, 4096)]] * 3, 16, norm=(0, 1, 2))


def test_fused_rejects_what_it_cannot_run(awq, small_group):
    import torch
    xs, Wdq, gpu, N = small_group[0]
    y = torch.empty((1, N), dtype=torch.float16, device="cuda")
    base = dict(x=dev(xs[:1]), qweight=gpu[0], scales=gpu[1], zeros=gpu[2], y=y, N=N)
    with pytest.raises(ValueError):
        awq.prepare_linear_fused_multi([base] * 25)
    with pytest.raises(ValueError):
        awq.prepare_linear_fused_multi([dict(base, norm=dev(np.ones(7, np.float16)))])
    # K = 11008 at M = 16 does not fit the register-resident activations of the streaming kernel
    case, s, xs16, ref, gpu2, Wdq2 = config_case(awq, 4096, 11008, 0.02, 1)
    y2 = torch.empty((16, 4096), dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.awq_w4a16_linear_fused_multi([dict(x=dev(xs16), qweight=gpu2[0], scales=gpu2[1], zeros=gpu2[2],
                                               y=y2, N=4096, norm=dev(np.ones(11008, np.float16)))])
    assert e.value.status == -2
    # ... but a lone linear with only a residual runs at every decode shape
    check_fused(awq, [(xs16, Wdq2, gpu2, 4096)], 16, in_place=(0,))
    check_fused(awq, [(xs16, Wdq2, gpu2, 4096)], 5, residual=(0,))


# ------------------------------------------------------------------- decode attention

ATT_TOL = 2e-3      # of max|v|: fp16 rounding of the output (2^-11) and fp32 sums / exponentials


@pytest.mark.parametrize("H,Hkv,pos,Lmax", [(32, 32, 0, 8), (32, 32, 5, 64), (8, 2, 63, 64), (32, 32, 256, 300),
                                            (64, 8, 1000, 1024), (32, 32, 2047, 2048), (4, 1, 2048, 4096)])
def test_decode_attention_against_the_oracle(awq, H, Hkv, pos, Lmax):
    import torch
    import oracle
    g = np.random.default_rng(200 + pos)
    D = 128
    q = g.standard_normal((H, D)).astype(np.float16)
    k = g.standard_normal((Hkv, D)).astype(np.float16)
    v = g.standard_normal((Hkv, D)).astype(np.float16)
    kc = np.zeros((Hkv, Lmax, D), np.float16)
    vc = np.zeros((Hkv, Lmax, D), np.float16)
    kc[:, :pos] = g.standard_normal((Hkv, pos, D)).astype(np.float16)
    vc[:, :pos] = g.standard_normal((Hkv, pos, D)).astype(np.float16)
    if pos > 10:
        kc[:, 3] *= 3                                   # a few sharp scores as well
    out_ref, kc_ref, vc_ref = oracle.decode_attention(q, k, v, kc, vc, pos)
    kc_gpu, vc_gpu = dev(kc), dev(vc)
    out_buf, check_out = guarded(H * D * 2, torch.float16)
    out_gpu = awq.awq_decode_attention(dev(q), dev(k), dev(v), kc_gpu, vc_gpu, pos, out=out_buf.view(H, D))
    check_out()
    out = host(out_gpu).astype(np.float64)
    assert np.all(np.isfinite(out))
    scale = np.abs(vc_ref[:, : pos + 1].astype(np.float64)).max()
    assert np.abs(out - out_ref.astype(np.float64)).max() <= ATT_TOL * scale
    # the caches: the value row exactly, the rotated key within one fp16 unit, nothing else touched
    kc_new, vc_new = host(kc_gpu), host(vc_gpu)
    assert np.array_equal(vc_new, vc_ref)
    assert np.array_equal(np.delete(kc_new, pos, axis=1), np.delete(kc_ref, pos, axis=1))
    a, b = kc_new[:, pos].astype(np.float64), kc_ref[:, pos].astype(np.float64)
    assert np.all(np.abs(a - b) <= np.abs(b) * 2.0 ** -10 + 1e-7)


def test_decode_attention_step_by_step_fills_the_cache(awq):
    """Twenty consecutive positions on one stream: every step sees the rows the earlier steps
    wrote; the last output and the final caches match the oracle run the same way."""
    import oracle
    g = np.random.default_rng(300)
    H, Hkv, D, Lmax = 16, 4, 128, 32
    kc, vc = np.zeros((Hkv, Lmax, D), np.float16), np.zeros((Hkv, Lmax, D), np.float16)
    kc_gpu, vc_gpu = dev(kc), dev(vc)
    for pos in range(20):
        q = g.standard_normal((H, D)).astype(np.float16)
        k = g.standard_normal((Hkv, D)).astype(np.float16)
        v = g.standard_normal((Hkv, D)).astype(np.float16)
        out_ref, kc, vc = oracle.decode_attention(q, k, v, kc, vc, pos)
        out = awq.awq_decode_attention(dev(q), dev(k), dev(v), kc_gpu, vc_gpu, pos)
    assert np.abs(host(out).astype(np.float64) - out_ref.astype(np.float64)).max() <= ATT_TOL * 4
    assert np.array_equal(host(vc_gpu), vc)
    assert np.all(np.abs(host(kc_gpu).astype(np.float64) - kc.astype(np.float64))
                  <= np.abs(kc.astype(np.float64)) * 2.0 ** -10 + 1e-7)


def test_decode_attention_rejects_bad_arguments(awq):
    import torch
    z = lambda *s: torch.zeros(s, dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.awq_decode_attention(z(8, 128), z(2, 128), z(2, 128), z(2, 16, 128), z(2, 16, 128), 16)
    assert e.value.status == -2                               # pos >= Lmax
    with pytest.raises(awq.AwqError) as e:
        awq.awq_decode_attention(z(6, 128), z(4, 128), z(4, 128), z(4, 16, 128), z(4, 16, 128), 0)
    assert e.value.status == -2                               # H % Hkv != 0
    with pytest.raises(awq.AwqError) as e:
        awq.awq_decode_attention(z(8, 64), z(2, 64), z(2, 64), z(2, 16, 64), z(2, 16, 64), 0)
    assert e.value.status == -2                               # D != 128
    with pytest.raises(awq.AwqError) as e:
        awq.awq_decode_attention(z(8, 128), z(2, 128), z(2, 128), z(2, 16, 128), z(2, 16, 128), 3,
                                 workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -5


def test_errors_surface_as_exceptions(awq):
    import torch
    W = torch.zeros((16, 100), dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.awq_quantize_pack(W)
    assert e.value.status == -2
