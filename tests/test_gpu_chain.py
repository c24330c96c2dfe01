"""awq_w4a16_linear_chain: the linears of a decode step in the order of their data dependences, in
one launch whose workgroups wait (bounded) for the stage in front (Sec. 4.2, kernel fusion).

Every stage's outputs are compared with the oracle applied to the inputs that stage really had --
the fp16 outputs the GPU produced for the stages before -- at the tolerance of the linear; all
intermediate buffers hold NaN before the launch, so a stage that read its input before the stage
in front had written it cannot pass.  The give-up path is forced from the host (flag set before the
launch, or a spin limit of one poll): the kernel must end, say so in sync[0], and work again after
the sync area has been zeroed."""
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
    awq.load()
    return awq


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


class Lin:
    """One quantized linear N x K with seeded weights: packed arrays on the GPU, dequantized on the host."""

    def __init__(self, awq, N, K, seed, sigma=0.02):
        import oracle
        g = np.random.default_rng(seed)
        W = (g.standard_normal((N, K)) * sigma).astype(np.float16)
        codes, scales, zeros = oracle.quantize(W, None)
        q, s, z = oracle.pack(codes, scales, zeros)
        import torch
        self.N, self.K = N, K
        self.gpu = (dev(q), dev(s).view(torch.float16), dev(z))
        self.Wdq = oracle.dequant(codes, scales, zeros)


def nan_buffer(M, N):
    import torch
    return torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")


def desc(lin, x, y, **kw):
    return dict(x=x, qweight=lin.gpu[0], scales=lin.gpu[1], zeros=lin.gpu[2], y=y, N=lin.N, **kw)


def check_stage(lin, x_host, y_gpu, norm=None, residual=None):
    """y_gpu against the oracle on the inputs the stage had (x_host: fp16 array)."""
    import oracle
    x_eff = x_host if norm is None else oracle.rmsnorm_inv_scale(x_host, norm, None, 1e-5)
    y_ref = oracle.matmul(x_eff, lin.Wdq)
    if residual is not None:
        y_ref = y_ref + residual.astype(np.float64)
    yh = host(y_gpu)
    assert np.all(np.isfinite(yh.astype(np.float32))), "a stage left NaN: it ran on unwritten input"
    err = oracle.norm_error(yh, y_ref, x_eff, lin.Wdq)
    den = np.linalg.norm(x_eff.astype(np.float64), axis=1)[:, None] * np.abs(lin.Wdq).max() + 1e-6
    allowed = TOL + 2.0 ** -11 * np.abs(y_ref) / den          # one rounding at the magnitude of residual + sum
    assert np.all(err <= allowed), f"max normalised error {err.max():.3e}"
    return yh


def run_decoder_like_chain(awq, H, F, M, seed, repeats=1, spin_limit=0, sync=None, expect_ok=True):
    """{q,k,v} -> {o (+hidden in place)} -> {gate, up (RMS norm in front)} -> {down (+hidden in
    place)} on hidden size H and MLP width F; o reads v's output (attention is not part of it)."""
    import torch
    g = np.random.default_rng(seed)
    lq, lk, lv, lo = (Lin(awq, H, H, seed + i) for i in range(4))
    lg, lu = Lin(awq, F, H, seed + 4), Lin(awq, F, H, seed + 5)
    ld = Lin(awq, H, F, seed + 6)
    x0 = g.standard_normal((M, H)).astype(np.float16)
    hid0 = g.standard_normal((M, H)).astype(np.float16)
    wn = g.uniform(0.5, 1.5, size=H).astype(np.float16)
    x0d, wnd = dev(x0), dev(wn)
    sync = awq.chain_sync() if sync is None else sync
    last = None
    for rep in range(repeats):
        yq, yk, yv = nan_buffer(M, H), nan_buffer(M, H), nan_buffer(M, H)
        yg, yu = nan_buffer(M, F), nan_buffer(M, F)
        hid = dev(hid0)
        stages = [
            [desc(lq, x0d, yq), desc(lk, x0d, yk), desc(lv, x0d, yv)],
            [desc(lo, yv, hid, residual=hid)],
            [desc(lg, hid, yg, norm=wnd), desc(lu, hid, yu, norm=wnd)],
            [desc(ld, yg, hid, residual=hid)],
        ]
        # hid is read by stage 3 and rewritten by stage 4: keep stage 2's value for the check
        awq.prepare_linear_chain(stages[:3], sync, spin_limit=spin_limit)()
        torch.cuda.synchronize()
        if not expect_ok:
            return sync, (yq, yk, yv, yg, yu, hid)
        assert int(sync.cpu().abs().sum()) == 0, "the sync area must be zero again after a normal end"
        for lin, y in ((lq, yq), (lk, yk), (lv, yv)):
            check_stage(lin, x0, y)
        hid1 = check_stage(lo, host(yv), hid, residual=hid0)
        yg_h = check_stage(lg, hid1, yg, norm=wn)
        check_stage(lu, hid1, yu, norm=wn)
        # the whole chain of four stages from the start again: the last stage adds into hid
        yq.fill_(float("nan")); yk.fill_(float("nan")); yv.fill_(float("nan"))
        yg.fill_(float("nan")); yu.fill_(float("nan"))
        hid.copy_(dev(hid0))
        awq.prepare_linear_chain(stages, sync, spin_limit=spin_limit)()
        torch.cuda.synchronize()
        assert int(sync.cpu().abs().sum()) == 0
        assert np.array_equal(host(yg).view(np.uint16), yg_h.view(np.uint16)), "a chain is deterministic"
        final = check_stage(ld, yg_h, hid, residual=hid1)
        if last is not None:
            assert np.array_equal(final.view(np.uint16), last.view(np.uint16))
        last = final
    return sync, None


@pytest.mark.parametrize("M,F", [(1, 1408), (2, 1408), (4, 1408), (7, 1408), (8, 1408), (16, 1024)])
def test_chain_small_shapes_every_stage_against_the_oracle(awq, M, F):
    # F = 1408: a ragged group count (11); at M = 16 a wave holds one batch, so K = 1408 (three
    # batches) cannot be split evenly over its waves and the shape is not served: 1024 there
    run_decoder_like_chain(awq, H=512, F=F, M=M, seed=900 + M, repeats=2)


def test_chain_llama7b_layer_full_size(awq):
    """The four dependent stages of a Llama-2-7B-shaped layer (configs[1]) in one launch, M = 1 and 4,
    three launches in a row on one sync area."""
    run_decoder_like_chain(awq, H=4096, F=11008, M=1, seed=1000, repeats=3)
    run_decoder_like_chain(awq, H=4096, F=11008, M=4, seed=1001, repeats=1)


def test_chain_gives_up_when_told_to_and_works_again(awq):
    import torch
    # the give-up flag set before the launch: every wait ends at its first poll, the kernel ends,
    # later stages never run (their outputs keep the NaN), the flag stays set
    sync = awq.chain_sync()
    sync[0] = 1
    sync, bufs = run_decoder_like_chain(awq, H=512, F=1408, M=2, seed=77, sync=sync, expect_ok=False)
    yq, yk, yv, yg, yu, hid = bufs
    s = sync.cpu()
    assert int(s[0]) != 0
    assert bool(torch.isnan(yg).all()) and bool(torch.isnan(yu).all()), "stage 3 must not have run"
    assert bool(torch.isfinite(yq.float()).all()), "stage 1 waits for nothing and runs"
    # a spin limit of one poll: workgroups that arrive early give up; whatever happens the kernel
    # ends and reports it
    sync.zero_()
    sync, bufs = run_decoder_like_chain(awq, H=512, F=1408, M=2, seed=78, sync=sync, spin_limit=1, expect_ok=False)
    torch.cuda.synchronize()
    gave_up = int(sync.cpu()[0]) != 0
    if not gave_up:
        assert int(sync.cpu().abs().sum()) == 0
    # zeroed again, the same area serves a normal call
    sync.zero_()
    run_decoder_like_chain(awq, H=512, F=1408, M=2, seed=79, sync=sync)


def test_chain_refuses_what_it_cannot_run(awq):
    import torch
    lin = Lin(awq, 4096, 11008, 5)            # K = 11008 does not fit the register slots at M = 16
    x = torch.zeros((16, 11008), dtype=torch.float16, device="cuda")
    y = torch.zeros((16, 4096), dtype=torch.float16, device="cuda")
    with pytest.raises(awq.AwqError) as e:
        awq.prepare_linear_chain([[desc(lin, x, y)]], awq.chain_sync())()
    assert e.value.status == -2
    with pytest.raises(ValueError):
        awq.prepare_linear_chain([[desc(lin, x[:1], y[:1])]] * 5, awq.chain_sync())
