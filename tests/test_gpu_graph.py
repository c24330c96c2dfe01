"""The launches of the library recorded into a HIP graph (through torch's capture) and replayed:
every replay must give the eager result bit for bit, with eager work and synchronisations between
the replays.  The library allocates nothing and clears nothing, so a captured call consists of its
kernels only."""
import numpy as np
import pytest

from test_gpu_parity import awq, dev, host, make_case  # noqa: F401  (awq is a fixture)

pytestmark = pytest.mark.gpu


def replay_and_compare(torch, run, outputs, disturb):
    """run(): the calls under test, writing `outputs`.  Eager first (also settles one-time kernel
    attributes), then captured, then three replays with other work in between."""
    run()
    torch.cuda.synchronize()
    want = [o.clone() for o in outputs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                        # warm-up on the capture stream's side
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for r in range(3):
        for o in outputs:
            o.fill_(float("nan"))
        disturb()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, w in zip(outputs, want):
            assert torch.equal(o.view(torch.int16), w.view(torch.int16)), f"replay {r} differs from the eager result"


def test_graph_replay_of_decode_prefill_and_low_bit_calls(awq):
    import torch
    import oracle
    N, K = 1024, 2048
    case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=70)
    W, sd = dev(case.W), dev(s)
    p4 = awq.awq_quantize_pack(W, sd)
    p3 = awq.awq_quantize_pack_w3(W, sd)
    p2 = awq.awq_quantize_pack_w2(W, sd)
    g = np.random.default_rng(70)
    x1, x16 = dev(xs[:1]), dev(xs)
    xbig = dev((np.tile(xs, (13, 1))[:200].astype(np.float32) * g.uniform(0.5, 1.5, size=(200, 1))).astype(np.float16))
    scratch = torch.empty(1 << 22, dtype=torch.float32, device="cuda")

    def disturb():                                   # eager work of the program between replays
        scratch.normal_()
        awq.awq_w4a16_linear(x16, *p4, N)

    # grouped decode, 4-bit / 3-bit / 2-bit, three linears each (the streaming kernels, M = 1)
    ys = [torch.empty((1, N), dtype=torch.float16, device="cuda") for _ in range(9)]
    c4 = awq.prepare_linear_multi([(x1, *p4, ys[i], N) for i in range(3)])
    c3 = awq.prepare_linear_multi_w3([(x1, *p3, ys[3 + i], N) for i in range(3)])
    c2 = awq.prepare_linear_multi_w2([(x1, *p2, ys[6 + i], N) for i in range(3)])
    replay_and_compare(torch, lambda: (c4(), c3(), c2()), ys, disturb)
    Wdq = oracle.dequant(*oracle.quantize(case.W, s))
    err = oracle.norm_error(host(ys[0]), oracle.matmul(xs[:1], Wdq), xs[:1], Wdq)
    assert err.max() <= 2e-3

    # single linears at 16 rows (batch kernels) and a prefill of 200 rows with K cut into ranges
    # (two kernels, the workspace brought by the caller)
    need = awq.awq_linear_workspace_bytes(200, N, K)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    y16 = torch.empty((16, N), dtype=torch.float16, device="cuda")
    y16_2 = torch.empty((16, N), dtype=torch.float16, device="cuda")
    ybig = torch.empty((200, N), dtype=torch.float16, device="cuda")

    def run():
        awq.awq_w4a16_linear(x16, *p4, N, out=y16)
        awq.awq_w2a16_linear(x16, *p2, N, out=y16_2)
        awq.awq_w4a16_linear(xbig, *p4, N, out=ybig, workspace=ws)
    replay_and_compare(torch, run, [y16, y16_2, ybig], disturb)
    xb = host(xbig)
    err = oracle.norm_error(host(ybig), oracle.matmul(xb, Wdq), xb, Wdq)
    assert err.max() <= 2e-3


def test_calls_on_two_streams_do_not_share_anything(awq):
    """The library keeps no scratch of its own: calls issued on two streams at the same time give
    the results of the same calls issued one after the other."""
    import torch
    cases = []
    for i, (N, K) in enumerate([(2048, 2048), (1024, 4096)]):
        case, s, xs = make_case(N, K, 16, 0.02, cfg=0, proj=80 + i)
        W, sd = dev(case.W), dev(s)
        cases.append((N, K, dev(xs), awq.awq_quantize_pack(W, sd), awq.awq_quantize_pack_w2(W, sd)))

    def work(c, outs):
        N, K, x, p4, p2 = c
        for rep in range(6):
            awq.awq_w4a16_linear_multi([(x[:1], *p4, outs[0], N), (x[:1], *p4, outs[1], N)])
            awq.awq_w4a16_linear(x, *p4, N, out=outs[2])
            awq.awq_w2a16_linear(x[:4], *p2, N, out=outs[3])

    def fresh(c):
        N = c[0]
        return [torch.zeros((m, N), dtype=torch.float16, device="cuda") for m in (1, 1, 16, 4)]

    want = []
    for c in cases:
        o = fresh(c)
        work(c, o)
        torch.cuda.synchronize()
        want.append(o)
    got = [fresh(c) for c in cases]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for c, o, st in zip(cases, got, streams):
        with torch.cuda.stream(st):
            work(c, o)
    torch.cuda.synchronize()
    for w, g_ in zip(want, got):
        for a, b in zip(w, g_):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))
