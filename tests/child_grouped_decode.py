"""Run as a child process by test_gpu_parity.py with planner overrides in the environment (they
are read once per process): a compact parity check of the grouped decode call, 4-bit and 3-bit,
against the oracle.  Prints OK on success."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    import torch
    import oracle
    import workloads
    import paper_2306_00978_amd as awq
    awq.load()
    TOL = 2e-3
    shapes = [(176, 1408), (64, 1408), (48, 2048), (320, 512), (1024, 4096)]
    for bits in (4, 3):
        probs = []
        for i, (N, K) in enumerate(shapes):
            case = workloads.linear_case("child", N, K, 16, 0.02, 0, proj=30 + i)
            s = oracle.act_scale(case.calib, 0.5).astype(np.float32)
            xs = oracle.apply_inv_scale(case.x, s)
            if bits == 4:
                c, sc, z = oracle.quantize(case.W, s)
                q, sp, zp = oracle.pack(c, sc, z)
            else:
                c, sc, z = oracle.quantize_w3(case.W, s)
                q, sp, zp = oracle.pack_w3(c, sc, z)
            gpu = (torch.from_numpy(q).cuda(), torch.from_numpy(sp.view(np.float16)).cuda(),
                   torch.from_numpy(zp).cuda())
            probs.append((xs, oracle.dequant(c, sc, z), gpu, N))
        for M in (1, 2, 4, 7, 16):
            linears = [(torch.from_numpy(np.ascontiguousarray(xs[:M])).cuda(), *gpu,
                        torch.empty((M, N), dtype=torch.float16, device="cuda"), N)
                       for xs, Wdq, gpu, N in probs]
            (awq.awq_w4a16_linear_multi if bits == 4 else awq.awq_w3a16_linear_multi)(linears)
            torch.cuda.synchronize()
            for (xs, Wdq, gpu, N), lin in zip(probs, linears):
                y = lin[4].cpu().numpy()
                y_ref = oracle.matmul(xs[:M], Wdq)
                err = oracle.norm_error(y, y_ref, xs[:M], Wdq)
                assert np.all(np.isfinite(y.astype(np.float32))) and err.max() <= TOL, (bits, M, N, err.max())
                # the single call of the same linear (its kernel has overrides of its own)
                one = (awq.awq_w4a16_linear if bits == 4 else awq.awq_w3a16_linear)(lin[0], *gpu, N)
                err = oracle.norm_error(one.cpu().numpy(), y_ref, xs[:M], Wdq)
                assert err.max() <= TOL, ("single", bits, M, N, err.max())
    print("OK")


if __name__ == "__main__":
    main()
