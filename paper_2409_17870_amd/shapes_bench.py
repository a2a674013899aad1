#!/usr/bin/env python3
"""Like-for-like rows against the paper's tables, and the ablation behind its Sec. 4.2 claim.

Run on an MI355X: ``python -m paper_2409_17870_amd.shapes_bench``.  Prints markdown.

1. GEMM-only times of the shapes of the paper's Table 1 (square MatMuls) and Table 2 (Llama-2-7B linear
   shapes at M = 1024) for W1A2 and W2A2, next to the latencies the paper prints for an RTX 3090.
2. Ablation for Sec. 4.2: the scheme the paper argues against, every 1-bit plane pair as a GEMM of its own
   whose 32-bit product goes to global memory, followed by a shift-and-add pass over those products,
   against the library's kernel, which keeps the recovery on chip.  The plane-pair GEMMs of the naive
   scheme use this library's own W1A1 kernel; the shift-and-add pass is plain PyTorch (it is the thing
   being argued against, not part of the product).

Inputs are random codes (integer GEMM time does not depend on the values).
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# paper Table 1 / Table 2, RTX 3090, microseconds
PAPER_US = {
    ("W1A2", 1024, 1024, 1024): 8.7, ("W1A2", 2048, 2048, 2048): 30.6, ("W1A2", 4096, 4096, 4096): 160.0,
    ("W2A2", 1024, 1024, 1024): 12.0, ("W2A2", 2048, 2048, 2048): 54.8, ("W2A2", 4096, 4096, 4096): 323.0,
    ("W1A2", 1024, 4096, 4096): 51.0, ("W1A2", 1024, 11008, 4096): 129.0, ("W1A2", 1024, 4096, 11008): 109.0,
    ("W2A2", 1024, 4096, 4096): 85.0, ("W2A2", 1024, 11008, 4096): 222.0, ("W2A2", 1024, 4096, 11008): 210.0,
}


def main():
    import torch
    from paper_2409_17870_amd import binding

    dev = torch.device("cuda:0")

    def timed(fn, iters):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    print("| scheme | M | N | K | this library, MI355X (us) | effective TOPS | paper, RTX 3090 (us) |")
    print("|---|---|---|---|---|---|---|")
    for (name, M, N, K), paper in PAPER_US.items():
        q, p = int(name[1]), int(name[3])
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        ap, wp = binding.apmm_pack_activations(a, p), binding.apmm_pack_weights(w, q)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        us = timed(lambda: binding.apmm_gemm(M, N, K, p, q, ap, wp, c_i32=c), 100)
        print("| %s | %d | %d | %d | %.1f | %.0f | %.1f |" % (name, M, N, K, us, 2.0 * M * N * K / us / 1e6, paper), flush=True)

    print()
    print("| scheme (4096^3) | fused kernel (us) | plane-pair GEMMs to global memory (us) | + shift-and-add pass (us) | naive total / fused |")
    print("|---|---|---|---|---|")
    M = N = K = 4096
    for (p, q) in ((2, 1), (2, 2), (4, 2)):
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        ap, wp = binding.apmm_pack_activations(a, p), binding.apmm_pack_weights(w, q)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        fused = timed(lambda: binding.apmm_gemm(M, N, K, p, q, ap, wp, c_i32=c), 50)
        a_planes = [binding.apmm_pack_activations(((a >> j) & 1).contiguous(), 1) for j in range(p)]
        w_planes = [binding.apmm_pack_weights(((w >> i) & 1).contiguous(), 1) for i in range(q)]
        d = [[torch.empty((M, N), dtype=torch.int32, device=dev) for _ in range(p)] for _ in range(q)]

        def pair_gemms():
            for i in range(q):
                for j in range(p):
                    binding.apmm_gemm(M, N, K, 1, 1, a_planes[j], w_planes[i], c_i32=d[i][j])

        def recover():
            out = torch.zeros((M, N), dtype=torch.int32, device=dev)
            for i in range(q):
                for j in range(p):
                    out.add_(d[i][j], alpha=1 << (i + j))
            return out

        pair_gemms()
        assert torch.equal(recover(), c), "the naive scheme must give the same result"
        t_pairs, t_rec = timed(pair_gemms, 10), timed(recover, 10)
        print("| W%dA%d | %.1f | %.1f | %.1f | %.1fx |" % (q, p, fused, t_pairs, t_rec, (t_pairs + t_rec) / fused), flush=True)


if __name__ == "__main__":
    main()
